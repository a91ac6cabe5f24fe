// Rank-based pruning of a k-NN graph by detourable routes (section 3.2, the CAGRA row of the
// table of pruning strategies; computing paradigm of section 5.2).  The position of a neighbour
// in a row stands for its distance.  For node A and its neighbour F at position p, a node D is
// a detour of the edge (A, F) when both its position in A's row and its position in F's row
// are below p; neighbours with more detours go first: the d_out neighbours with the smallest
// (count, position) stay.
//
// One wave per node A.  A's row goes into an id -> position map in LDS; the rows of the
// neighbours F are read 64 / k' at a time (k' = k rounded up to a power of two), one entry D
// per lane and only the entries in front of F's own position in A's row, and each lane looks
// its D up in the map.  A ballot per row gives the count.  Rows of different useful length are
// balanced as in the paper, by pairing positions q and k - 1 - q inside one group of lanes.
#include "tg_device.h"
#include "tg_kernels.h"

#define PRUNE_ENTRIES 256       // 128 buckets of two (id, position) entries for the at most 64 ids of a row
#define PRUNE_FREE 0xFFFFFFFFu
#define PRUNE_NOPOS 0xFFFFu
#define PRUNE_GRID 8192
#define PRUNE_PASSES 8

// What a lane does in pass t of a round of eight passes that starts at pair p0 depends only on the
// lane, t, p0 and k: which neighbour F of A it reads (the lane of A's row that holds F), which
// entry of F's row, and F's own position (0 when the lane has nothing to read: no position is
// below 0, so such a lane never reports a hit).
struct PruneLaneTable {
    int src[PRUNE_PASSES];      // byte address for ds_bpermute: 4 x (lane that holds F)
    int rr[PRUNE_PASSES];       // entry of F's row
    u32 jpos[PRUNE_PASSES];     // F's position in A's row, 0 if idle
};

__device__ inline void prune_fill_table(PruneLaneTable& T, int p0, int k, int kp, int per, int npairs, int my_row, int r)
{
#pragma unroll
    for (int t = 0; t < PRUNE_PASSES; ++t) {
        const int q = p0 + t * per + my_row;
        const int jlo = q, jhi = k - 1 - q;
        const bool lo = r < jlo;
        const int j = lo ? jlo : jhi;
        const int rr = lo ? r : r - jlo;
        const bool on = my_row < per && q < npairs && (lo || (jhi != jlo && rr < jhi));
        T.src[t] = on ? 4 * j : 0;
        T.rr[t] = on ? rr : 0;
        T.jpos[t] = on ? (u32)j : 0u;
    }
}

__global__ __launch_bounds__(256) void prune_rank_kernel(const int32_t* __restrict__ ids, int64_t n, int k, int kp, int d_out,
                                                         int32_t* __restrict__ out_ids, int32_t* __restrict__ counts)
{
    __shared__ __align__(16) u32 maps[4][2 * PRUNE_ENTRIES];      // entry e: word 2e = id, word 2e + 1 = position
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    u32* map = maps[wave];
    const int per = 64 / kp;                         // rows of neighbours per pass
    const int my_row = lane / kp, r = lane - my_row * kp;
    const int npairs = (k + 1) >> 1;
    const bool one_round = npairs <= PRUNE_PASSES * per;          // k <= 32: the table never changes
    PruneLaneTable T;
    prune_fill_table(T, 0, k, kp, per, npairs, my_row, r);
    // the count of position P = lane comes out of the pass that serves pair q = min(P, k - 1 - P):
    // in that pass's ballot its hits start at bit (row of the pair) x k' (+ q for the far partner), P bits long
    const int myq = min(lane, k - 1 - lane);
    const int lp = 31 - __clz(per);                  // per is a power of two
    const u32 n32 = (u32)n;                          // n < 2^30
    for (int64_t A = (int64_t)blockIdx.x * 4 + wave; A < n; A += (int64_t)gridDim.x * 4) {
        const int32_t a = lane < k ? ids[A * k + lane] : -1;
        const bool a_ok = (u32)a < n32;
        for (int i = lane; i < PRUNE_ENTRIES; i += 64) *reinterpret_cast<uint2*>(map + 2 * i) = make_uint2(PRUNE_FREE, PRUNE_NOPOS);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // A's row into the map (a bucket is read with one 16-byte load later); an id listed twice
        // keeps its first position
        {
            bool pending = a_ok;
            u32 e = (((u32)a * 0x9E3779B1u) >> 25) << 1;
            while (__ballot(pending)) {
                if (pending) {
                    const u32 old = atomicCAS(map + 2 * e, PRUNE_FREE, (u32)a);
                    if (old == PRUNE_FREE || old == (u32)a) { atomicMin(map + 2 * e + 1, (u32)lane); pending = false; }
                    else e = (e + 1) & (PRUNE_ENTRIES - 1);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // Rows are taken in pairs (positions q and k - 1 - q): the first needs its q entries in
        // front, the second k - 1 - q, together k - 1 lanes of a group of k' (the balanced
        // pairing of section 5.2).  64 / k' pairs per pass; the loads of eight passes are in
        // flight before the first look-up.
        u32 c = 0u;
        for (int p0 = 0; p0 < npairs; p0 += PRUNE_PASSES * per) {
            if (!one_round) prune_fill_table(T, p0, k, kp, per, npairs, my_row, r);
            int32_t D[PRUNE_PASSES];
#pragma unroll
            for (int t = 0; t < PRUNE_PASSES; ++t) {
                const int32_t F = __builtin_amdgcn_ds_bpermute(T.src[t], a);
                const bool scan = (T.jpos[t] != 0u) & ((u32)F < n32);        // one unsigned compare also rejects negative ids
                const int32_t got = ids[(u64)(u32)(scan ? F : 0) * (u32)k + (u32)T.rr[t]];      // row 0 when there is nothing to read
                D[t] = scan ? got : -1;
            }
            u64 mine = 0ull;                      // the ballot of the pass that serves this lane's position
#pragma unroll
            for (int t = 0; t < PRUNE_PASSES; ++t) {
                if (p0 + t * per >= npairs) break;           // uniform
                // look D up: its home bucket first (almost always decisive), then entry by entry.
                // -1 matches a free entry, whose position is below nothing.
                const u32 d = (u32)D[t];
                u32 e = ((d * 0x9E3779B1u) >> 25) << 1;
                const uint4 b = *reinterpret_cast<const uint4*>(map + 2 * e);
                // (no short cuts: every lane evaluates everything, nothing branches)
                const bool e0 = b.x == d, e1 = b.z == d;
                bool hit = (e0 & (b.y < T.jpos[t])) | (e1 & (b.w < T.jpos[t]));
                bool pending = !e0 & !e1 & (b.x != PRUNE_FREE) & (b.z != PRUNE_FREE);
                e = (e + 2) & (PRUNE_ENTRIES - 1);
                while (__ballot(pending)) {
                    if (pending) {
                        const uint2 w = *reinterpret_cast<const uint2*>(map + 2 * e);
                        if (w.x == d) { hit = w.y < T.jpos[t]; pending = false; }
                        else if (w.x == PRUNE_FREE) pending = false;
                        else e = (e + 1) & (PRUNE_ENTRIES - 1);
                    }
                }
                const u64 hits = __ballot(hit);
                if (((myq - p0) >> lp) == t) mine = hits;          // (a pair of an earlier round gives a negative number)
            }
            const int rel = myq - p0;
            if (lane < k && rel >= 0 && rel < PRUNE_PASSES * per) {
                const int row = rel & (per - 1);
                const int shift = row * kp + (lane == myq ? 0 : myq);       // the near partner's hits come first
                c = (u32)__popcll((mine >> shift) & ((1ull << lane) - 1ull));
            }
        }
        if (counts && lane < k) counts[A * k + lane] = (int32_t)c;
        // smallest (count, position) first
        u32 key = lane < k ? ((c << 8) | (u32)lane) : 0xFFFFFFFFu;
        key = tg_wave_sort32(key);
        const int32_t keep = __shfl(a, (int)(key & 63u));
        if (lane < d_out) out_ids[A * d_out + lane] = keep;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

void tg_launch_prune_rank(const int32_t* ids, int64_t n, int k, int d_out, int32_t* out_ids, int32_t* counts, hipStream_t s)
{
    int kp = 1;
    while (kp < k) kp <<= 1;
    int64_t wgs = (n + 3) / 4;
    if (wgs > PRUNE_GRID) wgs = PRUNE_GRID;
    hipLaunchKernelGGL(prune_rank_kernel, dim3((unsigned)wgs), dim3(256), 0, s, ids, n, k, kp, d_out, out_ids, counts);
}
