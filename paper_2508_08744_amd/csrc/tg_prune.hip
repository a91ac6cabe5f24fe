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

#define PRUNE_MAP_WORDS 256     // 128 buckets of two ids for the at most 64 ids of a row
#define PRUNE_FREE 0xFFFFFFFFu
#define PRUNE_GRID 8192

__global__ __launch_bounds__(256) void prune_rank_kernel(const int32_t* __restrict__ ids, int64_t n, int k, int kp, int d_out,
                                                         int32_t* __restrict__ out_ids, int32_t* __restrict__ counts)
{
    __shared__ u32 keys[4][PRUNE_MAP_WORDS];
    __shared__ u32 poss[4][PRUNE_MAP_WORDS];
    __shared__ u32 cnts[4][64];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    u32* mk = keys[wave];
    u32* mp = poss[wave];
    u32* mc = cnts[wave];
    const int per = 64 / kp;                         // rows of neighbours per pass
    const int my_row = lane / kp, r = lane - my_row * kp;
    for (int64_t A = (int64_t)blockIdx.x * 4 + wave; A < n; A += (int64_t)gridDim.x * 4) {
        const int32_t a = lane < k ? ids[A * k + lane] : -1;
        const bool a_ok = a >= 0 && a < n;
        for (int i = lane; i < PRUNE_MAP_WORDS; i += 64) { mk[i] = PRUNE_FREE; mp[i] = 0xFFFFu; }
        mc[lane] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // A's row into the map (buckets of two words, read with one 8-byte load later); an id
        // listed twice keeps its first position
        {
            bool pending = a_ok;
            u32 h = (((u32)a * 0x9E3779B1u) >> 25) << 1;
            while (__ballot(pending)) {
                if (pending) {
                    const u32 old = atomicCAS(mk + h, PRUNE_FREE, (u32)a);
                    if (old == PRUNE_FREE || old == (u32)a) { atomicMin(mp + h, (u32)lane); pending = false; }
                    else h = (h + 1) & (PRUNE_MAP_WORDS - 1);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // Rows are taken in pairs (positions q and k - 1 - q): the first needs its q entries in
        // front, the second k - 1 - q, together k - 1 lanes of a group of k' (the balanced
        // pairing of section 5.2).  64 / k' pairs per pass; the loads of eight passes are in
        // flight before the first look-up.
        const int npairs = (k + 1) >> 1;
        for (int p0 = 0; p0 < npairs; p0 += 8 * per) {
            int32_t D[8];
            int jj[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int q = p0 + t * per + my_row;
                const int jlo = q, jhi = k - 1 - q;
                const bool lo = r < jlo;
                const int j = lo ? jlo : jhi;
                const int rr = lo ? r : r - jlo;
                const bool on = my_row < per && q < npairs && (lo || (jhi != jlo && rr < jhi));
                const int32_t F = __shfl(a, on ? j : 0);
                const bool scan = on && F >= 0 && F < n;
                D[t] = scan ? ids[(int64_t)F * k + rr] : -1;
                jj[t] = j;
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int q = p0 + t * per + my_row;
                if (p0 + t * per >= npairs) break;           // uniform
                // look D up: its home bucket first (almost always decisive), then word by word
                const bool live = D[t] >= 0 && D[t] < n;
                u32 h = (((u32)D[t] * 0x9E3779B1u) >> 25) << 1;
                const uint2 b2 = *reinterpret_cast<const uint2*>(mk + h);
                bool hit = false;
                bool pending = false;
                if (live) {
                    if (b2.x == (u32)D[t]) hit = mp[h] < (u32)jj[t];
                    else if (b2.y == (u32)D[t]) hit = mp[h + 1] < (u32)jj[t];
                    else pending = b2.x != PRUNE_FREE && b2.y != PRUNE_FREE;
                }
                h = (h + 2) & (PRUNE_MAP_WORDS - 1);
                while (__ballot(pending)) {
                    if (pending) {
                        const u32 w = mk[h];
                        if (w == (u32)D[t]) { hit = mp[h] < (u32)jj[t]; pending = false; }
                        else if (w == PRUNE_FREE) pending = false;
                        else h = (h + 1) & (PRUNE_MAP_WORDS - 1);
                    }
                }
                const u64 hits = __ballot(hit);
                if (r == 0 && my_row < per && q < npairs) {
                    const int jlo = q, jhi = k - 1 - q;
                    const int base = my_row * kp;
                    const u64 mlo = jlo ? (((1ull << jlo) - 1ull) << base) : 0ull;
                    const u64 mhi = (jhi >= 64 ? ~0ull : ((1ull << jhi) - 1ull)) << (base + jlo);
                    mc[jlo] = (u32)__popcll(hits & mlo);
                    if (jhi != jlo) mc[jhi] = (u32)__popcll(hits & mhi);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const u32 c = lane < k ? mc[lane] : 0u;
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
