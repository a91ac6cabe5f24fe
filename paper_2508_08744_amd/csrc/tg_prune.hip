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
// its D up in the map.  A ballot per row gives the count.  The paper balances warps that scan
// rows of different useful length by pairing candidates; here a lane that has nothing to scan
// simply idles inside a wave that is busy with the other rows, and the kernel is bound by the
// gather of the rows (4 k^2 / 2 bytes per node), not by the scan.
#include "tg_device.h"
#include "tg_kernels.h"

#define PRUNE_MAP_WORDS 256     // more than twice the 64 ids of a row
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
        // A's row into the map; an id listed twice keeps its first position
        {
            bool pending = a_ok;
            u32 h = ((u32)a * 0x9E3779B1u) >> 24;
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
        for (int j0 = 0; j0 < k; j0 += per) {
            const int j = j0 + my_row;               // position (from 0) of this lane's F in A's row
            const int32_t F = __shfl(a, j < k ? j : 0);
            const bool scan = my_row < per && j < k && r < j && F >= 0 && F < n;
            const int32_t D = scan ? ids[(int64_t)F * k + r] : -1;
            bool pending = scan && D >= 0 && D < n, hit = false;
            u32 h = ((u32)D * 0x9E3779B1u) >> 24;
            while (__ballot(pending)) {
                if (pending) {
                    const u32 t = mk[h];
                    if (t == (u32)D) { hit = mp[h] < (u32)j; pending = false; }
                    else if (t == PRUNE_FREE) pending = false;
                    else h = (h + 1) & (PRUNE_MAP_WORDS - 1);
                }
            }
            const u64 hits = __ballot(hit);
            const u64 rowmask = (kp == 64 ? ~0ull : ((1ull << kp) - 1ull)) << (my_row * kp);
            if (r == 0 && my_row < per && j < k) mc[j] = (u32)__popcll(hits & rowmask);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const u32 c = lane < k ? mc[lane] : 0u;
        if (counts && lane < k) counts[A * k + lane] = (int32_t)c;
        // smallest (count, position) first
        u64 key = lane < k ? (((u64)c << 8) | (u64)lane) : TG_EMPTY_KEY;
        key = tg_wave_sort(key);
        const int32_t keep = __shfl(a, (int)(key & 63ull));
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
