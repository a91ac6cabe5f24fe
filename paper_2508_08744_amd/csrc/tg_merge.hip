// Merge of a local index into the global neighbour lists (section 6.1: every node belongs to
// its closest clusters, each cluster gets a local index, and a node's list becomes
// merge(list so far, its list in the local index)).  The paper merges on the CPU because two
// indexes would not fit a 24 GB card beside the construction; 288 GB of HBM hold both.
//
// One wave per node of the local index.  Its global row (one entry per lane) and its local
// row, ids translated to global numbering through the cluster's id table, go into an id map
// in LDS that keeps for every id the first entry that brought it (global entries come first);
// the survivors of both rows are sorted as (distance, id) keys with the wave's bitonic network,
// merged, and the first k are written back.  Rows shorter than k end in id -1, distance +inf.
#include "tg_device.h"
#include "tg_kernels.h"

#define MERGE_MAP_WORDS 256          // at most 128 ids per node
#define MERGE_FREE 0xFFFFFFFFu
#define MERGE_GRID 16384

__device__ inline u32 merge_map_insert(u32* keys, u32* owner, u32 id, u32 entry, bool active)
{
    bool pending = active;
    u32 h = (id * 0x9E3779B1u) >> 24;
    while (__ballot(pending)) {
        if (pending) {
            const u32 old = atomicCAS(keys + h, MERGE_FREE, id);
            if (old == MERGE_FREE || old == id) { atomicMin(owner + h, entry); pending = false; }
            else h = (h + 1) & (MERGE_MAP_WORDS - 1);
        }
    }
    return h;
}

// the keys that are not empty move to the front, order kept (tmp: 64 words of 8 bytes private to the wave)
__device__ inline u64 merge_close_up(u64 key, u64* tmp, int lane)
{
    const bool has = key != TG_EMPTY_KEY;
    const u64 mask = __ballot(has);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (has) tmp[__popcll(mask & tg_lanemask_lt())] = key;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return lane < __popcll(mask) ? tmp[lane] : TG_EMPTY_KEY;
}
// true when the keys ascend across the wave (uniform)
__device__ inline bool merge_ascending(u64 key, int lane)
{
    const u64 prev = tg_shfl64(key, lane > 0 ? lane - 1 : 0);
    return __ballot(lane > 0 && prev > key) == 0ull;
}

__global__ __launch_bounds__(256) void merge_local_kernel(int32_t* __restrict__ g_ids, float* __restrict__ g_dist, int64_t n, int k,
                                                          const int32_t* __restrict__ l_ids, const float* __restrict__ l_dist,
                                                          int64_t n_local, int k_local, const int32_t* __restrict__ l2g)
{
    __shared__ __align__(16) u32 s_keys[4][MERGE_MAP_WORDS];
    __shared__ u32 s_owner[4][MERGE_MAP_WORDS];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    u32* keys = s_keys[wave];
    u32* owner = s_owner[wave];
    for (int64_t i = (int64_t)blockIdx.x * 4 + wave; i < n_local; i += (int64_t)gridDim.x * 4) {
        const int64_t v = l2g[i];
        if (v < 0 || v >= n) continue;                       // a node without a global row (uniform over the wave)
        for (int j = lane; j < MERGE_MAP_WORDS; j += 64) { keys[j] = MERGE_FREE; owner[j] = 0xFFFFFFFFu; }
        const int32_t a_id = lane < k ? g_ids[v * k + lane] : -1;
        const float a_dist = lane < k ? g_dist[v * k + lane] : 0.f;
        const int32_t c = lane < k_local ? l_ids[i * k_local + lane] : -1;
        const float b_dist = lane < k_local ? l_dist[i * k_local + lane] : 0.f;
        const int32_t b_id = (c >= 0 && c < n_local) ? l2g[c] : -1;
        const bool a_ok = a_id >= 0 && a_id < n && a_id != v;
        const bool b_ok = b_id >= 0 && b_id < n && b_id != v;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // an id counts once: the first entry that brought it, global entries in front of local ones
        const u32 ha = merge_map_insert(keys, owner, (u32)a_id, (u32)lane, a_ok);
        const u32 hb = merge_map_insert(keys, owner, (u32)b_id, 64u + (u32)lane, b_ok);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const bool a_in = a_ok && owner[ha] == (u32)lane;
        const bool b_in = b_ok && owner[hb] == 64u + (u32)lane;
        u64 ka = a_in ? tg_key(a_dist, (u32)a_id, 0u) : TG_EMPTY_KEY;
        u64 kb = b_in ? tg_key(b_dist, (u32)b_id, 0u) : TG_EMPTY_KEY;
        // Rows that tg_knn_build wrote are ascending already; an entry that fell out above leaves a
        // gap.  Closing the gaps (through the map's words, free again by now) keeps the order, and a
        // row whose neighbours in lanes are then in order needs no sorting network.
        ka = merge_close_up(ka, reinterpret_cast<u64*>(keys), lane);
        kb = merge_close_up(kb, reinterpret_cast<u64*>(keys) + 64, lane);
        if (!merge_ascending(ka, lane)) ka = tg_wave_sort(ka);
        if (!merge_ascending(kb, lane)) kb = tg_wave_sort(kb);
        const u64 m = tg_wave_merge_low(ka, kb);
        if (lane < k) {
            const bool none = m == TG_EMPTY_KEY;
            g_ids[v * k + lane] = none ? -1 : (int32_t)tg_key_id(m);
            g_dist[v * k + lane] = none ? __builtin_inff() : tg_key_dist(m);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

void tg_launch_merge_local(int32_t* g_ids, float* g_dist, int64_t n, int k, const int32_t* l_ids, const float* l_dist,
                           int64_t n_local, int k_local, const int32_t* l2g, hipStream_t s)
{
    if (n_local == 0) return;
    int64_t wgs = (n_local + 3) / 4;
    if (wgs > MERGE_GRID) wgs = MERGE_GRID;
    hipLaunchKernelGGL(merge_local_kernel, dim3((unsigned)wgs), dim3(256), 0, s, g_ids, g_dist, n, k, l_ids, l_dist, n_local,
                       k_local, l2g);
}
