// Phase-1 sampling (step (1) of section 3.1.1): forward samples are read straight from
// the lists (first S new and first S old entries in list order); this file builds the
// bounded reverse samples.  Every sampled edge v -> u is numbered at u (one atomic add, done
// by the kernel that wrote the list where possible), a prefix sum turns the counts into
// segments, the edges are stored at their numbers inside the segments, and the wave
// that owns node u keeps, per class, the R arrivals with the smallest
// (hash(round, source, u), source): a uniform subset that does not depend on arrival order.
// The same wave then assembles the anchor's block and stores it for the join.
#include "tg_device.h"
#include "tg_kernels.h"

// ---- walk over the sampled edges: each group of KP lanes (KP = power of two >= k) owns one list
template <class F>
__device__ inline void for_each_sampled_edge(const TgGraph& g, int S, int kp, int64_t v0, F f)
{
    const int lane = tg_lane();
    const int per_wave = 64 / kp;
    const int64_t wave_id = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int sub = lane & (kp - 1), grp = lane / kp;
    const int64_t v = v0 + wave_id * per_wave + grp;
    const bool live = v < g.n && sub < g.k;
    u32 w = live ? g.gid[v * g.k + sub] : 0u;
    const bool fresh = live && (w >> 31);
    const bool old = live && !(w >> 31);
    const u64 gmask = (kp == 64 ? ~0ull : ((1ull << kp) - 1ull)) << (grp * kp);
    const u64 below = tg_lanemask_lt() & gmask;
    const u64 mf = __ballot(fresh), mo = __ballot(old);
    const bool take_new = fresh && __popcll(mf & below) < S;
    const bool take_old = old && __popcll(mo & below) < S;
    if (take_new || take_old) f((u32)v, w & TG_ID_MASK, take_old ? 1u : 0u);
}

// Arrival numbers: every sampled edge v -> u takes the next number at u (deg[u] counts the
// arrivals) and remembers it in epos, so that the scatter below needs no second atomic.  The
// kernels that write the lists (initial lists, list update) number the edges of the lists they
// have just written in the same way; this kernel serves the cases where that has not happened.
__global__ __launch_bounds__(256) void rev_count_kernel(TgGraph g, int S, int kp, u32* deg, u32* epos, int64_t v0)
{
    const int sub = tg_lane() & (kp - 1);
    for_each_sampled_edge(g, S, kp, v0, [&](u32 v, u32 u, u32) { epos[(int64_t)v * g.k + sub] = atomicAdd(deg + u, 1u); });
}

// edge v -> u with arrival number a goes to csr[off[u] + a]
__global__ __launch_bounds__(256) void rev_fill_kernel(TgGraph g, int S, int kp, const u32* __restrict__ epos,
                                                       const u64* __restrict__ off, u32* __restrict__ csr, int64_t v0)
{
    const int sub = tg_lane() & (kp - 1);
    for_each_sampled_edge(g, S, kp, v0, [&](u32 v, u32 u, u32 cls) {
        csr[off[u] + epos[(int64_t)v * g.k + sub]] = v | (cls << 31);
    });
}

// ---- exclusive prefix sum of deg[0..n) into off[0..n], three passes -------------------------
#define SCAN_BLOCK 1024   // elements per workgroup (256 threads x 4)

__global__ __launch_bounds__(256) void scan_partial_kernel(const u32* deg, int64_t n, u64* block_sums)
{
    __shared__ u64 red[4];
    int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK + threadIdx.x * 4;
    u64 s = 0;
    for (int i = 0; i < 4; ++i) if (base + i < n) s += deg[base + i];
    for (int o = 32; o > 0; o >>= 1) s += tg_shfl_xor64(s, o);
    if (tg_lane() == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
// one workgroup scans the block sums in place (exclusive), and writes the grand total to off[n]
__global__ __launch_bounds__(256) void scan_sums_kernel(u64* block_sums, int64_t nblocks, u64* off_total)
{
    __shared__ u64 carry_s;
    __shared__ u64 wsum[4];
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < nblocks; base += 256) {
        int64_t i = base + threadIdx.x;
        u64 x = i < nblocks ? block_sums[i] : 0;
        u64 incl = x;
        for (int o = 1; o < 64; o <<= 1) {
            u64 y = tg_shfl64(incl, max(tg_lane() - o, 0));
            if (tg_lane() >= o) incl += y;
        }
        if (tg_lane() == 63) wsum[threadIdx.x >> 6] = incl;
        __syncthreads();
        u64 pre = carry_s;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) pre += wsum[w];
        if (i < nblocks) block_sums[i] = pre + incl - x;
        __syncthreads();
        if (threadIdx.x == 255) carry_s = pre + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) *off_total = carry_s;
}
__global__ __launch_bounds__(256) void scan_final_kernel(u32* deg, int64_t n, const u64* block_sums, u64* off)
{
    __shared__ u64 wsum[4];
    int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK + threadIdx.x * 4;
    u32 x[4];
    u64 s = 0;
    for (int i = 0; i < 4; ++i) { x[i] = base + i < n ? deg[base + i] : 0u; s += x[i]; }
    u64 incl = s;
    for (int o = 1; o < 64; o <<= 1) {
        u64 y = tg_shfl64(incl, max(tg_lane() - o, 0));
        if (tg_lane() >= o) incl += y;
    }
    if (tg_lane() == 63) wsum[threadIdx.x >> 6] = incl;
    __syncthreads();
    u64 pre = block_sums[blockIdx.x];
    for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) pre += wsum[w];
    u64 run = pre + incl - s;
    for (int i = 0; i < 4; ++i) {
        if (base + i < n) {
            off[base + i] = run;
            deg[base + i] = 0u;     // counted anew for the next round
        }
        run += x[i];
    }
}
size_t tg_scan_tmp_elems(int64_t n) { return (size_t)((n + SCAN_BLOCK - 1) / SCAN_BLOCK) + 1; }

// ---- per node: keep the R smallest (priority, source) of each class, then assemble the block --
// Block of anchor v:  NEW = new_fwd ++ (new_rev not yet there),
//                     OLD = (old_fwd not in NEW) ++ (old_rev in neither).
// fwd entries sit one per lane (lanes < k), rn / ro are the kept reverse arrivals, ascending
// by (priority, source), one per lane (lanes < cn / co).
// A small id -> tag map in LDS for the cross checks between the forward and the reverse samples
// (open addressing, 256 words for at most 64 ids; ids inside one list are distinct).
#define ASM_WORDS 256
#define ASM_FREE 0xFFFFFFFFu
__device__ inline int asm_insert(u32* keys, u32 id, bool active)
{
    int slot = -1;
    bool pending = active;
    u32 h = (id * 0x9E3779B1u) >> 24;
    while (__ballot(pending)) {
        if (pending) {
            const u32 old = atomicCAS(keys + h, ASM_FREE, id);
            if (old == ASM_FREE) { slot = (int)h; pending = false; }
            else h = (h + 1) & (ASM_WORDS - 1);
        }
    }
    return slot;
}
__device__ inline int asm_find(const u32* keys, u32 id, bool active)
{
    int slot = -1;
    bool pending = active;
    u32 h = (id * 0x9E3779B1u) >> 24;
    while (__ballot(pending)) {
        if (pending) {
            const u32 t = keys[h];
            if (t == id) { slot = (int)h; pending = false; }
            else if (t == ASM_FREE) pending = false;
            else h = (h + 1) & (ASM_WORDS - 1);
        }
    }
    return slot;
}
__device__ inline void assemble_block(const TgGraph& g, const TgSample& sm, int64_t v, u32 rn, int cn, u32 ro, int co,
                                      u32* keys, u32* tags)
{
    const int lane = tg_lane();
    const int k = g.k, S = sm.S;
    const u64 lt = tg_lanemask_lt();
    const u32 w = lane < k ? g.gid[v * k + lane] : 0u;
    const bool fr = lane < k && (w >> 31);
    const bool ol = lane < k && !(w >> 31);
    const u64 mf = __ballot(fr), mo = __ballot(ol);
    const bool is_nf = fr && __popcll(mf & lt) < S;     // sampled new forward entry
    const bool is_of = ol && __popcll(mo & lt) < S;     // sampled old forward entry
    const u32 fid = w & TG_ID_MASK;
    const u64 m_nf = __ballot(is_nf);
    // forward samples into the map: tag 1 = new, 2 = old (4 is added when a reverse-new arrival repeats it)
    for (int i = lane; i < ASM_WORDS; i += 64) keys[i] = ASM_FREE;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int fslot = asm_insert(keys, fid, is_nf || is_of);
    if (fslot >= 0) tags[fslot] = is_nf ? 1u : 2u;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int sn = asm_find(keys, rn, lane < cn);
    const int so = asm_find(keys, ro, lane < co);
    const u32 tn = sn >= 0 ? tags[sn] : 0u;
    const bool rn_dup = tn == 1u;                       // already there as a new forward sample
    const bool ro_dup = so >= 0;                        // already there as a forward sample of either class
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (tn == 2u) tags[sn] = 6u;                        // the old forward sample is NEW through the reverse side
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const bool of_drop = is_of && (tags[fslot >= 0 ? fslot : 0] & 4u);
    const bool keep_rn = lane < cn && !rn_dup;
    const bool keep_of = is_of && !of_drop;
    const bool keep_ro = lane < co && !ro_dup;
    const u64 m_krn = __ballot(keep_rn), m_kof = __ballot(keep_of), m_kro = __ballot(keep_ro);
    const int n_nf = __popcll(m_nf);
    const int nN = n_nf + __popcll(m_krn);
    const int n_kof = __popcll(m_kof);
    const int nT = nN + n_kof + __popcll(m_kro);
    u32* ids = sm.blk + v * (int64_t)sm.BC;
    if (is_nf) ids[__popcll(m_nf & lt)] = fid;
    if (keep_rn) ids[n_nf + __popcll(m_krn & lt)] = rn;
    if (keep_of) ids[nN + __popcll(m_kof & lt)] = fid;
    if (keep_ro) ids[nN + n_kof + __popcll(m_kro & lt)] = ro;
    if (lane == 0) sm.bsz[v] = (u32)nN | ((u32)nT << 8);
}

__global__ __launch_bounds__(256) void rev_select_kernel(TgGraph g, TgSample sm, u64 hs_rev, int64_t v0)
{
    __shared__ u64 part[4][2][64];
    __shared__ u32 asm_keys[4][ASM_WORDS], asm_tags[4][ASM_WORDS];
    const int lane = tg_lane(), wave = threadIdx.x >> 6;
    const int64_t u = v0 + (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (u >= g.n) return;
    const u64 beg = sm.off[u], end = sm.off[u + 1];
    const u64 lt = tg_lanemask_lt();
    u64 best_new = TG_EMPTY_KEY, best_old = TG_EMPTY_KEY;   // ascending across the wave
    int tot_new = 0, tot_old = 0;
    for (u64 base = beg; base < end; base += 64) {
        // key = priority | class << 31 | source: one sort orders both classes; the class bit sits
        // below the priority, so inside a class the order is (priority, source)
        u64 key = TG_EMPTY_KEY;
        if (base + lane < end) {
            const u32 e = sm.csr[base + lane];
            const u32 v = e & TG_ID_MASK;
            key = (tg_hash_xy(hs_rev, (u64)v, (u64)u) & 0xFFFFFFFF00000000ull) | (u64)e;
        }
        key = tg_wave_sort(key);
        const bool is_old = key != TG_EMPTY_KEY && (((u32)key) >> 31);
        const bool is_new = key != TG_EMPTY_KEY && !(((u32)key) >> 31);
        const u64 mn = __ballot(is_new), mo = __ballot(is_old);
        const int cn = __popcll(mn), co = __popcll(mo);
        // split into two ascending runs through LDS
        if (is_new) part[wave][0][__popcll(mn & lt)] = key;
        if (is_old) part[wave][1][__popcll(mo & lt)] = key & ~0x80000000ull;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const u64 kn = lane < cn ? part[wave][0][lane] : TG_EMPTY_KEY;
        const u64 ko = lane < co ? part[wave][1][lane] : TG_EMPTY_KEY;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (base == beg) {
            best_new = kn;
            best_old = ko;
        } else {
            if (cn) best_new = tg_wave_merge_low(best_new, kn);
            if (co) best_old = tg_wave_merge_low(best_old, ko);
        }
        tot_new += cn;
        tot_old += co;
    }
    assemble_block(g, sm, u, (u32)best_new, min(tot_new, sm.R), (u32)best_old, min(tot_old, sm.R), asm_keys[wave], asm_tags[wave]);
}

// blocks as stored -> the boundary's fixed n x 128 layout (padding -1) and (|NEW|, |OLD|)
__global__ void dump_blocks_kernel(TgGraph g, TgSample sm, int32_t* blk, int32_t* sizes)
{
    size_t total = (size_t)g.n * TG_BLOCK_COLS;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < total; i += stride) {
        const size_t v = i / TG_BLOCK_COLS;
        const int c = (int)(i % TG_BLOCK_COLS);
        const u32 z = sm.bsz[v];
        const int nN = (int)(z & 0xFFu), nT = (int)(z >> 8);
        blk[i] = c < nT ? (int32_t)sm.blk[v * sm.BC + c] : -1;
        if (c == 0) { sizes[v * 2] = nN; sizes[v * 2 + 1] = nT - nN; }
    }
}
void tg_launch_dump_blocks(const TgGraph& g, const TgSample& sm, int32_t* blk, int32_t* sizes, hipStream_t s)
{
    size_t total = (size_t)g.n * TG_BLOCK_COLS;
    size_t grid = (total + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL(dump_blocks_kernel, dim3((unsigned)grid), dim3(256), 0, s, g, sm, blk, sizes);
}

void tg_launch_reverse(const TgGraph& g, const TgSample& sm, uint64_t hs_rev, bool counted, hipStream_t s)
{
    int kp = 1;
    while (kp < g.k) kp <<= 1;
    const int per_wave = 64 / kp;
    auto edge_blocks = [&](int64_t cnt) { return dim3((unsigned)(((cnt + per_wave - 1) / per_wave + 3) / 4)); };
    const int64_t nsb = (g.n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    if (!counted)
        tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
            hipLaunchKernelGGL(rev_count_kernel, edge_blocks(cnt), dim3(256), 0, s, g, sm.S, kp, sm.deg, g.gid_next, v0);
        });
    hipLaunchKernelGGL(scan_partial_kernel, dim3((unsigned)nsb), dim3(256), 0, s, sm.deg, g.n, sm.scan_tmp);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, s, sm.scan_tmp, nsb, sm.off + g.n);
    hipLaunchKernelGGL(scan_final_kernel, dim3((unsigned)nsb), dim3(256), 0, s, sm.deg, g.n, sm.scan_tmp, sm.off);
    tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
        hipLaunchKernelGGL(rev_fill_kernel, edge_blocks(cnt), dim3(256), 0, s, g, sm.S, kp, (const u32*)g.gid_next, (const u64*)sm.off,
                           sm.csr, v0);
    });
    tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
        hipLaunchKernelGGL(rev_select_kernel, dim3((unsigned)((cnt + 3) / 4)), dim3(256), 0, s, g, sm, hs_rev, v0);
    });
}
