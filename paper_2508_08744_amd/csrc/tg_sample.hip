// Phase-1 sampling (step (1) of section 3.1.1): forward samples are read straight from
// the lists (first S new and first S old entries in list order); this file builds the
// bounded reverse samples.  The sampled edges v -> u are brought together by target in two
// steps that write runs, not single words: the targets are cut into buckets of 2^bshift
// consecutive nodes; a workgroup walks a chunk of lists, counts its edges per bucket in LDS,
// takes one run per bucket with one atomic and stores its edges there (bucket step); then one
// workgroup per bucket counts the bucket's edges per target in LDS, stores them grouped by target
// and, a wave per target, keeps per class the R arrivals with the smallest
// (hash(round, source, u), source): a uniform subset that does not depend on arrival order.
// The same wave then assembles the anchor's block and stores it for the join.
#include "tg_device.h"
#include "tg_kernels.h"

// ---- walk of a workgroup over the sampled edges of the lists [vbeg, vend): each group of KP lanes
// (KP = power of two >= k) owns one list at a time
template <class F>
__device__ inline void for_chunk_edges(const TgGraph& g, int S, int kp, int64_t vbeg, int64_t vend, F f)
{
    const int lane = tg_lane(), wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int per_wave = 64 / kp;
    const int sub = lane & (kp - 1), grp = lane / kp;
    const u64 gmask = (kp == 64 ? ~0ull : ((1ull << kp) - 1ull)) << (grp * kp);
    const u64 below = tg_lanemask_lt() & gmask;
    for (int64_t base = vbeg + (int64_t)wave * per_wave; base < vend; base += (int64_t)nwaves * per_wave) {
        const int64_t v = base + grp;
        const bool live = v < vend && sub < g.k;
        const u32 w = live ? g.gid[v * g.k + sub] : 0u;
        const bool fresh = live && (w >> 31);
        const bool old = live && !(w >> 31);
        const u64 mf = __ballot(fresh), mo = __ballot(old);
        const bool take_new = fresh && __popcll(mf & below) < S;
        const bool take_old = old && __popcll(mo & below) < S;
        if (take_new || take_old) f((u32)v, w & TG_ID_MASK, take_old ? 1u : 0u);
    }
}

// Bucket step.  Both kernels count the chunk's edges per bucket in LDS (buckets b0 .. b0 + nb of this launch;
// edges to other buckets belong to another launch).  The first adds the counts to bcnt; once a prefix sum has
// turned bcnt into the buckets' places (boff), the second takes its runs off bcnt again (which so ends at zero,
// ready for the next round) and stores every edge as target % 2^bshift << 32 | class << 31 | source.
#define REV_BUCKET_THREADS 1024      // many waves on one table of counters: the walk is a chain of dependent accesses
template <bool FILL>
__global__ __launch_bounds__(REV_BUCKET_THREADS) void rev_bucket_kernel(TgGraph g, int S, int kp, int bshift, int64_t b0, int nb, int64_t chunk,
                                                         u32* bcnt, const u64* __restrict__ boff, u64* __restrict__ ebuf)
{
    __shared__ u32 hist[TG_REV_BUCKETS];
    for (int i = threadIdx.x; i < nb; i += REV_BUCKET_THREADS) hist[i] = 0u;
    __syncthreads();
    const int64_t vbeg = (int64_t)blockIdx.x * chunk, vend = vbeg + chunk < g.n ? vbeg + chunk : g.n;
    for_chunk_edges(g, S, kp, vbeg, vend, [&](u32, u32 u, u32) {
        const int64_t b = (int64_t)(u >> bshift) - b0;
        if (b >= 0 && b < nb) atomicAdd(&hist[b], 1u);
    });
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += REV_BUCKET_THREADS) {
        const u32 c = hist[i];
        if (!FILL) {
            if (c) atomicAdd(bcnt + b0 + i, c);
        } else if (c) {
            hist[i] = atomicSub(bcnt + b0 + i, c) - c;       // where this workgroup's run begins inside the bucket
        }
    }
    if (!FILL) return;
    __syncthreads();
    const u32 tmask = (1u << bshift) - 1u;
    for_chunk_edges(g, S, kp, vbeg, vend, [&](u32 v, u32 u, u32 cls) {
        const int64_t b = (int64_t)(u >> bshift) - b0;
        if (b >= 0 && b < nb) {
            const u32 pos = atomicAdd(&hist[b], 1u);
            ebuf[boff[b0 + b] + pos] = ((u64)(u & tmask) << 32) | (u64)(v | (cls << 31));
        }
    });
}

// ---- exclusive prefix sum of cnt[0..n) into off[0..n], three passes (cnt stays) -------------------------
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
__global__ __launch_bounds__(256) void scan_final_kernel(const u32* deg, int64_t n, const u64* block_sums, u64* off)
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
        if (base + i < n) off[base + i] = run;
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
__device__ inline void assemble_block(const TgGraph& g, const TgSample& sm, int64_t v, u32 w /* list entry of lane < k */, u32 rn, int cn,
                                      u32 ro, int co, u32* keys, u32* tags)
{
    const int lane = tg_lane();
    const int k = g.k, S = sm.S;
    const u64 lt = tg_lanemask_lt();
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

// One workgroup per bucket: its edges are counted per target in LDS, stored grouped by target (csr, at the
// bucket's own place: one workgroup writes and reads it, so it stays in that workgroup's cache), and every
// target's arrivals are then cut down to its reverse samples by one wave, which also assembles its block.
__global__ __launch_bounds__(256) void rev_select_kernel(TgGraph g, TgSample sm, u64 hs_rev, int64_t bfirst)
{
    __shared__ u32 tpos[TG_REV_MAX_W];
    __shared__ u64 part[4][2][64];
    __shared__ u32 asm_keys[4][ASM_WORDS], asm_tags[4][ASM_WORDS];
    const int lane = tg_lane(), wave = threadIdx.x >> 6;
    const int64_t b = bfirst + blockIdx.x;
    if (b >= sm.nbuckets) return;
    const int W = 1 << sm.bshift;
    const u64 beg = sm.boff[b], end = sm.boff[b + 1];
    const u64* eb = sm.ebuf;
    for (int i = threadIdx.x; i < W; i += 256) tpos[i] = 0u;
    __syncthreads();
    for (u64 e0 = beg + threadIdx.x; e0 < end; e0 += 4 * 256) {       // four loads on their way at a time
        u64 rec[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rec[j] = e0 + 256 * j < end ? eb[e0 + 256 * j] : ~0ull;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + 256 * j < end) atomicAdd(&tpos[(u32)(rec[j] >> 32) & (u32)(W - 1)], 1u);
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive prefix sum over the W targets: a lane takes W / 64 neighbouring ones
        const int per = W >> 6;
        u32 sum = 0;
        for (int i = 0; i < per; ++i) sum += tpos[lane * per + i];
        u32 incl = sum;
        for (int o = 1; o < 64; o <<= 1) {
            const u32 y = (u32)__shfl((int)incl, max(lane - o, 0));
            if (lane >= o) incl += y;
        }
        u32 run = incl - sum;
        for (int i = 0; i < per; ++i) {
            const u32 c = tpos[lane * per + i];
            tpos[lane * per + i] = run;
            run += c;
        }
    }
    __syncthreads();
    for (u64 e0 = beg + threadIdx.x; e0 < end; e0 += 4 * 256) {
        u64 rec[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) rec[j] = e0 + 256 * j < end ? eb[e0 + 256 * j] : ~0ull;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e0 + 256 * j < end) {
                const u32 pos = atomicAdd(&tpos[(u32)(rec[j] >> 32) & (u32)(W - 1)], 1u);
                sm.csr[beg + pos] = (u32)rec[j];
            }
    }
    __syncthreads();          // (the stores above are waited for and seen by the whole workgroup)
    // now tpos[t] is where the arrivals of target t end, and those of t + 1 begin
    const u64 lt = tg_lanemask_lt();
    // a wave's targets one after the other; the first arrivals and the list of the next target travel while this one is worked on
    const int k = g.k;
    auto arrivals_of = [&](int t, u64& abeg, u64& aend) {
        abeg = beg + (t ? tpos[t - 1] : 0u);
        aend = beg + tpos[t];
    };
    auto target_ok = [&](int t) { return t < W && (b << sm.bshift) + t < g.n; };
    u64 abeg = 0, aend = 0;
    u32 e_first = 0u, w_list = 0u;
    if (target_ok(wave)) {
        arrivals_of(wave, abeg, aend);
        e_first = abeg + lane < aend ? sm.csr[abeg + lane] : 0u;
        w_list = lane < k ? g.gid[((b << sm.bshift) + wave) * k + lane] : 0u;
    }
    for (int t = wave; target_ok(t); t += 4) {
        const int64_t u = (b << sm.bshift) + t;
        u64 nbeg = 0, nend = 0;
        u32 e_next = 0u, w_next = 0u;
        if (target_ok(t + 4)) {
            arrivals_of(t + 4, nbeg, nend);
            e_next = nbeg + lane < nend ? sm.csr[nbeg + lane] : 0u;
            w_next = lane < k ? g.gid[(u + 4) * k + lane] : 0u;
        }
        u64 best_new = TG_EMPTY_KEY, best_old = TG_EMPTY_KEY;   // ascending across the wave
        int tot_new = 0, tot_old = 0;
        for (u64 base = abeg; base < aend; base += 64) {
            // key = priority | class << 31 | source: one sort orders both classes; the class bit sits
            // below the priority, so inside a class the order is (priority, source)
            u64 key = TG_EMPTY_KEY;
            if (base + lane < aend) {
                const u32 e = base == abeg ? e_first : sm.csr[base + lane];
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
            if (base == abeg) {
                best_new = kn;
                best_old = ko;
            } else {
                if (cn) best_new = tg_wave_merge_low(best_new, kn);
                if (co) best_old = tg_wave_merge_low(best_old, ko);
            }
            tot_new += cn;
            tot_old += co;
        }
        assemble_block(g, sm, u, w_list, (u32)best_new, min(tot_new, sm.R), (u32)best_old, min(tot_old, sm.R), asm_keys[wave], asm_tags[wave]);
        abeg = nbeg; aend = nend; e_first = e_next; w_list = w_next;
    }
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

void tg_launch_reverse(const TgGraph& g, const TgSample& sm, uint64_t hs_rev, hipStream_t s)
{
    int kp = 1;
    while (kp < g.k) kp <<= 1;
    const int per_step = (REV_BUCKET_THREADS / 64) * (64 / kp);   // lists a workgroup reads at a time
    // about 2^14 edges per workgroup (measured: many short walks beat long runs per bucket)
    int64_t chunk = (1 << 14) / g.k;
    chunk = (chunk + per_step - 1) / per_step * per_step;
    const unsigned grid = (unsigned)((g.n + chunk - 1) / chunk);
    for (int pass = 0; pass < 2; ++pass) {
        for (int64_t b0 = 0; b0 < sm.nbuckets; b0 += TG_REV_BUCKETS) {
            const int nb = (int)(sm.nbuckets - b0 < TG_REV_BUCKETS ? sm.nbuckets - b0 : TG_REV_BUCKETS);
            if (pass == 0)
                hipLaunchKernelGGL(rev_bucket_kernel<false>, dim3(grid), dim3(REV_BUCKET_THREADS), 0, s, g, sm.S, kp, sm.bshift, b0, nb, chunk, sm.bcnt,
                                   (const u64*)sm.boff, sm.ebuf);
            else
                hipLaunchKernelGGL(rev_bucket_kernel<true>, dim3(grid), dim3(REV_BUCKET_THREADS), 0, s, g, sm.S, kp, sm.bshift, b0, nb, chunk, sm.bcnt,
                                   (const u64*)sm.boff, sm.ebuf);
        }
        if (pass == 0) {
            const int64_t nsb = (sm.nbuckets + SCAN_BLOCK - 1) / SCAN_BLOCK;
            hipLaunchKernelGGL(scan_partial_kernel, dim3((unsigned)nsb), dim3(256), 0, s, sm.bcnt, sm.nbuckets, sm.scan_tmp);
            hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, s, sm.scan_tmp, nsb, sm.boff + sm.nbuckets);
            hipLaunchKernelGGL(scan_final_kernel, dim3((unsigned)nsb), dim3(256), 0, s, (const u32*)sm.bcnt, sm.nbuckets, sm.scan_tmp, sm.boff);
        }
    }
    for (int64_t bf = 0; bf < sm.nbuckets; bf += (1 << 20))
        hipLaunchKernelGGL(rev_select_kernel, dim3((unsigned)(sm.nbuckets - bf < (1 << 20) ? sm.nbuckets - bf : (1 << 20))), dim3(256), 0, s, g, sm,
                           hs_rev, bf);
}
// buckets of 2^shift targets: 128 (measured: the smaller the faster, down to there), more where the bucket step would otherwise
// need more than four launches, each of which reads every list
int tg_rev_bucket_shift(int64_t n)
{
    int sh = 7;
    while (sh < TG_REV_MAX_SHIFT && ((n + (1ll << sh) - 1) >> sh) > 4 * TG_REV_BUCKETS) ++sh;
    return sh;
}
