// Phase-1 local join (section 4.2, first part): one workgroup per anchor v.
//   1. one wave assembles the anchor's block from the shared samples:
//        NEW = new_fwd ++ (new_rev not yet there), OLD = (old_fwd not in NEW) ++ (old_rev in neither)
//   2. the block's vectors are gathered into LDS, a slab of DK columns at a time;
//   3. the Gram tile NEW x (NEW ++ OLD) is accumulated with v_mfma_f32_16x16x4_f32 and turned
//      into distances |x|^2 + |y|^2 - 2<x,y>  (or -<x,y>, or 1 - cos);
//   4. retention: for every row node and column-tile group, and every column node and row-tile
//      group, the closest partner under the target's threshold is kept (the paper keeps one per
//      node and warp sub-tile) and handed to the target's candidate slots by atomic minimum.
// Only pairs (a,b) with a NEW and position a < b are used, so every new-new and new-old
// pair counts once and old-old pairs never.
#include "tg_device.h"
#include "tg_kernels.h"

#define JOIN_THREADS 256
#define JOIN_HDR_BYTES 3104   // kth[128] u64, hA[128] u64, ids[128], aux[128], sizes[4]  (16-byte multiple)

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// Block assembly by one full wave.  ids: LDS int[128]; sizes: LDS int[2] = (|NEW|, |NEW|+|OLD|).
// ---------------------------------------------------------------------------------------
__device__ inline void build_block(const TgGraph& g, const TgSample& sm, int64_t v, int* ids, int* sizes)
{
    const int lane = tg_lane();
    const int k = g.k, S = sm.S, R = sm.R;
    const u64 lt = tg_lanemask_lt();
    const u32 w = lane < k ? g.gid[v * k + lane] : 0u;
    const bool fr = lane < k && (w >> 31);
    const bool ol = lane < k && !(w >> 31);
    const u64 mf = __ballot(fr), mo = __ballot(ol);
    const bool is_nf = fr && __popcll(mf & lt) < S;     // sampled new forward entry
    const bool is_of = ol && __popcll(mo & lt) < S;     // sampled old forward entry
    const u32 fid = w & TG_ID_MASK;
    const int cn = sm.cnt_new[v], co = sm.cnt_old[v];
    const u32 rn = lane < cn ? sm.rev_new[v * R + lane] : 0xFFFFFFFFu;
    const u32 ro = lane < co ? sm.rev_old[v * R + lane] : 0xFFFFFFFFu;
    const u64 m_nf = __ballot(is_nf), m_of = __ballot(is_of);
    bool rn_dup = false, ro_dup = false, of_drop = false;
    for (int q = 0; q < k; ++q) {
        const u32 f = (u32)__builtin_amdgcn_readlane((int)fid, q);
        if ((m_nf >> q) & 1ull) { rn_dup |= (rn == f); ro_dup |= (ro == f); }
        else if ((m_of >> q) & 1ull) ro_dup |= (ro == f);
    }
    for (int q = 0; q < cn; ++q) of_drop |= (fid == (u32)__builtin_amdgcn_readlane((int)rn, q));
    const bool keep_rn = lane < cn && !rn_dup;
    const bool keep_of = is_of && !of_drop;
    const bool keep_ro = lane < co && !ro_dup;
    const u64 m_krn = __ballot(keep_rn), m_kof = __ballot(keep_of), m_kro = __ballot(keep_ro);
    const int n_nf = __popcll(m_nf);
    const int nN = n_nf + __popcll(m_krn);
    const int n_kof = __popcll(m_kof);
    const int nT = nN + n_kof + __popcll(m_kro);
    if (is_nf) ids[__popcll(m_nf & lt)] = (int)fid;
    if (keep_rn) ids[n_nf + __popcll(m_krn & lt)] = (int)rn;
    if (keep_of) ids[nN + __popcll(m_kof & lt)] = (int)fid;
    if (keep_ro) ids[nN + n_kof + __popcll(m_kro & lt)] = (int)ro;
    if (lane == 0) { sizes[0] = nN; sizes[1] = nT; }
}

__global__ __launch_bounds__(256) void dump_blocks_kernel(TgGraph g, TgSample sm, int32_t* blk, int32_t* sizes)
{
    __shared__ int s_ids[4][TG_BLOCK_COLS];
    __shared__ int s_sz[4][2];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int64_t v = (int64_t)blockIdx.x * 4 + wave;
    if (v >= g.n) return;
    build_block(g, sm, v, s_ids[wave], s_sz[wave]);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int nT = s_sz[wave][1];
    for (int i = lane; i < TG_BLOCK_COLS; i += 64) blk[v * TG_BLOCK_COLS + i] = i < nT ? s_ids[wave][i] : -1;
    if (lane == 0) { sizes[v * 2] = s_sz[wave][0]; sizes[v * 2 + 1] = nT - s_sz[wave][0]; }
}
void tg_launch_dump_blocks(const TgGraph& g, const TgSample& sm, int32_t* blk, int32_t* sizes, hipStream_t s)
{
    hipLaunchKernelGGL(dump_blocks_kernel, dim3((unsigned)((g.n + 3) / 4)), dim3(256), 0, s, g, sm, blk, sizes);
}

// ---------------------------------------------------------------------------------------
__device__ inline u64 rowmin16(u64 x)
{
    x = tg_min64(x, tg_shfl_xor64(x, 1));
    x = tg_min64(x, tg_shfl_xor64(x, 2));
    x = tg_min64(x, tg_shfl_xor64(x, 4));
    x = tg_min64(x, tg_shfl_xor64(x, 8));
    return x;
}

__device__ inline void emit_candidate(const TgCand& cd, const int* s_ids, const u64* s_hA, int tpos, u64 key)
{
    const u32 t = (u32)s_ids[tpos];
    const u32 c = tg_key_id(key);
    const u32 slot = (u32)(tg_mix64(s_hA[tpos] + (u64)c) >> 32) & (u32)(cd.C - 1);
    atomicMin(cd.slots + (int64_t)t * cd.C + slot, key);
}

// MODE 0: emit candidates.  MODE 1: write the distance tile of caller-given blocks.
template <int DK, int NGR, int NGC, int MODE>
__global__ __launch_bounds__(JOIN_THREADS) void join_kernel(TgGraph g, TgSample sm, TgCand cd, u64 hs_slot,
                                                            u64* stat_bins, const int32_t* xblk,
                                                            const int32_t* xsizes, float* xout)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    u64* s_kth = reinterpret_cast<u64*>(smem_raw);
    u64* s_hA = s_kth + TG_BLOCK_COLS;
    int* s_ids = reinterpret_cast<int*>(s_hA + TG_BLOCK_COLS);
    float* s_aux = reinterpret_cast<float*>(s_ids + TG_BLOCK_COLS);
    int* s_sz = reinterpret_cast<int*>(s_aux + TG_BLOCK_COLS);
    float* tile = reinterpret_cast<float*>(smem_raw + JOIN_HDR_BYTES);
    constexpr int LDT = DK + 4;          // LDS row stride in floats (16-byte pad against bank conflicts)

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t v = blockIdx.x;
    if (MODE == 0) {
        if (wave == 0) build_block(g, sm, v, s_ids, s_sz);
    } else {
        if (tid < TG_BLOCK_COLS) s_ids[tid] = xblk[v * TG_BLOCK_COLS + tid];
        if (tid == 0) { s_sz[0] = xsizes[v * 2]; s_sz[1] = xsizes[v * 2] + xsizes[v * 2 + 1]; }
    }
    __syncthreads();
    const int nN = s_sz[0], nT = s_sz[1];
    if (nN == 0 || nT < 2) return;
    if (tid < nT) {
        const int id = s_ids[tid];
        s_aux[tid] = g.metric == 2 ? g.rnorm[id] : g.nrm[id];
        if (MODE == 0) {
            s_kth[tid] = g.kth[id];
            s_hA[tid] = tg_mix64(hs_slot + (u64)id);
        }
    }
    if (MODE == 0 && stat_bins && tid == 0) {
        const u64 pairs = (u64)nN * (u64)(nN - 1) / 2 + (u64)nN * (u64)(nT - nN);
        atomicAdd(stat_bins + (blockIdx.x & (TG_STAT_BINS - 1)), pairs);
        atomicAdd(stat_bins + TG_STAT_BINS + (blockIdx.x & (TG_STAT_BINS - 1)), (u64)nT);
    }

    const int MT = (nN + 15) >> 4, NT = (nT + 15) >> 4;
    const int wr = wave & 1, wc = wave >> 1;
    const int g4 = lane >> 4, c16 = lane & 15;
    // this wave's tiles: rows {wr, wr+2}, columns {wc, wc+2, wc+4, wc+6}; a tile is needed
    // when it lies inside the block and is not strictly below the diagonal
    bool act[2][4];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) {
            const int i = wr + 2 * ti, j = wc + 2 * tj;
            act[ti][tj] = i < MT && j < NT && j >= i;
        }
    floatx4 acc[2][4];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) acc[ti][tj] = (floatx4){0.f, 0.f, 0.f, 0.f};

    constexpr int F4 = DK / 4;
    for (int ks = 0; ks < g.ld; ks += DK) {
        __syncthreads();
        const int total = nT * F4;
        for (int e = tid; e < total; e += JOIN_THREADS) {
            const int row = e / F4, c4 = e % F4;
            const int col = ks + c4 * 4;
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col < g.ld) val = *reinterpret_cast<const float4*>(g.X + (int64_t)s_ids[row] * g.ld + col);
            *reinterpret_cast<float4*>(tile + row * LDT + c4 * 4) = val;
        }
        __syncthreads();
        const int kend = min(DK, (g.ld - ks + 15) & ~15);
        // Lane (r, q) = (lane % 16, lane / 16) reads 4 consecutive columns 16*s + 4*q .. +3 of its
        // row; step t of the four MFMAs then contracts columns {16*s + 4*q + t : q = 0..3}.  The
        // same column permutation is applied to both operands, so the sum is the full dot product.
        for (int kk = 0; kk < kend; kk += 16) {
            float4 av[2], bv[4];
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
                if (wr + 2 * ti < MT) av[ti] = *reinterpret_cast<const float4*>(tile + ((wr + 2 * ti) * 16 + c16) * LDT + kk + 4 * g4);
#pragma unroll
            for (int tj = 0; tj < 4; ++tj)
                if (wc + 2 * tj < NT) bv[tj] = *reinterpret_cast<const float4*>(tile + ((wc + 2 * tj) * 16 + c16) * LDT + kk + 4 * g4);
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                for (int tj = 0; tj < 4; ++tj)
                    if (act[ti][tj]) {
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].x, bv[tj].x, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].y, bv[tj].y, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].z, bv[tj].z, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].w, bv[tj].w, acc[ti][tj], 0, 0, 0);
                    }
        }
    }

    // ---- epilogue.  Accumulator element e of tile (i, j) in lane (c16, g4) is the pair
    // (row a = 16 i + 4 g4 + e, column b = 16 j + c16).
    u64 colbest[4][NGR / 2];
#pragma unroll
    for (int tj = 0; tj < 4; ++tj)
#pragma unroll
        for (int rg = 0; rg < NGR / 2; ++rg) colbest[tj][rg] = TG_EMPTY_KEY;

#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
        const int i = wr + 2 * ti;
        if (i >= MT) continue;
#pragma unroll
        for (int cg = 0; cg < NGC / 2; ++cg) {
            u64 best[4] = {TG_EMPTY_KEY, TG_EMPTY_KEY, TG_EMPTY_KEY, TG_EMPTY_KEY};
            bool any = false;
#pragma unroll
            for (int tj = 0; tj < 4; ++tj) {
                if ((tj & (NGC / 2 - 1)) != cg) continue;
                if (!act[ti][tj]) continue;
                any = true;
                const int b = 16 * (wc + 2 * tj) + c16;
                const bool b_ok = b < nT;
                const int bb = b_ok ? b : 0;
                const float aux_b = s_aux[bb];
                const u32 id_b = (u32)s_ids[bb];
                const u64 kth_b = MODE == 0 ? s_kth[bb] : 0ull;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int a = 16 * i + 4 * g4 + e;
                    const bool ok = b_ok && a < nN && b > a;
                    const int aa = a < nN ? a : 0;
                    const float gram = acc[ti][tj][e];
                    float dist;
                    if (g.metric == 0) dist = fmaxf(0.0f, fmaf(-2.0f, gram, s_aux[aa] + aux_b));
                    else if (g.metric == 1) dist = -gram;
                    else dist = 1.0f - gram * s_aux[aa] * aux_b;
                    if (MODE == 1) {
                        if (ok) xout[((int64_t)v * TG_BLOCK_ROWS + a) * TG_BLOCK_COLS + b] = dist;
                    } else {
                        const u64 hi = (u64)tg_ord(dist) << 32;
                        u64 kr = hi | (u64)((id_b << 2) | 3u);
                        u64 kc = hi | (u64)(((u32)s_ids[aa] << 2) | 3u);
                        if (!ok || kr >= s_kth[aa]) kr = TG_EMPTY_KEY;
                        if (!ok || kc >= kth_b) kc = TG_EMPTY_KEY;
                        best[e] = tg_min64(best[e], kr);
                        colbest[tj][ti & (NGR / 2 - 1)] = tg_min64(colbest[tj][ti & (NGR / 2 - 1)], kc);
                    }
                }
            }
            if (MODE == 0 && any) {
#pragma unroll
                for (int e = 0; e < 4; ++e) best[e] = rowmin16(best[e]);
                const u64 mine = c16 == 0 ? best[0] : c16 == 1 ? best[1] : c16 == 2 ? best[2] : best[3];
                const int a = 16 * i + 4 * g4 + c16;
                if (c16 < 4 && mine != TG_EMPTY_KEY) emit_candidate(cd, s_ids, s_hA, a, mine);
            }
        }
    }
    if (MODE == 0) {
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) {
            const int j = wc + 2 * tj;
            if (j >= NT) continue;
#pragma unroll
            for (int rg = 0; rg < NGR / 2; ++rg) {
                u64 x = colbest[tj][rg];
                x = tg_min64(x, tg_shfl_xor64(x, 16));
                x = tg_min64(x, tg_shfl_xor64(x, 32));
                const int b = 16 * j + c16;
                if (g4 == 0 && x != TG_EMPTY_KEY) emit_candidate(cd, s_ids, s_hA, b, x);
            }
        }
    }
}

static size_t join_lds_bytes(int DK) { return JOIN_HDR_BYTES + (size_t)TG_BLOCK_COLS * (DK + 4) * sizeof(float); }

// LDS beyond 64 KB per workgroup has to be asked for once per kernel
template <class K>
static void allow_large_lds(K kernel, size_t bytes)
{
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int DK, int NGR, int NGC>
static void launch_join_t(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, hipStream_t s)
{
    static bool once = (allow_large_lds(join_kernel<DK, NGR, NGC, 0>, join_lds_bytes(DK)), true);
    (void)once;
    hipLaunchKernelGGL((join_kernel<DK, NGR, NGC, 0>), dim3((unsigned)g.n), dim3(JOIN_THREADS), join_lds_bytes(DK), s,
                       g, sm, c, hs_slot, stat_bins, (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr);
}
template <int DK>
static void launch_join_dk(const TgGraph& g, const TgSample& sm, const TgCand& c, int ngr, int ngc, u64 hs_slot,
                           u64* stat_bins, hipStream_t s)
{
    if (ngr == 2 && ngc == 2) launch_join_t<DK, 2, 2>(g, sm, c, hs_slot, stat_bins, s);
    else if (ngr == 2 && ngc == 4) launch_join_t<DK, 2, 4>(g, sm, c, hs_slot, stat_bins, s);
    else if (ngr == 2 && ngc == 8) launch_join_t<DK, 2, 8>(g, sm, c, hs_slot, stat_bins, s);
    else if (ngr == 4 && ngc == 2) launch_join_t<DK, 4, 2>(g, sm, c, hs_slot, stat_bins, s);
    else if (ngr == 4 && ngc == 4) launch_join_t<DK, 4, 4>(g, sm, c, hs_slot, stat_bins, s);
    else launch_join_t<DK, 4, 8>(g, sm, c, hs_slot, stat_bins, s);
}
static int join_slab(int ld) { return ld <= 64 ? 64 : 128; }

void tg_launch_join(const TgGraph& g, const TgSample& sm, const TgCand& c, int ng_row, int ng_col, uint64_t hs_slot,
                    unsigned long long* stat_bins, hipStream_t s)
{
    if (join_slab(g.ld) == 64) launch_join_dk<64>(g, sm, c, ng_row, ng_col, hs_slot, stat_bins, s);
    else launch_join_dk<128>(g, sm, c, ng_row, ng_col, hs_slot, stat_bins, s);
}

void tg_launch_join_distances(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out,
                              hipStream_t s)
{
    TgSample sm = {};
    TgCand c = {};
    static bool once = (allow_large_lds(join_kernel<64, 2, 2, 1>, join_lds_bytes(64)),
                        allow_large_lds(join_kernel<128, 2, 2, 1>, join_lds_bytes(128)), true);
    (void)once;
    if (join_slab(g.ld) == 64)
        hipLaunchKernelGGL((join_kernel<64, 2, 2, 1>), dim3((unsigned)nb), dim3(JOIN_THREADS), join_lds_bytes(64), s, g, sm,
                           c, 0ull, (u64*)nullptr, blk, sizes, out);
    else
        hipLaunchKernelGGL((join_kernel<128, 2, 2, 1>), dim3((unsigned)nb), dim3(JOIN_THREADS), join_lds_bytes(128), s, g,
                           sm, c, 0ull, (u64*)nullptr, blk, sizes, out);
}
