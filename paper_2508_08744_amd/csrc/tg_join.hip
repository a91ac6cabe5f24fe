// Phase-1 local join (section 4.2, first part).  The sampling kernel has stored every
// anchor's block (NEW ids, then OLD ids).  Anchors are first sorted into work lists by block
// size; small blocks of low-dimensional data go to a register-resident one-wave-per-anchor
// kernel, the rest to a workgroup kernel that
//   2. gathers the block's vectors into LDS, a slab of DK columns at a time;
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
#define JOIN_HDR_BYTES 2560   // salt[128], kd[128], spare[128], ids[128], aux[128]
#define JOIN_CELL_BYTES (TG_BLOCK_COLS * 8 * 8)   // one cell per member and opponent group (workgroup kernel)

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------
// cross-lane helpers: rotations inside a row of 16 lanes are DPP operand modifiers (no LDS)
template <int N>
__device__ inline float ror16_f(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + N, 0xF, 0xF, false));
}
template <int N>
__device__ inline u32 ror16_u(u32 x)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + N, 0xF, 0xF, false);
}
#define TG_NO_ID 0x7FFFFFFFu
// minimum of (dist, id) pairs over the 16 lanes of a row; every lane gets the result
__device__ inline void rowmin16f(float& dist, u32& id)
{
    float m = dist;
    m = fminf(m, ror16_f<8>(m));
    m = fminf(m, ror16_f<4>(m));
    m = fminf(m, ror16_f<2>(m));
    m = fminf(m, ror16_f<1>(m));
    u32 c = dist == m ? id : TG_NO_ID;
    c = min(c, ror16_u<8>(c));
    c = min(c, ror16_u<4>(c));
    c = min(c, ror16_u<2>(c));
    c = min(c, ror16_u<1>(c));
    dist = m;
    id = c;
}
// the same on ordered distances (tg_ord: unsigned order = float order)
__device__ inline void rowmin16(u32& dist, u32& id)
{
    u32 m = dist;
    m = min(m, ror16_u<8>(m));
    m = min(m, ror16_u<4>(m));
    m = min(m, ror16_u<2>(m));
    m = min(m, ror16_u<1>(m));
    u32 c = dist == m ? id : TG_NO_ID;
    c = min(c, ror16_u<8>(c));
    c = min(c, ror16_u<4>(c));
    c = min(c, ror16_u<2>(c));
    c = min(c, ror16_u<1>(c));
    dist = m;
    id = c;
}
__device__ inline void pairmin(float& bd, u32& bi, float d, u32 i)
{
    const bool take = (d < bd) | ((d == bd) & (i < bi));
    bd = take ? d : bd;
    bi = take ? i : bi;
}
// Gram value -> distance.  aux = squared norms (L2) or inverse norms (cosine).
template <int METRIC>
__device__ inline float gram_to_dist(float gram, float aux_a, float aux_b)
{
    if (METRIC == 0) return fmaxf(0.0f, fmaf(-2.0f, gram, aux_a + aux_b));
    if (METRIC == 1) return -gram + 0.0f;
    return 1.0f - gram * (aux_a * aux_b) + 0.0f;   // symmetric in the two nodes, bit for bit
}
// May a candidate at this distance precede the target's last list entry, whose distance is kd?  The id of
// that entry is not looked at: a candidate at exactly kd with a larger id passes too, and the list update,
// which keeps the k smallest (distance, id), drops it again; nothing that belongs in the list is held back.
__device__ inline bool reaches(float dist, float kd)
{
    return dist <= kd;
}

// Candidate c of the member at block position tpos (node t), found by anchor v's block in
// partner group q < 8.  A (t, v) pair owns one 64-byte line of t's slot row, picked by a hash,
// and the candidate of group q goes to word (q + rotation) % 8 of it, where it stays if it is
// the smaller (dist, id): one 64-bit atomic minimum, no order dependence.  All candidates one
// block has for t share a line, so they can travel in one memory transaction.
__device__ inline void emit_candidate(const TgCand& cd, const int* s_ids, const u32* s_salt, int tpos, u64 key, u32 v, int q)
{
    const u32 t = (u32)s_ids[tpos];
    u32 h = (s_salt[tpos] + v) * 0x9E3779B1u;
    h ^= h >> 15;
    h *= 0x85EBCA77u;
    h ^= h >> 13;
    const u32 line = h >> (36 - __ffs(cd.C));        // C / 8 lines
    const u32 slot = line * 8u + ((u32)(q + (int)(h & 7u)) & 7u);
    atomicMin(cd.slots + (int64_t)t * cd.C + slot, key);
}

// MODE 0: emit candidates for the stored blocks.  MODE 1: write the distance tile of caller-given blocks.
// NARROW: the rows come from the fp16 copy; a slab then holds 2 DK columns in the same bytes, and a
// step of 32 columns is one v_mfma_f32_16x16x32_f16 per tile.
// ROWS: the most members a block may have here, 64 or 128.  Blocks of at most 64 members need half the
// registers for a slab on its way, so two slabs travel while a third is multiplied; with 128 it is one.
template <int DK, int NGR, int NGC, int MODE, bool NARROW = false, int ROWS = TG_BLOCK_COLS>
__global__ __launch_bounds__(JOIN_THREADS, ROWS <= 64 ? 3 : 2) void join_kernel(TgGraph g, TgSample sm, TgCand cd, u64 hs_slot,
                                                            u64* stat_bins, const int32_t* xblk,
                                                            const int32_t* xsizes, float* xout, const u64* wl,
                                                            const u32* wl_cnt, int64_t direct_count, int skip_le)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    u32* s_salt = reinterpret_cast<u32*>(smem_raw);                     // slot-hash salt of each member
    float* s_kd = reinterpret_cast<float*>(s_salt + TG_BLOCK_COLS);     // threshold: distance of the member's last entry
    int* s_ids = reinterpret_cast<int*>(s_kd + 2 * TG_BLOCK_COLS);     // (128 words behind the thresholds are spare)
    float* s_aux = reinterpret_cast<float*>(s_ids + TG_BLOCK_COLS);     // squared norm (or 1/|x| for cosine)
    u64* s_cell = reinterpret_cast<u64*>(smem_raw + JOIN_HDR_BYTES);   // candidates of the block in hand
    unsigned char* tile = smem_raw + JOIN_HDR_BYTES + JOIN_CELL_BYTES;
    constexpr int LDTB = 4 * DK + 16;    // LDS row stride in bytes (16-byte pad against bank conflicts)
    constexpr int F4 = DK / 4;           // 16-byte pieces per row and slab
    constexpr int ES = NARROW ? 2 : 4;   // bytes per value
    constexpr int CS = 4 * DK / ES;      // columns per slab
    const int ldx = NARROW ? g.ldh : g.ld;                                   // columns per stored row
    const unsigned char* xbase = NARROW ? reinterpret_cast<const unsigned char*>(g.Xh) : reinterpret_cast<const unsigned char*>(g.X);
    constexpr int PER = ROWS * F4 / JOIN_THREADS;            // float4 per thread and slab, at most
    constexpr int DEPTH = ROWS <= 64 ? 2 : 1;                // slabs on their way
    constexpr int TJ = ROWS / 32;                            // column tiles per wave

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (g.f16_ok && (*g.f16_ok != 0u) != NARROW) return;      // the other variant's turn
    const int64_t count = wl ? (int64_t)*wl_cnt : direct_count;
    if (MODE == 0) {
        for (int c = tid; c < TG_BLOCK_COLS * 8; c += JOIN_THREADS) s_cell[c] = TG_EMPTY_KEY;
    }
    for (int64_t w = blockIdx.x; w < count; w += gridDim.x) {
    const int64_t v = wl ? (int64_t)(u32)wl[w] : w;
    int nN, nT;
    const u32* bids;
    if (MODE == 0) {
        const u32 z = sm.bsz[v];
        nN = (int)(z & 0xFFu);
        nT = (int)(z >> 8);
        bids = sm.blk + v * (int64_t)sm.BC;
    } else {
        nN = xsizes[v * 2];
        nT = nN + xsizes[v * 2 + 1];
        bids = reinterpret_cast<const u32*>(xblk) + v * TG_BLOCK_COLS;
    }
    if (nN == 0 || nT < 2 || nT > ROWS || ((nT + 15) >> 4) <= skip_le) continue;      // (the lists never hold a larger block)
    __syncthreads();                       // the previous block's epilogue has left the LDS header

    // gather of one slab: global -> registers now, registers -> LDS once the tile is free.
    // A thread fetches the same column part of the same PER rows in every slab, so the row
    // addresses are formed once per block and the loads are unconditional (rows and columns
    // past the end read a valid address and are zeroed).
    float4 pre[DEPTH][PER];
    const int cpart = (tid % F4) * (16 / ES);          // first column of this thread's 16-byte piece
    const unsigned char* rp[PER];
    bool rv[PER];
#pragma unroll
    for (int it = 0; it < PER; ++it) {
        const int row = (tid + JOIN_THREADS * it) / F4;
        rv[it] = row < nT;
        rp[it] = xbase + ((int64_t)bids[rv[it] ? row : 0] * ldx + cpart) * ES;
    }
    auto issue = [&](int ks, float4 (&dst)[PER]) {
        const bool cv = ks + cpart < ldx;
        const int kso = cv ? ks : -cpart;
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const float4 val = *reinterpret_cast<const float4*>(rp[it] + (int64_t)kso * ES);
            dst[it] = (rv[it] & cv) ? val : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto commit = [&](const float4 (&src)[PER]) {
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const int e = tid + JOIN_THREADS * it;
            const int row = e / F4;
            if (row < nT) *reinterpret_cast<float4*>(tile + row * LDTB + (e % F4) * 16) = src[it];
        }
    };
    issue(0, pre[0]);
    if (DEPTH == 2 && CS < ldx) issue(CS, pre[DEPTH - 1]);

    if (tid < nT) {
        const int id = (int)bids[tid];
        s_ids[tid] = id;
        s_aux[tid] = (MODE == 0) ? __uint_as_float((u32)g.kth[id]) : (g.metric == 2 ? g.rnorm[id] : g.nrm[id]);
        if (MODE == 0) {
            const u64 kth = g.kth[id];                       // threshold distance and norm in one word
            s_kd[tid] = tg_unord((u32)(kth >> 32));
            s_salt[tid] = (u32)tg_mix64(hs_slot + (u64)id);
        }
    }
    if (MODE == 0 && stat_bins && tid == 0) {
        const u64 pairs = (u64)nN * (u64)(nN - 1) / 2 + (u64)nN * (u64)(nT - nN);
        atomicAdd(stat_bins + (v & (TG_STAT_BINS - 1)), pairs);
        atomicAdd(stat_bins + TG_STAT_BINS + (v & (TG_STAT_BINS - 1)), (u64)nT);
    }

    const int MT = (nN + 15) >> 4, NT = (nT + 15) >> 4;
    const int wr = wave & 1, wc = wave >> 1;
    const int g4 = lane >> 4, c16 = lane & 15;
    // this wave's tiles: rows {wr, wr+2}, columns {wc, wc+2, wc+4, wc+6} (the first two for blocks of at
    // most 64 members); a tile is needed when it lies inside the block and is not strictly below the diagonal
    bool act[2][TJ];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) {
            const int i = wr + 2 * ti, j = wc + 2 * tj;
            act[ti][tj] = i < MT && j < NT && j >= i;
        }
    floatx4 acc[2][TJ];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) acc[ti][tj] = (floatx4){0.f, 0.f, 0.f, 0.f};

    // one slab: its values go from the registers into the tile, the registers take the slab DEPTH further on
    // (which travels while the slabs before it are multiplied), the tile is multiplied
    auto slab = [&](int ks, float4 (&stage)[PER]) {
        __syncthreads();
        commit(stage);
        __syncthreads();
        if (ks + DEPTH * CS < ldx) issue(ks + DEPTH * CS, stage);
        if (NARROW) {
            // lane (r, q) reads the 8 consecutive columns 32 s + 8 q .. + 7 of its row: one matrix instruction per step
            const int kend = min(CS, ldx - ks);         // rows of the fp16 copy are whole steps, zero padded
            for (int kk = 0; kk < kend; kk += 32) {
                float4 av[2], bv[TJ];
#pragma unroll
                for (int ti = 0; ti < 2; ++ti)
                    if (wr + 2 * ti < MT) av[ti] = *reinterpret_cast<const float4*>(tile + ((wr + 2 * ti) * 16 + c16) * LDTB + (kk + 8 * g4) * 2);
#pragma unroll
                for (int tj = 0; tj < TJ; ++tj)
                    if (wc + 2 * tj < NT) bv[tj] = *reinterpret_cast<const float4*>(tile + ((wc + 2 * tj) * 16 + c16) * LDTB + (kk + 8 * g4) * 2);
#pragma unroll
                for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                    for (int tj = 0; tj < TJ; ++tj)
                        if (act[ti][tj])
                            acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, av[ti]),
                                                                                  __builtin_bit_cast(halfx8, bv[tj]), acc[ti][tj], 0, 0, 0);
            }
            return;
        }
        const int kend = min(DK, (g.ld - ks + 15) & ~15);
        // Lane (r, q) = (lane % 16, lane / 16) reads 4 consecutive columns 16*s + 4*q .. +3 of its
        // row; step t of the four MFMAs then contracts columns {16*s + 4*q + t : q = 0..3}.  The
        // same column permutation is applied to both operands, so the sum is the full dot product.
        for (int kk = 0; kk < kend; kk += 16) {
            float4 av[2], bv[TJ];
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
                if (wr + 2 * ti < MT) av[ti] = *reinterpret_cast<const float4*>(tile + ((wr + 2 * ti) * 16 + c16) * LDTB + (kk + 4 * g4) * 4);
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
                if (wc + 2 * tj < NT) bv[tj] = *reinterpret_cast<const float4*>(tile + ((wc + 2 * tj) * 16 + c16) * LDTB + (kk + 4 * g4) * 4);
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                for (int tj = 0; tj < TJ; ++tj)
                    if (act[ti][tj]) {
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].x, bv[tj].x, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].y, bv[tj].y, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].z, bv[tj].z, acc[ti][tj], 0, 0, 0);
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ti].w, bv[tj].w, acc[ti][tj], 0, 0, 0);
                    }
        }
    };
    for (int ks = 0; ks < ldx; ks += DEPTH * CS) {
        slab(ks, pre[0]);
        if (DEPTH == 2 && ks + CS < ldx) slab(ks + CS, pre[DEPTH - 1]);
    }

    // ---- epilogue.  Accumulator element e of tile (i, j) in lane (c16, g4) is the pair
    // (row a = 16 i + 4 g4 + e, column b = 16 j + c16).  "Empty" is (inf, TG_NO_ID).
    const float INF = __builtin_inff();
    float cbd[TJ][NGR / 2];
    u32 cbi[TJ][NGR / 2];
#pragma unroll
    for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
        for (int rg = 0; rg < NGR / 2; ++rg) { cbd[tj][rg] = INF; cbi[tj][rg] = TG_NO_ID; }

#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
        const int i = wr + 2 * ti;
        if (i >= MT) continue;
        // per-lane row data for e = 0..3
        float aux_a[4], kd_a[4];
        u32 id_a[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int a = 16 * i + 4 * g4 + e;
            const int aa = a < nN ? a : 0;
            aux_a[e] = s_aux[aa];
            id_a[e] = (u32)s_ids[aa];
            if (MODE == 0) kd_a[e] = s_kd[aa];
        }
#pragma unroll
        for (int cg = 0; cg < NGC / 2; ++cg) {
            float rbd[4] = {INF, INF, INF, INF};
            u32 rbi[4] = {TG_NO_ID, TG_NO_ID, TG_NO_ID, TG_NO_ID};
            bool any = false;
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj) {
                if ((tj & (NGC / 2 - 1)) != cg) continue;
                if (!act[ti][tj]) continue;
                any = true;
                const int b = 16 * (wc + 2 * tj) + c16;
                const bool b_ok = b < nT;
                const int bb = b_ok ? b : 0;
                const float aux_b = s_aux[bb];
                const u32 id_b = (u32)s_ids[bb];
                const float kd_b = MODE == 0 ? s_kd[bb] : 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int a = 16 * i + 4 * g4 + e;
                    const bool ok = b_ok & (a < nN) & (b > a);
                    const float gram = acc[ti][tj][e];
                    const float dist = g.metric == 0 ? gram_to_dist<0>(gram, aux_a[e], aux_b)
                                     : g.metric == 1 ? gram_to_dist<1>(gram, aux_a[e], aux_b)
                                                     : gram_to_dist<2>(gram, aux_a[e], aux_b);
                    if (MODE == 1) {
                        if (ok) xout[((int64_t)v * TG_BLOCK_ROWS + a) * TG_BLOCK_COLS + b] = dist;
                    } else {
                        // row node a meets column node b: b is a candidate of a and a of b, each
                        // only if it would precede the last entry of the target's list
                        const bool pr = ok & reaches(dist, kd_a[e]);
                        const bool pc = ok & reaches(dist, kd_b);
                        pairmin(rbd[e], rbi[e], pr ? dist : INF, pr ? id_b : TG_NO_ID);
                        pairmin(cbd[tj][ti & (NGR / 2 - 1)], cbi[tj][ti & (NGR / 2 - 1)], pc ? dist : INF, pc ? id_a[e] : TG_NO_ID);
                    }
                }
            }
            if (MODE == 0 && any) {
#pragma unroll
                for (int e = 0; e < 4; ++e) rowmin16f(rbd[e], rbi[e]);
                const float md = c16 == 0 ? rbd[0] : c16 == 1 ? rbd[1] : c16 == 2 ? rbd[2] : rbd[3];
                const u32 mi = c16 == 0 ? rbi[0] : c16 == 1 ? rbi[1] : c16 == 2 ? rbi[2] : rbi[3];
                const int a = 16 * i + 4 * g4 + c16;
                if (c16 < 4 && mi != TG_NO_ID) atomicMin(s_cell + a * 8 + (wc + 2 * cg), ((u64)tg_ord(md) << 32) | (u64)((mi << 2) | 3u));
            }
        }
    }
    if (MODE == 0) {
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) {
            const int j = wc + 2 * tj;
            if (j >= NT) continue;
#pragma unroll
            for (int rg = 0; rg < NGR / 2; ++rg) {
                float d0 = cbd[tj][rg];
                u32 i0 = cbi[tj][rg];
                pairmin(d0, i0, __shfl_xor(d0, 16), (u32)__shfl_xor((int)i0, 16));
                pairmin(d0, i0, __shfl_xor(d0, 32), (u32)__shfl_xor((int)i0, 32));
                const int b = 16 * j + c16;
                if (g4 == 0 && i0 != TG_NO_ID) atomicMin(s_cell + b * 8 + (wr + 2 * rg), ((u64)tg_ord(d0) << 32) | (u64)((i0 << 2) | 3u));
            }
        }
        // Hand-over: the eight cells of a member sit in eight neighbouring lanes and their slots
        // share a 64-byte line, so a member's candidates travel as one transaction.  The cells
        // are left empty for the next block.
        __syncthreads();
        for (int c = tid; c < ((nT + 3) & ~3) * 8; c += JOIN_THREADS) {
            const u64 key = s_cell[c];
            if (key != TG_EMPTY_KEY) {
                s_cell[c] = TG_EMPTY_KEY;
                emit_candidate(cd, s_ids, s_salt, c >> 3, key, (u32)v, c & 7);
            }
        }
    }
    }   // work-list loop
}


// ---------------------------------------------------------------------------------------
// Register-resident variant for small blocks and d <= 128: one wave per anchor, no LDS tile
// and no barrier.  The wave keeps the whole block in VGPRs in MFMA operand layout: lane
// (r, q) = (lane % 16, lane / 16) holds, for every 16-row group t < GMAX and column step
// s < KS, columns 16 s + 4 q .. + 3 of row 16 t + r, so that one load instruction reads 64
// contiguous bytes of each of 16 rows (a step-major split would touch four lines per row).
// Tile (i, j) is then 4 KS v_mfma_f32_16x16x4_f32 on registers X[i][s], X[j][s]: both operands
// use the same column permutation, so the sum is the full dot product.  Retention is per
// 16 x 16 tile (ng_row = 4, ng_col = 8), so every tile hands its survivors over at once.
//
// Waves walk a work list of anchors whose blocks have at most GMAX row groups, and the walk
// is software pipelined: while block w is multiplied, the ids, thresholds and norms of block
// w + 1 are fetched, and as soon as tile row i of block w is finished its registers X[i] are
// refilled with row group i of block w + 1.  MODE as in join_kernel.
// ---------------------------------------------------------------------------------------
struct WaveItem {
    int64_t v;
    const u32* bids;
    int nN, nT, MT, NT;       // MT = NT = 0: nothing to do for this item
};
// work record: anchor | |NEW| << 32 | (|NEW|+|OLD|) << 40
__device__ inline u64 pack_rec(u32 v, int nN, int nT) { return (u64)v | ((u64)nN << 32) | ((u64)nT << 40); }

// NARROW: the rows come from the fp16 copy (g.Xh, rows of 32 KS values, zero padded): a register
// then holds eight values, columns 32 s + 8 q .. + 7, and a tile step is one
// v_mfma_f32_16x16x32_f16 (fp32 accumulation) in place of eight fp32 matrix instructions.
template <int GMAX, int MODE, int METRIC, int KS, bool FULL, bool NARROW>
__global__ __launch_bounds__(256) void join_wave_kernel(TgGraph g, TgSample sm, TgCand cd, u64 hs_slot, u64* stat_bins,
                                                        const int32_t* xblk, const int32_t* xsizes, float* xout,
                                                        const u64* __restrict__ wl, const u32* __restrict__ wl_cnt,
                                                        int64_t direct_count, int gmin)
{
    __shared__ u32 sh_salt[4][2][64];
    __shared__ u32 sh_okd[4][2][64];
    __shared__ int sh_ids[4][2][64];
    __shared__ float sh_aux[4][2][64];
    // candidates of one block, one cell per (member, partner group); handed over a block later
    __shared__ u64 sh_cell[4][2][64 * GMAX];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = tg_lane();
    const int r16 = lane & 15, q4 = lane >> 4;
    const float INF = __builtin_inff();
    if (g.f16_ok && (*g.f16_ok != 0u) != NARROW) return;      // the other variant's turn
    const int64_t count = wl ? (int64_t)*wl_cnt : direct_count;
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    // A record past the end of the list becomes an empty block at anchor 0, so that every load
    // below can be issued unconditionally (the load counters then stay exact and nothing has to
    // wait for more than it needs).
    auto load_rec = [&](int64_t w) -> u64 {
        const int64_t wc = w < count ? w : count - 1;
        u64 rec;
        if (MODE == 0) rec = wl[wc];
        else rec = pack_rec((u32)wc, xsizes[wc * 2], xsizes[wc * 2] + xsizes[wc * 2 + 1]);
        return w < count ? rec : 0ull;
    };
    auto decode = [&](u64 rec) {
        WaveItem it;
        it.v = (int64_t)(u32)rec;
        const int nN = (int)((rec >> 32) & 0xFFu), nT = (int)((rec >> 40) & 0xFFu);
        it.bids = MODE == 0 ? sm.blk + it.v * (int64_t)sm.BC : reinterpret_cast<const u32*>(xblk) + it.v * TG_BLOCK_COLS;
        const int NT = (nT + 15) >> 4;
        const bool serve = nN > 0 && nT >= 2 && NT <= GMAX && NT >= gmin;
        it.nN = serve ? nN : 0;
        it.nT = serve ? nT : 0;
        it.MT = serve ? (nN + 15) >> 4 : 0;
        it.NT = serve ? NT : 0;
        return it;
    };
    // ids of this lane's row in every group (rows past the block repeat row 0: they are masked later)
    auto fetch_row_ids = [&](const WaveItem& it, u32 (&idr)[GMAX]) {
#pragma unroll
        for (int t = 0; t < GMAX; ++t) {
            const int row = 16 * t + r16;
            idr[t] = it.bids[row < it.nT ? row : 0];
        }
    };
    float4 X[GMAX][KS];
    auto load_group = [&](int t, u32 id) {      // t is a compile-time constant at every call site
        if (NARROW) {
            const uint16_t* xh = g.Xh + (int64_t)id * g.ldh;
#pragma unroll
            for (int s8 = 0; s8 < KS; ++s8) X[t][s8] = *reinterpret_cast<const float4*>(xh + 32 * s8 + 8 * q4);
            return;
        }
        const float* x = g.X + (int64_t)id * g.ld;
#pragma unroll
        for (int s8 = 0; s8 < KS; ++s8) {
            const int col = 16 * s8 + 4 * q4;
            if (FULL) {
                // rows of exactly 16 KS floats: nothing to mask
                X[t][s8] = *reinterpret_cast<const float4*>(x + col);
            } else {
                // unconditional load at a clamped column, zeroed afterwards when the column is padding
                const bool real = col < g.ld;
                const float4 val = *reinterpret_cast<const float4*>(x + (real ? col : 0));
                X[t][s8] = real ? val : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    // per-member data (one member per lane): fetched into registers, parked in LDS one block ahead
    // the threshold of a member's list and its norm come in one word (MODE 1 has no lists: the norm alone)
    auto fetch_member = [&](int id, float& aux, u64& kth) {
        if (MODE == 0) {
            kth = g.kth[id];
            aux = __uint_as_float((u32)kth);
        } else {
            kth = 0ull;
            aux = METRIC == 2 ? g.rnorm[id] : g.nrm[id];
        }
    };
    auto park_member = [&](const WaveItem& it, int id, float aux, u64 kth, int buf) {
        if (lane < it.nT) {
            sh_ids[wave][buf][lane] = id;
            sh_aux[wave][buf][lane] = aux;
            if (MODE == 0) {
                sh_okd[wave][buf][lane] = (u32)(kth >> 32);
                sh_salt[wave][buf][lane] = (u32)tg_mix64(hs_slot + (u64)id);
            }
        }
    };

    // Hand the cells of a finished block to the slot rows.  Lanes q = 0..GMAX-1 of a member sit
    // side by side and their slots share a 64-byte line, so the atomics of one member travel
    // as one transaction.
    constexpr int CELLS = 64 * GMAX;
    auto flush_cells = [&](int fbuf, u32 fv, int fnT) {
        const u64* cells = sh_cell[wave][fbuf];
        const u32* f_salt = sh_salt[wave][fbuf];
        const int* f_ids = sh_ids[wave][fbuf];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int p = 16 * s4 + (lane >> 2), q = lane & 3;
            if (16 * s4 < fnT) {
                const bool in = p < fnT && q < GMAX;
                const u64 key = in ? cells[p * GMAX + (q < GMAX ? q : 0)] : TG_EMPTY_KEY;
                if (key != TG_EMPTY_KEY) {
                    const u32 t = (u32)f_ids[p];
                    u32 h = (f_salt[p] + fv) * 0x9E3779B1u;
                    h ^= h >> 15;
                    h *= 0x85EBCA77u;
                    h ^= h >> 13;
                    const u32 line = h >> (36 - __ffs(cd.C));
                    const u32 slot = line * 8u + ((u32)(q + (int)(h & 7u)) & 7u);
                    atomicMin(cd.slots + (int64_t)t * cd.C + slot, key);
                }
            }
        }
    };
    auto clear_cells = [&](int cbuf) {
#pragma unroll
        for (int c = 0; c < CELLS; c += 64) sh_cell[wave][cbuf][c + lane] = TG_EMPTY_KEY;
    };

    int64_t w = (int64_t)blockIdx.x * 4 + wave;
    if (w >= count) return;
    WaveItem cur = decode(load_rec(w));
    WaveItem nxt = decode(load_rec(w + nwaves));
    u64 rec2 = load_rec(w + 2 * nwaves);
    u32 idn[GMAX];
    int mid;
    {
        u32 idr[GMAX];
        fetch_row_ids(cur, idr);
#pragma unroll
        for (int t = 0; t < GMAX; ++t) load_group(t, idr[t]);
        const int m0 = (int)cur.bids[lane < cur.nT ? lane : 0];
        float a0;
        u64 k0;
        fetch_member(m0, a0, k0);
        park_member(cur, m0, a0, k0, 0);
        fetch_row_ids(nxt, idn);
        mid = (int)nxt.bids[lane < nxt.nT ? lane : 0];
    }
    int buf = 0;
    u32 prev_v = 0;
    int prev_nT = 0;      // members of the block whose cells still wait in LDS

    // In round w: block w is multiplied, the rows, norms and thresholds of block w + 1 are
    // fetched (their ids came in one round earlier), and the ids of block w + 2 start travelling.
    for (; w < count; w += nwaves) {
        const WaveItem nxt2 = decode(rec2);
        rec2 = load_rec(w + 3 * nwaves);
        u32 idn2[GMAX];
        fetch_row_ids(nxt2, idn2);
        const int mid2 = (int)nxt2.bids[lane < nxt2.nT ? lane : 0];
        float m_aux = 0.f;
        u64 m_kth = 0;

        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const u32* s_okd = sh_okd[wave][buf];
        const int* s_ids = sh_ids[wave][buf];
        const float* s_aux = sh_aux[wave][buf];
        const int64_t v = cur.v;
        const int nN = cur.nN, nT = cur.nT, MT = cur.MT, NT = cur.NT;
        u64* cells = sh_cell[wave][buf];
        if (MODE == 0) {
            if (prev_nT > 0) flush_cells(buf ^ 1, prev_v, prev_nT);
            clear_cells(buf);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (MODE == 0 && stat_bins && lane == 0 && MT > 0) {
            const u64 pairs = (u64)nN * (u64)(nN - 1) / 2 + (u64)nN * (u64)(nT - nN);
            atomicAdd(stat_bins + (v & (TG_STAT_BINS - 1)), pairs);
            atomicAdd(stat_bins + TG_STAT_BINS + (v & (TG_STAT_BINS - 1)), (u64)nT);
        }

#pragma unroll
        for (int i = 0; i < GMAX; ++i) {
            if (i < MT) {
                // Row side of this tile row: accumulator element e of lane (r16, q4) is row
                // a = 16 i + 4 q4 + e.  Everything below works on "ordered" distances (tg_ord:
                // unsigned order = float order); a pair that must not count gets +inf added, so
                // no validity masks have to be carried around.
                float aux_a[4], pen_a[4];
                u32 id_a[4], okd_max = 0u;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int a = 16 * i + 4 * q4 + e;
                    const int aa = a < nN ? a : 0;
                    pen_a[e] = a < nN ? 0.f : INF;
                    // L2: the penalty rides on the norm (norm + 0 is the norm, bit for bit)
                    aux_a[e] = METRIC == 0 ? s_aux[aa] + pen_a[e] : s_aux[aa];
                    id_a[e] = (u32)s_ids[aa];
                    if (MODE == 0) okd_max = max(okd_max, s_okd[aa]);
                }
                // the lane that will speak for row 16 i + 4 q4 + (r16 & 3) keeps that row's threshold
                const int a_mine = 16 * i + 4 * q4 + (r16 & 3);
                const u32 okd_mine = MODE == 0 ? s_okd[a_mine < nN ? a_mine : 0] : 0u;
#pragma unroll
                for (int j = i; j < GMAX; ++j) {
                    if (j >= NT) continue;
                    floatx4 acc = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s8 = 0; s8 < KS; ++s8) {
                        if (NARROW) {
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, X[i][s8]),
                                                                          __builtin_bit_cast(halfx8, X[j][s8]), acc, 0, 0, 0);
                        } else {
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s8].x, X[j][s8].x, acc, 0, 0, 0);
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s8].y, X[j][s8].y, acc, 0, 0, 0);
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s8].z, X[j][s8].z, acc, 0, 0, 0);
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s8].w, X[j][s8].w, acc, 0, 0, 0);
                        }
                    }
                    // column side: lane (r16, .) is column b = 16 j + r16
                    const int b = 16 * j + r16;
                    const int bb = b < nT ? b : 0;
                    const float pen_b = b < nT ? 0.f : INF;
                    const float aux_b = METRIC == 0 ? s_aux[bb] + pen_b : s_aux[bb];
                    const u32 id_b = (u32)s_ids[bb];
                    u32 o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float dist = gram_to_dist<METRIC>(acc[e], aux_a[e], aux_b);
                        if (METRIC != 0) dist += pen_a[e] + pen_b;
                        // only the diagonal tile has pairs on or below the diagonal to drop
                        if (i == j) dist += (r16 > 4 * q4 + e) ? 0.f : INF;
                        if (MODE == 1) {
                            if (dist < INF) xout[((int64_t)v * TG_BLOCK_ROWS + 16 * i + 4 * q4 + e) * TG_BLOCK_COLS + b] = dist;
                        }
                        o[e] = METRIC == 0 ? (__float_as_uint(dist) | 0x80000000u) : tg_ord(dist);
                    }
                    if (MODE == 0) {
                        const u32 okd_b = s_okd[bb];
                        // nothing in this tile can precede any threshold: the common case in late rounds
                        const u32 omin = min(min(o[0], o[1]), min(o[2], o[3]));
                        if (__ballot(omin <= max(okd_max, okd_b)) == 0) continue;
                        // Row nodes: closest column node of the tile for each of the lane's four rows,
                        // reduced over the 16 lanes of the row group; then one threshold test by the
                        // lane that speaks for the row (if the closest fails, every other pair fails).
                        u32 ro[4], ri[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ro[e] = o[e];
                            ri[e] = id_b;
                            rowmin16(ro[e], ri[e]);
                        }
                        const int e_mine = r16 & 3;
                        const u32 mo = e_mine == 0 ? ro[0] : e_mine == 1 ? ro[1] : e_mine == 2 ? ro[2] : ro[3];
                        const u32 mi = e_mine == 0 ? ri[0] : e_mine == 1 ? ri[1] : e_mine == 2 ? ri[2] : ri[3];
                        // (at the threshold's own distance a candidate passes whatever its id: the list update sorts that out)
                        if (r16 < 4 && mo <= okd_mine)
                            atomicMin(cells + a_mine * GMAX + j, ((u64)mo << 32) | (u64)((mi << 2) | 3u));
                        // Column node b: closest row node of the tile over the lane's four rows.
                        u64 cb = ((u64)o[0] << 32) | id_a[0];
#pragma unroll
                        for (int e = 1; e < 4; ++e) cb = tg_min64(cb, ((u64)o[e] << 32) | id_a[e]);
                        // (the four row quarters meet in the cell: it takes the minimum)
                        const u32 co = (u32)(cb >> 32), ci = (u32)cb;
                        if (co <= okd_b)
                            atomicMin(cells + b * GMAX + i, ((u64)co << 32) | (u64)((ci << 2) | 3u));
                    }
                }
            }
            if (i == 0) {
                // the next block's ids have arrived behind the first tile row: ask for its norms and thresholds
                fetch_member(mid, m_aux, m_kth);
            }
            // Row group i is used by tile rows min(i, MT - 1) and earlier: once tile row i is done
            // (and it is not the last one) its registers can take in the next block.
            if (i + 1 < MT) load_group(i, idn[i]);
        }
        // whatever the last tile row still needed
#pragma unroll
        for (int i = 0; i < GMAX; ++i)
            if (i + 1 >= MT) load_group(i, idn[i]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (MODE == 0) {
            // the block's cells wait in LDS for one more round; its member data are needed for
            // that, so the next block's member data go to the buffer of the block before
            prev_v = (u32)v;
            prev_nT = MT > 0 ? nT : 0;
        }
        park_member(nxt, mid, m_aux, m_kth, buf ^ 1);
        cur = nxt;
        nxt = nxt2;
#pragma unroll
        for (int t = 0; t < GMAX; ++t) idn[t] = idn2[t];
        mid = mid2;
        buf ^= 1;
    }
    if (MODE == 0 && prev_nT > 0) flush_cells(buf ^ 1, prev_v, prev_nT);
}

// ---------------------------------------------------------------------------------------
// Work lists: anchors with something to join, by block size.  List 0: at most 3 row groups,
// list 1: exactly 4, list 2: more.  Without the wave kernel (longer rows) list 1 takes every block
// of at most 4 row groups and list 0 stays empty.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bin_kernel(TgSample sm, int64_t n, int wave_ok)
{
    __shared__ u32 wcnt[3][4];
    __shared__ u32 base[3];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t v = (int64_t)blockIdx.x * 256 + tid;
    int bin = -1, rec_nN = 0, rec_nT = 0;
    if (v < n) {
        const u32 z = sm.bsz[v];
        const int nN = (int)(z & 0xFFu), nT = (int)(z >> 8);
        rec_nN = nN;
        rec_nT = nT;
        if (nN > 0 && nT >= 2) {
            const int NT = (nT + 15) >> 4;
            bin = NT > 4 ? 2 : (NT == 4 || !wave_ok) ? 1 : 0;
        }
    }
    u32 mypos = 0;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const u64 m = __ballot(bin == b);
        if (lane == 0) wcnt[b][wave] = (u32)__popcll(m);
        if (bin == b) mypos = (u32)__popcll(m & tg_lanemask_lt());
    }
    __syncthreads();
    if (tid < 3) {
        const u32 tot = wcnt[tid][0] + wcnt[tid][1] + wcnt[tid][2] + wcnt[tid][3];
        base[tid] = tot ? atomicAdd(sm.wl_cnt + tid, tot) : 0u;
    }
    __syncthreads();
    if (bin >= 0) {
        u32 pos = base[bin] + mypos;
        for (int w2 = 0; w2 < wave; ++w2) pos += wcnt[bin][w2];
        sm.wl[(int64_t)bin * n + pos] = pack_rec((u32)v, rec_nN, rec_nT);
    }
}

static size_t join_lds_bytes(int DK, int rows) { return JOIN_HDR_BYTES + JOIN_CELL_BYTES + (size_t)rows * (DK + 4) * sizeof(float); }

// LDS beyond 64 KB per workgroup has to be asked for once per kernel
template <class K>
static void allow_large_lds(K kernel, size_t bytes)
{
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

#define JOIN_GRID 2048     // persistent launches: workgroups walk the work list with this stride

// the workgroup kernel on one work list; ROWS = the most members a block of that list has
template <int DK, int NGR, int NGC, int ROWS>
static void launch_join_list(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list, hipStream_t s)
{
    static bool once = (allow_large_lds(join_kernel<DK, NGR, NGC, 0, false, ROWS>, join_lds_bytes(DK, ROWS)),
                        allow_large_lds(join_kernel<DK, NGR, NGC, 0, true, ROWS>, join_lds_bytes(DK, ROWS)), true);
    (void)once;
    const int rows = sm.BC < ROWS ? sm.BC : ROWS;   // a stored block never exceeds BC rows
    const unsigned grid = (unsigned)(g.n < JOIN_GRID ? g.n : JOIN_GRID);
    // with the device flag both variants are launched, and the one it does not name ends at once
    if (g.Xh)
        hipLaunchKernelGGL((join_kernel<DK, NGR, NGC, 0, true, ROWS>), dim3(grid), dim3(JOIN_THREADS), join_lds_bytes(DK, rows), s, g, sm, c,
                           hs_slot, stat_bins, (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr,
                           (const u64*)(sm.wl + (int64_t)list * g.n), (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_kernel<DK, NGR, NGC, 0, false, ROWS>), dim3(grid), dim3(JOIN_THREADS), join_lds_bytes(DK, rows), s, g, sm, c,
                           hs_slot, stat_bins, (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr,
                           (const u64*)(sm.wl + (int64_t)list * g.n), (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
}
// wave_done: the register-resident kernel has served lists 0 and 1
template <int DK, int NGR, int NGC>
static void launch_join_t(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, bool wave_done, hipStream_t s)
{
    if (!wave_done) launch_join_list<DK, NGR, NGC, 64>(g, sm, c, hs_slot, stat_bins, 1, s);
    launch_join_list<DK, NGR, NGC, TG_BLOCK_COLS>(g, sm, c, hs_slot, stat_bins, 2, s);
}
static void launch_join_ng(const TgGraph& g, const TgSample& sm, const TgCand& c, int ngr, int ngc, u64 hs_slot,
                           u64* stat_bins, bool wave_done, hipStream_t s)
{
    if (ngr == 2 && ngc == 2) launch_join_t<64, 2, 2>(g, sm, c, hs_slot, stat_bins, wave_done, s);
    else if (ngr == 2 && ngc == 4) launch_join_t<64, 2, 4>(g, sm, c, hs_slot, stat_bins, wave_done, s);
    else if (ngr == 2 && ngc == 8) launch_join_t<64, 2, 8>(g, sm, c, hs_slot, stat_bins, wave_done, s);
    else if (ngr == 4 && ngc == 2) launch_join_t<64, 4, 2>(g, sm, c, hs_slot, stat_bins, wave_done, s);
    else if (ngr == 4 && ngc == 4) launch_join_t<64, 4, 4>(g, sm, c, hs_slot, stat_bins, wave_done, s);
    else if (g.ld > 64 || (g.Xh && g.ldh > 128)) launch_join_t<128, 4, 8>(g, sm, c, hs_slot, stat_bins, wave_done, s);   // half as many slabs and barriers
    else launch_join_t<64, 4, 8>(g, sm, c, hs_slot, stat_bins, wave_done, s);
}

template <int GMAX, int METRIC, int KS>
static void launch_wave_k(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list,
                          hipStream_t s)
{
    const int64_t wgs = (g.n + 3) / 4;
    const unsigned grid = (unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID);
    if (g.Xh)       // rows of the fp16 copy are whole steps of 32 values: KS / 2 of them
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS / 2, true, true>), dim3(grid), dim3(256), 0, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * g.n),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    if (g.Xh && !g.f16_ok) return;
    if (g.ld == 16 * KS)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS, true, false>), dim3(grid), dim3(256), 0, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * g.n),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    else
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS, false, false>), dim3(grid), dim3(256), 0, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * g.n),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
}
template <int GMAX, int METRIC, int KS>
static void launch_wave_dump_k(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out, int gmin,
                               hipStream_t s)
{
    TgSample sm = {};
    TgCand c = {};
    const int64_t wgs = (nb + 3) / 4;
    if (g.Xh)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 1, METRIC, KS / 2, true, true>), dim3((unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID)),
                           dim3(256), 0, s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr, (const u32*)nullptr, nb, gmin);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 1, METRIC, KS, false, false>), dim3((unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID)),
                           dim3(256), 0, s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr, (const u32*)nullptr, nb, gmin);
}
// rows of at most 64 / 96 / 128 floats take 4 / 6 / 8 column steps per lane quarter
template <int GMAX, int METRIC>
static void launch_wave_m(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list,
                          hipStream_t s)
{
    if (g.ld <= 64) launch_wave_k<GMAX, METRIC, 4>(g, sm, c, hs_slot, stat_bins, list, s);
    else if (g.ld <= 96) launch_wave_k<GMAX, METRIC, 6>(g, sm, c, hs_slot, stat_bins, list, s);
    else launch_wave_k<GMAX, METRIC, 8>(g, sm, c, hs_slot, stat_bins, list, s);
}
template <int GMAX>
static void launch_wave_t(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list,
                          hipStream_t s)
{
    if (g.metric == 0) launch_wave_m<GMAX, 0>(g, sm, c, hs_slot, stat_bins, list, s);
    else if (g.metric == 1) launch_wave_m<GMAX, 1>(g, sm, c, hs_slot, stat_bins, list, s);
    else launch_wave_m<GMAX, 2>(g, sm, c, hs_slot, stat_bins, list, s);
}
template <int GMAX, int METRIC>
static void launch_wave_dump(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out, int gmin,
                             hipStream_t s)
{
    if (g.ld <= 64) launch_wave_dump_k<GMAX, METRIC, 4>(g, blk, sizes, nb, out, gmin, s);
    else if (g.ld <= 96) launch_wave_dump_k<GMAX, METRIC, 6>(g, blk, sizes, nb, out, gmin, s);
    else launch_wave_dump_k<GMAX, METRIC, 8>(g, blk, sizes, nb, out, gmin, s);
}

// The register-resident kernel applies to rows of at most 128 floats with per-tile retention.
static bool wave_path(const TgGraph& g, int ng_row, int ng_col) { return g.ld <= 128 && ng_row == 4 && ng_col == 8; }

void tg_launch_join(const TgGraph& g, const TgSample& sm, const TgCand& c, int ng_row, int ng_col, uint64_t hs_slot,
                    unsigned long long* stat_bins, hipStream_t s)
{
    const bool wv = wave_path(g, ng_row, ng_col);
    tg_launch_fill_u32(sm.wl_cnt, 4, 0u, s);
    hipLaunchKernelGGL(bin_kernel, dim3((unsigned)((g.n + 255) / 256)), dim3(256), 0, s, sm, g.n, wv ? 1 : 0);
    if (wv) {
        launch_wave_t<3>(g, sm, c, hs_slot, stat_bins, 0, s);
        launch_wave_t<4>(g, sm, c, hs_slot, stat_bins, 1, s);
    }
    launch_join_ng(g, sm, c, ng_row, ng_col, hs_slot, stat_bins, wv, s);
}

void tg_launch_join_distances(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out,
                              hipStream_t s)
{
    TgSample sm = {};
    TgCand c = {};
    static bool once = (allow_large_lds(join_kernel<64, 2, 2, 1, false>, join_lds_bytes(64, TG_BLOCK_COLS)),
                        allow_large_lds(join_kernel<64, 2, 2, 1, true>, join_lds_bytes(64, TG_BLOCK_COLS)), true);
    (void)once;
    int skip_le = 0;
    if (wave_path(g, 4, 8)) {      // same routing by block size as the production join
        if (g.metric == 0) { launch_wave_dump<3, 0>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 0>(g, blk, sizes, nb, out, 4, s); }
        else if (g.metric == 1) { launch_wave_dump<3, 1>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 1>(g, blk, sizes, nb, out, 4, s); }
        else { launch_wave_dump<3, 2>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 2>(g, blk, sizes, nb, out, 4, s); }
        skip_le = 4;
    }
    if (g.Xh)
        hipLaunchKernelGGL((join_kernel<64, 2, 2, 1, true>), dim3((unsigned)(nb < JOIN_GRID ? nb : JOIN_GRID)), dim3(JOIN_THREADS),
                           join_lds_bytes(64, TG_BLOCK_COLS), s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr,
                           (const u32*)nullptr, nb, skip_le);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_kernel<64, 2, 2, 1, false>), dim3((unsigned)(nb < JOIN_GRID ? nb : JOIN_GRID)), dim3(JOIN_THREADS),
                           join_lds_bytes(64, TG_BLOCK_COLS), s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr,
                           (const u32*)nullptr, nb, skip_le);
}
