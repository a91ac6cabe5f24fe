// Phase-1 local join (section 4.2, first part).  The sampling kernel has stored every
// anchor's block (NEW ids, then OLD ids).  Anchors are first sorted into work lists by block
// size and by part (a round is carried out in parts: the anchors v = p mod parts, with a list
// update after every part); small blocks of low-dimensional data go to a register-resident
// one-wave-per-anchor kernel, the rest to a workgroup kernel.  Before them a kernel of its own
//   1. finds out which members of a block already sit in which member's list (an exact id
//      look-up of every list entry in a small table of the block's ids in LDS) and stores it as
//      one bit per pair of members: such a node is no candidate for that member (the list update
//      would drop it anyway, but in the join it would take the place of a useful one).
// Either join kernel then
//   2. gathers the block's vectors (into registers, or into LDS a slab of columns at a time);
//   3. accumulates the Gram tile NEW x (NEW ++ OLD) with v_mfma_f32_16x16x4_f32 and turns it
//      into distances |x|^2 + |y|^2 - 2<x,y>  (or -<x,y>, or 1 - cos);
//   4. retention: every member keeps, for each group of eight consecutive block positions, the
//      closest candidate under its threshold (the paper keeps one per node and warp sub-tile),
//      in LDS cells; the eight cells of a member travel to one 64-byte line of that member's
//      candidate slots, word by word by atomic minimum.
// Only pairs (a,b) with a NEW and position a < b are used, so every new-new and new-old
// pair counts once and old-old pairs never.
#include "tg_device.h"
#include "tg_kernels.h"

#define JOIN_THREADS 256
#define JOIN_CELLS 8                                   // cells per member: one per group of eight positions (mod 8)
#define JOIN_CELL_BYTES (TG_BLOCK_COLS * JOIN_CELLS * 8)   // workgroup kernel: all cells of a block
#define T8_SLOTS 4096                                  // table of a block's ids: hash -> block position, one byte each
#define T8_FREE 255u                                   // "no member" (positions are 0..127)

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------
// cross-lane helpers: exchanges inside a row of 16 lanes are DPP operand modifiers (no LDS)
template <int CTRL>
__device__ inline u32 dpp_mov(u32 x)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
#define TG_NO_ID 0x7FFFFFFFu
// minimum of (ordered distance, id) pairs over each group of 8 lanes (lanes 0-7 and 8-15 of a row); every lane gets
// its group's result.  quad_perm 1,0,3,2 / quad_perm 2,3,0,1 / mirror of 8 lanes.
__device__ inline void groupmin8(u32& dist, u32& id)
{
    u32 m = dist;
    m = min(m, dpp_mov<0xB1>(m));
    m = min(m, dpp_mov<0x4E>(m));
    m = min(m, dpp_mov<0x141>(m));
    u32 c = dist == m ? id : TG_NO_ID;
    c = min(c, dpp_mov<0xB1>(c));
    c = min(c, dpp_mov<0x4E>(c));
    c = min(c, dpp_mov<0x141>(c));
    dist = m;
    id = c;
}
// Gram value -> distance.  aux = squared norms (L2) or inverse norms (cosine).
template <int METRIC>
__device__ inline float gram_to_dist(float gram, float aux_a, float aux_b)
{
    if (METRIC == 0) return fmaxf(0.0f, fmaf(-2.0f, gram, aux_a + aux_b));
    if (METRIC == 1) return -gram + 0.0f;
    return 1.0f - gram * (aux_a * aux_b) + 0.0f;   // symmetric in the two nodes, bit for bit
}
// A candidate may precede the target's last list entry when its distance does not exceed that entry's.  The id of
// that entry is not looked at: a candidate at exactly that distance with a larger id passes too, and the list update,
// which keeps the k smallest (distance, id), drops it again; nothing that belongs in the list is held back.

// ---------------------------------------------------------------------------------------
// Which members of a block sit in which member's list already: sm.adj, per anchor of the part
// (slot v / parts) and member p, adj_words words whose bit x says "the node at position x of
// the block is in p's list".  One wave per anchor.  The block's ids (distinct) go into an
// open-addressed table in LDS, T8[hash(id) + probes] = block position, a byte each.  The members'
// lists are then read as one run of 16-byte pieces, 64 pieces per load, so consecutive lanes
// read consecutive pieces of one list; every id of a piece is looked up (hash, table byte, the
// id at that position, the next byte while the place is taken by another id) and a hit sets its
// bit in LDS, from where the words go out in one run.
// The lists are read as they stand when this part of the round begins.
// ---------------------------------------------------------------------------------------
__device__ inline u32 t8_hash(u32 id)
{
    const u32 x = id ^ (id >> 11);
    return (u32)__umul24(x, 0x9E3779u) >> 20;      // 12 bits of a 24 x 24 bit product (the intrinsic's type is signed)
}
#define ADJ_WAVES 4
#define ADJ_UNROLL 8
struct AdjShared {
    int ids[TG_BLOCK_COLS + 4];
    u32 adjw[(TG_BLOCK_COLS + 1) * 4];      // the last row takes what lanes past the end of the block look up
    unsigned char T8[T8_SLOTS];
};
template <bool VEC>
__global__ __launch_bounds__(64 * ADJ_WAVES) void adj_kernel(TgGraph g, TgSample sm, int part, int64_t nslots)
{
    __shared__ AdjShared shs[ADJ_WAVES];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = tg_lane();
    AdjShared& sh = shs[wave];
    const int k = g.k;
    const u32 idmax = (u32)(g.n - 1);
    constexpr int W = VEC ? 4 : 1;                 // ids per piece; VEC: rows of the lists are 16-byte aligned (k % 4 == 0)
    const int per = k / W;                         // pieces per list
    const int per_sh = (per & (per - 1)) == 0 ? __ffs(per) - 1 : -1;
    const int aw = sm.adj_words, aw_sh = __ffs(aw) - 1;
    auto lds_fence = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    for (int c = lane; c < T8_SLOTS / 4; c += 64) reinterpret_cast<u32*>(sh.T8)[c] = 0xFFFFFFFFu;
    if (lane < 4) sh.ids[TG_BLOCK_COLS + lane] = -1;
    u32 my_s[2] = {0u, 0u};
    bool my_in[2] = {false, false};
    for (int64_t a = (int64_t)blockIdx.x * ADJ_WAVES + wave; a < nslots; a += (int64_t)gridDim.x * ADJ_WAVES) {
        const int64_t v = a * sm.parts + part;
        if (v >= g.n) continue;
        const u32 z = sm.bsz[v];
        const int nN = (int)(z & 0xFFu), nT = (int)(z >> 8);
        if (nN == 0 || nT < 2 || nT > sm.BC || nT > TG_BLOCK_COLS || nN > nT) continue;      // no join for this anchor
        const u32* bids = sm.blk + v * (int64_t)sm.BC;
        // The table of the block's ids: the last block's entries out, this block's in.  Lanes meet in the table
        // (a lane reads back the byte it wrote to learn whether another lane's id took the place), so these
        // accesses are volatile: the value read is the one in LDS, never one the compiler remembers having stored.
        volatile unsigned char* T8v = sh.T8;
        lds_fence();
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (my_in[h]) T8v[my_s[h]] = (unsigned char)T8_FREE;
        for (int c = lane; c < nT * 4; c += 64) sh.adjw[c] = 0u;
        lds_fence();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int p = lane + 64 * h;
            my_in[h] = p < nT;
            const u32 id = my_in[h] ? min(bids[p], idmax) : 0u;
            my_s[h] = t8_hash(id);
            sh.ids[p] = my_in[h] ? (int)id : -1;
        }
        for (int h = 0; h < (nT > 64 ? 2 : 1); ++h) {
            const u32 p = (u32)(lane + 64 * h);
            bool pending = my_in[h];
            while (__ballot(pending)) {                  // at most nT turns: the table has room for every member
                if (pending && T8v[my_s[h]] == T8_FREE) T8v[my_s[h]] = (unsigned char)p;
                lds_fence();
                if (pending) {
                    if (T8v[my_s[h]] == p) pending = false;
                    else my_s[h] = (my_s[h] + 1u) & (T8_SLOTS - 1);
                }
                lds_fence();
            }
        }
        lds_fence();
        const int total = nT * per;
        for (int base = 0; base < total; base += 64 * ADJ_UNROLL) {
            u32 lid[ADJ_UNROLL][W];
            int mm[ADJ_UNROLL];
#pragma unroll
            for (int u = 0; u < ADJ_UNROLL; ++u) {
                const int idx = base + 64 * u + lane;
                const bool ok = idx < total;
                const int ii = ok ? idx : 0;
                const int m = per_sh >= 0 ? ii >> per_sh : ii / per;
                const int q = ii - m * per;
                const u32* src = g.gid + (int64_t)sh.ids[m] * k + q * W;
                if (VEC) {
                    const uint4 t = *reinterpret_cast<const uint4*>(src);
                    lid[u][0] = t.x; lid[u][W > 1 ? 1 : 0] = t.y; lid[u][W > 2 ? 2 : 0] = t.z; lid[u][W > 3 ? 3 : 0] = t.w;
                } else {
                    lid[u][0] = *src;
                }
                mm[u] = ok ? m : TG_BLOCK_COLS;
            }
#pragma unroll
            for (int u = 0; u < ADJ_UNROLL; ++u) {
                if (base + 64 * u >= total) break;       // (wave-uniform)
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    const u32 cid = lid[u][w] & TG_ID_MASK;
                    u32 s = t8_hash(cid);
                    u32 e = (u32)sh.T8[s];
                    while (e != T8_FREE) {               // ends at a free place: the table is never full
                        if ((u32)sh.ids[e] == cid) {
                            atomicOr(&sh.adjw[mm[u] * 4 + (int)(e >> 5)], 1u << (e & 31u));
                            break;
                        }
                        s = (s + 1u) & (T8_SLOTS - 1);
                        e = sh.T8[s];
                    }
                }
            }
        }
        lds_fence();
        u32* out = sm.adj + a * sm.BC * (int64_t)aw;
        for (int c = lane; c < nT * aw; c += 64) out[c] = sh.adjw[(c >> aw_sh) * 4 + (c & (aw - 1))];
    }
}
void tg_launch_adj(const TgGraph& g, const TgSample& sm, int part, hipStream_t s)
{
    const int64_t nslots = (g.n + sm.parts - 1) / sm.parts;
    const int64_t wgs = (nslots + ADJ_WAVES - 1) / ADJ_WAVES;
    const dim3 grid((unsigned)(wgs < 16384 ? wgs : 16384)), block(64 * ADJ_WAVES);
    if ((g.k & 3) == 0) hipLaunchKernelGGL(adj_kernel<true>, grid, block, 0, s, g, sm, part, nslots);
    else hipLaunchKernelGGL(adj_kernel<false>, grid, block, 0, s, g, sm, part, nslots);
}

// the stored adjacency words of one part -> the boundary's fixed n x 128 x 4 layout (test interface)
__global__ void dump_adj_kernel(TgSample sm, int64_t n, int part, uint32_t* out)
{
    const size_t total = (size_t)((n + sm.parts - 1) / sm.parts) * TG_BLOCK_COLS * 4;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < total; i += stride) {
        const int64_t a = (int64_t)(i / (TG_BLOCK_COLS * 4));
        const int p = (int)((i / 4) % TG_BLOCK_COLS), wd = (int)(i % 4);
        const int64_t v = a * sm.parts + part;
        if (v >= n) continue;
        const u32 z = sm.bsz[v];
        const int nN = (int)(z & 0xFFu), nT = (int)(z >> 8);
        const bool joined = nN > 0 && nT >= 2 && nT <= sm.BC;
        out[((size_t)v * TG_BLOCK_COLS + p) * 4 + wd] = (joined && p < nT && wd < sm.adj_words) ? sm.adj[(a * sm.BC + p) * (int64_t)sm.adj_words + wd] : 0u;
    }
}
void tg_launch_dump_adj(const TgGraph& g, const TgSample& sm, int part, uint32_t* out, hipStream_t s)
{
    tg_launch_adj(g, sm, part, s);
    hipLaunchKernelGGL(dump_adj_kernel, dim3(1024), dim3(256), 0, s, sm, g.n, part, out);
}

// Candidate slot of member t (salt: its slot-hash salt) for the cell q of anchor v's block: the pair (t, v) owns
// one 64-byte line of t's slot row, picked by a hash, and cell q goes to word (q + rotation) % 8 of it, where it
// stays if it is the smaller (dist, id): one 64-bit atomic minimum, no order dependence.  All candidates one block
// has for t share a line, so they travel in one memory transaction.
__device__ inline void emit_candidate(const TgCand& cd, u32 t, u32 tmax, u32 salt, u64 key, u32 v, int q)
{
    if (t > tmax) return;                            // (no id from LDS becomes an address unchecked)
    u32 h = (salt + v) * 0x9E3779B1u;
    h ^= h >> 15;
    h *= 0x85EBCA77u;
    h ^= h >> 13;
    const u32 line = h >> (36 - __ffs(cd.C));        // C / 8 lines
    const u32 slot = line * 8u + ((u32)(q + (int)(h & 7u)) & 7u);
    atomicMin(cd.slots + (int64_t)t * cd.C + slot, key);
}

// ---------------------------------------------------------------------------------------
// Workgroup kernel.  MODE 0: emit candidates for the stored blocks.  MODE 1: write the distance tile of
// caller-given blocks.
// NARROW: the rows come from the fp16 copy; a slab then holds 2 DK columns in the same bytes, and a
// step of 32 columns is one v_mfma_f32_16x16x32_f16 per tile.
// ROWS: the most members a block may have here, 64 or 128.  Blocks of at most 64 members need half the
// registers for a slab on its way, so two slabs travel while a third is multiplied; with 128 it is one.
// LDS: header (salt, threshold, ids, norms), the adjacency words, the cells, the tile.
// ---------------------------------------------------------------------------------------
#define JOIN_HDR_BYTES (4 * (TG_BLOCK_COLS + 4) * 4)
#define JOIN_ADJ_BYTES (TG_BLOCK_COLS * 4 * 4)
template <int DK, int MODE, bool NARROW = false, int ROWS = TG_BLOCK_COLS>
__global__ __launch_bounds__(JOIN_THREADS, ROWS <= 64 ? 3 : 2) void join_kernel(TgGraph g, TgSample sm, TgCand cd, u64 hs_slot,
                                                            u64* stat_bins, const int32_t* xblk,
                                                            const int32_t* xsizes, float* xout, const u64* wl,
                                                            const u32* wl_cnt, int64_t direct_count, int skip_le)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr int HW = TG_BLOCK_COLS + 4;                               // words per header array
    u32* s_salt = reinterpret_cast<u32*>(smem_raw);                     // slot-hash salt of each member
    u32* s_okd = s_salt + HW;                                           // threshold: ordered distance of the member's last entry
    int* s_ids = reinterpret_cast<int*>(s_okd + HW);                    // ids; entry TG_BLOCK_COLS is no id
    float* s_aux = reinterpret_cast<float*>(s_ids + HW);                // squared norm (or 1/|x| for cosine)
    u32* s_adj = reinterpret_cast<u32*>(smem_raw + JOIN_HDR_BYTES);     // member p: four words, bit x = position x is in p's list
    u64* s_cell = reinterpret_cast<u64*>(smem_raw + JOIN_HDR_BYTES + JOIN_ADJ_BYTES);   // candidates of the block in hand
    unsigned char* tile = smem_raw + JOIN_HDR_BYTES + JOIN_ADJ_BYTES + JOIN_CELL_BYTES;
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
        for (int c = tid; c < TG_BLOCK_COLS * JOIN_CELLS; c += JOIN_THREADS) s_cell[c] = TG_EMPTY_KEY;
    }
    for (int64_t w = blockIdx.x; w < count; w += gridDim.x) {
    const int64_t v = wl ? (int64_t)(u32)wl[w] : w;
    if (v >= (MODE == 0 ? g.n : direct_count)) continue;
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
    if (nN == 0 || nN > nT || nN > TG_BLOCK_ROWS || nT < 2 || nT > ROWS || (MODE == 0 && nT > sm.BC) || ((nT + 15) >> 4) <= skip_le) continue;      // (the lists never hold a larger block)
    __syncthreads();                       // the previous block's epilogue has left the LDS header and the tile

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
        rp[it] = xbase + ((int64_t)min(bids[rv[it] ? row : 0], (u32)(g.n - 1)) * ldx + cpart) * ES;
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
        const int id = (int)min(bids[tid], (u32)(g.n - 1));
        s_ids[tid] = id;
        s_aux[tid] = (MODE == 0) ? __uint_as_float((u32)g.kth[id]) : (g.metric == 2 ? g.rnorm[id] : g.nrm[id]);
        if (MODE == 0) {
            const u64 kth = g.kth[id];                       // threshold distance and norm in one word
            s_okd[tid] = (u32)(kth >> 32);
            s_salt[tid] = (u32)tg_mix64(hs_slot + (u64)id);
        }
    }
    if (MODE == 0 && stat_bins && tid == 0) {
        const u64 pairs = (u64)nN * (u64)(nN - 1) / 2 + (u64)nN * (u64)(nT - nN);
        atomicAdd(stat_bins + (v & (TG_STAT_BINS - 1)), pairs);
        atomicAdd(stat_bins + TG_STAT_BINS + (v & (TG_STAT_BINS - 1)), (u64)nT);
    }
    if (MODE == 0 && tid < TG_BLOCK_COLS) {
        // which members sit in which member's list (adj_kernel): four words per member here
        const u32* aw = sm.adj + ((v / sm.parts) * sm.BC + tid) * (int64_t)sm.adj_words;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) s_adj[tid * 4 + wd] = (tid < nT && wd < sm.adj_words) ? aw[wd] : 0u;
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

    // ---- epilogue, in the "ordered integer" domain (tg_ord: unsigned order = float order).  Accumulator
    // element e of tile (i, j) in lane (c16, g4) is the pair (row a = 16 i + 4 g4 + e, column b = 16 j + c16).
    // A pair that must not count for a target gets every bit set in place of its distance.
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
        const int i = wr + 2 * ti;
        if (i >= MT) continue;
        float aux_a[4];
        u32 id_a[4], okd_a[4], adj_a[4][TJ];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int a = 16 * i + 4 * g4 + e;
            const int aa = a < nN ? a : 0;
            aux_a[e] = s_aux[aa];
            id_a[e] = (u32)s_ids[aa];
            if (MODE == 0) {
                okd_a[e] = a < nN ? s_okd[aa] : 0u;             // rows past the NEW part pass nothing
#pragma unroll
                for (int tj = 0; tj < TJ; ++tj) adj_a[e][tj] = s_adj[aa * 4 + ((wc + 2 * tj) >> 1)];
            }
        }
        const int a_mine = 16 * i + 4 * g4 + (c16 & 3);
        const u32 okd_mine = MODE == 0 ? (a_mine < nN ? s_okd[a_mine] : 0u) : 0u;
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) {
            if (!act[ti][tj]) continue;
            const int j = wc + 2 * tj;
            const int b = 16 * j + c16;
            const bool b_ok = b < nT;
            const int bb = b_ok ? b : 0;
            const float aux_b = s_aux[bb];
            const u32 id_b = (u32)s_ids[bb];
            u32 o[4];
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
                }
                o[e] = ok ? tg_ord(dist) : 0xFFFFFFFFu;
            }
            if (MODE == 0) {
                const u32 okd_b = b_ok ? s_okd[bb] : 0u;
                const u32 adj_b = s_adj[bb * 4 + (i >> 1)];                  // bit 16 (i & 1) + 4 g4 + e: row a sits in b's list
                // row node a meets column node b: b is a candidate of a unless a's list holds it, and a of b likewise
                u32 orow[4], ocol[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    orow[e] = o[e] | (u32)__builtin_amdgcn_sbfe((int)adj_a[e][tj], 16 * (j & 1) + c16, 1);
                    ocol[e] = o[e] | (u32)__builtin_amdgcn_sbfe((int)adj_b, 16 * (i & 1) + 4 * g4 + e, 1);
                }
                const u32 rmin = min(min(orow[0], orow[1]), min(orow[2], orow[3]));
                const u32 cmin = min(min(ocol[0], ocol[1]), min(ocol[2], ocol[3]));
                const u32 okd_amax = max(max(okd_a[0], okd_a[1]), max(okd_a[2], okd_a[3]));
                if (__ballot((rmin <= okd_amax && rmin != 0xFFFFFFFFu) || (cmin <= okd_b && cmin != 0xFFFFFFFFu)) == 0) continue;
                // row nodes: closest column node of each half of the tile (a group of eight positions)
                u32 ro[4], ri[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ro[e] = orow[e];
                    ri[e] = id_b;
                    groupmin8(ro[e], ri[e]);
                }
                const int e_mine = c16 & 3;
                const u32 mo = e_mine == 0 ? ro[0] : e_mine == 1 ? ro[1] : e_mine == 2 ? ro[2] : ro[3];
                const u32 mi = e_mine == 0 ? ri[0] : e_mine == 1 ? ri[1] : e_mine == 2 ? ri[2] : ri[3];
                if ((c16 & 7) < 4 && mo != 0xFFFFFFFFu && mo <= okd_mine)
                    atomicMin(s_cell + a_mine * JOIN_CELLS + ((2 * j + (c16 >> 3)) & 7), ((u64)mo << 32) | (u64)((mi << 2) | 3u));
                // column node b: closest row node over the lane's four rows (the two row quarters of a group meet in the cell)
                u64 cb = ((u64)ocol[0] << 32) | id_a[0];
#pragma unroll
                for (int e = 1; e < 4; ++e) cb = tg_min64(cb, ((u64)ocol[e] << 32) | id_a[e]);
                const u32 co = (u32)(cb >> 32), ci = (u32)cb;
                if (co != 0xFFFFFFFFu && co <= okd_b)
                    atomicMin(s_cell + b * JOIN_CELLS + ((2 * i + (g4 >> 1)) & 7), ((u64)co << 32) | (u64)((ci << 2) | 3u));
            }
        }
    }
    if (MODE == 0) {
        // Hand-over: the eight cells of a member sit in eight neighbouring lanes and their slots
        // share a 64-byte line, so a member's candidates travel as one transaction.  The cells
        // are left empty for the next block.
        __syncthreads();
        for (int c = tid; c < nT * JOIN_CELLS; c += JOIN_THREADS) {
            const u64 key = s_cell[c];
            if (key != TG_EMPTY_KEY) {
                s_cell[c] = TG_EMPTY_KEY;
                emit_candidate(cd, (u32)s_ids[c >> 3], (u32)(g.n - 1), s_salt[c >> 3], key, (u32)v, c & 7);
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
// use the same column permutation, so the sum is the full dot product.
//
// Waves walk a work list of anchors whose blocks have at most GMAX row groups, and the walk
// is software pipelined: while block w is multiplied, the ids, thresholds, norms and adjacency
// words of block w + 1 are fetched, and as soon as tile row i of block w is finished its
// registers X[i] are refilled with row group i of block w + 1.  MODE as in join_kernel.
// ---------------------------------------------------------------------------------------
struct WaveItem {
    int64_t v;
    const u32* bids;
    int nN, nT, MT, NT;       // MT = NT = 0: nothing to do for this item
};
// work record: anchor | |NEW| << 32 | (|NEW|+|OLD|) << 40
__device__ inline u64 pack_rec(u32 v, int nN, int nT) { return (u64)v | ((u64)nN << 32) | ((u64)nT << 40); }

struct WaveShared {
    u32 salt[2][64];
    u32 okd[2][64];
    int ids[2][64];
    float aux[2][64];
    u32 adj[2][64][2];         // member p, bit x: position x of the block is in p's list already
    u64 cell[2][64 * JOIN_CELLS];   // candidates of one block, one cell per (member, group of positions); handed over a block later
};

// NARROW: the rows come from the fp16 copy (g.Xh, rows of 32 KS values, zero padded): a register
// then holds eight values, columns 32 s + 8 q .. + 7, and a tile step is one
// v_mfma_f32_16x16x32_f16 (fp32 accumulation) in place of eight fp32 matrix instructions.
template <int GMAX, int MODE, int METRIC, int KS, bool FULL, bool NARROW>
__global__ __launch_bounds__(256) void join_wave_kernel(TgGraph g, TgSample sm, TgCand cd, u64 hs_slot, u64* stat_bins,
                                                        const int32_t* xblk, const int32_t* xsizes, float* xout,
                                                        const u64* __restrict__ wl, const u32* __restrict__ wl_cnt,
                                                        int64_t direct_count, int gmin)
{
    extern __shared__ __align__(16) unsigned char wave_smem[];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = tg_lane();
    WaveShared& sh = reinterpret_cast<WaveShared*>(wave_smem)[wave];
    const int r16 = lane & 15, q4 = lane >> 4;
    const float INF = __builtin_inff();
    if (g.f16_ok && (*g.f16_ok != 0u) != NARROW) return;      // the other variant's turn
    const int64_t count = wl ? (int64_t)*wl_cnt : direct_count;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const u32 idmax = (u32)(g.n - 1);

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
        const int nN = (int)((rec >> 32) & 0xFFu), nT = (int)((rec >> 40) & 0xFFu);
        const bool sane = MODE != 0 || ((u32)rec <= idmax && nN <= nT && nT <= sm.BC);
        it.v = sane ? (int64_t)(u32)rec : 0;
        it.bids = MODE == 0 ? sm.blk + it.v * (int64_t)sm.BC : reinterpret_cast<const u32*>(xblk) + it.v * TG_BLOCK_COLS;
        const int NT = (nT + 15) >> 4;
        const bool serve = sane && nN > 0 && nT >= 2 && NT <= GMAX && NT >= gmin;
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
            idr[t] = min(it.bids[row < it.nT ? row : 0], idmax);      // (a row past the block may hold anything)
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
    auto fetch_member = [&](const WaveItem& it, int id, float& aux, u64& kth, u64& adj) {
        if (MODE == 0) {
            kth = g.kth[id];
            aux = __uint_as_float((u32)kth);
            // which positions of the block this member's list holds already (adj_kernel); any lane reads a valid word
            adj = *reinterpret_cast<const u64*>(sm.adj + ((it.v >> sm.parts_shift) * sm.BC + (lane < it.nT ? lane : 0)) * (int64_t)sm.adj_words);
        } else {
            adj = 0ull;
            kth = 0ull;
            aux = METRIC == 2 ? g.rnorm[id] : g.nrm[id];
        }
    };
    auto park_member = [&](const WaveItem& it, int id, float aux, u64 kth, u64 adj, int buf) {
        if (lane < it.nT) {
            sh.ids[buf][lane] = id;
            sh.aux[buf][lane] = aux;
            if (MODE == 0) {
                sh.okd[buf][lane] = (u32)(kth >> 32);
                sh.salt[buf][lane] = (u32)tg_mix64(hs_slot + (u64)id);
                sh.adj[buf][lane][0] = (u32)adj;
                sh.adj[buf][lane][1] = (u32)(adj >> 32);
            }
        }
    };

    // Hand the cells of a finished block to the slot rows.  The eight cells of a member sit in eight
    // neighbouring lanes and their slots share a 64-byte line, so the atomics of one member travel
    // as one transaction.
    constexpr int CELLS = 64 * JOIN_CELLS;
    auto flush_cells = [&](int fbuf, u32 fv, int fnT) {
        const u64* cells = sh.cell[fbuf];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            const int p = 8 * s8 + (lane >> 3), q = lane & 7;
            if (8 * s8 < fnT) {
                const u64 key = p < fnT ? cells[p * JOIN_CELLS + q] : TG_EMPTY_KEY;
                if (key != TG_EMPTY_KEY) emit_candidate(cd, (u32)sh.ids[fbuf][p], idmax, sh.salt[fbuf][p], key, fv, q);
            }
        }
    };
    auto clear_cells = [&](int cbuf) {
#pragma unroll
        for (int c = 0; c < CELLS; c += 64) sh.cell[cbuf][c + lane] = TG_EMPTY_KEY;
    };
    auto lds_fence = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
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
        const int m0 = (int)min(cur.bids[lane < cur.nT ? lane : 0], idmax);
        float a0;
        u64 k0, j0;
        fetch_member(cur, m0, a0, k0, j0);
        park_member(cur, m0, a0, k0, j0, 0);
        fetch_row_ids(nxt, idn);
        mid = (int)min(nxt.bids[lane < nxt.nT ? lane : 0], idmax);
    }
    int buf = 0;
    u32 prev_v = 0;
    int prev_nT = 0;      // members of the block whose cells still wait in LDS

    // In round w: block w is multiplied, the rows, norms, thresholds and lists of block w + 1 are
    // fetched (their ids came in one round earlier), and the ids of block w + 2 start travelling.
    for (; w < count; w += nwaves) {
        const WaveItem nxt2 = decode(rec2);
        rec2 = load_rec(w + 3 * nwaves);
        u32 idn2[GMAX];
        fetch_row_ids(nxt2, idn2);
        const int mid2 = (int)min(nxt2.bids[lane < nxt2.nT ? lane : 0], idmax);
        float m_aux = 0.f;
        u64 m_kth = 0, m_adj = 0;

        lds_fence();
        const u32* s_okd = sh.okd[buf];
        const int* s_ids = sh.ids[buf];
        const float* s_aux = sh.aux[buf];
        const int64_t v = cur.v;
        const int nN = cur.nN, nT = cur.nT, MT = cur.MT, NT = cur.NT;
        u64* cells = sh.cell[buf];
        if (MODE == 0) {
            if (prev_nT > 0) flush_cells(buf ^ 1, prev_v, prev_nT);
            clear_cells(buf);
            lds_fence();
        }
        if (MODE == 0 && stat_bins && lane == 0 && MT > 0) {
            const u64 pairs = (u64)nN * (u64)(nN - 1) / 2 + (u64)nN * (u64)(nT - nN);
            atomicAdd(stat_bins + (v & (TG_STAT_BINS - 1)), pairs);
            atomicAdd(stat_bins + TG_STAT_BINS + (v & (TG_STAT_BINS - 1)), (u64)nT);
        }

#pragma unroll
        for (int i = 0; i < GMAX; ++i) {
            // Row side of this tile row: accumulator element e of lane (r16, q4) is row
            // a = 16 i + 4 q4 + e.  Everything below works on "ordered" distances (tg_ord:
            // unsigned order = float order); a pair that must not count gets +inf added, so
            // no validity masks have to be carried around.
            float aux_a[4], pen_a[4];
            u32 ida_key[4], okd_a[4], adj_a[4] = {0u, 0u, 0u, 0u};
            const int rowc = (16 * i + 4 * q4) * JOIN_CELLS + (r16 >> 3);      // cell (first of the lane's rows, column group 0) of this lane's half of a tile
            if (i < MT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int a = 16 * i + 4 * q4 + e;
                    const int aa = a < nN ? a : 0;
                    pen_a[e] = a < nN ? 0.f : INF;
                    // L2: the penalty rides on the norm (norm + 0 is the norm, bit for bit)
                    aux_a[e] = METRIC == 0 ? s_aux[aa] + pen_a[e] : s_aux[aa];
                    ida_key[e] = ((u32)s_ids[aa] << 2) | 3u;
                    okd_a[e] = (MODE == 0 && a < nN) ? s_okd[aa] : 0u;
                }
            }
            const int colc = r16 * JOIN_CELLS + (q4 >> 1);     // cell (column r16 of column group 0, row group 0)
            {
#pragma unroll
                for (int j = i; j < GMAX; ++j) {
                    if (i >= MT) continue;
                    if (MODE == 0 && (j == i || (j == 2 && i < 2))) {
                        // the half of the rows' adjacency words that covers the columns from here on
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int a = 16 * i + 4 * q4 + e;
                            adj_a[e] = sh.adj[buf][a < nN ? a : 0][j >> 1];
                        }
                    }
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
                        const u32 okd_b = b < nT ? s_okd[bb] : 0u;
                        const u32 adj_b = sh.adj[buf][bb][i >> 1];        // bit 16 (i & 1) + 4 q4 + e: row a sits in b's list
                        const u32 idb_key = (id_b << 2) | 3u;
                        // b is a candidate of a unless a's list holds it, and a of b likewise: such a pair gets every bit set
                        // (the ordered +inf of a masked pair is 0xFF800000: neither passes any threshold of a finite list).
                        // Every pair that may precede its target's last entry goes straight to the target's cell for this
                        // group of eight positions, which keeps the minimum (ds_min_u64): the closest of the group arrives
                        // there whatever else does, and nothing else is asked of the cell.  (At the threshold's own distance a
                        // candidate passes whatever its id: the list update sorts that out.)
                        u32 orow[4], ocol[4];
                        bool prow[4], pcol[4], any = false;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            orow[e] = o[e] | (u32)__builtin_amdgcn_sbfe((int)adj_a[e], 16 * (j & 1) + r16, 1);
                            ocol[e] = o[e] | (u32)__builtin_amdgcn_sbfe((int)adj_b, 16 * (i & 1) + 4 * q4 + e, 1);
                            prow[e] = orow[e] <= okd_a[e];
                            pcol[e] = ocol[e] <= okd_b;
                            any |= prow[e] | pcol[e];
                        }
                        // nothing in this tile can precede any threshold: the common case in late rounds
                        if (__ballot(any) == 0) continue;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (prow[e]) atomicMin(cells + rowc + (e * JOIN_CELLS + 2 * j), ((u64)orow[e] << 32) | (u64)idb_key);
                            if (pcol[e]) atomicMin(cells + colc + (16 * j * JOIN_CELLS + 2 * i), ((u64)ocol[e] << 32) | (u64)ida_key[e]);
                        }
                    }
                }
            }
            if (i == 0) {
                // the next block's ids have arrived behind the first tile row: ask for its norms and thresholds
                fetch_member(nxt, mid, m_aux, m_kth, m_adj);
            }
            // Row group i is used by tile rows min(i, MT - 1) and earlier: once tile row i is done
            // (and it is not the last one) its registers can take in the next block.
            if (i + 1 < MT) load_group(i, idn[i]);
        }
        // whatever the last tile row still needed
#pragma unroll
        for (int i = 0; i < GMAX; ++i)
            if (i + 1 >= MT) load_group(i, idn[i]);
        lds_fence();
        if (MODE == 0) {
            // the block's cells wait in LDS for one more round; its member data are needed for
            // that, so the next block's member data go to the buffer of the block before
            prev_v = (u32)v;
            prev_nT = MT > 0 ? nT : 0;
        }
        park_member(nxt, mid, m_aux, m_kth, m_adj, buf ^ 1);
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
// Work lists: anchors with something to join, by part of the round (v mod parts) and by block size.
// List 0: at most 3 row groups, list 1: exactly 4, list 2: more.  Without the wave kernel (longer rows
// or lists) list 1 takes every block of at most 4 row groups and list 0 stays empty.  The list of
// (part, size class) is wl + (part * 3 + class) * cap with cap = ceil(n / parts) records.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bin_kernel(TgSample sm, int64_t n, int wave_ok, int parts, int64_t cap)
{
    __shared__ u32 lcnt[TG_WL_LISTS], lbase[TG_WL_LISTS];
    const int tid = threadIdx.x;
    if (tid < TG_WL_LISTS) lcnt[tid] = 0u;
    __syncthreads();
    const int64_t v = (int64_t)blockIdx.x * 256 + tid;
    int list = -1, nN = 0, nT = 0;
    if (v < n) {
        const u32 z = sm.bsz[v];
        nN = (int)(z & 0xFFu);
        nT = (int)(z >> 8);
        if (nN > 0 && nT >= 2) {
            const int NT = (nT + 15) >> 4;
            const int bin = NT > 4 ? 2 : (NT == 4 || !wave_ok) ? 1 : 0;
            list = (int)(v % parts) * 3 + bin;
        }
    }
    // place inside the workgroup's share of the list, then one global atomic per workgroup and list
    const u32 mypos = list >= 0 ? atomicAdd(lcnt + list, 1u) : 0u;
    __syncthreads();
    if (tid < TG_WL_LISTS) lbase[tid] = lcnt[tid] ? atomicAdd(sm.wl_cnt + tid, lcnt[tid]) : 0u;
    __syncthreads();
    if (list >= 0 && (int64_t)lbase[list] + mypos < cap) sm.wl[(int64_t)list * cap + lbase[list] + mypos] = pack_rec((u32)v, nN, nT);
}

static size_t join_lds_bytes(int DK, int rows)
{
    return JOIN_HDR_BYTES + JOIN_ADJ_BYTES + JOIN_CELL_BYTES + (size_t)rows * (DK + 4) * sizeof(float);
}

// LDS beyond 64 KB per workgroup has to be asked for once per kernel
template <class K>
static void allow_large_lds(K kernel, size_t bytes)
{
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

#define JOIN_GRID 2048     // persistent launches: workgroups walk the work list with this stride

static int64_t wl_cap(int64_t n, int parts) { return (n + parts - 1) / parts; }

// the workgroup kernel on one work list; ROWS = the most members a block of that list has
template <int DK, int ROWS>
static void launch_join_list(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list, int parts,
                             hipStream_t s)
{
    static bool once = (allow_large_lds(join_kernel<DK, 0, false, ROWS>, join_lds_bytes(DK, ROWS)),
                        allow_large_lds(join_kernel<DK, 0, true, ROWS>, join_lds_bytes(DK, ROWS)), true);
    (void)once;
    const int rows = sm.BC < ROWS ? sm.BC : ROWS;   // a stored block never exceeds BC rows
    const int64_t cap = wl_cap(g.n, parts);
    const unsigned grid = (unsigned)(cap < JOIN_GRID ? cap : JOIN_GRID);
    // with the device flag both variants are launched, and the one it does not name ends at once
    if (g.Xh)
        hipLaunchKernelGGL((join_kernel<DK, 0, true, ROWS>), dim3(grid), dim3(JOIN_THREADS), join_lds_bytes(DK, rows), s, g, sm, c,
                           hs_slot, stat_bins, (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr,
                           (const u64*)(sm.wl + (int64_t)list * cap), (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_kernel<DK, 0, false, ROWS>), dim3(grid), dim3(JOIN_THREADS), join_lds_bytes(DK, rows), s, g, sm, c,
                           hs_slot, stat_bins, (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr,
                           (const u64*)(sm.wl + (int64_t)list * cap), (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
}
// wave_done: the register-resident kernel has served the classes 0 and 1
static void launch_join_wg(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, bool wave_done,
                           int part, int parts, hipStream_t s)
{
    if (g.ld > 64 || (g.Xh && g.ldh > 128)) {           // half as many slabs and barriers
        if (!wave_done) launch_join_list<128, 64>(g, sm, c, hs_slot, stat_bins, part * 3 + 1, parts, s);
        launch_join_list<128, TG_BLOCK_COLS>(g, sm, c, hs_slot, stat_bins, part * 3 + 2, parts, s);
    } else {
        if (!wave_done) launch_join_list<64, 64>(g, sm, c, hs_slot, stat_bins, part * 3 + 1, parts, s);
        launch_join_list<64, TG_BLOCK_COLS>(g, sm, c, hs_slot, stat_bins, part * 3 + 2, parts, s);
    }
}

template <int GMAX, int METRIC, int KS>
static void launch_wave_k(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list, int parts,
                          hipStream_t s)
{
    const int64_t cap = wl_cap(g.n, parts);
    const int64_t wgs = (cap + 3) / 4;
    const unsigned grid = (unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID);
    const size_t shm = 4 * sizeof(WaveShared);
    if (g.Xh)       // rows of the fp16 copy are whole steps of 32 values: KS / 2 of them
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS / 2, true, true>), dim3(grid), dim3(256), shm, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * cap),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    if (g.Xh && !g.f16_ok) return;
    if (g.ld == 16 * KS)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS, true, false>), dim3(grid), dim3(256), shm, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * cap),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
    else
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 0, METRIC, KS, false, false>), dim3(grid), dim3(256), shm, s, g, sm, c, hs_slot, stat_bins,
                           (const int32_t*)nullptr, (const int32_t*)nullptr, (float*)nullptr, (const u64*)(sm.wl + (int64_t)list * cap),
                           (const u32*)(sm.wl_cnt + list), (int64_t)0, 0);
}
template <int GMAX, int METRIC, int KS>
static void launch_wave_dump_k(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out, int gmin,
                               hipStream_t s)
{
    TgSample sm = {};
    TgCand c = {};
    const int64_t wgs = (nb + 3) / 4;
    const size_t shm = 4 * sizeof(WaveShared);
    if (g.Xh)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 1, METRIC, KS / 2, true, true>), dim3((unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID)),
                           dim3(256), shm, s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr, (const u32*)nullptr, nb, gmin);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_wave_kernel<GMAX, 1, METRIC, KS, false, false>), dim3((unsigned)(wgs < JOIN_GRID ? wgs : JOIN_GRID)),
                           dim3(256), shm, s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr, (const u32*)nullptr, nb, gmin);
}
// rows of at most 64 / 96 / 128 floats take 4 / 6 / 8 column steps per lane quarter
template <int GMAX, int METRIC>
static void launch_wave_m(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list, int parts,
                          hipStream_t s)
{
    if (g.ld <= 64) launch_wave_k<GMAX, METRIC, 4>(g, sm, c, hs_slot, stat_bins, list, parts, s);
    else if (g.ld <= 96) launch_wave_k<GMAX, METRIC, 6>(g, sm, c, hs_slot, stat_bins, list, parts, s);
    else launch_wave_k<GMAX, METRIC, 8>(g, sm, c, hs_slot, stat_bins, list, parts, s);
}
template <int GMAX>
static void launch_wave_t(const TgGraph& g, const TgSample& sm, const TgCand& c, u64 hs_slot, u64* stat_bins, int list, int parts,
                          hipStream_t s)
{
    if (g.metric == 0) launch_wave_m<GMAX, 0>(g, sm, c, hs_slot, stat_bins, list, parts, s);
    else if (g.metric == 1) launch_wave_m<GMAX, 1>(g, sm, c, hs_slot, stat_bins, list, parts, s);
    else launch_wave_m<GMAX, 2>(g, sm, c, hs_slot, stat_bins, list, parts, s);
}
template <int GMAX, int METRIC>
static void launch_wave_dump(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out, int gmin,
                             hipStream_t s)
{
    if (g.ld <= 64) launch_wave_dump_k<GMAX, METRIC, 4>(g, blk, sizes, nb, out, gmin, s);
    else if (g.ld <= 96) launch_wave_dump_k<GMAX, METRIC, 6>(g, blk, sizes, nb, out, gmin, s);
    else launch_wave_dump_k<GMAX, METRIC, 8>(g, blk, sizes, nb, out, gmin, s);
}

// The register-resident kernel applies to rows of at most 128 floats.
static bool wave_path(const TgGraph& g) { return g.ld <= 128; }

void tg_launch_bin(const TgGraph& g, const TgSample& sm, int parts, hipStream_t s)
{
    tg_launch_fill_u32(sm.wl_cnt, TG_WL_LISTS, 0u, s);
    hipLaunchKernelGGL(bin_kernel, dim3((unsigned)((g.n + 255) / 256)), dim3(256), 0, s, sm, g.n, wave_path(g) ? 1 : 0, parts,
                       wl_cap(g.n, parts));
}

void tg_launch_join(const TgGraph& g, const TgSample& sm, const TgCand& c, int part, int parts, uint64_t hs_slot,
                    unsigned long long* stat_bins, hipStream_t s)
{
    const bool wv = wave_path(g);
    if (wv) {
        launch_wave_t<3>(g, sm, c, hs_slot, stat_bins, part * 3 + 0, parts, s);
        launch_wave_t<4>(g, sm, c, hs_slot, stat_bins, part * 3 + 1, parts, s);
    }
    launch_join_wg(g, sm, c, hs_slot, stat_bins, wv, part, parts, s);
}

void tg_launch_join_distances(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out,
                              hipStream_t s)
{
    TgSample sm = {};
    TgCand c = {};
    static bool once = (allow_large_lds(join_kernel<64, 1, false>, join_lds_bytes(64, TG_BLOCK_COLS)),
                        allow_large_lds(join_kernel<64, 1, true>, join_lds_bytes(64, TG_BLOCK_COLS)), true);
    (void)once;
    int skip_le = 0;
    if (wave_path(g)) {      // same routing by block size as the production join
        if (g.metric == 0) { launch_wave_dump<3, 0>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 0>(g, blk, sizes, nb, out, 4, s); }
        else if (g.metric == 1) { launch_wave_dump<3, 1>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 1>(g, blk, sizes, nb, out, 4, s); }
        else { launch_wave_dump<3, 2>(g, blk, sizes, nb, out, 0, s); launch_wave_dump<4, 2>(g, blk, sizes, nb, out, 4, s); }
        skip_le = 4;
    }
    if (g.Xh)
        hipLaunchKernelGGL((join_kernel<64, 1, true>), dim3((unsigned)(nb < JOIN_GRID ? nb : JOIN_GRID)), dim3(JOIN_THREADS),
                           join_lds_bytes(64, TG_BLOCK_COLS), s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr,
                           (const u32*)nullptr, nb, skip_le);
    if (!g.Xh || g.f16_ok)
        hipLaunchKernelGGL((join_kernel<64, 1, false>), dim3((unsigned)(nb < JOIN_GRID ? nb : JOIN_GRID)), dim3(JOIN_THREADS),
                           join_lds_bytes(64, TG_BLOCK_COLS), s, g, sm, c, 0ull, (u64*)nullptr, blk, sizes, out, (const u64*)nullptr,
                           (const u32*)nullptr, nb, skip_le);
}
