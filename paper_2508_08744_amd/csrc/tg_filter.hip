// Distance-based and angle-based pruning of a k-NN graph in the Collect-Filter-Store procedure
// (section 5.1; the NSG, Vamana and NSSG rows of the table of pruning strategies, section 3.2).
// For node p the candidates are its neighbours (hops = 1) or those and their neighbours
// (hops = 2), ordered by (dis(p, c), id) and cut to cand_size; they are taken closest first and
// p' is inserted iff, for every p* inserted before,
//   distance rule:  dis(p, p') < alpha dis(p*, p')   (distances are squared here: alpha^2), or
//   angle rule:     the angle between p -> p* and p -> p' exceeds gamma; with the squared
//                   lengths a = |p p*|^2, b = |p p'|^2, c = |p* p'|^2 and t = a + b - c that is
//                   t < 0 or t^2 < 4 cos^2(gamma) a b   (no square root, no division),
// until d_out are in.  The dispersion rule (DPG) has no threshold: the nearest candidate is
// inserted first, then again and again the candidate whose angles at p to the inserted nodes add
// up to the most (equal sums: the nearer one), until d_out are in or none is left.
//
// One wave per node.  Section 5.2 evaluates a batch of candidates against the neighbour that
// was inserted last, one batch per insertion.  Here the candidate rows (at most 64) are loaded
// once into registers in matrix-core operand layout and ALL their pairwise products are
// formed at once (a Gram matrix on v_mfma_f32_16x16x4_f32, upper triangle of 16 x 16 tiles);
// what remains of the serial rule is bit arithmetic: every candidate gets the 64-bit set of
// the candidates in front of it that would occlude it, and the set of inserted candidates is the
// fixed point of "inserted iff no inserted candidate occludes me", found in a few passes.  The rows are the only large HBM traffic
// (4 d bytes per candidate); the products are cheap next to it.
//
// Lane (r, q) = (lane % 16, lane / 16) holds, for row group t and column step s, columns
// 16 s + 4 q .. + 3 of the current chunk of columns of candidate 16 t + r: one load instruction
// reads 64 contiguous bytes of each of 16 rows.  dis(p, c) is summed in difference form from
// the same registers.
#include "tg_device.h"
#include "tg_kernels.h"

// Collect: the neighbours; those and theirs for rows of at most 32 ids; the same for rows of up to 64 ids
// (a larger id set and queue per wave, which leaves room for three waves per workgroup)
#define FILTER_ONE_HOP 1
#define FILTER_TWO_HOPS 2
#define FILTER_TWO_HOPS_WIDE 3
// id set (a power of two, at most half full) and queue of the 2-hop collection: at most k + k * k ids
__host__ __device__ constexpr int filter_set_words(int collect) { return collect == FILTER_TWO_HOPS_WIDE ? 8192 : 2048; }
__host__ __device__ constexpr int filter_queue_words(int collect) { return collect == FILTER_TWO_HOPS_WIDE ? 4224 : 1088; }
__host__ __device__ constexpr int filter_waves(int collect) { return collect == FILTER_TWO_HOPS_WIDE ? 3 : 4; }
#define FILTER_GRID 16384
#define FILTER_FREE 0xFFFFFFFFu

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct FilterArgs {
    const float* X;
    int64_t n;
    int32_t d;
    const int32_t* ids;
    int32_t k, kp;          // kp: k rounded up to a power of two
    int32_t hops, cand_size;
    float thr;              // alpha^2 (distance rule) or 4 cos^2(gamma) (angle rule)
    int32_t d_out;
    int32_t* out_ids;
    int32_t* out_deg;
};

__device__ inline float4 filter_load4(const float* row, int col, int d, bool full, bool vec)
{
    if (full) return *reinterpret_cast<const float4*>(row + col);
    if (vec) return col < d ? *reinterpret_cast<const float4*>(row + col) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 v;
    v.x = col + 0 < d ? row[col + 0] : 0.f;
    v.y = col + 1 < d ? row[col + 1] : 0.f;
    v.z = col + 2 < d ? row[col + 2] : 0.f;
    v.w = col + 3 < d ? row[col + 3] : 0.f;
    return v;
}

// Loads the chunk [c0, c0 + 16 KS) of the rows cid[0 .. cnt) (16 NG >= cnt; rows past cnt repeat
// row 0) and adds this lane's share of the squared differences to node p's row into dp[t].
template <int NG, int KS, bool FULL, bool VEC>
__device__ inline void filter_load_chunk(const FilterArgs& A, const float* xp, const int* cid, int cnt, int c0,
                                         float4 (&X)[NG][KS], float (&dp)[NG])
{
    const int lane = tg_lane(), r16 = lane & 15, q4 = lane >> 4;
    const float* rp[NG];
#pragma unroll
    for (int t = 0; t < NG; ++t) {
        const int row = 16 * t + r16;
        rp[t] = A.X + (int64_t)cid[row < cnt ? row : 0] * A.d;
    }
#pragma unroll
    for (int t = 0; t < NG; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s) X[t][s] = filter_load4(rp[t], c0 + 16 * s + 4 * q4, A.d, FULL, VEC);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const float4 a = filter_load4(xp, c0 + 16 * s + 4 * q4, A.d, FULL, VEC);
#pragma unroll
        for (int t = 0; t < NG; ++t) {
            const float t0 = a.x - X[t][s].x, t1 = a.y - X[t][s].y, t2 = a.z - X[t][s].z, t3 = a.w - X[t][s].w;
            dp[t] += t0 * t0 + t1 * t1 + t2 * t2 + t3 * t3;
        }
    }
}

// the four quarter sums of a row meet: afterwards every lane (r, q) holds the whole sum of row 16 t + r
template <int NG>
__device__ inline void filter_reduce_quarters(float (&dp)[NG])
{
#pragma unroll
    for (int t = 0; t < NG; ++t) {
        dp[t] += __shfl_xor(dp[t], 16);
        dp[t] += __shfl_xor(dp[t], 32);
    }
}

template <int NG>
__device__ inline float filter_own(const float (&dp)[NG], int q4)
{
    // lane 16 q + r speaks for row 16 q + r (bit selects: an indexed read would go through scratch)
    if (NG == 1) return dp[0];
    if (NG == 2) return (q4 & 1) ? dp[1] : dp[0];
    const float lo = (q4 & 1) ? dp[1] : dp[0];
    const float hi = (q4 & 1) ? dp[NG - 1] : dp[2];
    return (q4 & 2) ? hi : lo;
}

template <int WORDS>
__device__ inline bool filter_set_insert(u32* tab, u32 id, bool active)
{
    bool present = false, pending = active;
    u32 h = (id * 0x9E3779B1u) >> (WORDS == 8192 ? 19 : 21);          // the top log2(WORDS) bits
    while (__ballot(pending)) {
        if (pending) {
            const u32 old = atomicCAS(tab + h, FILTER_FREE, id);
            if (old == FILTER_FREE) pending = false;
            else if (old == id) { present = true; pending = false; }
            else h = (h + 1) & (WORDS - 1);
        }
    }
    return present;
}

// Angle at p between p -> r and p -> c from the squared lengths a = |p r|^2, b = |p c|^2, c = |r c|^2:
// acos((a + b - c) / (2 sqrt(a b))), the arc cosine from the eight-term polynomial of Abramowitz and
// Stegun 4.4.46 (acos x = sqrt(1 - x) (a0 + .. + a7 x^7) on [0, 1], pi - acos(-x) below 0).  Every
// operation is rounded once, in this order, so that a host program can follow it bit for bit.
// A node at p's position (a b = 0) has no direction: angle 0.
__device__ inline float filter_angle_at(float a, float b, float c)
{
#pragma clang fp contract(off)
    const float ab = a * b;
    const float den = 2.0f * sqrtf(ab);
    const float t = (a + b) - c;
    float x = t / den;
    x = x > 1.0f ? 1.0f : x;
    x = x < -1.0f ? -1.0f : x;
    const float ax = fabsf(x);
    float pol = -0.0012624911f;
    pol = fmaf(pol, ax, 0.0066700901f);
    pol = fmaf(pol, ax, -0.0170881256f);
    pol = fmaf(pol, ax, 0.0308918810f);
    pol = fmaf(pol, ax, -0.0501743046f);
    pol = fmaf(pol, ax, 0.0889789874f);
    pol = fmaf(pol, ax, -0.2145988016f);
    pol = fmaf(pol, ax, 1.5707963050f);
    const float r = sqrtf(1.0f - ax) * pol;
    const float th = x < 0.0f ? 3.14159265358979323846f - r : r;
    return ab > 0.0f ? th : 0.0f;
}

__global__ void angle_at_kernel(const float* a, const float* b, const float* c, float* out, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = filter_angle_at(a[i], b[i], c[i]);
}
void tg_launch_angle_at(const float* a, const float* b, const float* c, float* out, int64_t count, hipStream_t s)
{
    hipLaunchKernelGGL(angle_at_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, a, b, c, out, count);
}

// maximum over the wave: xor butterfly by DPP inside each row of 16 lanes, then the four rows meet in scalar registers
__device__ inline u32 filter_wave_max(u32 x)
{
    x = max(x, tg_partner32<1>(x));
    x = max(x, tg_partner32<2>(x));
    x = max(x, tg_partner32<7>(x));
    x = max(x, tg_partner32<15>(x));
    const u32 r0 = (u32)__builtin_amdgcn_readlane((int)x, 0), r1 = (u32)__builtin_amdgcn_readlane((int)x, 16);
    const u32 r2 = (u32)__builtin_amdgcn_readlane((int)x, 32), r3 = (u32)__builtin_amdgcn_readlane((int)x, 48);
    return max(max(r0, r1), max(r2, r3));
}

__device__ inline void filter_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

#define FILTER_RULE_DIST 0
#define FILTER_RULE_ANGLE 1
#define FILTER_RULE_DISPERSION 2
// words of dynamic LDS per wave: the id set and queue of the 2-hop collection, and, later in the same
// words, the matrix of angles of the dispersion rule (rows of 16 NG + 1 words)
__host__ __device__ constexpr int filter_dyn_words(int ng, int collect, int rule)
{
    const int ids = collect == FILTER_ONE_HOP ? 0 : filter_set_words(collect) + filter_queue_words(collect);
    const int angles = rule == FILTER_RULE_DISPERSION ? 16 * ng * (16 * ng + 1) : 0;
    return ids > angles ? ids : angles;
}

template <int NG, int KS, bool FULL, bool VEC, int COLLECT, int RULE>
__global__ __launch_bounds__(256) void filter_dist_kernel(FilterArgs A)
{
    constexpr bool TWO_HOPS = COLLECT != FILTER_ONE_HOP;
    constexpr int WAVES = filter_waves(COLLECT);
    constexpr int SET_WORDS = filter_set_words(COLLECT);
    constexpr bool ANGLE = RULE == FILTER_RULE_ANGLE;
    constexpr int DYN = filter_dyn_words(NG, COLLECT, RULE);
    constexpr int AS = 16 * NG + 1;      // row stride of the matrix of angles
    extern __shared__ u32 dyn[];         // per wave: see filter_dyn_words
    __shared__ int s_cid[4][64];
    __shared__ __align__(16) float s_dpc[4][64];
    __shared__ __align__(16) float s_nrm[4][64];
    __shared__ u32 s_occ[4][128];
    __shared__ __align__(16) u64 s_key[4][64];       // the candidates' (distance, id) keys, read by every lane
    __shared__ u32 s_twin[4][256];                   // 1-hop: id -> first lane that lists it (128 ids, 128 lanes)
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int r16 = lane & 15, q4 = lane >> 4;
    int* cid = s_cid[wave];
    float* dpc = s_dpc[wave];
    float* nrm = s_nrm[wave];
    u32* occ = s_occ[wave];
    u64* skey = s_key[wave];
    const int k = A.k;
    const int nchunks = (A.d + 16 * KS - 1) / (16 * KS);

    for (int64_t p = (int64_t)blockIdx.x * WAVES + wave; p < A.n; p += (int64_t)gridDim.x * WAVES) {
        const float* xp = A.X + p * A.d;
        int m = 0;
        // ---- Collect ----
        const int32_t u = lane < k ? A.ids[p * k + lane] : -1;
        bool u_ok = u >= 0 && u < A.n && u != p;
        if (!TWO_HOPS) {
            // candidate l is entry l of the row; an entry that is no candidate (padding, p itself, an
            // id that an earlier entry lists already) keeps its place as a dead one and reads p's own row
            m = k;
            u32* tw = s_twin[wave];
            for (int i = lane; i < 256; i += 64) tw[i] = FILTER_FREE;
            filter_wave_sync();
            {
                bool pending = u_ok;
                u32 h = ((u32)u * 0x9E3779B1u) >> 25;
                while (__ballot(pending)) {
                    if (pending) {
                        const u32 old = atomicCAS(tw + h, FILTER_FREE, (u32)u);
                        if (old == FILTER_FREE || old == (u32)u) { atomicMin(tw + 128 + h, (u32)lane); pending = false; }
                        else h = (h + 1) & 127u;
                    }
                }
                filter_wave_sync();
                u_ok = u_ok && tw[128 + h] == (u32)lane;
            }
            cid[lane] = u_ok ? u : (int)p;
            filter_wave_sync();
        } else {
            u32* set = dyn + wave * DYN;
            int* queue = reinterpret_cast<int*>(set + SET_WORDS);
            for (int i = lane; i < SET_WORDS; i += 64) set[i] = FILTER_FREE;
            filter_wave_sync();
            int Q = 0;
            {
                const bool fresh = u_ok && !filter_set_insert<SET_WORDS>(set, (u32)u, u_ok);
                const u64 mask = __ballot(fresh);
                if (fresh) queue[__popcll(mask & tg_lanemask_lt())] = u;
                Q = __popcll(mask);
            }
            const int per = 64 / A.kp;
            const int my_row = lane / A.kp, r = lane - my_row * A.kp;
            for (int j0 = 0; j0 < k; j0 += per) {
                const int j = j0 + my_row;
                const bool on = my_row < per && j < k && r < k;
                const int32_t uj = __shfl(u, on ? j : 0);
                const bool uj_ok = __shfl((int)u_ok, on ? j : 0) != 0;
                const int32_t w = (on && uj_ok) ? A.ids[(int64_t)uj * k + r] : -1;
                const bool w_ok = w >= 0 && w < A.n && w != p;
                const bool fresh = w_ok && !filter_set_insert<SET_WORDS>(set, (u32)w, w_ok);
                const u64 mask = __ballot(fresh);
                if (fresh) queue[Q + __popcll(mask & tg_lanemask_lt())] = w;
                Q += __popcll(mask);
            }
            filter_wave_sync();
            // distance to p of everything collected, 64 at a time; the 64 closest stay, in order
            u64 best = TG_EMPTY_KEY;
            for (int b0 = 0; b0 < Q; b0 += 64) {
                const int cnt = min(64, Q - b0);
                float dp[4] = {0.f, 0.f, 0.f, 0.f};
                for (int c = 0; c < nchunks; ++c) {
                    float4 X[4][KS];
                    filter_load_chunk<4, KS, FULL, VEC>(A, xp, queue + b0, cnt, c * 16 * KS, X, dp);
                }
                filter_reduce_quarters<4>(dp);
                const float own = filter_own<4>(dp, q4);
                u64 key = lane < cnt ? tg_key(own, (u32)queue[b0 + lane], 0u) : TG_EMPTY_KEY;
                key = tg_wave_sort(key);
                best = b0 == 0 ? key : tg_wave_merge_low(best, key);
            }
            m = min(min(Q, 64), A.cand_size);
            if (lane < m) cid[lane] = (int)tg_key_id(best);
            filter_wave_sync();
        }
        if (m > 16 * NG) m = 16 * NG;          // never true: the launcher sizes NG for the largest candidate set
        if (m == 0) {
            if (lane < A.d_out) A.out_ids[p * A.d_out + lane] = -1;
            if (A.out_deg && lane == 0) A.out_deg[p] = 0;
            filter_wave_sync();
            continue;
        }

        // ---- Filter: rows into registers, dis(p, c) and the Gram matrix of the candidates ----
        floatx4 acc[NG][NG];
#pragma unroll
        for (int i = 0; i < NG; ++i)
#pragma unroll
            for (int j = 0; j < NG; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        float dp[NG];
#pragma unroll
        for (int t = 0; t < NG; ++t) dp[t] = 0.f;
        const int groups = (m + 15) >> 4;
        for (int c = 0; c < nchunks; ++c) {
            float4 X[NG][KS];
            filter_load_chunk<NG, KS, FULL, VEC>(A, xp, cid, m, c * 16 * KS, X, dp);
#pragma unroll
            for (int i = 0; i < NG; ++i) {
                if (i >= groups) break;                           // uniform
#pragma unroll
                for (int j = i; j < NG; ++j) {
                    if (j >= groups) break;
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s].x, X[j][s].x, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s].y, X[j][s].y, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s].z, X[j][s].z, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(X[i][s].w, X[j][s].w, acc[i][j], 0, 0, 0);
                    }
                }
            }
        }
        filter_reduce_quarters<NG>(dp);
        // accumulator register e of lane (r, q) in tile (i, j) is the product of rows 16 i + 4 q + e
        // and 16 j + r; the diagonal of tile (t, t) gives the squared norms
#pragma unroll
        for (int t = 0; t < NG; ++t) {
            const floatx4 a = acc[t][t];
            const float lo = (r16 & 1) ? a.y : a.x, hi = (r16 & 1) ? a.w : a.z;
            if (q4 == (r16 >> 2)) nrm[16 * t + r16] = (r16 & 2) ? hi : lo;
            if (q4 == 0) dpc[16 * t + r16] = dp[t];
        }
        occ[lane] = 0u;
        occ[lane + 64] = 0u;
        filter_wave_sync();
        // occ[C] = the candidates R that would occlude C: not dis(p, C) < alpha^2 dis(R, C), or an angle
        // at p of at most gamma (that relation is symmetric in R and C).  The lane holds its column's
        // four rows as a nibble; the mirrored pairs (rows and columns exchanged) of a tile off the
        // diagonal come out of ballots.
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            if (i >= groups) break;
            const float4 nR = *reinterpret_cast<const float4*>(nrm + 16 * i + 4 * q4);
            const float4 dR = *reinterpret_cast<const float4*>(dpc + 16 * i + 4 * q4);
#pragma unroll
            for (int j = i; j < NG; ++j) {
                if (j >= groups) break;
                const float nC = nrm[16 * j + r16];
                const float dC = dp[j];
                const floatx4 g = acc[i][j];
                const float rc0 = (nR.x + nC) - 2.0f * g.x;        // dis(R, C)
                const float rc1 = (nR.y + nC) - 2.0f * g.y;
                const float rc2 = (nR.z + nC) - 2.0f * g.z;
                const float rc3 = (nR.w + nC) - 2.0f * g.w;
                if (RULE == FILTER_RULE_DISPERSION) {
                    // the angle of every pair, stored both ways round (row R, column C and the reverse)
                    float* ang = reinterpret_cast<float*>(dyn + wave * DYN);
                    const int R = 16 * i + 4 * q4, C = 16 * j + r16;
                    const float th0 = filter_angle_at(dR.x, dC, rc0), th1 = filter_angle_at(dR.y, dC, rc1);
                    const float th2 = filter_angle_at(dR.z, dC, rc2), th3 = filter_angle_at(dR.w, dC, rc3);
                    ang[(R + 0) * AS + C] = th0; ang[(R + 1) * AS + C] = th1;
                    ang[(R + 2) * AS + C] = th2; ang[(R + 3) * AS + C] = th3;
                    ang[C * AS + R + 0] = th0; ang[C * AS + R + 1] = th1;
                    ang[C * AS + R + 2] = th2; ang[C * AS + R + 3] = th3;
                    continue;
                }
                bool o0, o1, o2, o3, m0, m1, m2, m3;               // R occludes C; C occludes R
                if (ANGLE) {
                    const float t0 = (dR.x + dC) - rc0, t1 = (dR.y + dC) - rc1, t2 = (dR.z + dC) - rc2, t3 = (dR.w + dC) - rc3;
                    o0 = m0 = !((t0 < 0.0f) | (t0 * t0 < A.thr * (dR.x * dC)));
                    o1 = m1 = !((t1 < 0.0f) | (t1 * t1 < A.thr * (dR.y * dC)));
                    o2 = m2 = !((t2 < 0.0f) | (t2 * t2 < A.thr * (dR.z * dC)));
                    o3 = m3 = !((t3 < 0.0f) | (t3 * t3 < A.thr * (dR.w * dC)));
                } else {
                    const float rhs0 = A.thr * rc0, rhs1 = A.thr * rc1, rhs2 = A.thr * rc2, rhs3 = A.thr * rc3;
                    o0 = !(dC < rhs0); o1 = !(dC < rhs1); o2 = !(dC < rhs2); o3 = !(dC < rhs3);
                    m0 = !(dR.x < rhs0); m1 = !(dR.y < rhs1); m2 = !(dR.z < rhs2); m3 = !(dR.w < rhs3);
                }
                const u32 nib = (u32)o0 | ((u32)o1 << 1) | ((u32)o2 << 2) | ((u32)o3 << 3);
                atomicOr(occ + 2 * (16 * j + r16) + (i >> 1), nib << (16 * (i & 1) + 4 * q4));
                if (j > i) {
                    const u64 b0 = __ballot(m0);
                    const u64 b1 = __ballot(m1);
                    const u64 b2 = __ballot(m2);
                    const u64 b3 = __ballot(m3);
                    if (r16 == 0) {
                        const int R = 16 * i + 4 * q4, sh = 16 * q4, word = j >> 1, up = 16 * (j & 1);
                        atomicOr(occ + 2 * (R + 0) + word, (u32)((b0 >> sh) & 0xFFFFull) << up);
                        atomicOr(occ + 2 * (R + 1) + word, (u32)((b1 >> sh) & 0xFFFFull) << up);
                        atomicOr(occ + 2 * (R + 2) + word, (u32)((b2 >> sh) & 0xFFFFull) << up);
                        atomicOr(occ + 2 * (R + 3) + word, (u32)((b3 >> sh) & 0xFFFFull) << up);
                    }
                }
            }
        }
        // before = the candidates in front of this lane's under (dis(p, c), id); dead entries have the
        // largest key and are in front of nothing
        const float own = filter_own<NG>(dp, q4);
        const int my_id = lane < m ? cid[lane] : 0;
        const bool dead = TWO_HOPS ? lane >= m : !u_ok;
        const u64 key = dead ? TG_EMPTY_KEY : tg_key(own, (u32)my_id, 0u);
        skey[lane] = key;
        filter_wave_sync();
        // one bit per other candidate, shifted in from below: after J steps candidate j sits at bit J - 1 - j
        u32 lt_lo = 0u, lt_hi = 0u;
        const int J = (m + 7) & ~7, J_lo = min(J, 32);
        for (int j0 = 0; j0 < J_lo; j0 += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) lt_lo = lt_lo + lt_lo + (skey[j0 + j] < key ? 1u : 0u);
        }
        for (int j0 = 32; j0 < J; j0 += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) lt_hi = lt_hi + lt_hi + (skey[j0 + j] < key ? 1u : 0u);
        }
        lt_lo = __brev(lt_lo) >> (32 - J_lo);
        lt_hi = J > 32 ? __brev(lt_hi) >> (64 - J) : 0u;
        const u64 live = ~__ballot(dead);
        const u64 before = (((u64)lt_hi << 32) | lt_lo) & live;
        filter_wave_sync();
        const u64 occ_by = (((u64)occ[2 * lane + 1] << 32) | occ[2 * lane]) & before;
        // ---- the serial rule as a fixed point ----
        // c is inserted iff no inserted candidate in front of it occludes it.  Starting from "all
        // inserted", every pass settles at least the next candidate in order, so the set stops
        // changing after at most m passes, and what it then holds obeys the rule.
        const bool in_cut = !dead && __popcll(before) < A.cand_size;       // the cut to cand_size counts candidates only
        if (RULE == FILTER_RULE_DISPERSION) {
            // ---- greedy insertion: one candidate per pass ----
            const float* ang = reinterpret_cast<const float*>(dyn + wave * DYN);
            const int want = min(A.d_out, __popcll(__ballot(in_cut)));
            const u32 rnk = (u32)__popcll(before);                  // place among the candidates, nearest first
            float score = 0.0f;                                     // sum of the angles to the inserted nodes
            bool open = in_cut;
            int my_pos = -1;
            u64 pick = __ballot(in_cut && rnk == 0u);               // the nearest candidate goes first
            for (int it = 0; it < want && pick != 0ull; ++it) {
                const int r_new = __ffsll((unsigned long long)pick) - 1;
                if (lane == r_new) { my_pos = it; open = false; }
                if (it + 1 >= want) break;
                score += lane < 16 * NG ? ang[r_new * AS + lane] : 0.0f;
                // sums are no less than +0, so their bit patterns order them; + 1 puts every open lane above the rest
                const u32 sb = open ? __float_as_uint(score) + 1u : 0u;
                const u32 top = filter_wave_max(sb);
                const bool first = open && sb == top;
                const u32 near = 64u - filter_wave_max(first ? 64u - rnk : 0u);
                pick = __ballot(first && rnk == near);
            }
            if (my_pos >= 0) A.out_ids[p * A.d_out + my_pos] = my_id;
            if (lane >= want && lane < A.d_out) A.out_ids[p * A.d_out + lane] = -1;
            if (A.out_deg && lane == 0) A.out_deg[p] = want;
            filter_wave_sync();
            continue;
        }
        u64 K = __ballot(in_cut);
        for (int pass = 0; pass < 65; ++pass) {
            const u64 Kn = __ballot(in_cut && (occ_by & K) == 0ull);
            if (Kn == K) break;
            K = Kn;
        }
        // ---- Store: insertion order is the order of the candidates; the first d_out are in ----
        const bool kept = (K >> lane) & 1ull;
        const int pos = __popcll(K & before);
        const int deg = min(__popcll(K), A.d_out);
        if (kept && pos < A.d_out) A.out_ids[p * A.d_out + pos] = my_id;
        if (lane >= deg && lane < A.d_out) A.out_ids[p * A.d_out + lane] = -1;
        if (A.out_deg && lane == 0) A.out_deg[p] = deg;
        filter_wave_sync();
    }
}

template <class K>
static void filter_launch(K kernel, const FilterArgs& A, int waves, size_t shm, hipStream_t s)
{
    // more than 64 KB of dynamic LDS has to be asked for
    if (shm > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
    int64_t wgs = (A.n + waves - 1) / waves;        // a wave per node; workgroups beyond the grid walk on
    if (wgs > FILTER_GRID) wgs = FILTER_GRID;
    hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(64 * waves), shm, s, A);
}

template <int NG, int COLLECT, int RULE>
static void launch_filter(const FilterArgs& A, bool vec, hipStream_t s)
{
    constexpr int grid = filter_waves(COLLECT);     // waves per workgroup; filter_launch sizes the grid from it
    const size_t shm = (size_t)filter_waves(COLLECT) * filter_dyn_words(NG, COLLECT, RULE) * sizeof(u32);
    // two row groups take their columns in chunks of 64, four in chunks of 32: few registers, so that
    // four (three) waves per SIMD cover each other's loads
    constexpr int KS = NG > 2 ? 2 : 4;
    const bool full = vec && (A.d % (16 * KS) == 0);         // no column guards needed
    if (full) filter_launch(filter_dist_kernel<NG, KS, true, true, COLLECT, RULE>, A, grid, shm, s);
    else if (vec) filter_launch(filter_dist_kernel<NG, KS, false, true, COLLECT, RULE>, A, grid, shm, s);
    else filter_launch(filter_dist_kernel<NG, KS, false, false, COLLECT, RULE>, A, grid, shm, s);
}

template <int RULE>
static void launch_filter_rule(const FilterArgs& A, bool vec, int most, hipStream_t s)
{
    // the 2-hop collection measures 64 candidates at a time, which needs the four-group instance
    if (A.hops == 2 && A.k > 32) launch_filter<4, FILTER_TWO_HOPS_WIDE, RULE>(A, vec, s);
    else if (A.hops == 2) launch_filter<4, FILTER_TWO_HOPS, RULE>(A, vec, s);
    else if (most <= 32) launch_filter<2, FILTER_ONE_HOP, RULE>(A, vec, s);
    else launch_filter<4, FILTER_ONE_HOP, RULE>(A, vec, s);
}

void tg_launch_filter(const float* X, int64_t n, int d, const int32_t* ids, int k, int hops, int cand_size, int rule, float thr,
                      int d_out, int32_t* out_ids, int32_t* out_deg, hipStream_t s)
{
    FilterArgs A;
    A.X = X; A.n = n; A.d = d; A.ids = ids; A.k = k;
    A.kp = 1;
    while (A.kp < k) A.kp <<= 1;
    A.hops = hops; A.cand_size = cand_size;
    A.thr = thr;
    A.d_out = d_out; A.out_ids = out_ids; A.out_deg = out_deg;
    const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const int most = hops == 1 ? k : (cand_size < 64 ? cand_size : 64);      // candidates that reach the filter
    if (rule == FILTER_RULE_DISPERSION) launch_filter_rule<FILTER_RULE_DISPERSION>(A, vec, most, s);
    else if (rule == FILTER_RULE_ANGLE) launch_filter_rule<FILTER_RULE_ANGLE>(A, vec, most, s);
    else launch_filter_rule<FILTER_RULE_DIST>(A, vec, most, s);
}
