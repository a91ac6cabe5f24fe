// Neighbour-list kernels: norms, random initial lists (Algorithm 1, initialisation), the
// lock-free list update of section 4.2, the phase-2 expand-and-update round
// (Algorithm 1, phase-2 loop), finalize, and state export/import.
//
// Ownership rule that makes the update lock-free: exactly one wavefront reads and
// rewrites a given list in a given kernel; other nodes reach a list only through its
// candidate slots (atomic minimum) or through the previous round's snapshot.
#include <hip/hip_fp16.h>
#include "tg_device.h"
#include "tg_kernels.h"

#define LISTS_WAVES 4   // wavefronts (= nodes) per workgroup

// ---------------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------------
__global__ void fill_u64_kernel(u64* p, size_t count, u64 v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = v;
}
__global__ void fill_u32_kernel(u32* p, size_t count, u32 v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = v;
}
static int grid_for(size_t count, int block)
{
    size_t g = (count + block - 1) / block;
    if (g > 65536) g = 65536;
    if (g < 1) g = 1;
    return (int)g;
}
void tg_launch_fill_u64(u64* p, size_t count, u64 v, hipStream_t s)
{
    if (count) hipLaunchKernelGGL(fill_u64_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, p, count, v);
}
void tg_launch_fill_u32(u32* p, size_t count, u32 v, hipStream_t s)
{
    if (count) hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, p, count, v);
}

// rows of d floats -> rows of ld floats, zero padded
__global__ void pad_rows_kernel(const float* __restrict__ X, int64_t n, int d, float* __restrict__ Xp, int ld)
{
    size_t total = (size_t)n * ld;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < total; i += stride) {
        size_t r = i / ld;
        int c = (int)(i - r * ld);
        Xp[i] = c < d ? X[r * (size_t)d + c] : 0.0f;
    }
}
void tg_launch_pad_rows(const float* X, int64_t n, int d, float* Xp, int ld, hipStream_t s)
{
    hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for((size_t)n * ld, 256)), dim3(256), 0, s, X, n, d, Xp, ld);
}

// ---------------------------------------------------------------------------------------
// squared norms: 16 lanes per row, float4 loads; workgroups walk the rows with the stride of
// the grid.  With `range` (words 0 and 1, ordered bits) the smallest and the largest value of X are
// found on the way, for the grid of the 8-bit codes of phase 2, and word TG_RANGE_NONINT is set when a
// value is not a whole number (finalize_kernel asks).  With `undefined`, rows that have no
// defined distance are counted there: a squared norm that is not a finite number (an infinite or
// undefined value in the row, or an overflow), and a zero norm where the reciprocal is asked for.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void norms_kernel(const float* __restrict__ X, int64_t n, int d, int ld,
                                                    float* __restrict__ nrm, float* __restrict__ rnorm, u32* __restrict__ range,
                                                    u32* __restrict__ undefined)
{
    __shared__ u32 s_lo[16], s_hi[16];
    const int sub = threadIdx.x & 15;
    float lo = __builtin_inff(), hi = -__builtin_inff();
    bool nonint = false;
    for (int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); row < n; row += (int64_t)gridDim.x * 16) {
        const float* x = X + row * (int64_t)ld;
        float acc = 0.0f;
        for (int c = sub * 4; c < ld; c += 64) {
            const float4 v = *reinterpret_cast<const float4*>(x + c);
            acc += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            if (range) {
                const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (c + i < d) { lo = fminf(lo, e[i]); hi = fmaxf(hi, e[i]); nonint |= !(e[i] == rintf(e[i])); }       // padding columns are no values
            }
        }
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        acc += __shfl_xor(acc, 4);
        acc += __shfl_xor(acc, 8);
        if (sub == 0) {
            nrm[row] = acc;
            if (rnorm) rnorm[row] = 1.0f / sqrtf(acc);
            if (undefined && (!(acc < __builtin_inff()) || (rnorm && !(acc > 0.0f)))) atomicAdd(undefined, 1u);
        }
    }
    if (!range) return;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if (sub == 0) { s_lo[threadIdx.x >> 4] = tg_ord(lo); s_hi[threadIdx.x >> 4] = tg_ord(hi); }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 a = s_lo[0], b = s_hi[0];
        for (int i = 1; i < 16; ++i) { a = min(a, s_lo[i]); b = max(b, s_hi[i]); }
        atomicMin(range + 0, a);
        atomicMax(range + 1, b);
    }
    if (__ballot(nonint) != 0ull && tg_lane() == 0 && range[TG_RANGE_NONINT] == 0u) range[TG_RANGE_NONINT] = 1u;
}
void tg_launch_norms(const TgGraph& g, uint32_t* range, uint32_t* undefined, hipStream_t s)
{
    if (undefined) tg_launch_fill_u32(undefined, 1, 0u, s);
    if (range) {
        tg_launch_fill_u32(range + 0, 1, 0xFF800000u, s);      // ordered +infinity: the smallest value so far
        tg_launch_fill_u32(range + 1, 1, 0x007FFFFFu, s);      // ordered -infinity
        tg_launch_fill_u32(range + TG_RANGE_NONINT, 1, 0u, s);
    }
    const int64_t wgs = (g.n + 15) / 16;
    hipLaunchKernelGGL(norms_kernel, dim3((unsigned)(wgs < 2048 ? wgs : 2048)), dim3(256), 0, s, g.X, g.n, g.d, g.ld, g.nrm,
                       g.metric == 2 ? g.rnorm : (float*)nullptr, range, undefined);
}

// ---------------------------------------------------------------------------------------
// 8-bit screening copy of X for phase 2.  One grid for the whole data set: lo = the smallest value
// of X, s = (the largest - lo) / 255; row x becomes the codes q_i = round((x_i - lo) / s) in 0..255,
// i.e. the vector xq_i = lo + s q_i.  Then |xq - yq|^2 = s^2 sum (qx_i - qy_i)^2 and <xq, yq> follow
// from integer dot products of the codes alone (nothing but the codes has to be fetched for a
// candidate), and |x - y| >= |xq - yq| - 2 err bounds the true distance from below, err being the
// largest |x - xq| of any row.  Byte-valued data have lo = 0, s = 1 and err = 0: the bound is the distance.
// grid: [0] ordered bits of lo, [1] of the largest value (both found by the kernel of the norms), [2] float bits of err.
// ---------------------------------------------------------------------------------------
// lo and s of the grid from its first two words (the same expressions wherever they are needed)
__device__ inline void quantize_grid(const u32* grid, float& lo, float& s)
{
    lo = tg_unord(grid[0]);
    const float hi = tg_unord(grid[1]);
    s = hi > lo ? (hi - lo) / 255.0f : 1.0f;
}
__global__ __launch_bounds__(256) void quantize_kernel(TgGraph g, uint8_t* __restrict__ Xq, u32* __restrict__ grid)
{
    __shared__ float s_err[16];
    const int sub = threadIdx.x & 15;
    float lo, s;
    quantize_grid(grid, lo, s);
    const float inv = 1.0f / s;
    const float alo = fabsf(lo);
    const int dq = g.ldq;
    float worst = 0.0f;          // largest |x - xq| of the rows this group of 16 lanes has coded
    for (int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); row < g.n; row += (int64_t)gridDim.x * 16) {
        const float* x = g.X + row * (int64_t)g.ld;
        uint8_t* out = Xq + row * (int64_t)g.ldq;
        float err2 = 0.0f, an2 = 0.0f;
        for (int c = sub * 4; c < dq; c += 64) {
            u32 packed = 0u;
            if (c < g.ld) {
                const float4 v = *reinterpret_cast<const float4*>(x + c);
                const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (c + i < g.d) {
                        const float q = fminf(255.0f, fmaxf(0.0f, rintf((e[i] - lo) * inv)));
                        const float r = fmaf(s, q, lo);
                        const float t = e[i] - r, a = fmaf(s, q, alo);
                        err2 = fmaf(t, t, err2);
                        an2 = fmaf(a, a, an2);
                        packed |= (u32)q << (8 * i);
                    }
                }
            }
            *reinterpret_cast<u32*>(out + c) = packed;
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            err2 += __shfl_xor(err2, o);
            an2 += __shfl_xor(an2, o);
        }
        // |x - xq| for the exact grid point xq: the measured distance to its fp32 value, rounded up, plus the
        // rounding of that value itself (half an ulp per component: far below 1e-6 of |lo| + s q)
        worst = fmaxf(worst, sqrtf(err2) * 1.0001f + 1e-6f * sqrtf(an2));
    }
    if (sub == 0) s_err[threadIdx.x >> 4] = worst;
    __syncthreads();
    if (threadIdx.x == 0) {
        float e = s_err[0];
        for (int i = 1; i < 16; ++i) e = fmaxf(e, s_err[i]);
        atomicMax(grid + 2, __float_as_uint(e));          // not negative: the bit patterns order the values
    }
}
void tg_launch_quantize(const TgGraph& g, uint8_t* Xq, float* Xqm, hipStream_t s)
{
    // the first two words of the grid (smallest and largest value of X) were found together with the norms
    u32* grid = reinterpret_cast<u32*>(Xqm);
    tg_launch_fill_u32(grid + 2, 1, 0u, s);
    const int64_t range_wgs = (g.n + 15) / 16;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)(range_wgs < 2048 ? range_wgs : 2048)), dim3(256), 0, s, g, Xq, grid);
}

// ---------------------------------------------------------------------------------------
// fp16 copy of the rows for the local join: round to nearest even, eight values per thread,
// zero beyond column d.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void narrow_kernel(TgGraph g, uint16_t* __restrict__ Xh, u32* exact_flag, u32* overflow_rows)
{
    bool inexact = false;
    const int per_row = g.ldh >> 3;
    const size_t total = (size_t)g.n * per_row;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const size_t row = i / per_row;
        const int c0 = (int)(i - row * per_row) * 8;
        const float* x = g.X + row * (size_t)g.ld;
        u32 h[8];
        bool over = false;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float val = c0 + e < g.d ? x[c0 + e] : 0.f;
            const __half hv = __float2half_rn(val);
            inexact |= __half2float(hv) != val;
            over |= fabsf(val) <= 3.4028234e38f && fabsf(__half2float(hv)) > 65504.f;      // a finite value that fp16 cannot hold
            h[e] = (u32)__half_as_ushort(hv);
        }
        if (over && overflow_rows) {
            // such a row is counted once: by the piece that holds its first such value (rare: the columns before are read again)
            bool first = true;
            for (int c = 0; c < c0 && first; ++c) first = !(fabsf(x[c]) > 65504.f && fabsf(x[c]) <= 3.4028234e38f);
            if (first) atomicAdd(overflow_rows, 1u);
        }
        *reinterpret_cast<uint4*>(Xh + row * (size_t)g.ldh + c0) =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
    // one store per wave that met such a value, and none once the flag is down
    if (exact_flag && __ballot(inexact) != 0ull && tg_lane() == 0 && *exact_flag != 0u) *exact_flag = 0u;
}
void tg_launch_narrow(const TgGraph& g, uint16_t* Xh, uint32_t* exact_flag, uint32_t* overflow_rows, hipStream_t s)
{
    hipLaunchKernelGGL(narrow_kernel, dim3(grid_for((size_t)g.n * (g.ldh >> 3), 256)), dim3(256), 0, s, g, Xh, exact_flag, overflow_rows);
}

// ---------------------------------------------------------------------------------------
// Distances from node v (its vector staged in LDS at xs, ld floats) to one candidate id per
// lane (cid < 0: none), computed directly from the vectors: sum (x-y)^2, -<x,y> or
// 1 - <x,y>/(|x||y|).  Candidates are compacted first so that only live rows are fetched.
// 16 lanes share one candidate row; a pass covers 4 NB candidates (NB per lane quarter) and
// 128 columns, with all 2 NB row loads of a lane in flight before the first is used: the wave
// is latency bound, so the number of dependent round trips is what counts.  NB = 8 suits
// full lists (initial lists, finalize), NB = 1 the few survivors of the phase-2 screening.
// wscr: 128 words of LDS private to this wave.
// ---------------------------------------------------------------------------------------
template <int N>
__device__ inline float row16_ror(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + N, 0xF, 0xF, false));
}
template <bool L2, int NB>
__device__ inline void direct_pass(const float* X, int ld, const float* xs, const u32* wscr, int p0, int nv, float (&acc)[NB])
{
    const int lane = tg_lane();
    const int grp = lane >> 4, sub = lane & 15;
    const float* y[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int p = p0 + 4 * q + grp;
        y[q] = X + (int64_t)wscr[p < nv ? p : nv - 1] * ld;   // rows past the end repeat the last one
        acc[q] = 0.0f;
    }
    for (int cb = 0; cb < ld; cb += 128) {
        // two column chunks per pass; a chunk past the row is read at column 0 and not counted
        const int c0 = cb + 4 * sub, c1 = c0 + 64;
        const bool r0 = c0 < ld, r1 = c1 < ld;
        const int cc0 = r0 ? c0 : 0, cc1 = r1 ? c1 : 0;
        float4 b0[NB], b1[NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            b0[q] = *reinterpret_cast<const float4*>(y[q] + cc0);
            b1[q] = *reinterpret_cast<const float4*>(y[q] + cc1);
        }
        const float4 a0 = *reinterpret_cast<const float4*>(xs + cc0);
        const float4 a1 = *reinterpret_cast<const float4*>(xs + cc1);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            float s0, s1;
            if (L2) {
                const float t0 = a0.x - b0[q].x, t1 = a0.y - b0[q].y, t2 = a0.z - b0[q].z, t3 = a0.w - b0[q].w;
                const float u0 = a1.x - b1[q].x, u1 = a1.y - b1[q].y, u2 = a1.z - b1[q].z, u3 = a1.w - b1[q].w;
                s0 = t0 * t0 + t1 * t1 + t2 * t2 + t3 * t3;
                s1 = u0 * u0 + u1 * u1 + u2 * u2 + u3 * u3;
            } else {
                s0 = a0.x * b0[q].x + a0.y * b0[q].y + a0.z * b0[q].z + a0.w * b0[q].w;
                s1 = a1.x * b1[q].x + a1.y * b1[q].y + a1.z * b1[q].z + a1.w * b1[q].w;
            }
            acc[q] += (r0 ? s0 : 0.0f) + (r1 ? s1 : 0.0f);
        }
    }
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        acc[q] += row16_ror<8>(acc[q]);
        acc[q] += row16_ror<4>(acc[q]);
        acc[q] += row16_ror<2>(acc[q]);
        acc[q] += row16_ror<1>(acc[q]);
    }
}
template <int NB>
__device__ inline float wave_direct_dist(const TgGraph& g, const float* xs, float rn_v, int cid, u32* wscr)
{
    const int lane = tg_lane();
    const int grp = lane >> 4, sub = lane & 15;
    const bool valid = cid >= 0;
    const u64 mask = __ballot(valid);
    const int nv = __popcll(mask);
    const int pos = __popcll(mask & tg_lanemask_lt());
    if (valid) wscr[pos] = (u32)cid;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float* wd = reinterpret_cast<float*>(wscr + 64);
    for (int p0 = 0; p0 < nv; p0 += 4 * NB) {
        float acc[NB];
        if (g.metric == 0) direct_pass<true, NB>(g.X, g.ld, xs, wscr, p0, nv, acc);
        else direct_pass<false, NB>(g.X, g.ld, xs, wscr, p0, nv, acc);
        // lane `sub` of each quarter speaks for candidate p0 + 4 sub + grp (sub < NB)
        float mine = acc[0];
#pragma unroll
        for (int q = 1; q < NB; ++q) mine = sub == q ? acc[q] : mine;
        const int p = p0 + 4 * sub + grp;
        if (sub < NB && p < nv) {
            float dist = mine;
            if (g.metric == 1) dist = -mine;
            else if (g.metric == 2) dist = 1.0f - mine * rn_v * g.rnorm[wscr[p]];
            wd[p] = dist;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float out = valid ? wd[pos] : 0.0f;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return out;
}

// ---------------------------------------------------------------------------------------
// Screening for phase 2: of one candidate id per lane (cid < 0: none) keep those whose
// distance to node v may still precede kd, judged on the 8-bit copy.  With the codes qx of v
// and qy of the candidate (integer dot products sum qx qy, sum qy qy, sum qy) and the grid
// (lo, s, err >= |x - xq| for every row):
//   |x - y| >= s sqrt(sum (qx - qy)^2) - 2 err                                   (squared L2)
//   <x, y> <= <xq, yq> + err (|yq| + |x|),  <xq, yq> = d lo^2 + lo s (sum qx + sum qy) + s^2 sum qx qy,
//   |yq|^2 = d lo^2 + 2 lo s sum qy + s^2 sum qy qy, and | |y| - |yq| | <= err    (inner product, cosine)
// are rigorous; the margins below cover the fp32 rounding of both these estimates and the
// exact evaluation that follows, so a dropped candidate could never have entered the list.
// Eight lanes share a candidate row (16 bytes each per 128 columns); survivors come back one
// per lane in a new order.  xq_s: v's codes in LDS; qxx, qx1: sum qx qx and sum qx of v;
// wscr: 64 words of LDS private to this wave.
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ inline u32 dpp_u32(u32 x)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
struct ScreenGrid {
    float lo, s, err;
};
__device__ inline int wave_screen(const TgGraph& g, const ScreenGrid& grid, const uint4* xq_s, u32 qxx, u32 qx1, float norm_v,
                                  float rn_v, int cid, u32* wscr, float kd)
{
    const int lane = tg_lane();
    const int sub = lane & 7, c8 = lane >> 3;
    const bool valid = cid >= 0;
    const u64 mask = __ballot(valid);
    const int nv = __popcll(mask);
    if (nv == 0) return -1;
    if (valid) wscr[__popcll(mask & tg_lanemask_lt())] = (u32)cid;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int nch = g.ldq >> 4;
    const bool ragged = (nch & 7) != 0;
    const bool l2 = g.metric == 0;
    // the lane (c8, sub) speaks for candidate 8 sub + c8; the eight lanes of a group take the candidates
    // 8 q + c8, q = 0..7, four at a time (two turns keep the sums of four candidates in registers, not of eight)
    const int p = 8 * sub + c8;
    const bool mine = p < nv;
    const u32 row = wscr[mine ? p : nv - 1];
    u32 xy = 0u, yy = 0u, y1 = 0u;
#pragma unroll 1
    for (int h = 0; h < 8; h += 4) {
        if (8 * h >= nv) break;                   // none of these four candidates exists (uniform)
        u32 rows[4], dxy[4], dyy[4], dy1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int pq = 8 * (h + q) + c8;
            rows[q] = wscr[pq < nv ? pq : nv - 1];      // candidates past the end repeat the last one
            dxy[q] = 0u;
            dyy[q] = 0u;
            dy1[q] = 0u;
        }
        for (int ch0 = 0; ch0 < nch; ch0 += 8) {
            const int ch = ch0 + sub;
            const bool real = ch < nch;            // always, when a row is a whole number of 128 codes (uniform test)
            const int cc = real ? ch : 0;
            uint4 a = xq_s[cc];
            uint4 b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = *reinterpret_cast<const uint4*>(g.Xq + (int64_t)rows[q] * g.ldq + 16 * cc);
            if (ragged && !real) {
                a = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                for (int q = 0; q < 4; ++q) b[q] = make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32 t = dxy[q];
                t = __builtin_amdgcn_udot4(a.x, b[q].x, t, false);
                t = __builtin_amdgcn_udot4(a.y, b[q].y, t, false);
                t = __builtin_amdgcn_udot4(a.z, b[q].z, t, false);
                t = __builtin_amdgcn_udot4(a.w, b[q].w, t, false);
                dxy[q] = t;
                u32 u = dyy[q];
                u = __builtin_amdgcn_udot4(b[q].x, b[q].x, u, false);
                u = __builtin_amdgcn_udot4(b[q].y, b[q].y, u, false);
                u = __builtin_amdgcn_udot4(b[q].z, b[q].z, u, false);
                u = __builtin_amdgcn_udot4(b[q].w, b[q].w, u, false);
                dyy[q] = u;
                if (!l2) {
                    u32 w1 = dy1[q];
                    w1 = __builtin_amdgcn_udot4(b[q].x, 0x01010101u, w1, false);
                    w1 = __builtin_amdgcn_udot4(b[q].y, 0x01010101u, w1, false);
                    w1 = __builtin_amdgcn_udot4(b[q].z, 0x01010101u, w1, false);
                    w1 = __builtin_amdgcn_udot4(b[q].w, 0x01010101u, w1, false);
                    dy1[q] = w1;
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 t = dxy[q], u = dyy[q];
            t += dpp_u32<0xB1>(t);     // lane ^ 1
            t += dpp_u32<0x4E>(t);     // lane ^ 2
            t += dpp_u32<0x141>(t);    // mirror inside 8 lanes: the other quad
            u += dpp_u32<0xB1>(u);
            u += dpp_u32<0x4E>(u);
            u += dpp_u32<0x141>(u);
            xy = sub == h + q ? t : xy;
            yy = sub == h + q ? u : yy;
            if (!l2) {
                u32 w1 = dy1[q];
                w1 += dpp_u32<0xB1>(w1);
                w1 += dpp_u32<0x4E>(w1);
                w1 += dpp_u32<0x141>(w1);
                y1 = sub == h + q ? w1 : y1;
            }
        }
    }
    bool reject;
    if (l2) {
        // sum (qx - qy)^2 in integers: exact (below 2^31 for rows of up to 4096 codes)
        const u32 sq = (qxx + yy) - 2u * xy;
        const float r = grid.s * sqrtf((float)sq) * (1.0f - 1e-6f) - 2.0f * grid.err;
        const float lb = r > 0.0f ? r * r : 0.0f;
        reject = lb * (1.0f - 1e-4f) > kd;
    } else {
        const float a0 = (float)g.d * grid.lo * grid.lo, a1 = grid.lo * grid.s, a2 = grid.s * grid.s;
        const float s1 = (float)(qx1 + y1), fxy = (float)xy, fy1 = (float)y1, fyy = (float)yy;
        const float dotq = a0 + a1 * s1 + a2 * fxy;
        const float slack = 1e-6f * (a0 + fabsf(a1) * s1 + a2 * fxy);
        const float yq2 = a0 + 2.0f * a1 * fy1 + a2 * fyy;
        const float slack_y = 1e-6f * (a0 + 2.0f * fabsf(a1) * fy1 + a2 * fyy);
        const float yq_hi = sqrtf(fmaxf(yq2 + slack_y, 0.0f)) * (1.0f + 1e-6f);
        const float yq_lo = sqrtf(fmaxf(yq2 - slack_y, 0.0f)) * (1.0f - 1e-6f);
        // <x, y> <= <xq, yq> + err |yq| + |x| err
        const float ub = dotq + slack + grid.err * (yq_hi + norm_v) * 1.0001f;
        if (g.metric == 1) {
            reject = -ub - 1e-5f * norm_v * (yq_hi + grid.err) > kd;
        } else {
            // the largest cosine the bound allows: |y| is within err of |yq|
            const float y_lo = yq_lo - grid.err, y_hi = yq_hi + grid.err;
            const float cos_ub = ub >= 0.0f ? (y_lo > 0.0f ? ub * rn_v / y_lo * 1.0001f : __builtin_inff()) : ub * rn_v / y_hi * 0.9999f;
            reject = 1.0f - cos_ub - 1e-4f > kd;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return (mine && !reject) ? (int)row : -1;
}

// What the join needs of node v besides its vector, in one word: the ordered distance of the list's last
// entry above, the bits of the node's squared norm (inverse norm for cosine) below.
__device__ inline float join_aux(const TgGraph& g, int64_t v) { return g.metric == 2 ? g.rnorm[v] : g.nrm[v]; }
__device__ inline u64 join_word(float aux, u64 last_key)
{
    return (last_key & 0xFFFFFFFF00000000ull) | (u64)__float_as_uint(aux);
}

// stage row v of X into this wave's LDS slice
__device__ inline void stage_row(const TgGraph& g, int64_t v, float* xs)
{
    const float* x = g.X + v * (int64_t)g.ld;
    for (int col = tg_lane() * 4; col < g.ld; col += 256)
        *reinterpret_cast<float4*>(xs + col) = *reinterpret_cast<const float4*>(x + col);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ inline bool id_in_list(u32 id, u64 list_key, int k)
{
    // list_key: one list entry per lane (lanes < k); true if `id` equals any listed id
    bool hit = false;
    const u32 lid = tg_key_id(list_key);
    for (int q = 0; q < k; ++q) hit |= (id == (u32)__builtin_amdgcn_readlane((int)lid, q));
    return hit;
}

// ---------------------------------------------------------------------------------------
// Algorithm 1, initialisation.  Node v draws ids floor(n * u_t), t = 0,1,2,..., from the tagged
// hash and keeps the first k that differ from v and from all earlier draws.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * LISTS_WAVES) void init_kernel(TgGraph g, u64 hs_init, int64_t v0)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int64_t v = v0 + (int64_t)blockIdx.x * LISTS_WAVES + wave;
    if (v >= g.n) return;
    float* xs = smem + (size_t)wave * g.ld;
    u32* wscr = reinterpret_cast<u32*>(smem + (size_t)LISTS_WAVES * g.ld) + wave * 128;
    const float aux_v = join_aux(g, v);          // asked for now, needed at the end
    stage_row(g, v, xs);

    int cnt = 0;
    for (u64 t0 = 0; cnt < g.k; t0 += 64) {
        const u32 c = (u32)(((tg_hash_xy(hs_init, (u64)v, t0 + (u64)lane) >> 32) * (u64)g.n) >> 32);
        bool bad = (c == (u32)v);
        for (int q = 0; q < cnt; ++q) bad |= (c == wscr[q]);
        for (int q = 0; q < 63; ++q) {
            u32 cq = (u32)__builtin_amdgcn_readlane((int)c, q);
            bad |= (q < lane && cq == c);
        }
        const u64 ok = __ballot(!bad);
        const int rank = cnt + __popcll(ok & tg_lanemask_lt());
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (!bad && rank < g.k) wscr[rank] = c;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        cnt = min(g.k, cnt + __popcll(ok));
    }
    const int cid = lane < g.k ? (int)wscr[lane] : -1;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const float rn_v = g.metric == 2 ? g.rnorm[v] : 1.0f;
    const float dist = wave_direct_dist<8>(g, xs, rn_v, cid, wscr);
    u64 key = lane < g.k ? tg_key(dist, (u32)cid, 1u) : TG_EMPTY_KEY;
    key = tg_wave_sort(key);
    if (lane < g.k) {
        g.gid[v * g.k + lane] = tg_key_id(key) | 0x80000000u;
        g.gdist[v * g.k + lane] = tg_key_dist(key);
        if (lane == g.k - 1) g.kth[v] = join_word(aux_v, key);
    }
}
void tg_launch_init(const TgGraph& g, uint64_t hs_init, hipStream_t s)
{
    size_t shm = (size_t)LISTS_WAVES * g.ld * sizeof(float) + LISTS_WAVES * 128 * sizeof(u32);
    tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
        hipLaunchKernelGGL(init_kernel, dim3((unsigned)((cnt + LISTS_WAVES - 1) / LISTS_WAVES)), dim3(64 * LISTS_WAVES), shm, s, g,
                           hs_init, v0);
    });
}

// ---------------------------------------------------------------------------------------
// A set of node ids in LDS (open addressing, linear probing, `mask` + 1 words, always more
// words than ids, so every probe sequence ends at a free word).  Inserts `id` for the lanes
// with `active` and tells each whether the id was there already; of several lanes that bring
// the same new id exactly one is told "new".
// ---------------------------------------------------------------------------------------
#define TG_SET_FREE 0xFFFFFFFFu
__device__ inline bool lds_set_insert(u32* tab, u32 mask, int shift, u32 id, bool active)
{
    bool present = false, pending = active;
    u32 h = (id * 0x9E3779B1u) >> shift;
    while (__ballot(pending)) {
        if (pending) {
            const u32 old = atomicCAS(tab + h, TG_SET_FREE, id);
            if (old == TG_SET_FREE) pending = false;
            else if (old == id) { present = true; pending = false; }
            else h = (h + 1) & mask;
        }
    }
    return present;
}

// ---------------------------------------------------------------------------------------
// Section 4.2 list update (phase 1).  The wave that owns list v reads the list and v's
// candidate slots, drops candidates the list already holds, sorts the rest, merges the two
// ascending sequences and keeps the first k.  With `flip` (the first update after a sampling)
// the entries sampled as "new" this round become old; arrivals are new.  Used slots are handed
// back empty.  A node without candidates whose list needs neither flips nor numbers costs its
// slot row only.
// ---------------------------------------------------------------------------------------
#define UPDATE_MAX_C 256
#define UPDATE_SET_WORDS 512     // more than 64 + UPDATE_MAX_C ids
// REMEASURE (the join ranked on rows rounded to fp16): every arrival is measured again in fp32 from the
// vectors before the list is written, so the lists and their thresholds hold exact distances.
template <bool REMEASURE>
__global__ __launch_bounds__(64 * LISTS_WAVES) void update_kernel(TgGraph g, int S, TgCand cd, u64* updates, int flip, int64_t v0)
{
    extern __shared__ float smem[];      // REMEASURE: a row of X and 128 words of scratch per wave
    __shared__ u64 queue[LISTS_WAVES][UPDATE_MAX_C];
    __shared__ u32 seen_s[LISTS_WAVES][UPDATE_SET_WORDS];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int64_t v = v0 + (int64_t)blockIdx.x * LISTS_WAVES + wave;
    if (v >= g.n) return;
    const int k = g.k;
    // all filled slots of v, closed up in LDS (the slots are handed back empty)
    const u64 lt = tg_lanemask_lt();
    int nq = 0;
    u64* slot0 = cd.slots + v * (int64_t)cd.C + lane;
    u64 cks[UPDATE_MAX_C / 64];
#pragma unroll
    for (int j = 0; j < UPDATE_MAX_C / 64; ++j)          // every load is on its way before the first is looked at
        cks[j] = (64 * j + lane < cd.C) ? slot0[64 * j] : TG_EMPTY_KEY;
    u32 w = 0;
    float dist = 0.0f;
    if (!flip) {
        // nothing but candidates can change this list now: without any, the slot row was all there is to read
        bool some = false;
#pragma unroll
        for (int j = 0; j < UPDATE_MAX_C / 64; ++j) some |= cks[j] != TG_EMPTY_KEY;
        if (__ballot(some) == 0ull) return;
    }
    if (lane < k) {
        w = g.gid[v * k + lane];
        dist = g.gdist[v * k + lane];
    }
    const float aux_v = join_aux(g, v);          // asked for now, needed at the end
#pragma unroll
    for (int j = 0; j < UPDATE_MAX_C / 64; ++j) {
        const bool filled = cks[j] != TG_EMPTY_KEY;
        const u64 m = __ballot(filled);
        if (filled) {
            slot0[64 * j] = TG_EMPTY_KEY;
            queue[wave][nq + __popcll(m & lt)] = cks[j];
        }
        nq += __popcll(m);
    }
    u32 fresh = w >> 31;
    const u64 mf = __ballot(lane < k && fresh);
    if (flip && fresh && __popcll(mf & lt) < S) fresh = 0;
    u64 L = lane < k ? tg_key(dist, w & TG_ID_MASK, fresh) : TG_EMPTY_KEY;

    const bool any_cand = nq > 0;
    if (any_cand) {
        // ids of G[v], then every candidate: a candidate that is listed, or a repeat (the same
        // candidate may sit in several slots, one per block that found it), finds its id there
        u32* seen = seen_s[wave];
        int set_words = 128;
        while (set_words * 2 < 3 * (k + nq)) set_words *= 2;          // at most UPDATE_SET_WORDS
        const u32 set_mask = (u32)set_words - 1u;
        const int set_shift = 33 - __ffs(set_words);
        for (int i = lane; i < set_words; i += 64) seen[i] = TG_SET_FREE;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        (void)lds_set_insert(seen, set_mask, set_shift, w & TG_ID_MASK, lane < k);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int q0 = 0; q0 < nq; q0 += 64) {
            u64 ck = q0 + lane < nq ? queue[wave][q0 + lane] : TG_EMPTY_KEY;
            if (q0 > 0 && !(ck < tg_shfl64(L, k - 1))) ck = TG_EMPTY_KEY;      // cannot precede the last entry of the list as merged so far
            const u32 cid = tg_key_id(ck);
            const bool cand = ck != TG_EMPTY_KEY && cid != (u32)v;
            const bool known = lds_set_insert(seen, set_mask, set_shift, cid, cand);
            if (!cand || known) ck = TG_EMPTY_KEY;
            if (__ballot(ck != TG_EMPTY_KEY) == 0) continue;
            ck = tg_wave_sort(ck);
            L = tg_wave_merge_low(L, ck);
            if (lane >= k) L = TG_EMPTY_KEY;
            if (q0 == 0 && nq > 128) {
                // More than two batches (the first parts of the early rounds): the first merge has tightened the list, and most of
                // what waits cannot precede its last entry any more.  What still can is closed up, usually into one batch.
                const u64 last = tg_shfl64(L, k - 1);
                int wr = 64;
                for (int r0 = 64; r0 < nq; r0 += 64) {
                    const u64 c = r0 + lane < nq ? queue[wave][r0 + lane] : TG_EMPTY_KEY;
                    const bool keep = c < last;
                    const u64 mk = __ballot(keep);
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    if (keep) queue[wave][wr + __popcll(mk & lt)] = c;       // (never ahead of what has been read)
                    wr += __popcll(mk);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                nq = wr;
            }
        }
        if (REMEASURE) {
            const bool arrival = lane < k && (L & 2ull) != 0ull;
            if (__ballot(arrival) != 0ull) {
                float* xs = smem + (size_t)wave * g.ld;
                u32* wscr = reinterpret_cast<u32*>(smem + (size_t)LISTS_WAVES * g.ld) + wave * 128;
                stage_row(g, v, xs);
                const float rn_v = g.metric == 2 ? g.rnorm[v] : 1.0f;
                const float exact = wave_direct_dist<8>(g, xs, rn_v, arrival ? (int)tg_key_id(L) : -1, wscr);
                if (arrival) L = tg_key(exact, tg_key_id(L), (u32)L & 3u);
                L = tg_wave_sort(L);           // lanes past k hold the empty key and stay behind
            }
        }
    }
    if (!any_cand && (mf == 0 || !flip)) return;      // the list is what it was
    const int ins = __popcll(__ballot(lane < k && (L & 2ull)));
    if (lane < k) {
        g.gid[v * k + lane] = tg_key_id(L) | (((u32)L & 1u) << 31);
        g.gdist[v * k + lane] = tg_key_dist(L);
        if (lane == k - 1) g.kth[v] = join_word(aux_v, L);
    }
    if (ins && lane == 0) atomicAdd(updates + (v & (TG_STAT_BINS - 1)), (u64)ins);
}
void tg_launch_update(const TgGraph& g, const TgSample& sm, const TgCand& c, u64* updates, bool flip, hipStream_t s)
{
    if (c.C > UPDATE_MAX_C) return;    // the boundary refuses such C; the queue in LDS holds no more
    // rows rounded for the join whatever their values (not the mode that narrows only where that is exact): measure arrivals again
    const bool remeasure = g.Xh && !g.f16_ok;
    const size_t shm = remeasure ? (size_t)LISTS_WAVES * g.ld * sizeof(float) + LISTS_WAVES * 128 * sizeof(u32) : 0;
    tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
        const dim3 grid((unsigned)((cnt + LISTS_WAVES - 1) / LISTS_WAVES));
        if (remeasure)
            hipLaunchKernelGGL(update_kernel<true>, grid, dim3(64 * LISTS_WAVES), shm, s, g, sm.S, c, updates, flip ? 1 : 0, v0);
        else
            hipLaunchKernelGGL(update_kernel<false>, grid, dim3(64 * LISTS_WAVES), 0, s, g, sm.S, c, updates, flip ? 1 : 0, v0);
    });
}

// phase switch: every entry unvisited
__global__ void mark_fresh_kernel(u32* gid, size_t count)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) gid[i] |= 0x80000000u;
}
void tg_launch_mark_all_fresh(const TgGraph& g, hipStream_t s)
{
    size_t count = (size_t)g.n * g.k;
    hipLaunchKernelGGL(mark_fresh_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, g.gid, count);
}

// ---------------------------------------------------------------------------------------
// Algorithm 1, phase-2 loop, one wave per node v: take the first m unvisited entries u of
// G[v], mark them visited, read G[u] from the lists as they stood when the round began
// (g.gid; this round writes g.gid_next), measure v against the ids that are neither v nor
// listed nor met earlier in this round, and merge them into G[v].
// floor(64 / k) neighbour lists are handled per pass, one candidate per lane (k <= 64), so
// the usual m = 2, k <= 32 round is one gather of ids and one of vectors.  Membership in G[v]
// and repeats are settled through an id set in LDS; the few candidates that survive the
// screening are put into the list one by one (many: sorted and merged).
// ---------------------------------------------------------------------------------------
template <bool SCREEN>
__device__ __forceinline__ void phase2_node(const TgGraph& g, int64_t v, int m, int set_words, u64* updates, u64* stat_bins)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int k = g.k;
    float* xs = smem + (size_t)wave * g.ld;
    u32* wbase = reinterpret_cast<u32*>(smem + (size_t)LISTS_WAVES * g.ld);
    u32* wscr = wbase + wave * 128;
    u32* seen = wbase + LISTS_WAVES * 128 + wave * set_words;      // ids of G[v] and of every candidate met this round
    uint4* xq_s = reinterpret_cast<uint4*>(wbase + LISTS_WAVES * (128 + set_words)) + wave * ((g.ldq >> 4) + 2);
    const u32 set_mask = (u32)set_words - 1u;
    const int set_shift = 33 - __ffs(set_words);                    // top log2(set_words) bits of the hash

    u32 w = 0;
    float dist = 0.0f;
    if (lane < k) {
        w = g.gid[v * k + lane];
        dist = g.gdist[v * k + lane];
    }
    const float aux_v = join_aux(g, v);          // asked for now, needed at the end
    ScreenGrid grid = {0.0f, 1.0f, 0.0f};
    u32 qxx = 0u, qx1 = 0u;          // sum qx qx and sum qx over v's codes
    if (SCREEN) {
        const u32* gw = reinterpret_cast<const u32*>(g.Xqm);
        quantize_grid(gw, grid.lo, grid.s);
        grid.err = __uint_as_float(gw[2]);
        const int nch = g.ldq >> 4;
        const uint4* src = reinterpret_cast<const uint4*>(g.Xq + v * (int64_t)g.ldq);
        for (int i = lane; i < nch; i += 64) {
            const uint4 a = src[i];
            xq_s[i] = a;
            qxx = __builtin_amdgcn_udot4(a.x, a.x, qxx, false);
            qxx = __builtin_amdgcn_udot4(a.y, a.y, qxx, false);
            qxx = __builtin_amdgcn_udot4(a.z, a.z, qxx, false);
            qxx = __builtin_amdgcn_udot4(a.w, a.w, qxx, false);
            qx1 = __builtin_amdgcn_udot4(a.x, 0x01010101u, qx1, false);
            qx1 = __builtin_amdgcn_udot4(a.y, 0x01010101u, qx1, false);
            qx1 = __builtin_amdgcn_udot4(a.z, 0x01010101u, qx1, false);
            qx1 = __builtin_amdgcn_udot4(a.w, 0x01010101u, qx1, false);
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            qxx += (u32)__shfl_xor((int)qxx, o);
            qx1 += (u32)__shfl_xor((int)qx1, o);
        }
    }
    for (int i = lane; i < set_words; i += 64) seen[i] = TG_SET_FREE;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    u32 fresh = w >> 31;
    u64 mf = __ballot(lane < k && fresh);
    if (fresh && __popcll(mf & tg_lanemask_lt()) < m) fresh = 0;   // non-revisitation
    u64 L = lane < k ? tg_key(dist, w & TG_ID_MASK, fresh) : TG_EMPTY_KEY;
    const u32 my_id = w & TG_ID_MASK;
    (void)lds_set_insert(seen, set_mask, set_shift, my_id, lane < k);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const float rn_v = g.metric == 2 ? g.rnorm[v] : 1.0f;
    const float norm_v = g.metric != 0 ? sqrtf(g.nrm[v]) : 0.0f;
    const int nexp = min(m, __popcll(mf));
    const int per = 64 / k;
    bool staged = false;

    int evaluated = 0, measured = 0;
    for (int e0 = 0; e0 < nexp; e0 += per) {
        const int nb = min(per, nexp - e0);
        const int my_e = lane / k, j = lane - my_e * k;
        const bool in = my_e < nb;
        int src = 0;
        for (int q = 0; q < nb; ++q) {
            const int sbit = __ffsll((long long)mf) - 1;
            mf &= mf - 1;
            if (q == my_e) src = sbit;
        }
        const u32 u = (u32)__shfl((int)my_id, src);
        const u32 cid = in ? (g.gid[(int64_t)u * k + j] & TG_ID_MASK) : 0xFFFFFFFFu;
        // a candidate counts once per round, and not at all if it is v or sits in G[v]
        const bool fresh_id = in && cid != (u32)v;
        const bool drop = !fresh_id | lds_set_insert(seen, set_mask, set_shift, cid, fresh_id);
        evaluated += __popcll(__ballot(!drop));
        // candidates that provably cannot precede the list's last entry are dropped on the 8-bit copy
        int cand = drop ? -1 : (int)cid;
        if (SCREEN) {
            const float kd = tg_key_dist((u64)__builtin_amdgcn_readlane((int)(L >> 32), k - 1) << 32);
            cand = wave_screen(g, grid, xq_s, qxx, qx1, norm_v, rn_v, cand, wscr, kd);
        }
        const u64 alive = __ballot(cand >= 0);
        if (alive == 0) continue;
        const int nalive = __popcll(alive);
        measured += nalive;
        if (!staged) {
            stage_row(g, v, xs);
            staged = true;
        }
        const float cdist = wave_direct_dist<SCREEN ? 1 : 8>(g, xs, rn_v, cand, wscr);
        u64 ck = cand >= 0 ? tg_key(cdist, (u32)cand, 3u) : TG_EMPTY_KEY;
        if (nalive <= 4) {
            // a few survivors: put each at its rank, entries behind it move up by one
            u64 rem = alive;
            while (rem) {
                const int sl = __ffsll((long long)rem) - 1;
                rem &= rem - 1;
                const u64 key = ((u64)(u32)__builtin_amdgcn_readlane((int)(ck >> 32), sl) << 32) |
                                (u64)(u32)__builtin_amdgcn_readlane((int)(u32)ck, sl);
                const int pos = __popcll(__ballot(L < key));
                const u64 up = tg_shfl64(L, lane > 0 ? lane - 1 : 0);
                L = lane < pos ? L : (lane == pos ? key : up);
                if (lane >= k) L = TG_EMPTY_KEY;
            }
        } else {
            ck = tg_wave_sort(ck);
            L = tg_wave_merge_low(L, ck);
            if (lane >= k) L = TG_EMPTY_KEY;
        }
    }
    const int ins = __popcll(__ballot(lane < k && (L & 2ull)));
    if (lane < k) {
        g.gid_next[v * k + lane] = tg_key_id(L) | (((u32)L & 1u) << 31);
        g.gdist[v * k + lane] = tg_key_dist(L);
        if (lane == k - 1) g.kth[v] = join_word(aux_v, L);
    }
    if (lane == 0) {
        if (ins) atomicAdd(updates + (v & (TG_STAT_BINS - 1)), (u64)ins);
        if (stat_bins && evaluated) {
            atomicAdd(stat_bins + (v & (TG_STAT_BINS - 1)), (u64)evaluated);                          // pairs
            if (measured) atomicAdd(stat_bins + TG_STAT_BINS + (v & (TG_STAT_BINS - 1)), (u64)measured);  // fp32 vectors
        }
    }
}
// Workgroups walk the nodes with the stride of the grid.  Both variants are launched when a
// screening copy exists; the flag says whose turn it is, and the other one ends at once.
template <bool SCREEN>
__device__ __forceinline__ void phase2_body(const TgGraph& g, int m, int set_words, u64* updates, u64* stat_bins,
                                            const u32* __restrict__ screen_on)
{
    if (screen_on && (*screen_on != 0u) != SCREEN) return;
    const int wave = threadIdx.x >> 6;
    for (int64_t v = (int64_t)blockIdx.x * LISTS_WAVES + wave; v < g.n; v += (int64_t)gridDim.x * LISTS_WAVES) {
        phase2_node<SCREEN>(g, v, m, set_words, updates, stat_bins);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}
// the screening variant is latency bound: five waves per SIMD (96 registers) instead of four
__global__ __launch_bounds__(64 * LISTS_WAVES) __attribute__((amdgpu_waves_per_eu(5)))
void phase2_screen_kernel(TgGraph g, int m, int set_words, u64* updates, u64* stat_bins, const u32* screen_on)
{
    phase2_body<true>(g, m, set_words, updates, stat_bins, screen_on);
}
__global__ __launch_bounds__(64 * LISTS_WAVES) void phase2_plain_kernel(TgGraph g, int m, int set_words, u64* updates, u64* stat_bins,
                                                                        const u32* screen_on)
{
    phase2_body<false>(g, m, set_words, updates, stat_bins, screen_on);
}
// Screening pays when the 8-bit codes are nearly lossless (byte-valued features); on real-valued
// data in high dimension most candidates pass the bound and its reads are wasted.  After a
// screened round: if more than half of the candidates went on to the fp32 evaluation, the
// following rounds measure every candidate directly.
__global__ __launch_bounds__(256) void screen_decide_kernel(const u64* __restrict__ stat_bins, u32* screen_on)
{
    __shared__ u64 red[2][4];
    u64 pairs = 0, measured = 0;
    for (int i = threadIdx.x; i < TG_STAT_BINS; i += 256) {
        pairs += stat_bins[i];
        measured += stat_bins[TG_STAT_BINS + i];
    }
    for (int o = 32; o > 0; o >>= 1) {
        pairs += tg_shfl_xor64(pairs, o);
        measured += tg_shfl_xor64(measured, o);
    }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = pairs; red[1][threadIdx.x >> 6] = measured; }
    __syncthreads();
    if (threadIdx.x == 0) {
        pairs = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        measured = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        if (*screen_on != 0u && 2 * measured > pairs) *screen_on = 0u;
    }
}
#define PHASE2_GRID 16384
void tg_launch_phase2(const TgGraph& g, int m, u64* updates, u64* stat_bins, u32* screen_on, hipStream_t s)
{
    // the id set holds the k listed ids and at most m k candidates; half as many words again, as a power of two
    int set_words = 64;
    while (set_words * 2 < 3 * (g.k + m * g.k)) set_words *= 2;
    const size_t shm = (size_t)LISTS_WAVES * g.ld * sizeof(float) + LISTS_WAVES * (128 + (size_t)set_words) * sizeof(u32) +
                       (size_t)LISTS_WAVES * (g.Xq ? g.ldq + 32 : 0);
    int64_t blocks = (g.n + LISTS_WAVES - 1) / LISTS_WAVES;
    if (blocks > PHASE2_GRID) blocks = PHASE2_GRID;
    if (g.Xq) {
        hipLaunchKernelGGL(phase2_screen_kernel, dim3((unsigned)blocks), dim3(64 * LISTS_WAVES), shm, s, g, m, set_words, updates, stat_bins,
                           (const u32*)screen_on);
        hipLaunchKernelGGL(phase2_plain_kernel, dim3((unsigned)blocks), dim3(64 * LISTS_WAVES), shm, s, g, m, set_words, updates, stat_bins,
                           (const u32*)screen_on);
        hipLaunchKernelGGL(screen_decide_kernel, dim3(1), dim3(256), 0, s, (const u64*)stat_bins, screen_on);
    } else {
        hipLaunchKernelGGL(phase2_plain_kernel, dim3((unsigned)blocks), dim3(64 * LISTS_WAVES), shm, s, g, m, set_words, updates, stat_bins,
                           (const u32*)nullptr);
    }
}

// ---------------------------------------------------------------------------------------
// Output: optionally recompute every kept distance directly from the vectors (the join
// ranks with the norm-plus-Gram form, which loses digits to cancellation) and re-sort.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * LISTS_WAVES) void finalize_kernel(TgGraph g, int recompute, const u32* __restrict__ range, int32_t* out_ids,
                                                                    float* out_dist, int64_t v0)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int64_t v = v0 + (int64_t)blockIdx.x * LISTS_WAVES + wave;
    if (v >= g.n) return;
    const int k = g.k;
    float* xs = smem + (size_t)wave * g.ld;
    u32* wscr = reinterpret_cast<u32*>(smem + (size_t)LISTS_WAVES * g.ld) + wave * 128;
    int id = -1;
    float dist = 0.0f;
    if (lane < k) {
        id = (int)(g.gid[v * k + lane] & TG_ID_MASK);
        dist = g.gdist[v * k + lane];
    }
    if (recompute && range && g.metric != 2 && range[TG_RANGE_NONINT] == 0u) {
        // Whole numbers small enough that every fp32 sum of the norms, the inner products and their combination is exact
        // (2 d max|x|^2 <= 2^24): the distances in the lists are the directly computed ones already, bit for bit.
        const float m = fmaxf(fabsf(tg_unord(range[0])), fabsf(tg_unord(range[1])));
        if (2.0f * (float)g.d * m * m <= 16777216.0f) recompute = 0;
    }
    if (recompute) {
        stage_row(g, v, xs);
        const float rn_v = g.metric == 2 ? g.rnorm[v] : 1.0f;
        dist = wave_direct_dist<8>(g, xs, rn_v, id, wscr);
        u64 key = lane < k ? tg_key(dist, (u32)id, 0u) : TG_EMPTY_KEY;
        key = tg_wave_sort(key);
        id = (int)tg_key_id(key);
        dist = tg_key_dist(key);
    }
    if (lane < k) {
        out_ids[v * k + lane] = id;
        if (out_dist) out_dist[v * k + lane] = dist;
    }
}
void tg_launch_finalize(const TgGraph& g, int recompute, const uint32_t* range, int32_t* out_ids, float* out_dist, hipStream_t s)
{
    size_t shm = (size_t)LISTS_WAVES * g.ld * sizeof(float) + LISTS_WAVES * 128 * sizeof(u32);
    tg_for_node_chunks(g.n, [&](int64_t v0, int64_t cnt) {
        hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)((cnt + LISTS_WAVES - 1) / LISTS_WAVES)), dim3(64 * LISTS_WAVES), shm, s, g,
                           recompute, range, out_ids, out_dist, v0);
    });
}

// ---------------------------------------------------------------------------------------
// state export / import
// ---------------------------------------------------------------------------------------
__global__ void export_kernel(TgGraph g, int32_t* ids, float* dist, uint8_t* fresh)
{
    size_t count = (size_t)g.n * g.k;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) {
        u32 w = g.gid[i];
        if (ids) ids[i] = (int32_t)(w & TG_ID_MASK);
        if (dist) dist[i] = g.gdist[i];
        if (fresh) fresh[i] = (uint8_t)(w >> 31);
    }
}
void tg_launch_export(const TgGraph& g, int32_t* ids, float* dist, uint8_t* fresh, hipStream_t s)
{
    size_t count = (size_t)g.n * g.k;
    hipLaunchKernelGGL(export_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, g, ids, dist, fresh);
}
__global__ void import_kernel(TgGraph g, const int32_t* ids, const float* dist, const uint8_t* fresh)
{
    size_t count = (size_t)g.n * g.k;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) {
        g.gid[i] = (u32)ids[i] | ((u32)(fresh[i] != 0) << 31);
        g.gdist[i] = dist[i];
        if ((int)(i % g.k) == g.k - 1) g.kth[i / g.k] = join_word(join_aux(g, (int64_t)(i / g.k)), tg_key(dist[i], (u32)ids[i], 3u));
    }
}
void tg_launch_import(const TgGraph& g, const int32_t* ids, const float* dist, const uint8_t* fresh, hipStream_t s)
{
    size_t count = (size_t)g.n * g.k;
    hipLaunchKernelGGL(import_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, g, ids, dist, fresh);
}
