// Exhaustive exact k-NN of selected rows (the ground truth of the recall definition,
// section 7.1): every query is measured against every row of X, distances computed
// directly from the vectors in fp32, and the k smallest (distance, id) kept.
//
// One wave serves EXQ queries over one slice of the rows: 16 lanes share a row, each
// row chunk is loaded once and used for all EXQ queries, survivors of the running
// threshold are appended to a small LDS buffer per query and folded into the wave-wide
// sorted top list by a sort + merge when the buffer fills.  Slices are merged by a
// second kernel.
#include "tg_device.h"
#include "tg_kernels.h"

#define EXQ 4            // queries per wave
#define EX_BUF 64        // buffered survivors per query

__device__ inline void ex_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__global__ __launch_bounds__(256) void exact_scan_kernel(const float* __restrict__ X, int ld, const float* __restrict__ rnorm,
                                                                  int64_t n, int k, int metric, const int64_t* __restrict__ rows,
                                                                  int64_t nq, int nslices, u64* __restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char ex_smem[];
    const int wave = threadIdx.x >> 6, lane = tg_lane();
    const int grp = lane >> 4, sub = lane & 15;
    const int64_t qgroup = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    const int slice = blockIdx.y;
    if (qgroup * EXQ >= nq) return;
    // per-wave LDS: EXQ query vectors, EXQ survivor buffers
    const size_t per_wave = (size_t)EXQ * ld * sizeof(float) + (size_t)EXQ * EX_BUF * sizeof(u64);
    float* qs = reinterpret_cast<float*>(ex_smem + wave * per_wave);
    u64* buf = reinterpret_cast<u64*>(ex_smem + wave * per_wave + (size_t)EXQ * ld * sizeof(float));

    int64_t qrow[EXQ];
    float qrn[EXQ];
#pragma unroll
    for (int q = 0; q < EXQ; ++q) {
        const int64_t qi = qgroup * EXQ + q;
        const int64_t asked = qi < nq ? (rows ? rows[qi] : qi) : -1;
        qrow[q] = asked < n ? asked : -1;               // a row index outside [0, n) is no query: its output stays empty
        qrn[q] = (metric == 2 && qrow[q] >= 0) ? rnorm[qrow[q]] : 1.0f;
        for (int col = lane * 4; col < ld; col += 256) {
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            if (qrow[q] >= 0) z = *reinterpret_cast<const float4*>(X + qrow[q] * (int64_t)ld + col);
            *reinterpret_cast<float4*>(qs + (size_t)q * ld + col) = z;
        }
    }
    ex_sync();

    u64 top[EXQ];       // ascending across lanes, lanes >= k hold TG_EMPTY_KEY
    u64 tau[EXQ];       // key of the k-th best so far
    int cnt[EXQ];
#pragma unroll
    for (int q = 0; q < EXQ; ++q) { top[q] = TG_EMPTY_KEY; tau[q] = TG_EMPTY_KEY; cnt[q] = 0; }

    const int64_t per_slice = (n + nslices - 1) / nslices;
    const int64_t r0 = (int64_t)slice * per_slice;
    const int64_t r1 = min(n, r0 + per_slice);
    for (int64_t base = r0; base < r1; base += 4) {
        const int64_t row = base + grp;
        const bool live = row < r1;
        float acc[EXQ];
#pragma unroll
        for (int q = 0; q < EXQ; ++q) acc[q] = 0.0f;
        if (live) {
            const float* y = X + row * (int64_t)ld;
            for (int col = sub * 4; col < ld; col += 64) {
                const float4 b = *reinterpret_cast<const float4*>(y + col);
#pragma unroll
                for (int q = 0; q < EXQ; ++q) {
                    const float4 a = *reinterpret_cast<const float4*>(qs + (size_t)q * ld + col);
                    if (metric == 0) {
                        const float t0 = a.x - b.x, t1 = a.y - b.y, t2 = a.z - b.z, t3 = a.w - b.w;
                        acc[q] += t0 * t0 + t1 * t1 + t2 * t2 + t3 * t3;
                    } else {
                        acc[q] += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
                    }
                }
            }
        }
        const float rn_row = (metric == 2 && live) ? rnorm[row] : 1.0f;
#pragma unroll
        for (int q = 0; q < EXQ; ++q) {
            float s = acc[q];
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            s += __shfl_xor(s, 4);
            s += __shfl_xor(s, 8);
            float dist = s;
            if (metric == 1) dist = -s;
            else if (metric == 2) dist = 1.0f - s * qrn[q] * rn_row;
            const u64 key = tg_key(dist, (u32)row, 0u);
            const bool pass = live && sub == 0 && qrow[q] >= 0 && row != qrow[q] && key < tau[q];
            const u64 m = __ballot(pass);
            if (m) {
                if (pass) buf[q * EX_BUF + cnt[q] + __popcll(m & tg_lanemask_lt())] = key;
                cnt[q] += __popcll(m);
                if (cnt[q] > EX_BUF - 4) {
                    ex_sync();
                    u64 c = lane < cnt[q] ? buf[q * EX_BUF + lane] : TG_EMPTY_KEY;
                    ex_sync();
                    top[q] = tg_wave_merge_low(top[q], tg_wave_sort(c));
                    if (lane >= k) top[q] = TG_EMPTY_KEY;
                    tau[q] = tg_shfl64(top[q], k - 1);
                    cnt[q] = 0;
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < EXQ; ++q) {
        ex_sync();
        u64 c = lane < cnt[q] ? buf[q * EX_BUF + lane] : TG_EMPTY_KEY;
        top[q] = tg_wave_merge_low(top[q], tg_wave_sort(c));
        const int64_t qi = qgroup * EXQ + q;
        if (qi < nq && lane < k) partial[(qi * nslices + slice) * k + lane] = top[q];
    }
}

__global__ __launch_bounds__(256) void exact_merge_kernel(const u64* __restrict__ partial, int64_t nq, int k, int nslices,
                                                          int32_t* __restrict__ out_ids, float* __restrict__ out_dist)
{
    const int lane = tg_lane();
    const int64_t qi = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (qi >= nq) return;
    u64 top = TG_EMPTY_KEY;
    for (int s = 0; s < nslices; ++s) {
        u64 c = lane < k ? partial[(qi * nslices + s) * k + lane] : TG_EMPTY_KEY;
        top = tg_wave_merge_low(top, c);
        if (lane >= k) top = TG_EMPTY_KEY;
    }
    if (lane < k) {
        const bool none = top == TG_EMPTY_KEY;
        out_ids[qi * k + lane] = none ? -1 : (int32_t)tg_key_id(top);
        if (out_dist) out_dist[qi * k + lane] = none ? __builtin_inff() : tg_key_dist(top);
    }
}

// partial must hold nq * nslices * k keys; returns the slice count used for (n, nq)
int tg_exact_slices(int64_t n, int64_t nq)
{
    const int64_t groups = (nq + EXQ - 1) / EXQ;
    int64_t s = (8192 + groups - 1) / groups;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    while (s > 1 && (n + s - 1) / s < 1024) --s;
    return (int)s;
}

void tg_launch_exact_knn(const float* X, int ld, const float* nrm, const float* rnorm, int64_t n, int d, int k, int metric,
                         const int64_t* rows, int64_t nq, int32_t* out_ids, float* out_dist, u64* partial, int nslices,
                         hipStream_t s)
{
    (void)nrm; (void)d;
    const int64_t groups = (nq + EXQ - 1) / EXQ;
    const int waves = ld <= 1024 ? 4 : ld <= 2048 ? 2 : 1;     // independent waves per workgroup, bounded by LDS
    const size_t shm = (size_t)waves * ((size_t)EXQ * ld * sizeof(float) + (size_t)EXQ * EX_BUF * sizeof(u64));
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(exact_scan_kernel),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256), true);
    (void)once;
    dim3 grid((unsigned)((groups + waves - 1) / waves), (unsigned)nslices);
    hipLaunchKernelGGL(exact_scan_kernel, grid, dim3(64 * waves), shm, s, X, ld, rnorm, n, k, metric, rows, nq, nslices, partial);
    hipLaunchKernelGGL(exact_merge_kernel, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, partial, nq, k, nslices, out_ids, out_dist);
}
