// Kernels of the damped inversion (Sec. 3.3, Eq. 12) other than the GEMMs:
//   - trace_kernel:  pi^2 = (tr A / dA) / (tr G / dG) and the two damping values per layer;
//   - copy_damp_kernel: dst = src + damp * I (start of the blocked inversion);
//   - leaf_inverse_kernel: (X + damp I)^-1 for n <= 288 by Gauss-Jordan elimination held
//     entirely in registers of one 512- or 1024-thread workgroup (one matrix per workgroup, many
//     matrices per launch); only the pivot row goes through LDS.
#include "kfac_internal.h"

#include <type_traits>

namespace kfac {

// ------------------------------------------------------------------ trace / pi / damping
__global__ __launch_bounds__(256) void trace_kernel(const TraceJob *__restrict__ jobs, float gamma,
                                                    float *__restrict__ damp, float *__restrict__ pi_out)
{
    __shared__ double red[2][256];
    const TraceJob J = jobs[blockIdx.x];
    double sa = 0.0, sg = 0.0;
    for (int i = threadIdx.x; i < J.dA; i += 256) sa += (double)J.A[(long long)i * J.dA + i];
    for (int i = threadIdx.x; i < J.dG; i += 256) sg += (double)J.G[(long long)i * J.dG + i];
    red[0][threadIdx.x] = sa;
    red[1][threadIdx.x] = sg;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            red[0][threadIdx.x] += red[0][threadIdx.x + s];
            red[1][threadIdx.x] += red[1][threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double trA = red[0][0], trG = red[1][0];
        double pi = 1.0;
        if (trA > 0.0 && trG > 0.0) pi = sqrt((trA / J.dA) / (trG / J.dG));
        damp[3 * blockIdx.x + 0] = (float)pi;
        damp[3 * blockIdx.x + 1] = (float)(pi * (double)gamma);   // added to A
        damp[3 * blockIdx.x + 2] = (float)((double)gamma / pi);   // added to G
        if (pi_out) pi_out[blockIdx.x] = (float)pi;
    }
}

hipError_t launch_trace(const TraceJob *jobs_dev, int n_layers, float gamma, float *damp_dev,
                        float *pi_out, hipStream_t s)
{
    if (n_layers <= 0) return hipSuccess;
    trace_kernel<<<dim3(n_layers), dim3(256), 0, s>>>(jobs_dev, gamma, damp_dev, pi_out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ dst = src + damp I
constexpr int COPY_ROWS = 8;

__global__ __launch_bounds__(256) void copy_damp_kernel(const CopyJob *__restrict__ jobs, int n_jobs,
                                                        const float *__restrict__ damp)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const CopyJob J = jobs[lo];
    const float d = (J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f;
    const int r0 = (wg - J.wg_start) * COPY_ROWS;
    for (int r = r0; r < min(J.n, r0 + COPY_ROWS); ++r)
        for (int c = threadIdx.x; c < J.n; c += 256) {
            float v = J.src[(long long)r * J.lds + c];
            if (r == c) v += d;
            J.dst[(long long)r * J.ldd + c] = v;
        }
}

hipError_t launch_copy_damp(const CopyJob *jobs_dev, int n_jobs, int total_wgs, const float *damp_dev,
                            hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    copy_damp_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, damp_dev);
    return hipGetLastError();
}

__global__ void zero_i32_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t s)
{
    if (n <= 0 || !p) return hipSuccess;
    zero_i32_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(p, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------ in-register Gauss-Jordan
// Thread (ti, tj) of a TR x 32 thread grid holds the elements (ti + TR*bi, tj + 32*bj),
// bi < BR, bj < BC (so n <= TR*BR = 32*BC).  Gauss-Jordan without pivoting (safe for a
// positive definite matrix).  After pivots 0..k-1 the working matrix T has
// T[k][j] = -T[j][k] for j < k and T[k][j] = T[j][k] for j > k, so publishing row k alone
// also gives column k.  Step k:
//     p = 1/T[k][k];  T[i][j] -= T[i][k] p T[k][j]  (i, j != k);
//     T[k][j] *= p;   T[i][k] *= -p;   T[k][k] = p.
// One barrier per step (the pivot row buffer is double-buffered).  A non-positive pivot is
// reported through info.
// f(integral_constant<int, I>) for I = 0..N-1, unrolled at compile time.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int BR, int BC, int TR>
__global__ __launch_bounds__(TR * 32) void leaf_inverse_kernel(const LeafJob *__restrict__ jobs,
                                                               const float *__restrict__ damp,
                                                               int32_t *__restrict__ info)
{
    static_assert(TR * BR == 32 * BC, "row and column coverage must agree");
    static_assert(TR == 32 || TR == 16, "thread grid is 32x32 or 16x32");
    __shared__ float rowbuf[2][32 * BC];
    __shared__ int bad;
    const LeafJob J = jobs[blockIdx.x];
    const int n = J.n;
    const int tj = threadIdx.x & 31, ti = threadIdx.x >> 5;
    const float d = (J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f;
    if (threadIdx.x == 0) bad = 0;

    // 32-bit element offsets from the (uniform) base keep one address register per access
    const unsigned lds = (unsigned)J.lds, ldd = (unsigned)J.ldd;
    float a[BR][BC];
#pragma unroll
    for (int bi = 0; bi < BR; ++bi) {
#pragma unroll
        for (int bj = 0; bj < BC; ++bj) {
            const int i = ti + TR * bi, j = tj + 32 * bj;
            float v = (i == j) ? 1.f : 0.f;
            if (i < n && j < n) {
                v = J.src[(unsigned)i * lds + (unsigned)j];
                if (i == j) v += d;
            }
            a[bi][bj] = v;
        }
    }
    __syncthreads();

    // The pivot loop is split into BR compile-time blocks of TR pivots, so that the register
    // row (KBR) and register column (KBC) that hold pivot row/column k are compile-time
    // constants and the matrix never leaves its registers.
    static_for<0, BR>([&](auto KB) {
        constexpr int KBR = decltype(KB)::value;
        constexpr int KBC = (KBR * TR) / 32;
        const int kend = min(n, (KBR + 1) * TR);
        for (int k = KBR * TR; k < kend; ++k) {
            const int ktr = k - KBR * TR;   // row k lives in threads ti == ktr, register row KBR
            const int ktc = k & 31;         // column k lives in threads tj == ktc, register column KBC
            float *rb = rowbuf[k & 1];
            if (ti == ktr) {
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) rb[tj + 32 * bj] = a[KBR][bj];
            }
            __syncthreads();
            const float pivot = rb[k];
            // a non-positive pivot is recorded (first one wins); the elimination goes on and
            // its (meaningless) result is still written: no early exit keeps the loop simple
            if (!(pivot > 0.f) && threadIdx.x == 0 && bad == 0) bad = k + 1;
            const float p = 1.0f / pivot;
            float rj[BC], ci[BR];
#pragma unroll
            for (int bj = 0; bj < BC; ++bj) rj[bj] = rb[tj + 32 * bj];
#pragma unroll
            for (int bi = 0; bi < BR; ++bi) {
                const int i = ti + TR * bi;
                const float r = rb[i];
                ci[bi] = ((i < k) ? -r : r) * p;
            }
            // Row k and column k are special (T[k][j] <- p T[k][j], T[i][k] <- -p T[i][k],
            // T[k][k] <- p).  Their owners clear the old values and patch their multipliers
            // so that the one fused multiply-add below produces exactly those results.
            if (ti == ktr) {
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) a[KBR][bj] = 0.f;
                ci[KBR] = -p;
            }
            if (tj == ktc) {
#pragma unroll
                for (int bi = 0; bi < BR; ++bi) a[bi][KBC] = 0.f;
                rj[KBC] = 1.f;
            }
#pragma unroll
            for (int bi = 0; bi < BR; ++bi)
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) a[bi][bj] = fmaf(-ci[bi], rj[bj], a[bi][bj]);
        }
    });
    __syncthreads();
    if (threadIdx.x == 0 && bad != 0 && info && J.info_idx >= 0)
        atomicCAS(&info[J.info_idx], 0, J.pivot_base + bad);

    // the lower triangle is written and mirrored, so the result is exactly symmetric
#pragma unroll
    for (int bi = 0; bi < BR; ++bi) {
#pragma unroll
        for (int bj = 0; bj < BC; ++bj) {
            const int i = ti + TR * bi, j = tj + 32 * bj;
            if (i < n && j <= i) {
                J.dst[(unsigned)i * ldd + (unsigned)j] = a[bi][bj];
                if (j != i) J.dst[(unsigned)j * ldd + (unsigned)i] = a[bi][bj];
            }
        }
    }
}

hipError_t launch_leaf(const LeafJob *jobs_dev, int n_jobs, int size_class, const float *damp_dev,
                       int32_t *info, hipStream_t s)
{
    if (n_jobs <= 0) return hipSuccess;
    dim3 grid(n_jobs);
    switch (kLeafClasses[size_class]) {   // class value = n_max / 32
        case 2: leaf_inverse_kernel<2, 2, 32><<<grid, dim3(1024), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 3: leaf_inverse_kernel<3, 3, 32><<<grid, dim3(1024), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 4: leaf_inverse_kernel<4, 4, 32><<<grid, dim3(1024), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 5: leaf_inverse_kernel<5, 5, 32><<<grid, dim3(1024), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 7: leaf_inverse_kernel<14, 7, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 8: leaf_inverse_kernel<16, 8, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 9: leaf_inverse_kernel<18, 9, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace kfac
