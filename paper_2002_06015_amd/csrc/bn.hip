// Unit-wise natural gradient for BatchNorm (Sec. 4.2, Eq. 15-17).
//   bn_reduce_kernel: per-sample gradients of gamma/beta from dy and xhat ([N, C, HW]):
//     one wavefront per (n, c) row, lanes stride over the row, wavefront-shuffle reduction.
//     Pure streaming: HBM-bound.
//   bn_unit_kernel: one thread per channel builds the 2x2 Fisher block (3 unique numbers)
//     from the [N, C] per-sample gradients (coalesced over channels), folds it into the
//     running average and applies the closed-form 2x2 inverse to the mean gradient.
#include "kfac_internal.h"

namespace kfac {

typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void bn_reduce_kernel(const BnReduceJob *__restrict__ jobs, int n_jobs, int N)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const BnReduceJob J = jobs[lo];
    const long long row = (long long)(wg - J.wg_start) * 4 + (threadIdx.x >> 6);
    if (row >= (long long)N * J.C) return;
    const int lane = threadIdx.x & 63;
    const float *dy = J.dy + row * J.HW;
    const float *xh = J.xhat + row * J.HW;
    float sg = 0.f, sb = 0.f;
    const bool vec = ((J.HW & 3) == 0) && ((((uintptr_t)J.dy | (uintptr_t)J.xhat) & 15) == 0);
    if (vec) {
        for (int t = lane * 4; t < J.HW; t += 256) {
            const floatx4 a = *(const floatx4 *)(dy + t);
            const floatx4 b = *(const floatx4 *)(xh + t);
            sg += a[0] * b[0] + a[1] * b[1] + a[2] * b[2] + a[3] * b[3];
            sb += a[0] + a[1] + a[2] + a[3];
        }
    } else {
        for (int t = lane; t < J.HW; t += 64) {
            const float a = dy[t];
            sg += a * xh[t];
            sb += a;
        }
    }
    sg = wave_sum(sg);
    sb = wave_sum(sb);
    if (lane == 0) {
        J.g_gamma[row] = sg;
        J.g_beta[row] = sb;
    }
}

// The same from NHWC tensors ([N, HW, C]): a workgroup takes 64 channels of one sample, lanes along the channels
// (16 lanes x 16 bytes per position when C % 4 == 0, else 64 lanes x 4 bytes), 16 (4) positions at a time; the
// partial sums of the threads that share a channel are added through LDS in a fixed order.
__global__ __launch_bounds__(256) void bn_reduce_nhwc_kernel(const BnReduceJob *__restrict__ jobs, int n_jobs, int N)
{
    __shared__ float red[2][16][64];
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const BnReduceJob J = jobs[lo];
    const int chunks = (J.C + 63) / 64;
    const int local = wg - J.wg_start;
    const int n = local / chunks, c0 = (local - n * chunks) * 64;
    const float *dy = J.dy + (long long)n * J.HW * J.C;
    const float *xh = J.xhat + (long long)n * J.HW * J.C;
    const bool vec = ((J.C & 3) == 0) && ((((uintptr_t)J.dy | (uintptr_t)J.xhat) & 15) == 0);
    const int tid = threadIdx.x;
    if (vec) {
        const int c = c0 + 4 * (tid & 15), part = tid >> 4;   // 16 parts
        floatx4 sg = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
        if (c < J.C)
            for (int t = part; t < J.HW; t += 16) {
                const floatx4 a = *(const floatx4 *)(dy + (long long)t * J.C + c);
                const floatx4 b = *(const floatx4 *)(xh + (long long)t * J.C + c);
                sg += a * b;
                sb += a;
            }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            red[0][part][4 * (tid & 15) + e] = sg[e];
            red[1][part][4 * (tid & 15) + e] = sb[e];
        }
    } else {
        const int c = c0 + (tid & 63), part = tid >> 6;       // 4 parts
        float sg = 0.f, sb = 0.f;
        if (c < J.C)
            for (int t = part; t < J.HW; t += 4) {
                const float a = dy[(long long)t * J.C + c];
                sg += a * xh[(long long)t * J.C + c];
                sb += a;
            }
        red[0][part][tid & 63] = sg;
        red[1][part][tid & 63] = sb;
    }
    __syncthreads();
    if (tid < 128) {
        const int which = tid >> 6, cl = tid & 63;
        const int parts = vec ? 16 : 4;
        float sum = 0.f;
        for (int q = 0; q < parts; ++q) sum += red[which][q][cl];
        if (c0 + cl < J.C) (which ? J.g_beta : J.g_gamma)[(long long)n * J.C + c0 + cl] = sum;
    }
}

__global__ __launch_bounds__(256) void bn_unit_kernel(const BnJob *__restrict__ jobs, int n_jobs, int N,
                                                      float decay, float lambda)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const BnJob J = jobs[lo];
    const int i = (wg - J.wg_start) * 256 + threadIdx.x;
    if (i >= J.C) return;
    float a = 0.f, b = 0.f, d = 0.f, mg = 0.f, mb = 0.f;
    for (int n = 0; n < N; ++n) {
        const float gg = J.g_gamma[(long long)n * J.C + i];
        const float gb = J.g_beta[(long long)n * J.C + i];
        a = fmaf(gg, gg, a); b = fmaf(gg, gb, b); d = fmaf(gb, gb, d);
        mg += gg; mb += gb;
    }
    const float inv_n = 1.0f / (float)N;
    a *= inv_n; b *= inv_n; d *= inv_n; mg *= inv_n; mb *= inv_n;
    float *F = J.F_ema + (long long)3 * i;
    float f0 = (1.0f - decay) * a, f1 = (1.0f - decay) * b, f2 = (1.0f - decay) * d;
    if (decay != 0.0f) { f0 += decay * F[0]; f1 += decay * F[1]; f2 += decay * F[2]; }
    F[0] = f0; F[1] = f1; F[2] = f2;
    // (F + lambda I)^-1 [mg, mb]^T with [[a,b],[c,d]]^-1 = 1/(ad - bc) [[d,-b],[-c,a]]
    const float fa = f0 + lambda, fd = f2 + lambda;
    const float det = fa * fd - f1 * f1;
    J.out_gamma[i] = (fd * mg - f1 * mb) / det;
    J.out_beta[i] = (fa * mb - f1 * mg) / det;
}

hipError_t launch_bn(const BnJob *jobs_dev, int n_jobs, int total_wgs, int N, float decay, float lambda,
                     hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    bn_unit_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, N, decay, lambda);
    return hipGetLastError();
}

hipError_t launch_bn_reduce(const BnReduceJob *jobs_dev, int n_jobs, int total_wgs, int N, int nhwc, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    if (nhwc) bn_reduce_nhwc_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, N);
    else      bn_reduce_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, N);
    return hipGetLastError();
}

}  // namespace kfac
