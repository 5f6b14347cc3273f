// Staleness of statistics (Sec. 4.3, the similarity criterion under Algorithm 2):
//     ||X - P||_F / ||P||_F   and   ||X - Q||_F / ||Q||_F
// for a group of matrices X with their predecessors P = X_-1, Q = X_-2, in two passes over a
// device table of jobs.  HBM bound: every element of the three matrices is read once
// (12 bytes per element of X).  The sums are accumulated in double, per thread, per workgroup
// and per job always in the same order, so the result does not depend on scheduling.
#include "kfac_internal.h"

namespace kfac {

typedef float stale_vec4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, element alignment

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum of the four per-thread values over the workgroup, valid in thread 0.  The order is
// fixed: butterfly within each wavefront, then wavefront 0, 1, 2, 3.
__device__ __forceinline__ void block_sum4(double (&v)[4], double (*red)[4])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = wave_sum(v[k]);
    if (lane == 0)
#pragma unroll
        for (int k = 0; k < 4; ++k) red[wave][k] = v[k];
    __syncthreads();
    if (threadIdx.x == 0)
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = ((red[0][k] + red[1][k]) + red[2][k]) + red[3][k];
}

__global__ __launch_bounds__(256) void staleness_partial_kernel(const StaleJob *__restrict__ jobs, int n_jobs)
{
    __shared__ double red[4][4];
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const StaleJob J = jobs[lo];
    const int local = wg - J.wg_start;
    const long long e0 = (long long)local * kStaleChunk;
    const long long e1 = e0 + kStaleChunk < J.n ? e0 + kStaleChunk : J.n;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    // whole 4-element groups of the chunk: thread t takes groups t, t + 256, ... (all loads of a thread in flight at once)
    constexpr int GROUPS = kStaleChunk / 4 / 256;
    stale_vec4 x[GROUPS], p[GROUPS], q[GROUPS];
    bool in[GROUPS];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const long long e = e0 + 4LL * ((int)threadIdx.x + 256 * g);
        in[g] = e + 4 <= e1;
        x[g] = p[g] = q[g] = stale_vec4{0.f, 0.f, 0.f, 0.f};
        if (in[g]) {
            x[g] = __builtin_nontemporal_load((const stale_vec4 *)(J.X + e));
            if (J.P) p[g] = __builtin_nontemporal_load((const stale_vec4 *)(J.P + e));
            if (J.Q) q[g] = __builtin_nontemporal_load((const stale_vec4 *)(J.Q + e));
        }
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        if (!in[g]) continue;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const double xv = (double)x[g][k], pv = (double)p[g][k], qv = (double)q[g][k];
            acc[0] = fma(xv - pv, xv - pv, acc[0]);
            acc[1] = fma(pv, pv, acc[1]);
            acc[2] = fma(xv - qv, xv - qv, acc[2]);
            acc[3] = fma(qv, qv, acc[3]);
        }
    }
    // the last up to 3 elements of the matrix (only in its last chunk)
    const long long tail0 = e0 + ((e1 - e0) & ~3LL);
    if (threadIdx.x < (unsigned)(e1 - tail0)) {
        const long long e = tail0 + threadIdx.x;
        const double xv = (double)J.X[e], pv = J.P ? (double)J.P[e] : 0.0, qv = J.Q ? (double)J.Q[e] : 0.0;
        acc[0] = fma(xv - pv, xv - pv, acc[0]);
        acc[1] = fma(pv, pv, acc[1]);
        acc[2] = fma(xv - qv, xv - qv, acc[2]);
        acc[3] = fma(qv, qv, acc[3]);
    }
    block_sum4(acc, red);
    if (threadIdx.x == 0) {
        double *out = J.partial + 4LL * local;
        out[0] = acc[0]; out[1] = acc[1]; out[2] = acc[2]; out[3] = acc[3];
    }
}

__device__ __forceinline__ double stale_ratio(bool defined, double num, double den)
{
    if (!defined) return __builtin_huge_val();
    if (den == 0.0) return num == 0.0 ? 0.0 : __builtin_huge_val();
    return sqrt(num) / sqrt(den);
}

__global__ __launch_bounds__(256) void staleness_final_kernel(const StaleJob *__restrict__ jobs, int n_jobs)
{
    __shared__ double red[4][4];
    const StaleJob J = jobs[blockIdx.x];
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int w = threadIdx.x; w < J.wgs; w += 256) {
        const double *part = J.partial + 4LL * w;
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += part[k];
    }
    block_sum4(acc, red);
    if (threadIdx.x == 0) {
        J.out[0] = stale_ratio(J.P != nullptr, acc[0], acc[1]);
        J.out[1] = stale_ratio(J.Q != nullptr, acc[2], acc[3]);
    }
}

hipError_t launch_staleness(const StaleJob *jobs_dev, int n_jobs, int total_wgs, int pass, hipStream_t s)
{
    if (n_jobs <= 0) return hipSuccess;
    if (pass == 0) {
        if (total_wgs <= 0) return hipSuccess;
        staleness_partial_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    } else {
        staleness_final_kernel<<<dim3(n_jobs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    }
    return hipGetLastError();
}

}  // namespace kfac
