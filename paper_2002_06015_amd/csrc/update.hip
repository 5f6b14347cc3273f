// End of the optimisation step (Sec. 6.2 Eq. "paramupdate", Sec. 6.3 "Weights rescaling"):
//     w' = w - eta U + m (w - w_prev);     w_prev <- w;     w <- sqrt(2 d_out) w' / (||w'|| + eps)
// for a group of layers in three passes over a device table of jobs.  HBM bound: pass 0 reads
// U, w and w_prev and writes w' and w_prev (20 bytes per weight) and leaves the sum of squares
// of its chunk (in double, fixed order); pass 1 turns the sums of a layer into its scale
// factor; pass 2 multiplies w' by it (8 bytes per weight).  Without rescaling only pass 0 runs.
#include "kfac_internal.h"

namespace kfac {

typedef float upd_vec4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, element alignment

__device__ __forceinline__ const UpdateJob &upd_find(const UpdateJob *jobs, int n_jobs, int wg)
{
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    return jobs[lo];
}

__device__ __forceinline__ float upd_one(float w, float wp, float u, float eta, float m)
{
    return fmaf(m, w - wp, fmaf(-eta, u, w));
}

__global__ __launch_bounds__(256) void update_step_kernel(const UpdateJob *__restrict__ jobs, int n_jobs, float eta,
                                                          float momentum)
{
    __shared__ double red[4];
    const UpdateJob J = upd_find(jobs, n_jobs, blockIdx.x);
    const int local = blockIdx.x - J.wg_start;
    const long long e0 = (long long)local * kUpdateChunk;
    const long long e1 = e0 + kUpdateChunk < J.n ? e0 + kUpdateChunk : J.n;
    double ss = 0.0;
    constexpr int GROUPS = kUpdateChunk / 4 / 256;
    upd_vec4 w[GROUPS], wp[GROUPS], u[GROUPS];
    bool in[GROUPS];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const long long e = e0 + 4LL * ((int)threadIdx.x + 256 * g);
        in[g] = e + 4 <= e1;
        if (in[g]) {
            w[g] = *(const upd_vec4 *)(J.W + e);
            wp[g] = *(const upd_vec4 *)(J.W_prev + e);
            u[g] = __builtin_nontemporal_load((const upd_vec4 *)(J.U + e));
        }
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        if (!in[g]) continue;
        const long long e = e0 + 4LL * ((int)threadIdx.x + 256 * g);
        upd_vec4 nw;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            nw[k] = upd_one(w[g][k], wp[g][k], u[g][k], eta, momentum);
            ss = fma((double)nw[k], (double)nw[k], ss);
        }
        *(upd_vec4 *)(J.W + e) = nw;
        *(upd_vec4 *)(J.W_prev + e) = w[g];
    }
    const long long tail0 = e0 + ((e1 - e0) & ~3LL);
    if (threadIdx.x < (unsigned)(e1 - tail0)) {
        const long long e = tail0 + threadIdx.x;
        const float wv = J.W[e];
        const float nw = upd_one(wv, J.W_prev[e], J.U[e], eta, momentum);
        ss = fma((double)nw, (double)nw, ss);
        J.W[e] = nw;
        J.W_prev[e] = wv;
    }
    if (!J.partial) return;   // no rescaling: the sums are not needed
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (threadIdx.x == 0) J.partial[local] = ((red[0] + red[1]) + red[2]) + red[3];
}

__global__ __launch_bounds__(256) void update_scale_kernel(const UpdateJob *__restrict__ jobs, int n_jobs, float eps)
{
    __shared__ double red[4];
    const UpdateJob J = jobs[blockIdx.x];
    if (!J.partial) return;
    double ss = 0.0;
    for (int w = threadIdx.x; w < J.wgs; w += 256) ss += J.partial[w];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double norm = sqrt(((red[0] + red[1]) + red[2]) + red[3]);
        *J.scale = (float)(sqrt(2.0 * (double)J.d_out) / (norm + (double)eps));
    }
}

__global__ __launch_bounds__(256) void update_rescale_kernel(const UpdateJob *__restrict__ jobs, int n_jobs)
{
    const UpdateJob J = upd_find(jobs, n_jobs, blockIdx.x);
    if (!J.partial) return;
    const float sc = *J.scale;
    const long long e0 = (long long)(blockIdx.x - J.wg_start) * kUpdateChunk;
    const long long e1 = e0 + kUpdateChunk < J.n ? e0 + kUpdateChunk : J.n;
    constexpr int GROUPS = kUpdateChunk / 4 / 256;
    upd_vec4 w[GROUPS];
    bool in[GROUPS];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const long long e = e0 + 4LL * ((int)threadIdx.x + 256 * g);
        in[g] = e + 4 <= e1;
        if (in[g]) w[g] = *(const upd_vec4 *)(J.W + e);
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        if (!in[g]) continue;
        const long long e = e0 + 4LL * ((int)threadIdx.x + 256 * g);
        *(upd_vec4 *)(J.W + e) = w[g] * sc;
    }
    const long long tail0 = e0 + ((e1 - e0) & ~3LL);
    if (threadIdx.x < (unsigned)(e1 - tail0)) J.W[tail0 + threadIdx.x] *= sc;
}

hipError_t launch_update(const UpdateJob *jobs_dev, int n_jobs, int total_wgs, int pass, float eta, float momentum,
                         float eps, hipStream_t s)
{
    if (n_jobs <= 0 || total_wgs <= 0) return hipSuccess;
    if (pass == 0) update_step_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, eta, momentum);
    else if (pass == 1) update_scale_kernel<<<dim3(n_jobs), dim3(256), 0, s>>>(jobs_dev, n_jobs, eps);
    else update_rescale_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

}  // namespace kfac
