// Natural gradient on BatchNorm parameters with the Fisher block of the whole layer (Sec. 4.2,
// the dense 2c x 2c matrix the unit-wise approximation replaces; "fullBN" in Sec. 7).  With the
// per-sample gradient g_n in the order (gamma_1, beta_1, ..., gamma_c, beta_c):
//     F <- decay F + (1 - decay) / N  sum_n g_n g_n^T                 (pass 0, HBM bound)
//     gbar = mean_n g_n;  damping of the layer = lambda               (pass 1)
//     [out_gamma, out_beta] = (F + lambda I)^-1 gbar                  (pass 2, HBM bound GEMV)
// The inversion between passes 1 and 2 is the library's SPD inversion.
#include "kfac_internal.h"

namespace kfac {

__device__ __forceinline__ const BnFullJob *bnf_find(const BnFullJob *jobs, int n_jobs, int wg, int pass)
{
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start[pass] <= wg) lo = mid; else hi = mid;
    }
    return jobs + lo;
}

// element k of the interleaved per-sample gradient of sample n
__device__ __forceinline__ float bnf_elem(const float *g_gamma, const float *g_beta, int C, int n, int k)
{
    const float *src = (k & 1) ? g_beta : g_gamma;
    return src[(long long)n * C + (k >> 1)];
}

// Pass 0: one workgroup per 64 x 64 tile of F; 16 x 16 threads, 4 x 4 outputs each.  The rank-N
// update has only N terms per output, so the kernel is bound by reading and writing F
// (8 bytes per element); samples go through LDS 32 at a time.
__global__ __launch_bounds__(256) void bn_full_factor_kernel(const BnFullJob *__restrict__ jobs, int n_jobs, int N,
                                                             float decay)
{
    __shared__ float rows[32][64];
    __shared__ float cols[32][64];
    const BnFullJob *Jp = bnf_find(jobs, n_jobs, blockIdx.x, 0);
    const float *g_gamma = Jp->g_gamma, *g_beta = Jp->g_beta;
    float *F = Jp->F_ema;
    const int C = Jp->C;
    const int local = blockIdx.x - Jp->wg_start[0];
    const int d = 2 * C;
    const int tiles = (d + 63) / 64;
    const int r0 = (local / tiles) * 64, c0 = (local % tiles) * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    typedef float v4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, element alignment
    // whole tile (every tile when C is a multiple of 32): 16-byte accesses, and the old values are
    // requested before the products are formed
    const bool whole = r0 + 64 <= d && c0 + 64 <= d;
    float *base = F + (long long)(r0 + 4 * ty) * d + c0 + 4 * tx;
    v4 old[4];
    if (whole && decay != 0.f) {
#pragma unroll
        for (int i = 0; i < 4; ++i) old[i] = *(const v4 *)(base + (long long)i * d);
    }
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int n0 = 0; n0 < N; n0 += 32) {
        if (n0) __syncthreads();
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int e = threadIdx.x + 256 * q;     // 32 x 64 elements of each panel
            const int n = n0 + (e >> 6), k = e & 63;
            const bool ok = n < N;
            rows[e >> 6][k] = ok && r0 + k < d ? bnf_elem(g_gamma, g_beta, C, n, r0 + k) : 0.f;
            cols[e >> 6][k] = ok && c0 + k < d ? bnf_elem(g_gamma, g_beta, C, n, c0 + k) : 0.f;
        }
        __syncthreads();
        const int nn = N - n0 < 32 ? N - n0 : 32;
        for (int n = 0; n < nn; ++n) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = rows[n][4 * ty + i]; b[i] = cols[n][4 * tx + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
    }
    const float w = (1.0f - decay) / (float)N;
    if (whole) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = decay == 0.f ? w * acc[i][j] : fmaf(decay, old[i][j], w * acc[i][j]);
            *(v4 *)(base + (long long)i * d) = o;
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + 4 * ty + i;
        if (r >= d) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = c0 + 4 * tx + j;
            if (c >= d) continue;
            float *p = F + (long long)r * d + c;
            // decay == 0 must not read F (it may hold anything, NaN included, before the first step)
            *p = decay == 0.f ? w * acc[i][j] : fmaf(decay, *p, w * acc[i][j]);
        }
    }
}

// Pass 1: mean gradient in the order of w, and the layer's damping.
__global__ __launch_bounds__(256) void bn_full_mean_kernel(const BnFullJob *__restrict__ jobs, int n_jobs, int N,
                                                           float lambda, float *__restrict__ damp)
{
    const BnFullJob *Jp = bnf_find(jobs, n_jobs, blockIdx.x, 1);
    const float *g_gamma = Jp->g_gamma, *g_beta = Jp->g_beta;
    const int C = Jp->C, damp_idx = Jp->damp_idx;
    const int local = blockIdx.x - Jp->wg_start[1];
    const int k = local * 256 + threadIdx.x;
    if (local == 0 && threadIdx.x == 0 && damp_idx >= 0) damp[damp_idx] = lambda;
    if (k >= 2 * C) return;
    float s = 0.f;
    for (int n = 0; n < N; ++n) s += bnf_elem(g_gamma, g_beta, C, n, k);
    Jp->gbar[k] = s / (float)N;
}

// Pass 2: u = F_inv gbar, one wavefront per row, four rows per workgroup.
__global__ __launch_bounds__(256) void bn_full_apply_kernel(const BnFullJob *__restrict__ jobs, int n_jobs)
{
    typedef float v4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, element alignment
    const BnFullJob *Jp = bnf_find(jobs, n_jobs, blockIdx.x, 2);
    const int local = blockIdx.x - Jp->wg_start[2];
    const float *gbar = Jp->gbar;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = 2 * Jp->C;
    const int r = local * 4 + wave;
    if (r >= d) return;
    const float *row = Jp->F_inv + (long long)r * d;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if ((d & 3) == 0) {
        for (int k = 4 * lane; k < d; k += 256) {
            const v4 f = *(const v4 *)(row + k);
            const v4 g = *(const v4 *)(gbar + k);
            s0 = fmaf(f.x, g.x, s0); s1 = fmaf(f.y, g.y, s1); s2 = fmaf(f.z, g.z, s2); s3 = fmaf(f.w, g.w, s3);
        }
    } else {
        for (int k = lane; k < d; k += 64) s0 = fmaf(row[k], gbar[k], s0);
    }
    float s = (s0 + s1) + (s2 + s3);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) ((r & 1) ? Jp->out_beta : Jp->out_gamma)[r >> 1] = s;
}

hipError_t launch_bn_full(const BnFullJob *jobs_dev, int n_jobs, int total_wgs, int pass, int N, float decay,
                          float lambda, float *damp, hipStream_t s)
{
    if (n_jobs <= 0 || total_wgs <= 0) return hipSuccess;
    if (pass == 0) bn_full_factor_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, N, decay);
    else if (pass == 1) bn_full_mean_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, N, lambda, damp);
    else bn_full_apply_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

}  // namespace kfac
