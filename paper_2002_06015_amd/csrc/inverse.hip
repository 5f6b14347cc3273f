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
        damp[3 * J.idx + 0] = (float)pi;
        damp[3 * J.idx + 1] = (float)(pi * (double)gamma);   // added to A
        damp[3 * J.idx + 2] = (float)((double)gamma / pi);   // added to G
        if (pi_out) pi_out[J.idx] = (float)pi;
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
// T[k][j] = -T[j][k] for j < k and T[k][j] = T[j][k] for j > k, so publishing pivot rows
// alone also gives the pivot columns.  A single-pivot step would be
//     p = 1/T[k][k];  T[i][j] -= T[i][k] p T[k][j]  (i, j != k);
//     T[k][j] *= p;   T[i][k] *= -p;   T[k][k] = p;
// the kernel takes the pivots in pairs (see the loop).  One barrier per pair (the pivot row
// buffer is double-buffered).  A non-positive pivot is reported through info.
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
    static_assert((TR * BR) % 2 == 0, "pivots are taken in pairs");
    __shared__ float rowbuf[2][2][32 * BC];
    int bad = 0;
    const LeafJob J = jobs[blockIdx.x];
    const int n = J.n;
    const int tj = threadIdx.x & 31, ti = threadIdx.x >> 5;
    const float d = (J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f;

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

    // Two pivots per step (one barrier and one LDS round trip for both): with the pivot rows
    // R = T[{k,k+1}, :], the 2x2 pivot block P and Q = P^-1, a block Gauss-Jordan step is
    //     T[i][j] -= C[i,:] Q R[:,j],  T[K,j] = Q R[:,j],  T[i,K] = -C[i,:] Q,  T[K,K] = Q,
    // where the pivot columns follow from the rows: C[i,:] = s_i R[:,i]^T, s_i = -1 for
    // already eliminated i < k and +1 otherwise.  The owners of rows/columns k, k+1 clear
    // their old values and patch their multipliers so that the same two fused multiply-adds
    // produce exactly those special results.  The pivot loop is split into BR compile-time
    // blocks of TR pivots, so that the register row (KBR) and column (KBC) holding the pivot
    // rows/columns are compile-time constants and the matrix never leaves its registers.
    // An odd n takes the identity padding row n as its last second pivot.
    const int n_even = n + (n & 1);
    static_for<0, BR>([&](auto KB) {
        constexpr int KBR = decltype(KB)::value;
        constexpr int KBC = (KBR * TR) / 32;
        const int kend = min(n_even, (KBR + 1) * TR);
        for (int k = KBR * TR; k < kend; k += 2) {
            const int ktr = k - KBR * TR;   // rows k, k+1 live in threads ti == ktr, ktr+1, register row KBR
            const int ktc = k & 31;         // columns k, k+1 live in threads tj == ktc, ktc+1, register column KBC
            float *rb0 = rowbuf[(k >> 1) & 1][0], *rb1 = rowbuf[(k >> 1) & 1][1];
            if (ti == ktr) {
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) rb0[tj + 32 * bj] = a[KBR][bj];
            }
            if (ti == ktr + 1) {
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) rb1[tj + 32 * bj] = a[KBR][bj];
            }
            __syncthreads();
            const float pa = rb0[k], pb = rb0[k + 1], pd = rb1[k + 1];
            const float det = fmaf(pa, pd, -pb * pb);
            // non-positive pivots (the second one is det / pa) are recorded, first one wins,
            // tracked in a register by every thread alike; the elimination goes on and its
            // (meaningless) result is still written: no early exit, no branch
            const int badk = !(pa > 0.f) ? k + 1 : (!(det > 0.f) ? k + 2 : 0);
            bad = (bad == 0) ? badk : bad;
            const float idet = __builtin_amdgcn_rcpf(det);
            const float q00 = pd * idet, q01 = -pb * idet, q11 = pa * idet;
            float t0[BC], t1[BC], c0[BR], c1[BR];
#pragma unroll
            for (int bj = 0; bj < BC; ++bj) {
                const float r0 = rb0[tj + 32 * bj], r1 = rb1[tj + 32 * bj];
                t0[bj] = fmaf(q00, r0, q01 * r1);
                t1[bj] = fmaf(q01, r0, q11 * r1);
            }
#pragma unroll
            for (int bi = 0; bi < BR; ++bi) {
                const int i = ti + TR * bi;
                const float r0 = rb0[i], r1 = rb1[i];
                c0[bi] = (i < k) ? -r0 : r0;
                c1[bi] = (i < k) ? -r1 : r1;
            }
            if (ti == ktr || ti == ktr + 1) {
#pragma unroll
                for (int bj = 0; bj < BC; ++bj) a[KBR][bj] = 0.f;
                c0[KBR] = (ti == ktr) ? -1.f : 0.f;
                c1[KBR] = (ti == ktr) ? 0.f : -1.f;
            }
            if (tj == ktc || tj == ktc + 1) {
#pragma unroll
                for (int bi = 0; bi < BR; ++bi) a[bi][KBC] = 0.f;
                t0[KBC] = (tj == ktc) ? q00 : q01;
                t1[KBC] = (tj == ktc) ? q01 : q11;
            }
#pragma unroll
            for (int bi = 0; bi < BR; ++bi)
#pragma unroll
                for (int bj = 0; bj < BC; ++bj)
                    a[bi][bj] = fmaf(-c1[bi], t1[bj], fmaf(-c0[bi], t0[bj], a[bi][bj]));
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
        case 3: leaf_inverse_kernel<6, 3, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 4: leaf_inverse_kernel<8, 4, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 5: leaf_inverse_kernel<10, 5, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 7: leaf_inverse_kernel<14, 7, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 8: leaf_inverse_kernel<16, 8, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        case 9: leaf_inverse_kernel<18, 9, 16><<<grid, dim3(512), 0, s>>>(jobs_dev, damp_dev, info); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace kfac
