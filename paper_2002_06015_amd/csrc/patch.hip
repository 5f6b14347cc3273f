// Patch extraction (Sec. 3.3, Eq. 10: M_A = im2col(A) in R^{c_in k^2 x h w}) as a grouped,
// HBM-bound copy.  Output layout [c_in*k*k][ld] with the contraction index m = (n, y, x)
// contiguous, which is what the factor GEMM wants.  A wavefront owns one input plane
// (n, c): for each of the k*k taps it writes one contiguous run of h*w outputs (fully
// coalesced 256-byte stores); the plane itself is re-read k*k times out of L1/L2.
#include "kfac_internal.h"

namespace kfac {

constexpr int TCHUNK = 1024;  // output positions of one plane handled by one workgroup pass

template <typename T>
__device__ __forceinline__ void patch_plane(const PatchJob &J, int plane, int t0, int t1, int lane)
{
    const int n = plane / J.c_in, c = plane - n * J.c_in;
    const T *src = (const T *)J.src + (long long)plane * J.h_in * J.w_in;
    const int hw = J.h * J.w;
    const int kk = J.k * J.k;
    T *dst_row0 = (T *)J.dst + (long long)c * kk * J.ld + (long long)n * hw;
    for (int tap = 0; tap < kk; ++tap) {
        const int ky = tap / J.k, kx = tap - ky * J.k;
        T *dst = dst_row0 + (long long)tap * J.ld;
        for (int t = t0 + lane; t < t1; t += 64) {
            const int y = J.magic_w ? (int)__umulhi((unsigned)t, J.magic_w) : t / J.w;
            const int x = t - y * J.w;
            const int iy = y * J.stride + ky - J.pad, ix = x * J.stride + kx - J.pad;
            T v = (T)0;
            if (iy >= 0 && iy < J.h_in && ix >= 0 && ix < J.w_in) v = src[iy * J.w_in + ix];
            dst[t] = v;
        }
    }
}

// The same with four outputs per lane and one 16-byte (fp32) or 8-byte (bf16) store: needs
// h*w % 4 == 0 (so that a group of four starts aligned and stays inside the plane) and w >= 4
// (so that it wraps to the next output row at most once).  ld is a multiple of 32.
template <typename T>
__device__ __forceinline__ void patch_plane_vec4(const PatchJob &J, int plane, int t0, int t1, int lane)
{
    typedef T vec4 __attribute__((ext_vector_type(4)));
    const int n = plane / J.c_in, c = plane - n * J.c_in;
    const T *src = (const T *)J.src + (long long)plane * J.h_in * J.w_in;
    const int hw = J.h * J.w;
    const int kk = J.k * J.k;
    T *dst_row0 = (T *)J.dst + (long long)c * kk * J.ld + (long long)n * hw;
    for (int t = t0 + 4 * lane; t < t1; t += 256) {
        const int y0 = J.magic_w ? (int)__umulhi((unsigned)t, J.magic_w) : t / J.w;
        const int x0 = t - y0 * J.w;
        int iy[4], ix[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool wrap = x0 + e >= J.w;
            iy[e] = (y0 + (wrap ? 1 : 0)) * J.stride - J.pad;
            ix[e] = (x0 + e - (wrap ? J.w : 0)) * J.stride - J.pad;
        }
        for (int ky = 0; ky < J.k; ++ky)
            for (int kx = 0; kx < J.k; ++kx) {
                vec4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int yy = iy[e] + ky, xx = ix[e] + kx;
                    T u = (T)0;
                    if (yy >= 0 && yy < J.h_in && xx >= 0 && xx < J.w_in) u = src[yy * J.w_in + xx];
                    v[e] = u;
                }
                __builtin_nontemporal_store(v, (vec4 *)(dst_row0 + (long long)(ky * J.k + kx) * J.ld + t));
            }
    }
}

// The same for a kernel size and stride known at compile time and output rows that are a whole number of groups
// (w % 4 == 0: the four outputs of a group lie in one output row): per kernel row the lane gathers the
// 3 * S + K input values its four outputs touch once, and every tap takes its four values from that window
// (7 x 7 / stride 2: 91 loads per group instead of 196).
template <typename T, int K, int S>
__device__ __forceinline__ void patch_plane_window(const PatchJob &J, int plane, int t0, int t1, int lane)
{
    typedef T vec4 __attribute__((ext_vector_type(4)));
    constexpr int WIN = 3 * S + K;
    const int n = plane / J.c_in, c = plane - n * J.c_in;
    const T *src = (const T *)J.src + (long long)plane * J.h_in * J.w_in;
    const int hw = J.h * J.w;
    T *dst_row0 = (T *)J.dst + (long long)c * (K * K) * J.ld + (long long)n * hw;
    for (int t = t0 + 4 * lane; t < t1; t += 256) {
        const int y0 = J.magic_w ? (int)__umulhi((unsigned)t, J.magic_w) : t / J.w;
        const int x0 = t - y0 * J.w;
        const int ix0 = x0 * S - J.pad;
#pragma unroll
        for (int ky = 0; ky < K; ++ky) {
            const int iy = y0 * S - J.pad + ky;
            const bool row_in = iy >= 0 && iy < J.h_in;
            const T *line = src + (row_in ? iy : 0) * J.w_in;
            T win[WIN];
#pragma unroll
            for (int j = 0; j < WIN; ++j) {
                const int ix = ix0 + j;
                win[j] = (row_in && ix >= 0 && ix < J.w_in) ? line[ix] : (T)0;
            }
#pragma unroll
            for (int kx = 0; kx < K; ++kx) {
                const vec4 v = {win[kx], win[S + kx], win[2 * S + kx], win[3 * S + kx]};
                __builtin_nontemporal_store(v, (vec4 *)(dst_row0 + (long long)(ky * K + kx) * J.ld + t));
            }
        }
    }
}

__global__ __launch_bounds__(256) void patch_kernel(const PatchJob *__restrict__ jobs, int n_jobs)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const PatchJob &J = jobs[lo];
    const int local = wg - J.wg_start;
    const int hw = J.h * J.w;
    if (J.flat) {
        // pointwise layer with tiny planes (e.g. a fully-connected layer, hw = 1): one thread
        // per output element, P[c][n*hw + t] = src[n][c][t]
        const int M = J.N * hw;
        const int chunks_m = (M + 255) / 256;
        const int row = local / chunks_m;
        const int m = (local - row * chunks_m) * 256 + (int)threadIdx.x;
        if (m >= M) return;
        const int n = m / hw, t = m - n * hw;
        const long long so = ((long long)n * J.c_in + row) * hw + t;
        const long long d = (long long)row * J.ld + m;
        if (J.esize == 4) ((float *)J.dst)[d] = ((const float *)J.src)[so];
        else              ((unsigned short *)J.dst)[d] = ((const unsigned short *)J.src)[so];
        return;
    }
    const int chunks = (hw + TCHUNK - 1) / TCHUNK;
    const int chunk = local % chunks;
    const int plane = (local / chunks) * 4 + (threadIdx.x >> 6);
    if (plane >= J.N * J.c_in) return;
    const int t0 = chunk * TCHUNK, t1 = min(hw, t0 + TCHUNK);
    const bool vec = (hw & 3) == 0 && J.w >= 4 && (((uintptr_t)J.dst) & 15) == 0;   // TCHUNK is a multiple of 4
    const bool stem = vec && J.k == 7 && J.stride == 2 && (J.w & 3) == 0;   // the 7 x 7 / stride 2 first layer
    if (J.esize == 4) {
        if (stem)     patch_plane_window<float, 7, 2>(J, plane, t0, t1, threadIdx.x & 63);
        else if (vec) patch_plane_vec4<float>(J, plane, t0, t1, threadIdx.x & 63);
        else          patch_plane<float>(J, plane, t0, t1, threadIdx.x & 63);
    } else {
        if (stem)     patch_plane_window<unsigned short, 7, 2>(J, plane, t0, t1, threadIdx.x & 63);
        else if (vec) patch_plane_vec4<unsigned short>(J, plane, t0, t1, threadIdx.x & 63);
        else          patch_plane<unsigned short>(J, plane, t0, t1, threadIdx.x & 63);
    }
}

hipError_t launch_patch(const PatchJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    patch_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

}  // namespace kfac
