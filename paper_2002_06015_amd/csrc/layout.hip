// NHWC -> NCHW conversion of convolution inputs and output gradients (Sec. 5.2 names NHWC as the
// layout of the tensors around convolution layers; the statistics kernels read NCHW).  Per image a
// [HW, C] matrix is transposed into [C, HW] in 64 x 64 tiles through LDS, so that both the reads
// (along C) and the writes (along HW) are contiguous; 16-byte (fp32) / 8-byte (bf16) accesses where
// C resp. HW is a multiple of 4.  HBM bound: every element is read once and written once.
#include "kfac_internal.h"

namespace kfac {

template <typename T>
__global__ __launch_bounds__(256) void nhwc_to_nchw_kernel(const LayoutJob *__restrict__ jobs, int n_jobs)
{
    typedef T vec4 __attribute__((ext_vector_type(4), aligned(sizeof(T))));
    __shared__ T tile[64][65];   // [c][hw]; odd stride: the transposed accesses spread over the banks
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= (int)blockIdx.x) lo = mid; else hi = mid;
    }
    const LayoutJob *J = jobs + lo;
    const int C = J->C, HW = J->HW, tc = J->tiles_c, th = J->tiles_hw;
    int local = blockIdx.x - J->wg_start;
    const int n = local / (tc * th);
    local -= n * tc * th;
    const int h0 = (local / tc) * 64, c0 = (local % tc) * 64;
    const T *src = (const T *)J->src + (long long)n * HW * C;
    T *dst = (T *)J->dst + (long long)n * HW * C;
    const int g = threadIdx.x & 15, r = threadIdx.x >> 4;
    // read: rows of the tile are positions hw, 16 groups of 4 channels each
    if ((C & 3) == 0) {
        vec4 v[4];
        bool in[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int h = h0 + r + 16 * q, c = c0 + 4 * g;
            in[q] = h < HW && c < C;
            if (in[q]) v[q] = __builtin_nontemporal_load((const vec4 *)(src + (long long)h * C + c));
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (!in[q]) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) tile[4 * g + i][r + 16 * q] = v[q][i];
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int h = h0 + r + 16 * q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = c0 + g + 16 * i;        // consecutive lanes, consecutive channels
                if (h < HW && c < C) tile[g + 16 * i][r + 16 * q] = src[(long long)h * C + c];
            }
        }
    }
    __syncthreads();
    // write: rows of the tile are channels, 16 groups of 4 positions each
    if ((HW & 3) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + r + 16 * q, h = h0 + 4 * g;
            if (c < C && h < HW) {
                vec4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = tile[r + 16 * q][4 * g + i];
                *(vec4 *)(dst + (long long)c * HW + h) = v;
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + r + 16 * q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int h = h0 + g + 16 * i;
                if (c < C && h < HW) dst[(long long)c * HW + h] = tile[r + 16 * q][g + 16 * i];
            }
        }
    }
}

hipError_t launch_nhwc_to_nchw(const LayoutJob *jobs_dev, int n_jobs, int total_wgs, int esize, hipStream_t s)
{
    if (n_jobs <= 0 || total_wgs <= 0) return hipSuccess;
    if (esize == 4) nhwc_to_nchw_kernel<float><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    else nhwc_to_nchw_kernel<unsigned short><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

}  // namespace kfac
