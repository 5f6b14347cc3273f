// Symmetry-aware packing of the statistics (Sec. 5.2): a symmetric d x d matrix travels as its
// upper triangle, d (d + 1) / 2 elements -- row r contributes X[r][r .. d-1], rows in order,
// matrices back to back -- optionally rounded to bfloat16 (nearest, ties to even).
// Both directions are HBM bound and work on 64 x 64 tiles of the upper triangle, one workgroup
// per tile, one wavefront per row segment: a segment is contiguous in the matrix and in the
// packed buffer, so every access is a full 256-byte (128-byte for bf16) run.  Unpacking writes the
// mirror image through an LDS transpose, along rows as well.
#include "kfac_internal.h"

namespace kfac {

__device__ __forceinline__ void pack_tile_of(int t, int T, int &tr, int &tc)
{
    // upper-triangle tiles in row-major order: row tr holds T - tr tiles
    int r = 0, rem = t;
    while (rem >= T - r) { rem -= T - r; ++r; }
    tr = r; tc = r + rem;
}

__device__ __forceinline__ unsigned short pack_bf16(float x)
{
    const unsigned u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);   // NaN stays NaN
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ const PackJob &pack_find(const PackJob *jobs, int n_jobs, int wg)
{
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    return jobs[lo];
}

template <bool BF16>
__global__ __launch_bounds__(256) void pack_upper_kernel(const PackJob *__restrict__ jobs, int n_jobs, void *packed)
{
    const PackJob J = pack_find(jobs, n_jobs, blockIdx.x);
    int tr, tc;
    pack_tile_of(blockIdx.x - J.wg_start, J.tiles, tr, tc);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = 64 * tc + lane;
    // all 16 loads of a thread first (they are independent), then the stores
    float v[16];
    bool in[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int r = 64 * tr + wave + 4 * q;
        in[q] = r < J.d && c < J.d && c >= r;
        v[q] = in[q] ? __builtin_nontemporal_load(J.X + (long long)r * J.d + c) : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        if (!in[q]) continue;
        const int r = 64 * tr + wave + 4 * q;
        const long long k = J.off + (long long)r * J.d - (long long)r * (r - 1) / 2 + (c - r);
        if (BF16) ((unsigned short *)packed)[k] = pack_bf16(v[q]);
        else      ((float *)packed)[k] = v[q];
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void unpack_upper_kernel(const PackJob *__restrict__ jobs, int n_jobs,
                                                           const void *packed)
{
    __shared__ float tile[64][65];
    const PackJob J = pack_find(jobs, n_jobs, blockIdx.x);
    int tr, tc;
    pack_tile_of(blockIdx.x - J.wg_start, J.tiles, tr, tc);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *X = const_cast<float *>(J.X);
    const int c = 64 * tc + lane;
    float v[16];
    bool in[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int r = 64 * tr + wave + 4 * q;
        in[q] = r < J.d && c < J.d && c >= r;
        v[q] = 0.f;
        if (in[q]) {
            const long long k = J.off + (long long)r * J.d - (long long)r * (r - 1) / 2 + (c - r);
            v[q] = BF16 ? __uint_as_float((unsigned)((const unsigned short *)packed)[k] << 16) : ((const float *)packed)[k];
        }
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int rl = wave + 4 * q, r = 64 * tr + rl;
        if (in[q]) X[(long long)r * J.d + c] = v[q];
        tile[rl][lane] = v[q];
    }
    __syncthreads();
    // mirror image: element (c, r) for c > r, written along row c
    const int r = 64 * tr + lane;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int cl = wave + 4 * q, cc = 64 * tc + cl;
        if (cc < J.d && r < J.d && cc > r) X[(long long)cc * J.d + r] = tile[lane][cl];
    }
}

hipError_t launch_pack(const PackJob *jobs_dev, int n_jobs, int total_wgs, int bf16, int unpack, void *packed,
                       hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    if (!unpack) {
        if (bf16) pack_upper_kernel<true><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, packed);
        else      pack_upper_kernel<false><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, packed);
    } else {
        if (bf16) unpack_upper_kernel<true><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, packed);
        else      unpack_upper_kernel<false><<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, packed);
    }
    return hipGetLastError();
}

}  // namespace kfac
