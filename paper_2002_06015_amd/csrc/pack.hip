// Symmetry-aware packing of the statistics (Sec. 5.2): a symmetric d x d matrix travels as its
// upper triangle, d (d + 1) / 2 elements -- row r contributes X[r][r .. d-1], rows in order,
// matrices back to back -- optionally rounded to bfloat16 (nearest, ties to even).
// Both directions are HBM bound.  Packing walks the packed buffer (see pack_upper_kernel).
// Unpacking works on 64 x 64 tiles of the upper triangle, one workgroup per tile, one wavefront
// per row segment (contiguous in the matrix and in the packed buffer: 256-byte runs, 128 for
// bf16), and writes the mirror image through an LDS transpose, along rows as well.
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

// Packing is driven by the output: a workgroup produces 4096 consecutive elements of a matrix's
// triangle, a thread four groups of four.  The row of an element p follows from
// start(r) = r d - r (r - 1) / 2 <= p by the quadratic formula (in fp32, then corrected by exact integer steps);
// consecutive elements are consecutive in the matrix except at the ends of rows, so the reads are
// as contiguous as the writes.
__device__ __forceinline__ long long pack_row_start(int r, int d) { return (long long)r * d - (long long)r * (r - 1) / 2; }

template <bool BF16>
__global__ __launch_bounds__(256) void pack_upper_kernel(const PackJob *__restrict__ jobs, int n_jobs, void *packed)
{
    typedef float v4 __attribute__((ext_vector_type(4), aligned(4)));
    typedef unsigned short h4 __attribute__((ext_vector_type(4), aligned(2)));
    const PackJob *J = &pack_find(jobs, n_jobs, blockIdx.x);
    const int d = J->d;
    const float *X = J->X;
    const long long tri = (long long)d * (d + 1) / 2, off = J->off;
    const long long p0 = (long long)(blockIdx.x - J->wg_start) * kPackChunk;
    v4 v[4];
    // all loads of a thread first (they are independent), then the stores
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const long long p = p0 + 4LL * ((int)threadIdx.x + 256 * g);
        v[g] = v4{0.f, 0.f, 0.f, 0.f};
        if (p >= tri) continue;
        const float b = 2.0f * d + 1.0f;
        int r = (int)((b - sqrtf(b * b - 8.0f * (float)p)) * 0.5f);
        r = r < 0 ? 0 : (r > d - 1 ? d - 1 : r);
        while (r + 1 < d && pack_row_start(r + 1, d) <= p) ++r;
        while (r > 0 && pack_row_start(r, d) > p) --r;
        int c = r + (int)(p - pack_row_start(r, d));
        if (c + 3 < d) {
            v[g] = __builtin_nontemporal_load((const v4 *)(X + (long long)r * d + c));
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (p + k < tri) v[g][k] = X[(long long)r * d + c];
                if (++c == d) { ++r; c = r; }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const long long p = p0 + 4LL * ((int)threadIdx.x + 256 * g);
        if (p >= tri) continue;
        if (p + 3 < tri) {
            if (BF16) *(h4 *)((unsigned short *)packed + off + p) = h4{pack_bf16(v[g][0]), pack_bf16(v[g][1]), pack_bf16(v[g][2]), pack_bf16(v[g][3])};
            else      *(v4 *)((float *)packed + off + p) = v[g];
        } else {
            for (int k = 0; k < 4 && p + k < tri; ++k) {
                if (BF16) ((unsigned short *)packed)[off + p + k] = pack_bf16(v[g][k]);
                else      ((float *)packed)[off + p + k] = v[g][k];
            }
        }
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
