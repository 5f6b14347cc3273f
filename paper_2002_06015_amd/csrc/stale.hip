// Staleness of statistics (Sec. 4.3, the similarity criterion under Algorithm 2):
//     ||X - P||_F / ||P||_F   and   ||X - Q||_F / ||Q||_F
// for a group of matrices X with their predecessors P = X_-1, Q = X_-2, in two passes over a
// device table of jobs.  HBM bound: every element of the three matrices is read once
// (12 bytes per element of X).  The sums are accumulated in double, per thread, per workgroup
// and per job always in the same order, so the result does not depend on scheduling.
#include "../../include/kfac.h"
#include "kfac_internal.h"

#include <mutex>

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

// Sums of one chunk of kStaleChunk elements of job J (chunk `local`), written to J.partial.
__device__ __forceinline__ void stale_partial_chunk(const StaleJob &J, int local, double (*red)[4])
{
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
    stale_partial_chunk(J, wg - J.wg_start, red);
}

// Adds the chunk sums of job J in a fixed order and writes its two ratios.
__device__ __forceinline__ void stale_final_job(const StaleJob &J, double (*red)[4])
{
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

__global__ __launch_bounds__(256) void staleness_final_kernel(const StaleJob *__restrict__ jobs, int n_jobs)
{
    __shared__ double red[4][4];
    const StaleJob J = jobs[blockIdx.x];
    stale_final_job(J, red);
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

// ---- the variant that allocates nothing ------------------------------------------------------
// Chunk sums live in a fixed device array instead of the caller's workspace, and the job table
// travels in the kernel arguments instead of a device table, so a call needs no memory beyond
// its inputs and outputs.  One array per GPU, shared by every call on that GPU.
constexpr int kStaticChunks = 16384;     // chunk sums the array holds: 16384 * 4096 = 2^26 matrix elements
constexpr int kStaticBatch = 64;         // jobs per launch (the table must fit the kernel argument segment)
constexpr int kStaticMaxDevices = 64;

static __device__ __align__(256) double scratch[4 * kStaticChunks];   // 512 KiB

struct StaleBatch {
    struct Item {
        const float *X, *P, *Q;
        double *out;
        long long n;
        int wg_start, wgs;
    } item[kStaticBatch];
    int n_jobs;
};

__device__ __forceinline__ StaleJob stale_batch_job(const StaleBatch &B, int i, double *partial_base)
{
    StaleJob J;
    J.X = B.item[i].X; J.P = B.item[i].P; J.Q = B.item[i].Q;
    J.n = B.item[i].n;
    J.partial = partial_base + 4LL * B.item[i].wg_start;
    J.out = B.item[i].out;
    J.wgs = B.item[i].wgs;
    J.wg_start = B.item[i].wg_start;
    return J;
}

__global__ __launch_bounds__(256) void staleness_partial_static_kernel(const StaleBatch B, double *partial_base)
{
    __shared__ double red[4][4];
    const int wg = blockIdx.x;
    int lo = 0, hi = B.n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (B.item[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const StaleJob J = stale_batch_job(B, lo, partial_base);
    stale_partial_chunk(J, wg - J.wg_start, red);
}

__global__ __launch_bounds__(256) void staleness_final_static_kernel(const StaleBatch B, double *partial_base)
{
    __shared__ double red[4][4];
    const StaleJob J = stale_batch_job(B, blockIdx.x, partial_base);
    stale_final_job(J, red);
}

// Device address of this GPU's copy of `scratch` (each GPU holds its own), looked up once per
// device with that device current.  Returns null on failure.
static double *static_scratch_ptr()
{
    static std::mutex mu;
    static double *ptr[kStaticMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        double *p = nullptr;
        if (hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
}

}  // namespace kfac

extern "C" kfac_status kfac_staleness_static(void *hip_stream, int32_t n, const int32_t *dims, const float *const *X,
                                             const float *const *X_m1, const float *const *X_m2, double *ratios)
{
    using namespace kfac;
    if (n < 1 || n > 65536 || !dims || !X || !ratios) return KFAC_ERR_INVALID;
    for (int i = 0; i < n; ++i) {
        if (dims[i] < 1 || dims[i] > (1 << 20) || !X[i]) return KFAC_ERR_INVALID;
        if ((X_m1 && X_m1[i] == X[i]) || (X_m2 && X_m2[i] == X[i])) return KFAC_ERR_INVALID;
        const long long elems = (long long)dims[i] * dims[i];
        if ((elems + kStaleChunk - 1) / kStaleChunk > kStaticChunks) return KFAC_ERR_WORKSPACE;   // beyond the fixed array
    }
    double *base = static_scratch_ptr();
    if (!base) return KFAC_ERR_DEVICE;
    hipStream_t s = (hipStream_t)hip_stream;
    // launches in stream order share the array: a batch ends at kStaticBatch jobs or when the array is full
    int i = 0;
    while (i < n) {
        StaleBatch B;
        B.n_jobs = 0;
        int wgs = 0;
        while (i < n && B.n_jobs < kStaticBatch) {
            const long long elems = (long long)dims[i] * dims[i];
            const int w = (int)((elems + kStaleChunk - 1) / kStaleChunk);
            if (wgs + w > kStaticChunks) break;
            StaleBatch::Item &it = B.item[B.n_jobs++];
            it.X = X[i];
            it.P = X_m1 ? X_m1[i] : nullptr;
            it.Q = X_m2 ? X_m2[i] : nullptr;
            it.out = ratios + 2 * i;
            it.n = elems;
            it.wg_start = wgs;
            it.wgs = w;
            wgs += w;
            ++i;
        }
        staleness_partial_static_kernel<<<dim3(wgs), dim3(256), 0, s>>>(B, base);
        staleness_final_static_kernel<<<dim3(B.n_jobs), dim3(256), 0, s>>>(B, base);
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_DEVICE;
    }
    return KFAC_OK;
}
