// Kernels of the damped inversion (Sec. 3.3, Eq. 12) other than the GEMMs:
//   - trace_kernel:  pi^2 = (tr A / dA) / (tr G / dG) and the two damping values per layer;
//   - copy_damp_kernel: dst = src + damp * I (start of the blocked inversion), optionally with the
//     bias border of an A factor eliminated on the way (Schur complement), and border_kernel,
//     which puts the border back into the finished inverse;
//   - leaf_block_kernel: (X + damp I)^-1 for n <= 288 by a blocked symmetric sweep held in the
//     registers of one 1024-thread workgroup, block products on the matrix cores (one matrix per
//     workgroup, many matrices per launch).
#include "kfac_internal.h"


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
    const float *last = J.src + (long long)J.n * J.lds;   // the border row u^T, c (if any)
    const float ic = J.border ? 1.f / (last[J.n] + d) : 0.f;
    const int r1 = min(J.n, r0 + COPY_ROWS);
    // four adjacent columns per thread (16-byte accesses that only need element alignment: the
    // leading dimensions are odd for bordered factors), all rows of the workgroup in flight at once
    typedef float vec4 __attribute__((ext_vector_type(4), aligned(4)));
    const int n4 = J.n & ~3;
    for (int c = 4 * (int)threadIdx.x; c < n4; c += 1024) {
        vec4 v[COPY_ROWS];
#pragma unroll
        for (int q = 0; q < COPY_ROWS; ++q)
            if (r0 + q < r1) v[q] = *(const vec4 *)(J.src + (long long)(r0 + q) * J.lds + c);
        vec4 u = {0.f, 0.f, 0.f, 0.f};
        if (J.border) u = *(const vec4 *)(last + c);
#pragma unroll
        for (int q = 0; q < COPY_ROWS; ++q) {
            const int r = r0 + q;
            if (r >= r1) break;
            vec4 x = v[q];
            if (r >= c && r < c + 4) x[r - c] += d;
            if (J.border) {
                const float ur = last[r] * ic;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = fmaf(-ur, u[e], x[e]);
            }
            *(vec4 *)(J.dst + (long long)r * J.ldd + c) = x;
        }
    }
    for (int r = r0; r < r1; ++r) {
        const float ur = J.border ? last[r] * ic : 0.f;
        for (int c = n4 + (int)threadIdx.x; c < J.n; c += 256) {
            float v = J.src[(long long)r * J.lds + c];
            if (r == c) v += d;
            if (J.border) v = fmaf(-ur, last[c], v);
            J.dst[(long long)r * J.ldd + c] = v;
        }
    }
}

hipError_t launch_copy_damp(const CopyJob *jobs_dev, int n_jobs, int total_wgs, const float *damp_dev,
                            hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    copy_damp_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs, damp_dev);
    return hipGetLastError();
}

// ------------------------------------------------------------------ border of a bordered inverse
__global__ __launch_bounds__(256) void border_kernel(const BorderJob *__restrict__ jobs, int n_jobs, int pass,
                                                     const float *__restrict__ damp, int32_t *__restrict__ info)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (pass == 0) {
        // one wavefront per row i: w_i = sum_j X[i][j] u_j
        const int wg = blockIdx.x;
        int lo = 0, hi = n_jobs;
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
        }
        const BorderJob J = jobs[lo];
        const int i = (wg - J.wg_start) * 4 + wave;
        if (i >= J.n) return;
        const float *u = J.src + (long long)J.n * J.lds;
        const float *x = J.X + (long long)i * J.ldx;
        // 16-byte accesses that only need element alignment (the leading dimensions are odd)
        typedef float vec4 __attribute__((ext_vector_type(4), aligned(4)));
        float a4[4] = {0.f, 0.f, 0.f, 0.f};
        const int n4 = J.n & ~3;
        for (int j = 4 * lane; j < n4; j += 256) {
            const vec4 xv = *(const vec4 *)(x + j), uv = *(const vec4 *)(u + j);
#pragma unroll
            for (int e = 0; e < 4; ++e) a4[e] = fmaf(xv[e], uv[e], a4[e]);
        }
        float acc = (a4[0] + a4[1]) + (a4[2] + a4[3]);
        for (int j = n4 + lane; j < J.n; j += 64) acc = fmaf(x[j], u[j], acc);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) {
            const float c = u[J.n] + ((J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f);
            const float v = -acc / c;
            J.X[(long long)i * J.ldx + J.n] = v;
            J.X[(long long)J.n * J.ldx + i] = v;
        }
        return;
    }
    // corner: X[n][n] = (1 - sum_i u_i X[n][i]) / c   (X[n][i] = -w_i / c from pass 0)
    __shared__ float red[4];
    const BorderJob J = jobs[blockIdx.x];
    const float *u = J.src + (long long)J.n * J.lds;
    const float *xr = J.X + (long long)J.n * J.ldx;
    float acc = 0.f;
    for (int i = threadIdx.x; i < J.n; i += 256) acc = fmaf(u[i], xr[i], acc);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) red[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float c = u[J.n] + ((J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f);
        const float q = (red[0] + red[1]) + (red[2] + red[3]);
        J.X[(long long)J.n * J.ldx + J.n] = (1.f - q) / c;
        if (!(c > 0.f) && info && J.info_idx >= 0) atomicCAS(&info[J.info_idx], 0, J.n + 1);
    }
}

hipError_t launch_border(const BorderJob *jobs_dev, int n_jobs, int total_wgs, int pass, const float *damp_dev,
                         int32_t *info, hipStream_t s)
{
    if (n_jobs <= 0) return hipSuccess;
    border_kernel<<<dim3(pass == 0 ? total_wgs : n_jobs), dim3(256), 0, s>>>(jobs_dev, n_jobs, pass, damp_dev, info);
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

// ------------------------------------------------------------------ blocked leaf inverse on the matrix cores
// (X + damp I)^-1 for n <= 288 by one 1024-thread workgroup, as a symmetric block sweep with
// 32x32 blocks.  The matrix is first scaled to unit diagonal (s_i = 1/sqrt(x_ii), undone at
// the end), which makes every pivot of the elimination lie in (0, 1].  The workgroup holds
// N = -(scaled matrix), lower-triangle 32x32 tiles only, each tile in the accumulator layout of
// v_mfma_f32_32x32x2_f32 in the registers of one wavefront (tile t -> wavefront t % 16).
// Sweeping block k (all i, j != k; D = (-N_kk)^-1; the column panel R_i = N_ik, taken from
// tile (i,k) for i > k and from the transpose of tile (k,i) for i < k):
//     P_i   = R_i D             ->  new N_ik (and N_ki = P_i^T)
//     N_ij += P_i R_j^T         (symmetric: tiles i >= j only)
//     N_kk  = D
// After all blocks N = X^-1 (the usual sweep operator, written for -X so that every update
// is an accumulation).  R and P go through LDS; the products are MFMA.
// D comes from a scalar sweep of the 32x32 diagonal tile inside its owner wavefront, also on
// the matrix core: pivot p is the rank-1 update S += a b^T with b = row p (one accumulator
// register across the lanes) and a = -row p / d (the tile is symmetric), patched so that the
// same update leaves row and column p divided by d (a_p = 1/d - 1, b_p = d - 1; no cancellation
// because d <= 1); two pivots share one 32x32x2 instruction.  A non-positive pivot is reported.
typedef float lb_floatx16 __attribute__((ext_vector_type(16)));
typedef float lb_floatx4 __attribute__((ext_vector_type(4)));
constexpr int LB_MAXN = 288;

__device__ __forceinline__ float lb_readlane(float x, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}

// The panels live in LDS as three bf16 planes per value (x = h + m + l exactly, see split_pair): rows of
// LB_LQ bf16 (32 + 8 pad: 80-byte rows, conflict-free 16-byte fragment reads), plane stride given.
typedef __bf16 lb_bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short lb_ushortx8 __attribute__((ext_vector_type(8)));
constexpr int LB_LQ = 40;
constexpr int LB_PLANE = LB_MAXN * LB_LQ;     // plane stride of the R and P panels (bf16 elements)
constexpr int LB_DPLANE = 32 * LB_LQ;         // of D

// acc += A B^T for two 32 x 32 blocks given as plane rows: `pa`, `pb` point at the h plane of the lane's
// row (lane % 32) plus 8 * (lane / 32), the half-wave's part of each 16-wide k step.  Six bf16 matrix
// instructions per step form the product to fp32 accuracy: h h' + h m' + h l' + m h' + m m' + l h'.
__device__ __forceinline__ void lb_mma_planes(lb_floatx16 &acc, const unsigned short *pa, int plane_a,
                                              const unsigned short *pb, int plane_b)
{
    auto rd = [](const unsigned short *p) { return __builtin_bit_cast(lb_bf16x8, *(const lb_ushortx8 *)p); };
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const lb_bf16x8 ah = rd(pa + 16 * u), am = rd(pa + plane_a + 16 * u), al = rd(pa + 2 * plane_a + 16 * u);
        const lb_bf16x8 bh = rd(pb + 16 * u), bm = rd(pb + plane_b + 16 * u), bl = rd(pb + 2 * plane_b + 16 * u);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
    }
}

// A 32 x 32 tile held in the accumulator layout (register v: row 8 (v / 4) + 4 h + v % 4, lane % 32: column)
// into plane rows, split on the way.
//   lb_store_rows: tile element (row, column) goes to panel row row0 + row, position column  (2-byte stores)
//   lb_store_cols: ... to panel row row0 + column, position row: the transposed tile; the four rows of a
//                  register group are four adjacent positions, one 8-byte store per plane
__device__ __forceinline__ void lb_store_rows(unsigned short *panel, int plane, int row0, const lb_floatx16 &t, int l32, int h)
{
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
        unsigned hh, mm, ll;
        split_pair(t[v], t[v + 1], hh, mm, ll);
        unsigned short *d = panel + (row0 + 8 * (v >> 2) + 4 * h + (v & 3)) * LB_LQ + l32;
        d[0] = (unsigned short)hh; d[LB_LQ] = (unsigned short)(hh >> 16);
        d[plane] = (unsigned short)mm; d[plane + LB_LQ] = (unsigned short)(mm >> 16);
        d[2 * plane] = (unsigned short)ll; d[2 * plane + LB_LQ] = (unsigned short)(ll >> 16);
    }
}
__device__ __forceinline__ void lb_store_cols(unsigned short *panel, int plane, int row0, const lb_floatx16 &t, int l32, int h)
{
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint2 hh, mm, ll;
        split_pair(t[4 * g], t[4 * g + 1], hh.x, mm.x, ll.x);
        split_pair(t[4 * g + 2], t[4 * g + 3], hh.y, mm.y, ll.y);
        unsigned short *d = panel + (row0 + l32) * LB_LQ + 8 * g + 4 * h;
        *(uint2 *)d = hh;
        *(uint2 *)(d + plane) = mm;
        *(uint2 *)(d + 2 * plane) = ll;
    }
}

// Scalar sweep of the 32x32 diagonal tile of block k inside the wavefront that holds it
// (register slot `slot`): leaves D = (-N_kk)^-1 in the slot and in Dq.  Returns the 1-based
// index (within the matrix) of the first non-positive pivot, or 0.
template <int NSLOT>
__device__ __forceinline__ int lb_sweep_diag(lb_floatx16 (&acc)[NSLOT], int slot, int k, int l32, int h, unsigned short *Dq)
{
    lb_floatx16 sg;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        float x = acc[0][v];
#pragma unroll
        for (int s = 1; s < NSLOT; ++s) x = (slot == s) ? acc[s][v] : x;
        sg[v] = -x;
    }
    // Pivot p is the rank-1 update S += a b^T with
    //     a_i = -x_i / d (i != p),  a_p = 1/d - 1;    b_j = x_j (j != p),  b_p = d - 1
    // where x = row p and d = x_p: besides S_ij -= x_i x_j / d this leaves row and column p multiplied by
    // 1/d (sums of equal-signed terms, because d <= 1) and S_pp = 2 - 1/d instead of -1/d.  No later pivot
    // reads S_pp (pivot q reads row q only, and adds to S_pp), so the 2 is taken off once, at the end.
    // A wavefront cannot issue its vector arithmetic beside its own matrix instruction, so the pivots go
    // two per instruction: the rows of pivots p and p + 1 (p even: both in the same half-wave) are brought up
    // to date with fmas, row p + 1 by pivot p, and the two updates ride in the two k slots of one
    // 32x32x2 instruction (one half-wave each; v_permlane32_swap puts the second pair of vectors there).  The
    // row of pivot p + 2 is read from the tile as the previous instruction left it and corrected by both.
    int badl = 0;
    float xcur = sg[0];                 // row 0, valid in the half-wave that holds it
#pragma unroll
    for (int p = 0; p < 32; p += 2) {
        const int hp = (p >> 2) & 1;    // half-wave holding rows p and p + 1
        // pivot p
        const float d0 = lb_readlane(xcur, p + 32 * hp);
        badl = (badl == 0 && !(d0 > 0.f)) ? 32 * k + p + 1 : badl;
        const float r0 = __builtin_amdgcn_rcpf(d0);
        const float xr0 = xcur * r0;
        float b0 = l32 == p ? d0 - 1.f : xcur;
        float a0 = l32 == p ? r0 - 1.f : -xr0;
        // row p + 1 after pivot p, then pivot p + 1
        const int v1 = 4 * ((p + 1) >> 3) + ((p + 1) & 3);
        const float x1 = fmaf(-lb_readlane(xr0, p + 1 + 32 * hp), b0, sg[v1]);
        const float d1 = lb_readlane(x1, p + 1 + 32 * hp);
        badl = (badl == 0 && !(d1 > 0.f)) ? 32 * k + p + 2 : badl;
        const float r1 = __builtin_amdgcn_rcpf(d1);
        const float xr1 = x1 * r1;
        float b1 = l32 == p + 1 ? d1 - 1.f : x1;
        float a1 = l32 == p + 1 ? r1 - 1.f : -xr1;
        float xnext = 0.f;
        if (p + 2 < 32) {
            const int hn = ((p + 2) >> 2) & 1;
            const int v2 = 4 * ((p + 2) >> 3) + ((p + 2) & 3);
            const float al0 = lb_readlane(xr0, p + 2 + 32 * hp), al1 = lb_readlane(xr1, p + 2 + 32 * hp);
            float c0 = b0, c1 = b1;
            if (hn != hp) {             // row p + 2 lives in the other half-wave: the two b vectors go there
                const auto s0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(b0), __float_as_uint(b0), false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(b1), __float_as_uint(b1), false, false);
                c0 = __uint_as_float(hp == 0 ? s0[0] : s0[1]);
                c1 = __uint_as_float(hp == 0 ? s1[0] : s1[1]);
            }
            xnext = fmaf(-al1, c1, fmaf(-al0, c0, sg[v2]));
        }
        // operands: the half-wave that holds the rows keeps pivot p, the other one receives pivot p + 1
        // (swap(x, y) exchanges the upper half of x with the lower half of y)
        float a, b;
        if (hp == 0) {
            const auto sa = __builtin_amdgcn_permlane32_swap(__float_as_uint(a0), __float_as_uint(a1), false, false);
            const auto sb = __builtin_amdgcn_permlane32_swap(__float_as_uint(b0), __float_as_uint(b1), false, false);
            a = __uint_as_float(sa[0]); b = __uint_as_float(sb[0]);
        } else {
            const auto sa = __builtin_amdgcn_permlane32_swap(__float_as_uint(a1), __float_as_uint(a0), false, false);
            const auto sb = __builtin_amdgcn_permlane32_swap(__float_as_uint(b1), __float_as_uint(b0), false, false);
            a = __uint_as_float(sa[1]); b = __uint_as_float(sb[1]);
        }
        sg = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, sg, 0, 0, 0);
        xcur = xnext;
    }
    // sg = -(that tile)^-1 + 2 I = 2 I - D;  D is symmetric, so its planes can be written transposed (8-byte stores)
    const int drow = l32 - 4 * h;       // register v holds the diagonal element of its lane where this is 8 (v / 4) + v % 4
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        sg[v] = (drow == 8 * (v >> 2) + (v & 3) ? 2.f : 0.f) - sg[v];
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) acc[s][v] = (slot == s) ? sg[v] : acc[s][v];
    }
    lb_store_cols(Dq, LB_DPLANE, 0, sg, l32, h);
    return badl;
}

// Which wavefront holds which tile.  In step k the tiles of block row / column k only form the
// panel P, the other 36 (of 45, for 9 blocks) take 12 matrix instructions each, and the wavefront
// that holds the diagonal tile of block k + 1 updates and then sweeps it, which is the longest
// chain of the step.  The table below (found by annealing over assignments with at most 3 tiles per
// wavefront) gives every diagonal tile a wavefront of its own, lets the owner of diagonal tile b
// hold nothing else but tiles of block row / column b - 1 (idle while it sweeps), puts at most two
// panel tiles of a step on one wavefront and spreads the rest evenly over the four SIMDs (wavefront
// % 4).  Other sizes keep the plain order (tile t to wavefront t % 16).
__constant__ signed char kLeafTile9[16][3] = {{20, 25, -1}, {2, 3, 10}, {15, 23, 28}, {6, 14, 39}, {32, 43, 44}, {19, 29, 42},
                                              {4, 9, 12}, {11, 17, 21}, {27, 41, -1}, {0, 8, 36}, {5, 7, 37}, {22, 30, 38},
                                              {26, 35, -1}, {16, 24, 31}, {18, 34, 40}, {1, 13, 33}};
__constant__ signed char kLeafWave9[45] = {9, 15, 1, 1, 6, 10, 3, 10, 9, 6, 1, 7, 6, 15, 3, 2, 13, 7, 14, 5, 0, 7, 11,
                                           2, 13, 0, 12, 8, 2, 5, 11, 13, 4, 15, 14, 12, 9, 10, 11, 3, 14, 8, 5, 4, 4};
__constant__ signed char kLeafSlot9[45] = {0, 0, 0, 1, 0, 0, 0, 1, 1, 1, 2, 0, 2, 1, 1, 0, 0, 1, 0, 0, 0, 2, 0,
                                           1, 1, 1, 0, 0, 2, 1, 1, 2, 0, 2, 1, 1, 2, 2, 2, 2, 2, 1, 2, 1, 2};

template <int NSLOT>
__global__ __launch_bounds__(1024) void leaf_block_kernel(const LeafJob *__restrict__ jobs,
                                                          const float *__restrict__ damp,
                                                          int32_t *__restrict__ info)
{
    extern __shared__ __attribute__((aligned(16))) float lb_lds[];
    unsigned short *Rq = (unsigned short *)lb_lds;   // [3][LB_MAXN][LB_LQ] column panel R, three bf16 planes
    unsigned short *Pq = Rq + 3 * LB_PLANE;          // [3][LB_MAXN][LB_LQ] P = R D
    unsigned short *Dq = Pq + 3 * LB_PLANE;          // [3][32][LB_LQ]      D
    float *sc = (float *)(Dq + 3 * LB_DPLANE);       // [LB_MAXN]           diagonal scaling
    __shared__ int bad_s;

    const LeafJob J = jobs[blockIdx.x];
    const int n = J.n;
    const int T = (n + 31) >> 5;
    const int ntiles = T * (T + 1) / 2;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int l32_ = lane & 31, h_ = lane >> 5;
    const float d = (J.damp_idx >= 0) ? damp[J.damp_idx] : 0.f;
    const unsigned lds = (unsigned)J.lds, ldd = (unsigned)J.ldd;

    // my tiles: tile t is block (ti, tj), ti >= tj, in row-major order of the lower triangle; slot s
    // of wavefront w holds tile w + 16 s, or what the balanced table says for 9 blocks.
    // The raw loads are issued first; the scaling needs the diagonal (through LDS) and comes after.
    const bool balanced = NSLOT == 3 && T == 9;
    auto diag_owner = [&](int b) { const int t = b * (b + 1) / 2 + b; return balanced ? (int)kLeafWave9[t] : (t & 15); };
    auto diag_slot = [&](int b) { const int t = b * (b + 1) / 2 + b; return balanced ? (int)kLeafSlot9[t] : (t >> 4); };
    lb_floatx16 acc[NSLOT];
    int ti[NSLOT], tj[NSLOT];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        int t = w + 16 * s;
        if (balanced) { t = kLeafTile9[w][s < 3 ? s : 0]; t = t < 0 ? ntiles : t; }
        int r = 0;
        while ((r + 1) * (r + 2) / 2 <= t) ++r;
        ti[s] = t < ntiles ? r : -1;
        tj[s] = t - r * (r + 1) / 2;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 32 * r + 8 * (v >> 2) + 4 * h_ + (v & 3), j = 32 * tj[s] + l32_;
            float x = 0.f;
            if (t < ntiles && i < n && j < n) x = J.src[(unsigned)i * lds + (unsigned)j];
            acc[s][v] = x;
        }
    }
    if (tid < 32 * T) {
        float v = 1.f;
        if (tid < n) {
            const float a = J.src[(unsigned)tid * lds + (unsigned)tid] + d;
            v = a > 0.f ? rsqrtf(a) : 1.f;   // a non-positive diagonal shows up as a non-positive pivot
        }
        sc[tid] = v;
    }
    if (tid == 0) bad_s = 0;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 32 * ti[s] + 8 * (v >> 2) + 4 * h_ + (v & 3), j = 32 * tj[s] + l32_;
            float x = acc[s][v];
            if (ti[s] >= 0 && i < n && j < n) x = -(x + (i == j ? d : 0.f)) * sc[i] * sc[j];
            else x = (i == j) ? -1.f : 0.f;     // identity padding (of -X)
            acc[s][v] = x;
        }
    }

    // The diagonal tile of block k + 1 is swept by its owner during the trailing update of
    // block k (right after the owner has brought that tile up to date), so that the serial
    // sweep runs beside the other wavefronts' products instead of in front of them.
    if (w == diag_owner(0)) {
        int l32 = l32_, h = h_;
        asm volatile("" : "+v"(l32), "+v"(h));
        const int badl = lb_sweep_diag<NSLOT>(acc, diag_slot(0), 0, l32, h, Dq);
        if (badl != 0 && lane == 0) bad_s = badl;
    }
    __syncthreads();   // D of block 0 is in LDS
    for (int k = 0; k < T; ++k) {
        // (per-step copies of the lane coordinates: as loop invariants, the 32 lane masks of the
        // sweep and the LDS addresses below would be hoisted and kept live across the whole loop)
        int l32 = l32_, h = h_;
        asm volatile("" : "+v"(l32), "+v"(h));
        // ---- column panel R of block k into LDS (planes): R_i = N_ik, from tile (i,k) for i > k and from
        // the transpose of tile (k,i) for i < k
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            if (ti[s] < 0) continue;
            if (tj[s] == k && ti[s] > k) lb_store_rows(Rq, LB_PLANE, 32 * ti[s], acc[s], l32, h);
            else if (ti[s] == k && tj[s] < k) lb_store_cols(Rq, LB_PLANE, 32 * tj[s], acc[s], l32, h);
        }
        // A wavefront forms P from the panel rows it has just written itself and from D (in LDS since the
        // barrier that ended the previous step or the prologue): its own LDS accesses stay in order, so no
        // workgroup barrier is needed here, only the guarantee that they are not reordered.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---- the tiles of block row / column k take their new value P_i = R_i D (tile (i,k)) or its transpose
        // D R_i^T (tile (k,i)) straight from the product, and put P into LDS for everybody else
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            if (ti[s] < 0) continue;
            if (tj[s] == k && ti[s] > k) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
                lb_mma_planes(acc[s], Rq + (32 * ti[s] + l32) * LB_LQ + 8 * h, LB_PLANE, Dq + l32 * LB_LQ + 8 * h, LB_DPLANE);
                lb_store_rows(Pq, LB_PLANE, 32 * ti[s], acc[s], l32, h);
            } else if (ti[s] == k && tj[s] < k) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
                lb_mma_planes(acc[s], Dq + l32 * LB_LQ + 8 * h, LB_DPLANE, Rq + (32 * tj[s] + l32) * LB_LQ + 8 * h, LB_PLANE);
                lb_store_cols(Pq, LB_PLANE, 32 * tj[s], acc[s], l32, h);
            }
        }
        __syncthreads();   // P is in LDS; D of block k is no longer needed
        // ---- every other tile N_ij += P_i R_j^T
        const bool sweeps_next = k + 1 < T && w == diag_owner(k + 1);   // holds the diagonal tile of block k + 1
        if (sweeps_next) {
            const int slot = diag_slot(k + 1);
            // the update of that tile and its sweep are one long dependent chain and bound the step: they issue
            // ahead of the other wavefronts' products, which also leave the first LDS reads to this wavefront
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int s = 0; s < NSLOT; ++s)
                if (s == slot)
                    lb_mma_planes(acc[s], Pq + (32 * (k + 1) + l32) * LB_LQ + 8 * h, LB_PLANE,
                                  Rq + (32 * (k + 1) + l32) * LB_LQ + 8 * h, LB_PLANE);
            const int badl = lb_sweep_diag<NSLOT>(acc, slot, k + 1, l32, h, Dq);
            __builtin_amdgcn_s_setprio(0);
            if (badl != 0 && lane == 0 && bad_s == 0) bad_s = badl;   // blocks are swept in order: the first one stays
        } else if (k + 1 < T) {
            __builtin_amdgcn_s_sleep(3);
        }
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            if (ti[s] < 0) continue;
            const int i = ti[s], j = tj[s];
            if (i == k || j == k) continue;
            if (sweeps_next && i == k + 1 && j == k + 1) continue;
            lb_mma_planes(acc[s], Pq + (32 * i + l32) * LB_LQ + 8 * h, LB_PLANE, Rq + (32 * j + l32) * LB_LQ + 8 * h, LB_PLANE);
        }
        __syncthreads();
    }
    if (tid == 0 && bad_s != 0 && info && J.info_idx >= 0) atomicCAS(&info[J.info_idx], 0, J.pivot_base + bad_s);

    // undo the scaling; the lower triangle is written and mirrored, so the result is exactly
    // symmetric.  The mirror image goes through a per-wavefront 32x33 LDS tile (the panels are
    // dead by now) so that it is written along rows as well.
    float *stage = lb_lds + w * (32 * 33);
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        if (ti[s] < 0) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * h_ + (v & 3);
            const int i = 32 * ti[s] + r, j = 32 * tj[s] + l32_;
            float x = 0.f;
            if (i < n && j < n) x = acc[s][v] * sc[i] * sc[j];
            if (i < n && j <= i) J.dst[(unsigned)i * ldd + (unsigned)j] = x;
            stage[l32_ * 33 + r] = x;          // transposed
        }
        // rows of the transposed tile: element (r, c) is X[32 ti + c][32 tj + r], goes to dst[32 tj + r][32 ti + c]
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * h_ + (v & 3);
            const int i = 32 * ti[s] + l32_, j = 32 * tj[s] + r;
            if (i < n && j < i) J.dst[(unsigned)j * ldd + (unsigned)i] = stage[r * 33 + l32_];
        }
    }
}

template <int NSLOT>
static hipError_t launch_leaf_block(const LeafJob *jobs_dev, int n_jobs, const float *damp_dev, int32_t *info,
                                    hipStream_t s)
{
    constexpr size_t lds_bytes = (size_t)(6 * LB_PLANE + 3 * LB_DPLANE) * sizeof(unsigned short) + LB_MAXN * sizeof(float);
    static_assert(lds_bytes >= (size_t)16 * 32 * 33 * sizeof(float), "the per-wavefront staging tiles of the final store fit");
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)leaf_block_kernel<NSLOT>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    leaf_block_kernel<NSLOT><<<dim3(n_jobs), dim3(1024), lds_bytes, s>>>(jobs_dev, damp_dev, info);
    return hipGetLastError();
}

hipError_t launch_leaf(const LeafJob *jobs_dev, int n_jobs, int size_class, const float *damp_dev,
                       int32_t *info, hipStream_t s)
{
    if (n_jobs <= 0) return hipSuccess;
    switch (kLeafClasses[size_class]) {   // class value = n_max / 32: 16, 32 or 48 tile slots
        case 5: return launch_leaf_block<1>(jobs_dev, n_jobs, damp_dev, info, s);
        case 7: return launch_leaf_block<2>(jobs_dev, n_jobs, damp_dev, info, s);
        case 9: return launch_leaf_block<3>(jobs_dev, n_jobs, damp_dev, info, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kfac
