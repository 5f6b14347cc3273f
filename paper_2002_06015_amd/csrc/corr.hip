// The A factor of a 3x3 / stride 1 / pad 1 convolution without the patch matrix (Sec. 3.3,
// Eq. 10 and 11 define A = 1/(N hw) sum_n M_A M_A^T with M_A = im2col).  Entry
// ((c,ky,kx), (c',ky',kx')) of the sum is
//     sum_n sum_{(y,x)} a_c(n, y+ky-1, x+kx-1) a_c'(n, y+ky'-1, x+kx'-1)     (a = 0 outside)
// and, with u = (y+ky-1, x+kx-1) and D = (ky'-ky, kx'-kx), equals the full spatial
// cross-correlation  C_D[c,c'] = sum_n sum_u a_c(n,u) a_c'(n,u+D)  except that
//     ky = ky' = 2 leaves out the image row u_y = 0,   ky = ky' = 0 the row u_y = H-1,
//     kx = kx' = 2 leaves out the column u_x = 0,      kx = kx' = 0 the column u_x = W-1
// (every other bound on u coincides with u and u+D lying in the image).  So instead of the
// 81 C^2 products of the patch Gram matrix, 13 displacements D (the other 12 are transposes)
// are contracted over the image, plus corrections from the four border lines (1-D
// correlations) and the four corners (inclusion-exclusion), all by the grouped GEMM kernel:
//   - pad_kernel rewrites the activations as planes of Hp x Wp with (at least) two zero rows on
//     top and two zero columns on the left of each plane.  Because the planes follow each
//     other in memory, every position just outside an image (up to 2 away) is a zero of the
//     same or the next plane, and a(n, u+D) is simply the element dy*Wp+dx further on: a
//     shifted operand is the same buffer with an offset base pointer, no masks.
//     It also extracts the border lines [C][N][L+pad] and corners [C][N] for the corrections.
//   - assemble_kernel combines the 13 + 12 + 4 small Gram matrices into A (with the running
//     average and the bias border, whose sums come from the GEMM_BORDER row sums).
#include "kfac_internal.h"

namespace kfac {

typedef float corr_floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void pad_kernel(const PadJob *__restrict__ jobs, int n_jobs)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const PadJob &J = jobs[lo];
    const long long idx = (long long)(wg - J.wg_start) * 256 + threadIdx.x;
    const int H = J.H, W = J.W, Wp = J.Wp, PP = J.Hp * Wp, y0 = J.Hp - H, x0 = Wp - W;
    const long long planes = (long long)J.N * J.C;
    // part 1: the padded tensor including its zero slack in front and behind, 4 elements per thread
    const long long n4 = J.padded_floats / 4;
    if (idx < n4) {
        // coordinates of the first of the four positions by division (32-bit where the tensor allows), the others by stepping
        const long long g0 = idx * 4 - J.front_slack, total = planes * PP;
        long long plane = 0;
        int yp = 0, xp = 0;
        if (g0 > 0 && g0 < total) {
            int r;
            if (total < (1LL << 31)) {
                const unsigned q = (unsigned)g0 / (unsigned)PP;
                plane = q;
                r = (int)((unsigned)g0 - q * (unsigned)PP);
            } else {
                plane = g0 / PP;
                r = (int)(g0 - plane * PP);
            }
            yp = r / Wp;
            xp = r - yp * Wp;
        }
        const float *sp = J.src + plane * H * W;
        corr_floatx4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long long g = g0 + e;
            float x = 0.f;
            if (g >= 0 && g < total) {
                if (yp >= y0 && xp >= x0) x = sp[(yp - y0) * W + (xp - x0)];
                if (++xp == Wp) {
                    xp = 0;
                    if (++yp == J.Hp) { yp = 0; sp += H * W; }
                }
            }
            v[e] = x;
        }
        *(corr_floatx4 *)(J.padded + idx * 4) = v;
        return;
    }
    // part 2: border rows (top, bottom) [2][C][N][Lw], border columns (left, right) [2][C][N][Lh],
    // corners [4][C][N]; every line is followed by at least two zeros
    long long k = idx - n4;
    const long long row_elems = (long long)J.C * J.N * J.Lw, col_elems = (long long)J.C * J.N * J.Lh;
    if (k < 2 * row_elems + 4) {
        float x = 0.f;
        if (k < 2 * row_elems) {
            const int which = (int)(k / row_elems);
            const long long r = k - which * row_elems;
            const int q = (int)(r % J.Lw);
            const long long cn = r / J.Lw;
            const int n = (int)(cn % J.N), c = (int)(cn / J.N);
            if (q < W) x = J.src[((long long)n * J.C + c) * H * W + (long long)(which ? H - 1 : 0) * W + q];
        }
        J.rows[k] = x;
        return;
    }
    k -= 2 * row_elems + 4;
    if (k < 2 * col_elems + 4) {
        float x = 0.f;
        if (k < 2 * col_elems) {
            const int which = (int)(k / col_elems);
            const long long r = k - which * col_elems;
            const int p = (int)(r % J.Lh);
            const long long cn = r / J.Lh;
            const int n = (int)(cn % J.N), c = (int)(cn / J.N);
            if (p < H) x = J.src[((long long)n * J.C + c) * H * W + (long long)p * W + (which ? W - 1 : 0)];
        }
        J.cols[k] = x;
        return;
    }
    k -= 2 * col_elems + 4;
    if (k < 4LL * J.C * J.N) {
        const int which = (int)(k / ((long long)J.C * J.N));
        const long long r = k - (long long)which * J.C * J.N;
        const int n = (int)(r % J.N), c = (int)(r / J.N);
        const int p = (which & 2) ? H - 1 : 0, q = (which & 1) ? W - 1 : 0;
        J.corners[k] = J.src[((long long)n * J.C + c) * H * W + (long long)p * W + q];
    }
}

hipError_t launch_pad(const PadJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    pad_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

// bf16 activations: see PadJobBF16.  8 elements (16 bytes) per thread.
typedef unsigned short corr_ushortx8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void pad_bf16_kernel(const PadJobBF16 *__restrict__ jobs, int n_jobs)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const PadJobBF16 &J = jobs[lo];
    long long idx = (long long)(wg - J.wg_start) * 256 + threadIdx.x;
    const int H = J.H, W = J.W, Wp = J.Wp, PP = J.Hp * Wp, y0 = J.Hp - H, x0 = Wp - W;
    const long long planes = (long long)J.N * J.C;
    // part 1: the five shifted copies of the padded tensor.  One thread per aligned group of 8 positions:
    // it gathers the 12 values P(g0 - 2 .. g0 + 9) once (coordinates by one division, then stepped) and
    // writes the group of every copy from that window.
    const long long per_copy = J.copy_elems / 8;
    if (idx < per_copy) {
        const long long g0 = idx * 8 - J.front_slack - 2;
        const long long total = planes * PP;
        long long plane = 0;
        int yp = 0, xp = 0;
        if (g0 > 0 && g0 < total) {
            plane = g0 / PP;
            const int r = (int)(g0 - plane * PP);
            yp = r / Wp;
            xp = r - yp * Wp;
        }
        const unsigned short *sp = J.src + plane * H * W;
        unsigned short win[12];
#pragma unroll
        for (int e = 0; e < 12; ++e) {
            const long long g = g0 + e;
            unsigned short x = 0;
            if (g >= 0 && g < total) {
                if (g0 <= 0) {   // the window starts in the front slack: position g is (plane 0, g / Wp, g % Wp)
                    yp = (int)(g / Wp);
                    xp = (int)(g - (long long)yp * Wp);
                }
                if (yp >= y0 && xp >= x0) x = sp[(yp - y0) * W + (xp - x0)];
                if (++xp == Wp) {
                    xp = 0;
                    if (++yp == J.Hp) { yp = 0; sp += H * W; }
                }
            }
            win[e] = x;
        }
#pragma unroll
        for (int q = 0; q < 5; ++q) {
            corr_ushortx8 v;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = win[q + e];
            *(corr_ushortx8 *)(J.padded + (long long)q * J.copy_elems + idx * 8) = v;
        }
        return;
    }
    idx -= per_copy;
    // part 2: border rows, three copies shifted by 0, 1, 2 (one element per thread from here on)
    if (idx < 3 * J.rows_elems) {
        const int d = (int)(idx / J.rows_elems);
        const long long k = idx - d * J.rows_elems + d;      // copy d at position p holds the line buffer at p + d
        const long long row_elems = (long long)J.C * J.N * J.Lw;
        unsigned short x = 0;
        if (k < 2 * row_elems) {
            const int which = (int)(k / row_elems);
            const long long r = k - which * row_elems;
            const int qx = (int)(r % J.Lw);
            const long long cn = r / J.Lw;
            const int n = (int)(cn % J.N), c = (int)(cn / J.N);
            if (qx < W) x = J.src[((long long)n * J.C + c) * H * W + (long long)(which ? H - 1 : 0) * W + qx];
        }
        J.rows[idx] = x;
        return;
    }
    idx -= 3 * J.rows_elems;
    if (idx < 3 * J.cols_elems) {
        const int d = (int)(idx / J.cols_elems);
        const long long k = idx - d * J.cols_elems + d;
        const long long col_elems = (long long)J.C * J.N * J.Lh;
        unsigned short x = 0;
        if (k < 2 * col_elems) {
            const int which = (int)(k / col_elems);
            const long long r = k - which * col_elems;
            const int py = (int)(r % J.Lh);
            const long long cn = r / J.Lh;
            const int n = (int)(cn % J.N), c = (int)(cn / J.N);
            if (py < H) x = J.src[((long long)n * J.C + c) * H * W + (long long)py * W + (which ? W - 1 : 0)];
        }
        J.cols[idx] = x;
        return;
    }
    idx -= 3 * J.cols_elems;
    if (idx < 4LL * J.C * J.Ln) {
        const int which = (int)(idx / ((long long)J.C * J.Ln));
        const long long r = idx - (long long)which * J.C * J.Ln;
        const int n = (int)(r % J.Ln), c = (int)(r / J.Ln);
        const int py = (which & 2) ? H - 1 : 0, qx = (which & 1) ? W - 1 : 0;
        J.corners[idx] = n < J.N ? J.src[((long long)n * J.C + c) * H * W + (long long)py * W + qx] : (unsigned short)0;
    }
}

hipError_t launch_pad_bf16(const PadJobBF16 *jobs_dev, int n_jobs, int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    pad_bf16_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

// One workgroup per row i = (c, ky, kx) of A (plus one for the bias row), threads along the row.
// Which Gram matrices entry (c', ky', kx') comes from depends only on (ky, kx, ky', kx'): the
// workgroup first builds that table of 9 entries.  A displacement that is stored the other way
// round is read from the transposed copy the GEMM wrote alongside, so every read is along a
// row of a Gram matrix and every write along the row of A (the interleaving of the nine k'
// goes through LDS).
struct CorrSource {
    const float *full, *row, *col, *corner;   // row / col / corner: null if no such correction
    int ld_full, ld_row, ld_col;
};

__device__ __forceinline__ CorrSource corr_source(const AssembleJob &J, int ky, int kx, int kyp, int kxp)
{
    CorrSource S{};
    const int dy = kyp - ky, dx = kxp - kx;
    const bool fwd = dy > 0 || (dy == 0 && dx >= 0);
    const int ey = fwd ? dy : -dy, ex = fwd ? dx : -dx;
    const int slot = ey == 0 ? ex : 3 + (ey - 1) * 5 + (ex + 2);
    S.full = fwd ? J.full[slot] : J.full_t[slot];
    S.ld_full = J.ld_full[slot];
    const int row_out = (ky == kyp) ? (ky == 2 ? 0 : (ky == 0 ? 1 : -1)) : -1;   // 0: top row left out, 1: bottom
    const int col_out = (kx == kxp) ? (kx == 2 ? 0 : (kx == 0 ? 1 : -1)) : -1;   // 0: left column, 1: right
    if (row_out >= 0) {
        const int d = dx >= 0 ? dx : -dx;
        S.row = dx >= 0 ? J.rows[row_out][d] : J.rows_t[row_out][d];
        S.ld_row = J.ld_rows[row_out][d];
    }
    if (col_out >= 0) {
        const int d = dy >= 0 ? dy : -dy;
        S.col = dy >= 0 ? J.cols[col_out][d] : J.cols_t[col_out][d];
        S.ld_col = J.ld_cols[col_out][d];
    }
    if (row_out >= 0 && col_out >= 0) S.corner = J.corners[2 * row_out + col_out];
    return S;
}

// sum of the patch row (c, ky, kx) over all positions: the bias border
__device__ __forceinline__ float corr_row_sum(const AssembleJob &J, int c, int ky, int kx)
{
    const int row_out = ky == 2 ? 0 : (ky == 0 ? 1 : -1), col_out = kx == 2 ? 0 : (kx == 0 ? 1 : -1);
    float v = J.full[0][(long long)c * J.ld_full[0] + J.C];
    if (row_out >= 0) v -= J.rows[row_out][0][(long long)c * J.ld_rows[row_out][0] + J.C];
    if (col_out >= 0) v -= J.cols[col_out][0][(long long)c * J.ld_cols[col_out][0] + J.C];
    if (row_out >= 0 && col_out >= 0) v += J.corners[2 * row_out + col_out][(long long)c * J.ld_corner + J.C];
    return v;
}

__device__ __forceinline__ void corr_store(const AssembleJob &J, float *out, float v)
{
    float r = J.alpha * v;
    if (J.beta != 0.f) r = fmaf(J.beta, *out, r);
    *out = r;
}

__global__ __launch_bounds__(256) void assemble_kernel(const AssembleJob *__restrict__ jobs, int n_jobs)
{
    const int wg = blockIdx.x;
    int lo = 0, hi = n_jobs;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (jobs[mid].wg_start <= wg) lo = mid; else hi = mid;
    }
    const AssembleJob &J = jobs[lo];
    const int d0 = 9 * J.C;
    const int i = wg - J.wg_start;          // row of A
    float *out_row = J.A + (long long)i * J.ldA;
    if (i < d0) {
        const int c = i / 9, k = i - 9 * c, ky = k / 3, kx = k - 3 * ky;
        typedef float v4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, element alignment
        __shared__ CorrSource src[9];
        __shared__ float vals[9][257];   // 256 channels c' at a time: [k'][c']
        if (threadIdx.x < 9) src[threadIdx.x] = corr_source(J, ky, kx, threadIdx.x / 3, threadIdx.x % 3);
        __syncthreads();
        // Reads go along rows of the Gram matrices (consecutive threads, consecutive c'), writes along
        // the row of A (consecutive threads, consecutive (c', k')); LDS does the interleaving.
        for (int cp0 = 0; cp0 < J.C; cp0 += 256) {
            const int cp = cp0 + threadIdx.x;
            if (cp < J.C) {
#pragma unroll
                for (int kp = 0; kp < 9; ++kp) {
                    const CorrSource S = src[kp];
                    float v = S.full[(long long)c * S.ld_full + cp];
                    if (S.row) v -= S.row[(long long)c * S.ld_row + cp];
                    if (S.col) v -= S.col[(long long)c * S.ld_col + cp];
                    if (S.corner) v += S.corner[(long long)c * J.ld_corner + cp];
                    vals[kp][threadIdx.x] = v;
                }
            }
            __syncthreads();
            const int nout = 9 * min(256, J.C - cp0);
            float *dst = out_row + 9 * cp0;
            for (int e = 4 * threadIdx.x; e < nout; e += 1024) {
                if (e + 3 < nout) {
                    v4 r;
#pragma unroll
                    for (int q = 0; q < 4; ++q) r[q] = J.alpha * vals[(e + q) % 9][(e + q) / 9];
                    if (J.beta != 0.f) {
                        const v4 o = *(const v4 *)(dst + e);
#pragma unroll
                        for (int q = 0; q < 4; ++q) r[q] = fmaf(J.beta, o[q], r[q]);
                    }
                    *(v4 *)(dst + e) = r;
                } else {
                    for (int q = 0; e + q < nout; ++q) corr_store(J, dst + e + q, vals[(e + q) % 9][(e + q) / 9]);
                }
            }
            __syncthreads();
        }
        if (J.bias && threadIdx.x == 0) corr_store(J, out_row + d0, corr_row_sum(J, c, ky, kx));
    } else {
        // the bias row
        for (int j = threadIdx.x; j <= d0; j += 256) {
            const int c = j / 9, k = j - 9 * c;
            corr_store(J, out_row + j, j < d0 ? corr_row_sum(J, c, k / 3, k % 3) : J.count);
        }
    }
}

hipError_t launch_assemble(const AssembleJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    assemble_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(jobs_dev, n_jobs);
    return hipGetLastError();
}

}  // namespace kfac
