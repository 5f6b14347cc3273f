// Internal device-table layouts and launch entry points shared by the host planner
// (kfac_api.hip) and the kernel files.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kfac {

// ---- grouped NT GEMM -------------------------------------------------------------
// One operand of C[i][j] = sum_m a(i, m) * b(j, m): a matrix whose rows run along the
// contraction index m.  Element (r, m) lives at
//     base + (m / hw) * batch_stride + r * row_stride + (m % hw)
// so an NCHW tensor [N, rows, hw] is contracted in place over (n, t) (batch_stride =
// rows*hw, row_stride = hw) and a plain row-major matrix is the case hw >= K.
// Rows >= rows read as 0.
// A thread loads 16-byte chunks along m: fp32 operands need hw % 4 == 0 (or a plain
// matrix, any leading dimension); bf16 operands need hw % 8 == 0 or a plain matrix, and
// base, row_stride and batch_stride that keep every chunk 16-byte aligned.
// bf16 runs of 8q + 4 elements (14 x 14 planes): tail = 4, hw is the run length rounded up to
// 8q + 8 and the contraction runs over N * hw positions, of which the last four of every run
// read as 0 (the last chunk of a run is loaded as two halves; 8-byte alignment is enough then).
struct Operand {
    const void *base;
    long long row_stride;
    long long batch_stride;
    int rows;
    int hw;
    int tail;   // 0, or 4 (bf16 only): valid elements in the last 8-element chunk of a run
    int trans;  // 1 (fp32 in the product mode of three bf16 planes, or bf16): the operand is stored with its rows as
                // the contiguous direction, element (r, m) at base + m * row_stride + r (an NHWC tensor [N*hw, rows]
                // contracted in place); a chunk is 16 bytes of adjacent rows at one m, rows a whole number of chunks
};

// GEMM_SYM:    M == N and the product is symmetric (a == b, or a b^T symmetric by construction as in the Schur
//              complements of the inversion); only tiles tm >= tn are computed and mirrored.
// GEMM_BORDER: (with GEMM_SYM) C is (M+1) x (M+1): the product of the operand extended by
//              an all-ones row (the bias row of the patch matrix, Sec. 3.3).  The border is
//              not multiplied out: C[i][M] = C[M][i] = alpha * sum_m a(i, m) + beta * old
//              comes from row sums taken while the diagonal tiles stage their operand,
//              and C[M][M] = alpha * ones + beta * old.
// GEMM_TRANS:  both operands are stored transposed (Operand::trans).
enum : int { GEMM_SYM = 1, GEMM_BORDER = 2, GEMM_TRANS = 4 };

struct GemmProblem {
    Operand a, b;
    float *C;        // [M, N], leading dimension ldc (may be null if only Ct is wanted)
    float *Ct;       // optional transposed copy Ct[j][i], leading dimension ldct (or null)
    float *partial;  // split-K scratch: [tiles][splits][BM*BN] (null if splits == 1)
    float *partial_rs;  // split-K scratch of the border row sums: [tiles_m][splits][BM] (GEMM_BORDER, splits > 1)
    long long ldc, ldct;
    int M, N, K;
    int ones;                 // GEMM_BORDER: the sum of the all-ones row with itself (K, unless the contraction includes padding)
    int tiles_m, tiles_n, n_tiles;
    int splits, k_per_split;  // k_per_split is a multiple of 32
    int flags;
    int tile_cfg;             // 0: 128x128 tiles, 1: 64x64 tiles
    float alpha, beta;        // C = alpha * acc + beta * C   (beta == 0: C is not read)
};

// ---- patch extraction ------------------------------------------------------------
struct PatchJob {
    const void *src;  // [N, c_in, h_in, w_in]
    void *dst;        // [c_in*k*k, ld]
    long long ld;
    int N, c_in, k, stride, pad, h_in, w_in, h, w;
    int esize;        // 4 (f32) or 2 (bf16)
    int flat;         // 1: k == 1, stride 1, no padding, tiny planes: one thread per output element
    unsigned magic_w; // floor(2^32 / w) + 1: t / w == mulhi(t, magic_w) for t, w < 2^16
    int wg_start;     // first workgroup of this job in the grouped launch
};

// ---- A factor of 3x3 convolutions through spatial correlations (corr.hip) -------------
struct PadJob {
    const float *src;        // [N, C, H, W]
    float *padded;           // start of the allocation: front slack, N*C planes of Hp*Wp, back slack
    long long padded_floats; // size of that allocation (multiple of 4)
    int front_slack;         // floats before the first plane (multiple of 4)
    float *rows;             // [2][C][N][Lw] top / bottom image row, then 4 zeros
    float *cols;             // [2][C][N][Lh] left / right image column, then 4 zeros
    float *corners;          // [4][C][N]: (top,left), (top,right), (bottom,left), (bottom,right)
    int N, C, H, W, Lw, Lh;
    int Hp, Wp;              // padded plane: Hp - H >= 2 zero rows on top, Wp - W >= 2 zero columns on the left
    int wg_start;
};

// The same for bf16 activations.  The bf16 GEMM loader reads 16-byte chunks at 16-byte aligned addresses,
// so a displaced operand cannot simply be an offset base pointer: the padded tensor is written five times,
// copy q (q = 0..4) shifted by dx = q - 2 elements, so that copy q read at an aligned position g gives the
// padded tensor at g + dx; a displacement (dy, dx) is then copy dx + 2 at offset dy * Wp with Wp a multiple
// of 8.  Likewise three copies (shift 0, 1, 2) of the border lines.
struct PadJobBF16 {
    const unsigned short *src;   // [N, C, H, W]
    unsigned short *padded;      // 5 copies of copy_elems each: front slack, N*C planes of Hp*Wp, back slack
    long long copy_elems;        // multiple of 8
    int front_slack;             // multiple of 8
    unsigned short *rows;        // 3 copies of rows_elems: [2][C][N][Lw] top / bottom image row, then zeros
    unsigned short *cols;        // 3 copies of cols_elems: [2][C][N][Lh] left / right image column, then zeros
    unsigned short *corners;     // [4][C][Ln]: the four corner pixels per sample, rows padded with zeros to Ln
    long long rows_elems, cols_elems;   // multiples of 8
    int N, C, H, W, Lw, Lh, Ln;
    int Hp, Wp;                  // Hp - H >= 2 zero rows on top, Wp - W >= 2 zero columns on the left, Wp % 8 == 0
    int wg_start;
};

struct AssembleJob {
    // Gram matrices of the contractions, [c][c'] with the leading dimensions given; those of
    // displacement 0 carry the GEMM_BORDER column (row sums) at index C
    // (the *_t pointers are the transposed copies, same leading dimensions; for displacement 0
    // they are the matrices themselves)
    const float *full[13];   // displacement (dy,dx): slot dx for dy = 0 (dx = 0..2), 3 + 5(dy-1) + dx+2 for dy = 1, 2
    const float *full_t[13];
    int ld_full[13];
    const float *rows[2][3]; // [top, bottom][dx = 0..2]
    const float *rows_t[2][3];
    int ld_rows[2][3];
    const float *cols[2][3]; // [left, right][dy = 0..2]
    const float *cols_t[2][3];
    int ld_cols[2][3];
    const float *corners[4]; // all with the border column
    int ld_corner;
    float *A;                // [9C + bias][ldA]
    long long ldA;
    int C, bias;
    float alpha, beta;       // A = alpha * sums + beta * A
    float count;             // N * h * w: the sum of the all-ones bias row with itself
    int wg_start;
};

// ---- inversion ---------------------------------------------------------------------
struct TraceJob {   // one per layer
    const float *A, *G;
    int dA, dG;
    int idx;        // layer index: damp[3*idx .. 3*idx+2] and pi_out[idx] are written
};

struct CopyJob {    // dst[i][j] = src[i][j] + (i == j) * damp[damp_idx]   (i, j < n)
    const float *src;
    float *dst;
    long long lds, ldd;
    int n;
    int damp_idx;   // index into the damping array, or -1
    int border;     // 1: src is (n+1) x (n+1); its last row/column (the bias border of an A factor) is
                    // eliminated on the fly: with u = src[0:n, n], c = src[n][n] + damp the copy is
                    // the Schur complement  src[0:n,0:n] + damp I - u u^T / c
    int wg_start;
};

// Completes the inverse of a bordered matrix [[B, u], [u^T, c]] whose Schur complement
// S = B - u u^T / c has been inverted into X[0:n, 0:n]:
//   X[0:n, n] = X[n, 0:n] = -(X u) / c,   X[n][n] = 1/c + u^T X u / c^2.
struct BorderJob {
    const float *src;   // the (n+1) x (n+1) factor (u = its last row), leading dimension lds
    float *X;           // (n+1) x (n+1), leading dimension ldx
    long long lds, ldx;
    int n;
    int damp_idx;       // or -1
    int info_idx;       // or -1: a non-positive c is reported as pivot n + 1
    int wg_start;       // pass 0: one workgroup per 4 rows
};

struct LeafJob {    // dst = (src + damp I)^-1 inside one workgroup, n <= 288
    const float *src;
    float *dst;
    long long lds, ldd;
    int n;
    int damp_idx;   // or -1
    int info_idx;   // index into info (or -1), pivot indices are reported + pivot_base
    int pivot_base;
};

// ---- BatchNorm ---------------------------------------------------------------------
struct BnJob {
    const float *g_gamma, *g_beta;
    float *F_ema, *out_gamma, *out_beta;
    int C;
    int wg_start;
};

struct BnReduceJob {
    const float *dy, *xhat;
    float *g_gamma, *g_beta;
    int C, HW;
    int wg_start;   // NCHW: one wave per (n, c) row, 4 rows per workgroup; NHWC: one workgroup per sample and 64 channels
};

// One tensor [N, HW, C] -> [N, C, HW] (NHWC -> NCHW).
struct LayoutJob {
    const void *src;
    void *dst;
    int N, C, HW;
    int tiles_c, tiles_hw;   // 64 x 64 tiles per image
    int wg_start;
};

// BatchNorm layer treated with its whole 2C x 2C Fisher block (Sec. 4.2 before the unit-wise approximation).
struct BnFullJob {
    const float *g_gamma, *g_beta;   // [N, C] per-sample gradients
    float *F_ema;                    // [2C, 2C]
    const float *F_inv;              // [2C, 2C]
    float *gbar;                     // [2C] scratch: mean gradient, (gamma_i, beta_i) interleaved
    float *out_gamma, *out_beta;     // [C]
    int C;
    int damp_idx;                    // slot of the layer's damping; -1: the layer is not inverted
    int wg_start[3];                 // per pass: factor tiles, mean, apply
};

// Staleness of one statistic (Sec. 4.3): X against its predecessors P = X_-1 and Q = X_-2 (null: none).
struct StaleJob {
    const float *X, *P, *Q;
    long long n;        // elements
    double *partial;    // [wgs][4]: sum (x-p)^2, sum p^2, sum (x-q)^2, sum q^2 of each workgroup's chunk
    double *out;        // [2]: the two ratios
    int wgs;            // workgroups of the first pass (chunks of kStaleChunk elements)
    int wg_start;
};
constexpr int kStaleChunk = 4096;

// Parameter update of one layer (Sec. 6.2, 6.3): n = d_out * d_in weights.
struct UpdateJob {
    float *W, *W_prev;
    const float *U;
    long long n;
    double *partial;    // [wgs] sums of squares of the new weights per chunk; null: no rescaling
    float *scale;       // [1] sqrt(2 d_out) / (||w'|| + eps)
    int d_out;
    int wgs;            // chunks of kUpdateChunk weights
    int wg_start;
};
constexpr int kUpdateChunk = 4096;

// Upper triangle of one d x d matrix <-> its place in the packed buffer (Sec. 5.2).
struct PackJob {
    const float *X;     // the matrix (written by the unpack kernel)
    long long off;      // first element of this matrix in the packed buffer
    int d;
    int tiles;          // ceil(d / 64): unpacking takes tiles (tiles + 1) / 2 workgroups
    int wg_start;       // (packing: one workgroup per kPackChunk elements of the triangle)
};
constexpr int kPackChunk = 4096;

#ifdef __HIPCC__
// ---- fp32 as the exact sum of three bf16 values (8 + 8 + 8 significant bits) -------------------------
// two fp32 values -> their packed (h, m, l) bf16 pairs, low half = first value
__device__ __forceinline__ void split_pair(float x0, float x1, unsigned &h, unsigned &m, unsigned &l)
{
    const unsigned b0 = __float_as_uint(x0), b1 = __float_as_uint(x1);
    const float r0 = x0 - __uint_as_float(b0 & 0xFFFF0000u), r1 = x1 - __uint_as_float(b1 & 0xFFFF0000u);
    const unsigned c0 = __float_as_uint(r0), c1 = __float_as_uint(r1);
    const float q0 = r0 - __uint_as_float(c0 & 0xFFFF0000u), q1 = r1 - __uint_as_float(c1 & 0xFFFF0000u);
    h = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
    m = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
    l = __builtin_amdgcn_perm(__float_as_uint(q1), __float_as_uint(q0), 0x07060302u);
}

#endif

// ---- launchers (implemented in the kernel files) -----------------------------------
hipError_t launch_gemm(const GemmProblem *probs_dev, const int *tile_start_dev, int n_probs,
                       int total_wgs, int tile_cfg, int dtype, hipStream_t s);
hipError_t launch_gemm_reduce(const GemmProblem *probs_dev, const int *red_start_dev, int n_probs,
                              int total_wgs, hipStream_t s);
hipError_t launch_patch(const PatchJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s);
hipError_t launch_pad(const PadJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s);
hipError_t launch_pad_bf16(const PadJobBF16 *jobs_dev, int n_jobs, int total_wgs, hipStream_t s);
hipError_t launch_assemble(const AssembleJob *jobs_dev, int n_jobs, int total_wgs, hipStream_t s);
hipError_t launch_trace(const TraceJob *jobs_dev, int n_layers, float gamma, float *damp_dev,
                        float *pi_out, hipStream_t s);
hipError_t launch_copy_damp(const CopyJob *jobs_dev, int n_jobs, int total_wgs, const float *damp_dev,
                            hipStream_t s);
// pass 0: the border row/column (total_wgs workgroups); pass 1: the corner (one workgroup per job)
hipError_t launch_border(const BorderJob *jobs_dev, int n_jobs, int total_wgs, int pass, const float *damp_dev,
                         int32_t *info, hipStream_t s);
hipError_t launch_leaf(const LeafJob *jobs_dev, int n_jobs, int size_class, const float *damp_dev,
                       int32_t *info, hipStream_t s);
hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t s);
hipError_t launch_bn(const BnJob *jobs_dev, int n_jobs, int total_wgs, int N, float decay, float lambda,
                     hipStream_t s);
// pass 0: F update; 1: mean gradient and damping; 2: u = F_inv gbar
hipError_t launch_bn_full(const BnFullJob *jobs_dev, int n_jobs, int total_wgs, int pass, int N, float decay,
                          float lambda, float *damp, hipStream_t s);
hipError_t launch_nhwc_to_nchw(const LayoutJob *jobs_dev, int n_jobs, int total_wgs, int esize, hipStream_t s);
hipError_t launch_bn_reduce(const BnReduceJob *jobs_dev, int n_jobs, int total_wgs, int N, int nhwc, hipStream_t s);
// pass 0: per-chunk sums (total_wgs workgroups); pass 1: one workgroup per job adds them up and writes the ratios
hipError_t launch_pack(const PackJob *jobs_dev, int n_jobs, int total_wgs, int bf16, int unpack, void *packed,
                       hipStream_t s);
// pass 0: the update (+ sums of squares); 1: scale factor per layer; 2: rescale
hipError_t launch_update(const UpdateJob *jobs_dev, int n_jobs, int total_wgs, int pass, float eta, float momentum,
                         float eps, hipStream_t s);
hipError_t launch_staleness(const StaleJob *jobs_dev, int n_jobs, int total_wgs, int pass, hipStream_t s);

// leaf size classes: a class value B serves n <= 32*B (one launch per class and level)
static const int kLeafClasses[] = {5, 7, 9};
static const int kNumLeafClasses = 3;
static const int kLeafMax = 288;

}  // namespace kfac
