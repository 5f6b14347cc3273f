// Grouped "NT" GEMM on the gfx950 matrix cores: for every problem in a device table,
//     C[i][j] = alpha * sum_m a(i, m) * b(j, m) + beta * C[i][j]
// where both operands have their rows along the contraction index (see Operand).
// This one kernel carries every dense contraction of the K-FAC step:
//   - the Kronecker factors A = E[M_A M_A^T], G = E[D D^T] (Sec. 3.3, Eq. 9 and 11):
//     a == b, only lower-triangle tiles are computed and mirrored, the running average
//     is the alpha/beta epilogue, long contractions are split along K into partial tiles
//     that a second kernel sums in a fixed order (bitwise reproducible);
//   - the Schur-complement products of the blocked inverse (Eq. 12);
//   - the two products of the preconditioned gradient G^-1 dW A^-1 (Eq. 6).
//
// Tiling: a 256-thread workgroup (2x2 wavefronts of 64) owns a BM x BN tile; each
// wavefront owns TM x TN blocks of 32x32 computed with v_mfma_f32_32x32x2_f32 (fp32)
// or v_mfma_f32_32x32x16_bf16.  The contraction runs in tiles of 32 staged through LDS
// (one stage in LDS, the next one in flight in registers).
#include "kfac_internal.h"

namespace kfac {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushortx8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushortx4 __attribute__((ext_vector_type(4)));

constexpr int KT = 32;      // contraction tile
constexpr int LDF = 36;     // LDS row length in floats (32 + 4 pad: conflict-free 16-byte reads)
constexpr int LDH = 40;     // LDS row length in bf16 (32 + 8 pad)

__device__ __forceinline__ int find_problem(const int *start, int n, int wg)
{
    int lo = 0, hi = n;  // invariant: start[lo] <= wg < start[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (start[mid] <= wg) lo = mid; else hi = mid;
    }
    return lo;
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup i runs on XCD i % 8) and each
// XCD has its own L2.  This maps the hardware index to a logical index such that each XCD
// works through one contiguous eighth of the logical range, so that tiles which share
// operand panels (neighbours in the logical order) hit the same L2.  Bijective on [0, total).
__device__ __forceinline__ int xcd_remap(int wg, int total)
{
    const int x = wg & 7, q = wg >> 3;
    const int base = total >> 3, rem = total & 7;
    return x * base + min(x, rem) + q;
}

__device__ __forceinline__ void tri_decode(int t, int &tm, int &tn)
{
    int r = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while (r * (r + 1) / 2 > t) --r;
    while ((r + 1) * (r + 2) / 2 <= t) ++r;
    tm = r;
    tn = t - r * (r + 1) / 2;
}

// Final write of one element of C and of its mirror / transposed copy (element-wise form,
// used by the bf16 kernel).
__device__ __forceinline__ void store_result(const GemmProblem &P, bool diag_tile, int i, int j, float acc)
{
    if (i >= P.M || j >= P.N) return;
    const bool sym = (P.flags & GEMM_SYM) != 0;
    if (sym && diag_tile && j > i) return;  // the mirror of (j, i) writes this one
    float *c = P.C + (long long)i * P.ldc + j;
    float v = P.alpha * acc;
    if (P.beta != 0.0f) v += P.beta * (*c);
    *c = v;
    if (sym && i != j) P.C[(long long)j * P.ldc + i] = v;
    if (P.Ct) P.Ct[(long long)j * P.ldct + i] = v;
}

// Final write of a ROWS x COLS slab of accumulated sums held in LDS (T[r][c] at
// T[r * (COLS + 1) + c], global position (gi0 + r, gj0 + c)):
//     C[i][j] = alpha * T + beta * C[i][j]
// plus, for symmetric problems, the mirror image C[j][i] (for a tile on the diagonal only
// j <= i is written directly and j < i mirrored, which makes the result exactly symmetric),
// plus the optional transposed copy Ct[j][i].  Both passes write whole row segments with
// adjacent lanes on adjacent addresses; the transposition happens in the LDS reads.
// The mirror pass relies on the old C being exactly symmetric (it reads beta's operand at
// the mirrored position); Ct requires beta == 0.
typedef float floatx4_st __attribute__((ext_vector_type(4), aligned(4)));

template <int ROWS, int COLS>
__device__ __forceinline__ void store_slab(const GemmProblem &P, const float *T, int gi0, int gj0, bool diag_tile,
                                           int tid)
{
    constexpr int LDT = COLS + 1;
    const bool sym = (P.flags & GEMM_SYM) != 0;
    const float alpha = P.alpha, beta = P.beta;
    // direct pass: a thread owns 4 adjacent columns of one row
    {
        constexpr int TPR = COLS / 4, RPP = 256 / TPR;
        const int c = (tid % TPR) * 4, rr = tid / TPR;
        for (int r = rr; r < ROWS; r += RPP) {
            const int i = gi0 + r, j = gj0 + c;
            if (i >= P.M || j >= P.N) continue;
            const int jmax = min(diag_tile ? i : P.N - 1, P.N - 1);   // last column this row may write
            if (j > jmax) continue;
            float *dst = P.C + (long long)i * P.ldc + j;
            const float *t = T + r * LDT + c;
            if (j + 3 <= jmax) {
                floatx4 v = {alpha * t[0], alpha * t[1], alpha * t[2], alpha * t[3]};
                if (beta != 0.0f) {
                    const floatx4 o = *(const floatx4_st *)dst;
                    for (int e = 0; e < 4; ++e) v[e] = fmaf(beta, o[e], v[e]);   // same rounding in every path
                }
                *(floatx4_st *)dst = v;
            } else {
                for (int e = 0; e < 4 && j + e <= jmax; ++e) {
                    float v = alpha * t[e];
                    if (beta != 0.0f) v = fmaf(beta, dst[e], v);
                    dst[e] = v;
                }
            }
        }
    }
    // mirrored / transposed pass: a thread owns 4 adjacent rows i of one column j, which are
    // 4 adjacent addresses of row j of the mirror image
    float *mbase = sym ? P.C : P.Ct;
    if (mbase) {
        const long long ldm = sym ? P.ldc : P.ldct;
        const float mbeta = sym ? beta : 0.0f;
        constexpr int TPR = ROWS / 4, RPP = 256 / TPR;
        const int r = (tid % TPR) * 4, cc = tid / TPR;
        for (int c = cc; c < COLS; c += RPP) {
            const int i = gi0 + r, j = gj0 + c;
            if (i >= P.M || j >= P.N) continue;
            // rows i..i+3 that may be mirrored: i + e < M and, on a diagonal tile, j < i + e
            const int e0 = (sym && diag_tile) ? max(0, j + 1 - i) : 0;
            const int e1 = min(4, P.M - i);
            if (e0 >= e1) continue;
            float *dst = mbase + (long long)j * ldm + i;
            const float *t = T + r * LDT + c;
            if (e0 == 0 && e1 == 4) {
                floatx4 v = {alpha * t[0], alpha * t[LDT], alpha * t[2 * LDT], alpha * t[3 * LDT]};
                if (mbeta != 0.0f) {
                    const floatx4 o = *(const floatx4_st *)dst;
                    for (int e = 0; e < 4; ++e) v[e] = fmaf(mbeta, o[e], v[e]);
                }
                *(floatx4_st *)dst = v;
            } else {
                for (int e = e0; e < e1; ++e) {
                    float v = alpha * t[e * LDT];
                    if (mbeta != 0.0f) v = fmaf(mbeta, dst[e], v);
                    dst[e] = v;
                }
            }
        }
    }
}

// ------------------------------------------------------------------ operand loader (fp32)
// A thread owns one 4-wide k chunk (kq = 4 * (tid % 8)) of the rows r0 + 32*s (r0 = tid / 8)
// of the operand tile.  A chunk is one 16-byte load that only needs 4-byte alignment (any
// leading dimension works); the host guarantees that the 4 elements of a chunk are adjacent
// in memory (hw % 4 == 0 for NCHW operands).  Every load of the main loop has an
// unconditionally valid address and is masked by value afterwards, so the loads of a whole
// tile are issued back to back:
//   - rows outside the operand are clamped to its last row and replaced by 0 (or by 1 for
//     the virtual all-ones row);
//   - the contraction range of a workgroup is cut into full 32-wide tiles; a remaining
//     multiple of 4 is covered by one more full tile shifted back to end at the range end,
//     whose already-counted k positions are zeroed in ONE operand;
//   - a remaining K % 4 (only plain matrices have one) is added in the epilogue.
// Ranges shorter than 32 take a slow, careful tile instead.
typedef float floatx4_u __attribute__((ext_vector_type(4), aligned(4)));
typedef const float __attribute__((address_space(1))) *gfloat_ptr;
typedef const floatx4_u __attribute__((address_space(1))) *gfloat4_ptr;

template <int BR>
struct LoaderF32 {
    static constexpr int SLOTS = BR / 32;
    gfloat_ptr base;
    long long rowoff[SLOTS];   // clamped row * row_stride (loop invariant)
    unsigned dead;             // bit s: slot row is outside the operand
    unsigned ones;             // bit s: slot row is the virtual all-ones row
    long long batch_stride;
    int hw, kq, r0, m, n, t;
    bool zero_all;             // the tile held in registers is to be stored as zeros

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int tid)
    {
        base = (gfloat_ptr)op.base;
        batch_stride = op.batch_stride;
        hw = op.hw;
        kq = (tid & 7) * 4; r0 = tid >> 3;
        dead = 0; ones = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int row = tile_row0 + r0 + 32 * s;
            if (row >= op.rows) dead |= 1u << s;
            if (row == op.ones_row) ones |= 1u << s;
            rowoff[s] = (long long)min(row, op.rows - 1) * op.row_stride;
        }
        m = n = t = 0;
        zero_all = false;
    }
    __device__ __forceinline__ void seek(int tile_k0)   // position on the tile starting at tile_k0
    {
        m = tile_k0 + kq;
        n = m / hw;
        t = m - n * hw;
    }
    __device__ __forceinline__ void advance()
    {
        m += KT; t += KT;
        while (t >= hw) { t -= hw; ++n; }
    }
    // Raw loads only: the masks are applied in store_lds, one iteration later, so nothing
    // waits for the data before the matrix instructions of the current tile are issued.
    __device__ __forceinline__ void load_full(floatx4 (&reg)[SLOTS])
    {
        const long long col = (long long)n * batch_stride + t;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) reg[s] = *(gfloat4_ptr)(base + rowoff[s] + col);
        zero_all = false;
    }
    // the shifted tile: k positions below mlo were already covered by the full tiles
    __device__ __forceinline__ void zero_below(int mlo) { zero_all = m < mlo; }
    // careful tile for short ranges: chunks at or beyond kend4 are not read
    __device__ __forceinline__ void load_careful(floatx4 (&reg)[SLOTS], int kend4)
    {
        const long long col = (long long)n * batch_stride + t;
        const bool in = m < kend4;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (in) v = *(gfloat4_ptr)(base + rowoff[s] + col);
            reg[s] = v;
        }
        zero_all = !in;
    }
    __device__ __forceinline__ void store_lds(const floatx4 (&reg)[SLOTS], float *lds) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            floatx4 v = reg[s];
            const float fill = (ones >> s) & 1 ? 1.f : 0.f;
            if ((dead >> s) & 1) { v[0] = fill; v[1] = fill; v[2] = fill; v[3] = fill; }
            if (zero_all) { v[0] = 0.f; v[1] = 0.f; v[2] = 0.f; v[3] = 0.f; }
            *(floatx4 *)(lds + (r0 + 32 * s) * LDF + kq) = v;
        }
    }
    // K % 4 remainder tile (plain matrices only: hw > K): thread tid < BR fills LDS row tid
    // with the elements k4 .. kend-1 of its operand row followed by zeros
    __device__ __forceinline__ static void fill_remainder(const Operand &op, int tile_row0, int k4, int kend,
                                                          int tid, float *lds)
    {
        if (tid >= BR) return;
        const int row = tile_row0 + tid;
        floatx4 x = {0.f, 0.f, 0.f, 0.f};
        if (row == op.ones_row) {
            for (int e = 0; e < 3; ++e)
                if (k4 + e < kend) x[e] = 1.f;
        } else if (row < op.rows) {
            gfloat_ptr p = (gfloat_ptr)op.base + (long long)row * op.row_stride + k4;
            for (int e = 0; e < 3; ++e)
                if (k4 + e < kend) x[e] = p[e];
        }
        float *dst = lds + tid * LDF;
        *(floatx4 *)dst = x;
#pragma unroll
        for (int q = 1; q < 8; ++q) *(floatx4 *)(dst + 4 * q) = floatx4{0.f, 0.f, 0.f, 0.f};
    }
};

// ------------------------------------------------------------------ fp32 kernel
// Two LDS stages: iteration `it` stores the tile it already holds in registers into stage
// it & 1, issues the global loads of tile it + 1, then (one barrier) multiplies out of stage
// it & 1.  The stage written in iteration it + 1 was last read before the barrier of
// iteration it + 1, which every wavefront reaches only after finishing that read.
template <int TM, int TN, bool LIVE>
__device__ __forceinline__ void gemm_f32_mainloop(const GemmProblem &P, int tm, int tn, int tid,
                                                  LoaderF32<64 * TM> &la, LoaderF32<64 * TN> &lb, float *lds,
                                                  int k0, int k1, int wave_m, int wave_n, int l32, int half,
                                                  floatx16 (&acc)[TM][TN])
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int STAGE = (BM + BN) * LDF;
    // [k0, k0 + klen4) is covered by vector-loaded tiles; a K % 4 remainder [k0 + klen4, k1)
    // exists only in the last split of a plain-matrix problem and gets a tile of its own
    const int klen = max(k1 - k0, 0);
    const int klen4 = klen & ~3;
    const int nfull = klen4 / KT;
    const bool shifted = nfull > 0 && klen4 > nfull * KT;   // one more full tile ending at k0 + klen4
    const bool careful = nfull == 0 && klen4 > 0;
    const int nvec = nfull + ((shifted || careful) ? 1 : 0);
    const int nk = nvec + (klen4 < klen ? 1 : 0);
    floatx4 ra[BM / 32], rb[BN / 32];
    la.seek(k0); lb.seek(k0);
    if (nfull > 0) { la.load_full(ra); lb.load_full(rb); }
    else if (careful) { la.load_careful(ra, k0 + klen4); lb.load_careful(rb, k0 + klen4); }
    for (int it = 0; it < nk; ++it) {
        float *sa = lds + (it & 1) * STAGE, *sb = sa + BM * LDF;
        if (it < nvec) {
            la.store_lds(ra, sa);
            lb.store_lds(rb, sb);
        } else {
            LoaderF32<BM>::fill_remainder(P.a, tm * BM, k0 + klen4, k1, tid, sa);
            LoaderF32<BN>::fill_remainder(P.b, tn * BN, k0 + klen4, k1, tid, sb);
        }
        if (it + 1 < nfull) {
            la.advance(); lb.advance();
            la.load_full(ra); lb.load_full(rb);
        } else if (it + 1 < nvec) {
            la.seek(k0 + klen4 - KT); lb.seek(k0 + klen4 - KT);
            la.load_full(ra); lb.load_full(rb);
            la.zero_below(k0 + nfull * KT);
        }
        __syncthreads();
        if constexpr (LIVE) {
            // each half-wave takes 16 consecutive k of the tile (the same 16 for both operands)
            floatx4 fa[TM][4], fb[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float *p = sa + (wave_m * 32 * TM + i * 32 + l32) * LDF + half * 16;
#pragma unroll
                for (int q = 0; q < 4; ++q) fa[i][q] = *(const floatx4 *)(p + 4 * q);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float *p = sb + (wave_n * 32 * TN + j * 32 + l32) * LDF + half * 16;
#pragma unroll
                for (int q = 0; q < 4; ++q) fb[j][q] = *(const floatx4 *)(p + 4 * q);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][q][e], fb[j][q][e], acc[i][j], 0, 0, 0);
        }
    }
}

template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(const GemmProblem *__restrict__ probs,
                                                          const int *__restrict__ tile_start, int n_probs)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    extern __shared__ __attribute__((aligned(16))) float lds[];   // 2 stages of (BM + BN) * LDF floats

    const int wg = blockIdx.x;
    const int pi = find_problem(tile_start, n_probs, wg);
    const GemmProblem &P = probs[pi];
    // every problem starts at a multiple of 8 workgroups (padded with idle ones), so the XCD
    // of a workgroup is its local index % 8; neighbours in the logical order are
    // neighbouring tiles of the same K range
    const int n_local = P.n_tiles * P.splits;
    const int local = xcd_remap(wg - tile_start[pi], (n_local + 7) & ~7);
    if (local >= n_local) return;
    const int split = local / P.n_tiles;
    const int tile = local - split * P.n_tiles;
    int tm, tn;
    if (P.flags & GEMM_SYM) tri_decode(tile, tm, tn);
    else { tm = tile / P.tiles_n; tn = tile - tm * P.tiles_n; }
    const int k0 = split * P.k_per_split;
    const int k1 = min(P.K, k0 + P.k_per_split);
    const int tid = threadIdx.x;

    LoaderF32<BM> la;
    LoaderF32<BN> lb;
    la.init(P.a, tm * BM, tid);
    lb.init(P.b, tn * BN, tid);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int lane = tid & 63, wid = tid >> 6;
    const int wave_m = wid >> 1, wave_n = wid & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // A wavefront whose whole sub-tile lies outside the matrix, or above the diagonal of a
    // symmetric product, stores nothing: it only helps with the loads and skips the math.
    const bool diag_tile = (P.flags & GEMM_SYM) && tm == tn;
    const int wave_r0 = tm * BM + wave_m * 32 * TM, wave_c0 = tn * BN + wave_n * 32 * TN;
    const bool live = wave_r0 < P.M && wave_c0 < P.N && !(diag_tile && wave_c0 >= wave_r0 + 32 * TM);

    if (live) gemm_f32_mainloop<TM, TN, true>(P, tm, tn, tid, la, lb, lds, k0, k1, wave_m, wave_n, l32, half, acc);
    else      gemm_f32_mainloop<TM, TN, false>(P, tm, tn, tid, la, lb, lds, k0, k1, wave_m, wave_n, l32, half, acc);

    // accumulator layout of the 32x32 block: column = lane % 32,
    // row = 8 * (v / 4) + 4 * (lane / 32) + v % 4 for register v = 0..15
    if (P.splits > 1) {
        float *part = P.partial + ((long long)tile * P.splits + split) * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wave_m * 32 * TM + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    const int c = wave_n * 32 * TN + j * 32 + l32;
                    part[r * BN + c] = acc[i][j][v];
                }
    } else {
        // stage the tile in LDS (the operand stages are dead by now), then store whole rows
        __syncthreads();
        if (live) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = wave_m * 32 * TM + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                        const int c = wave_n * 32 * TN + j * 32 + l32;
                        lds[r * (BN + 1) + c] = acc[i][j][v];
                    }
        }
        __syncthreads();
        store_slab<BM, BN>(P, lds, tm * BM, tn * BN, diag_tile, tid);
    }
}

// ------------------------------------------------------------------ bf16 operand loader
// Operands are bf16 in memory; a tile row is 32 bf16 = 64 bytes in LDS (+ pad).
template <int BR>
struct LoaderBF16 {
    static constexpr int NREG = BR / 8;  // bf16 values held per thread for one tile
    const unsigned short *base;
    long long row_stride, batch_stride;
    int rows, hw, ones_row, vec;
    int row0, koff, r0, m, n, t, kend;

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int k0, int k1, int tid)
    {
        base = (const unsigned short *)op.base;
        row_stride = op.row_stride; batch_stride = op.batch_stride;
        rows = op.rows; hw = op.hw; ones_row = op.ones_row; vec = op.vec;
        row0 = tile_row0; kend = k1;
        if (vec == 4) { koff = (tid & 7) * 4; r0 = tid >> 3; }
        else          { koff = tid & 31;      r0 = tid >> 5; }
        m = k0 + koff;
        n = m / hw;
        t = m - n * hw;
    }
    __device__ __forceinline__ void advance()
    {
        m += KT; t += KT;
        while (t >= hw) { t -= hw; ++n; }
    }
    // Branch-free, as in the fp32 loader.
    __device__ __forceinline__ void load(unsigned short (&reg)[NREG]) const
    {
        const unsigned short one_bits = 0x3F80;  // 1.0 in bf16
        const long long col = (long long)n * batch_stride + t;
        if (vec == 4) {
#pragma unroll
            for (int s = 0; s < BR / 32; ++s) {
                const int row = row0 + r0 + 32 * s;
                const bool ok = (row < rows) && (m < kend);
                const long long off = ok ? (long long)row * row_stride + col : 0;
                ushortx4 v = *(const ushortx4 *)(base + off);
                const bool use = ok || row == ones_row;
                const unsigned short one = (row == ones_row) ? one_bits : (unsigned short)0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned short x = ok ? v[e] : one;
                    reg[4 * s + e] = (use && m + e < kend) ? x : (unsigned short)0;
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < BR / 8; ++s) {
                const int row = row0 + r0 + 8 * s;
                const bool ok = (row < rows) && (m < kend);
                const long long off = ok ? (long long)row * row_stride + col : 0;
                const unsigned short v = base[off];
                reg[s] = ok ? v : ((row == ones_row && m < kend) ? one_bits : (unsigned short)0);
            }
        }
    }
    __device__ __forceinline__ void store_lds(const unsigned short (&reg)[NREG], unsigned short *lds) const
    {
        if (vec == 4) {
#pragma unroll
            for (int s = 0; s < BR / 32; ++s) {
                ushortx4 v = {reg[4 * s], reg[4 * s + 1], reg[4 * s + 2], reg[4 * s + 3]};
                *(ushortx4 *)(lds + (r0 + 32 * s) * LDH + koff) = v;
            }
        } else {
#pragma unroll
            for (int s = 0; s < BR / 8; ++s) lds[(r0 + 8 * s) * LDH + koff] = reg[s];
        }
    }
};

// ------------------------------------------------------------------ bf16 kernel
template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(const GemmProblem *__restrict__ probs,
                                                           const int *__restrict__ tile_start, int n_probs)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    __shared__ __attribute__((aligned(16))) unsigned short lds_a[BM * LDH];
    __shared__ __attribute__((aligned(16))) unsigned short lds_b[BN * LDH];

    const int wg = blockIdx.x;
    const int pi = find_problem(tile_start, n_probs, wg);
    const GemmProblem &P = probs[pi];
    const int n_local = P.n_tiles * P.splits;
    const int local = xcd_remap(wg - tile_start[pi], (n_local + 7) & ~7);
    if (local >= n_local) return;
    const int split = local / P.n_tiles;
    const int tile = local - split * P.n_tiles;
    int tm, tn;
    if (P.flags & GEMM_SYM) tri_decode(tile, tm, tn);
    else { tm = tile / P.tiles_n; tn = tile - tm * P.tiles_n; }
    const int k0 = split * P.k_per_split;
    const int k1 = min(P.K, k0 + P.k_per_split);
    const int tid = threadIdx.x;

    LoaderBF16<BM> la;
    LoaderBF16<BN> lb;
    la.init(P.a, tm * BM, k0, k1, tid);
    lb.init(P.b, tn * BN, k0, k1, tid);
    unsigned short ra[BM / 8], rb[BN / 8];

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int lane = tid & 63, wid = tid >> 6;
    const int wave_m = wid >> 1, wave_n = wid & 1;
    const int l32 = lane & 31, half = lane >> 5;

    // A wavefront whose whole sub-tile lies outside the matrix, or above the diagonal of a
    // symmetric product, stores nothing: it only helps with the loads and skips the math.
    const bool diag_tile = (P.flags & GEMM_SYM) && tm == tn;
    const int wave_r0 = tm * BM + wave_m * 32 * TM, wave_c0 = tn * BN + wave_n * 32 * TN;
    [[maybe_unused]] const bool live = wave_r0 < P.M && wave_c0 < P.N && !(diag_tile && wave_c0 >= wave_r0 + 32 * TM);

    const int nk = (k1 - k0 + KT - 1) / KT;
    if (nk > 0) { la.load(ra); lb.load(rb); }
    for (int it = 0; it < nk; ++it) {
        __syncthreads();
        la.store_lds(ra, lds_a);
        lb.store_lds(rb, lds_b);
        __syncthreads();
        if (it + 1 < nk) {
            la.advance(); lb.advance();
            la.load(ra); lb.load(rb);
        }
        // v_mfma_f32_32x32x16_bf16: a lane supplies 8 consecutive k of row lane%32; the two
        // half-waves cover k groups {0..7},{8..15}.  Two issues cover the 32-wide tile:
        // issue u uses k = 16u + 8*half + 0..7, identically for both operands.
        ushortx8 fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const unsigned short *p = lds_a + (wave_m * 32 * TM + i * 32 + l32) * LDH + half * 8;
            fa[i][0] = *(const ushortx8 *)(p);
            fa[i][1] = *(const ushortx8 *)(p + 16);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const unsigned short *p = lds_b + (wave_n * 32 * TN + j * 32 + l32) * LDH + half * 8;
            fb[j][0] = *(const ushortx8 *)(p);
            fb[j][1] = *(const ushortx8 *)(p + 16);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, fa[i][u]), __builtin_bit_cast(bf16x8, fb[j][u]), acc[i][j], 0, 0, 0);
    }

    if (P.splits > 1) {
        float *part = P.partial + ((long long)tile * P.splits + split) * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wave_m * 32 * TM + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    const int c = wave_n * 32 * TN + j * 32 + l32;
                    part[r * BN + c] = acc[i][j][v];
                }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = tm * BM + wave_m * 32 * TM + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    const int c = tn * BN + wave_n * 32 * TN + j * 32 + l32;
                    store_result(P, diag_tile, r, c, acc[i][j][v]);
                }
    }
}

// ------------------------------------------------------------------ split-K reduction + epilogue
// One workgroup per 32-row slab of a partial tile: sums the partial tiles in split order
// (fixed order, so results are reproducible bit for bit) into LDS and applies the same
// row-wise epilogue.  red_start counts slabs.
template <int B>
__device__ __forceinline__ void reduce_slab(const GemmProblem &P, int tile, int slab, int tm, int tn, float *T)
{
    const bool diag_tile = (P.flags & GEMM_SYM) && tm == tn;
    const float *part = P.partial + (long long)tile * P.splits * (B * B) + slab * 32 * B;
    // 32 * B elements, 4 per thread per pass
    for (int e = threadIdx.x * 4; e < 32 * B; e += 1024) {
        floatx4 s = {0.f, 0.f, 0.f, 0.f};
        for (int q = 0; q < P.splits; ++q) s += *(const floatx4 *)(part + (long long)q * (B * B) + e);
        const int r = e / B, c = e - r * B;
        float *t = T + r * (B + 1) + c;
        t[0] = s[0]; t[1] = s[1]; t[2] = s[2]; t[3] = s[3];
    }
    __syncthreads();
    store_slab<32, B>(P, T, tm * B + slab * 32, tn * B, diag_tile, threadIdx.x);
}

__global__ __launch_bounds__(256) void gemm_reduce_kernel(const GemmProblem *__restrict__ probs,
                                                          const int *__restrict__ red_start, int n_probs)
{
    __shared__ float T[32 * 129];
    const int wg = blockIdx.x;
    const int pi = find_problem(red_start, n_probs, wg);
    const GemmProblem &P = probs[pi];
    if (P.splits <= 1) return;
    const int B = (P.tile_cfg == 0) ? 128 : 64;
    const int slabs = B / 32;
    const int local = wg - red_start[pi];
    const int tile = local / slabs;
    const int slab = local - tile * slabs;
    int tm, tn;
    if (P.flags & GEMM_SYM) tri_decode(tile, tm, tn);
    else { tm = tile / P.tiles_n; tn = tile - tm * P.tiles_n; }
    if (tm * B + slab * 32 >= P.M) return;
    if (B == 128) reduce_slab<128>(P, tile, slab, tm, tn, T);
    else          reduce_slab<64>(P, tile, slab, tm, tn, T);
}

template <int TM, int TN>
static hipError_t launch_f32(const GemmProblem *probs_dev, const int *tile_start_dev, int n_probs, int total_wgs,
                             hipStream_t s)
{
    constexpr size_t lds_bytes = 2 * (64 * TM + 64 * TN) * LDF * sizeof(float);
    static bool configured = false;   // the attribute is per function, set once per process
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_nt_f32_kernel<TM, TN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    gemm_nt_f32_kernel<TM, TN><<<dim3(total_wgs), dim3(256), lds_bytes, s>>>(probs_dev, tile_start_dev, n_probs);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmProblem *probs_dev, const int *tile_start_dev, int n_probs,
                       int total_wgs, int tile_cfg, int dtype, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    dim3 grid(total_wgs), block(256);
    if (dtype == 0) {
        if (tile_cfg == 0) return launch_f32<2, 2>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
        return launch_f32<1, 1>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    }
    if (tile_cfg == 0) gemm_nt_bf16_kernel<2, 2><<<grid, block, 0, s>>>(probs_dev, tile_start_dev, n_probs);
    else               gemm_nt_bf16_kernel<1, 1><<<grid, block, 0, s>>>(probs_dev, tile_start_dev, n_probs);
    return hipGetLastError();
}

hipError_t launch_gemm_reduce(const GemmProblem *probs_dev, const int *red_start_dev, int n_probs,
                              int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    gemm_reduce_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(probs_dev, red_start_dev, n_probs);
    return hipGetLastError();
}

}  // namespace kfac
