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
// (two stages in LDS, a third tile in flight in registers).
#include "kfac_internal.h"
#include <type_traits>

namespace kfac {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushortx8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushortx4 __attribute__((ext_vector_type(4)));

constexpr int KT = 32;      // contraction tile
constexpr int LDF = 36;     // LDS row length in floats (32 + 4 pad: conflict-free 16-byte reads)

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

// Tile index -> tile coordinates.  The tiles are numbered in bands of g tile rows, column by column inside a
// band, so that the run of consecutive tiles which an XCD works on at one time is a g x (run / g) block:
// it touches g + run / g operand panels instead of 1 + run (one tile row), and each panel is brought into that
// XCD's L2 once for the whole block.  g grows with the problem (about the square root of an XCD's share of the
// tiles, at most 8).  Symmetric problems number the tiles of the lower triangle (tn <= tm) the same way; the
// band that crosses the diagonal ends in a small triangle.  Bijective on [0, n_tiles); the partial tiles of
// split contractions and their reduction use the same numbering.
__device__ __forceinline__ void decode_tile(const GemmProblem &P, int t, int &tm, int &tn)
{
    const int g = min(8, max(1, (int)ceilf(sqrtf((float)P.n_tiles * 0.125f))));
    if (P.flags & GEMM_SYM) {
        // band s holds rows s g .. s g + rows - 1 and starts at tile number T(s g), T(r) = r (r + 1) / 2
        int r0;
        tri_decode(t, r0, tn);                       // r0: the row whose plain numbering contains t
        const int s = r0 / g, first = s * g;
        const int rows = min(g, P.tiles_m - first);
        const int u = t - first * (first + 1) / 2;   // index inside the band
        const int full = first * rows;               // tiles of the band left of its diagonal block
        if (u < full) {
            tn = u / rows;
            tm = first + (u - tn * rows);
        } else {
            int rr, cc;
            tri_decode(u - full, rr, cc);
            tm = first + rr;
            tn = first + cc;
        }
    } else {
        const int band = g * P.tiles_n;
        const int s = t / band, first = s * g;
        const int rows = min(g, P.tiles_m - first);
        const int u = t - s * band;
        tn = u / rows;
        tm = first + (u - tn * rows);
    }
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
    // The old values (beta != 0) of all rows of a pass are requested before the first store of
    // the pass: a load issued behind a store to the same matrix waits for it, and a pass of
    // load - store pairs then costs one memory round trip per row.
    // direct pass: a thread owns 4 adjacent columns of one row
    {
        constexpr int TPR = COLS / 4, RPP = 256 / TPR, NIT = (ROWS + RPP - 1) / RPP;
        const int c = (tid % TPR) * 4, rr = tid / TPR;
        const int j = gj0 + c;
        floatx4 old[NIT];
        if (beta != 0.0f) {
#pragma unroll
            for (int q = 0; q < NIT; ++q) {
                const int r = rr + q * RPP, i = gi0 + r;
                const int jmax = min(diag_tile ? i : P.N - 1, P.N - 1);
                old[q] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (r < ROWS && i < P.M && j + 3 <= jmax) old[q] = *(const floatx4_st *)(P.C + (long long)i * P.ldc + j);
            }
        }
#pragma unroll
        for (int q = 0; q < NIT; ++q) {
            const int r = rr + q * RPP, i = gi0 + r;
            if (r >= ROWS || i >= P.M || j >= P.N) continue;
            const int jmax = min(diag_tile ? i : P.N - 1, P.N - 1);   // last column this row may write
            if (j > jmax) continue;
            float *dst = P.C + (long long)i * P.ldc + j;
            const float *t = T + r * LDT + c;
            if (j + 3 <= jmax) {
                floatx4 v = {alpha * t[0], alpha * t[1], alpha * t[2], alpha * t[3]};
                if (beta != 0.0f)
                    for (int e = 0; e < 4; ++e) v[e] = fmaf(beta, old[q][e], v[e]);   // same rounding in every path
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
        constexpr int TPR = ROWS / 4, RPP = 256 / TPR, NIT = (COLS + RPP - 1) / RPP;
        const int r = (tid % TPR) * 4, cc = tid / TPR;
        const int i = gi0 + r;
        floatx4 old[NIT];
        if (mbeta != 0.0f) {
#pragma unroll
            for (int q = 0; q < NIT; ++q) {
                const int c = cc + q * RPP, j = gj0 + c;
                const int e0 = (sym && diag_tile) ? max(0, j + 1 - i) : 0;
                old[q] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (c < COLS && j < P.N && e0 == 0 && i + 4 <= P.M) old[q] = *(const floatx4_st *)(mbase + (long long)j * ldm + i);
            }
        }
#pragma unroll
        for (int q = 0; q < NIT; ++q) {
            const int c = cc + q * RPP, j = gj0 + c;
            if (c >= COLS || i >= P.M || j >= P.N) continue;
            // rows i..i+3 that may be mirrored: i + e < M and, on a diagonal tile, j < i + e
            const int e0 = (sym && diag_tile) ? max(0, j + 1 - i) : 0;
            const int e1 = min(4, P.M - i);
            if (e0 >= e1) continue;
            float *dst = mbase + (long long)j * ldm + i;
            const float *t = T + r * LDT + c;
            if (e0 == 0 && e1 == 4) {
                floatx4 v = {alpha * t[0], alpha * t[LDT], alpha * t[2 * LDT], alpha * t[3 * LDT]};
                if (mbeta != 0.0f)
                    for (int e = 0; e < 4; ++e) v[e] = fmaf(mbeta, old[q][e], v[e]);
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

// Border of a GEMM_BORDER problem: entry `row` of the extra row / column from the row sum
// of the operand, and the corner from the contraction length.
__device__ __forceinline__ void store_border(const GemmProblem &P, int row, float sum)
{
    float *pr = P.C + (long long)P.M * P.ldc + row;
    float v = P.alpha * sum;
    if (P.beta != 0.0f) v = fmaf(P.beta, *pr, v);
    *pr = v;
    P.C[(long long)row * P.ldc + P.M] = v;
}
__device__ __forceinline__ void store_corner(const GemmProblem &P)
{
    float *pc = P.C + (long long)P.M * P.ldc + P.M;
    float v = P.alpha * (float)P.ones;
    if (P.beta != 0.0f) v = fmaf(P.beta, *pc, v);
    *pc = v;
}

// ------------------------------------------------------------------ operand loader (fp32)
// A thread owns one 4-wide k chunk (kq = 4 * (tid % 8)) of the rows r0 + 32*s (r0 = tid / 8)
// of the operand tile.  A chunk is one 16-byte load that only needs 4-byte alignment (any
// leading dimension works); the host guarantees that the 4 elements of a chunk are adjacent
// in memory (hw % 4 == 0 for NCHW operands).  Every load of the main loop has an
// unconditionally valid address and is masked by value afterwards, so the loads of a whole
// tile are issued back to back:
//   - rows outside the operand are clamped to its last row and replaced by 0;
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
    long long batch_stride;
    long long col;             // offset of the thread's chunk within a row: n * batch_stride + t
    int hw, kq, r0, m, n, t;
    bool zero_all;             // the tile held in registers is to be stored as zeros

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int tid)
    {
        base = (gfloat_ptr)op.base;
        batch_stride = op.batch_stride;
        hw = op.hw;
        kq = (tid & 7) * 4; r0 = tid >> 3;
        dead = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int row = tile_row0 + r0 + 32 * s;
            if (row >= op.rows) dead |= 1u << s;
            rowoff[s] = (long long)min(row, op.rows - 1) * op.row_stride;
        }
        m = n = t = 0;
        col = 0;
        zero_all = false;
    }
    __device__ __forceinline__ void seek(int tile_k0)   // position on the tile starting at tile_k0
    {
        m = tile_k0 + kq;
        n = m / hw;
        t = m - n * hw;
        col = (long long)n * batch_stride + t;
    }
    __device__ __forceinline__ void advance()
    {
        m += KT; t += KT; col += KT;
        while (t >= hw) { t -= hw; col += batch_stride - hw; }
    }
    // the same for runs of at least one tile (hw >= KT): at most one wrap, no branch
    __device__ __forceinline__ void advance_once()
    {
        m += KT; t += KT; col += KT;
        const bool wrap = t >= hw;
        t -= wrap ? hw : 0;
        col += wrap ? batch_stride - hw : 0;
    }
    // Raw loads only: the masks are applied in store_lds, one iteration later, so nothing
    // waits for the data before the matrix instructions of the current tile are issued.
    __device__ __forceinline__ void load_full(floatx4 (&reg)[SLOTS])
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) reg[s] = *(gfloat4_ptr)(base + rowoff[s] + col);
        zero_all = false;
    }
    // the shifted tile: k positions below mlo were already covered by the full tiles
    __device__ __forceinline__ void zero_below(int mlo) { zero_all = m < mlo; }
    // careful tile for short ranges: chunks at or beyond kend4 are not read
    __device__ __forceinline__ void load_careful(floatx4 (&reg)[SLOTS], int kend4)
    {
        const bool in = m < kend4;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (in) v = *(gfloat4_ptr)(base + rowoff[s] + col);
            reg[s] = v;
        }
        zero_all = !in;
    }
    // RS: also add what is stored to the running row sums rs[s] of the rows r0 + 32*s
    template <bool RS>
    __device__ __forceinline__ void store_lds(const floatx4 (&reg)[SLOTS], float *lds, float (&rs)[SLOTS]) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            floatx4 v = reg[s];
            if (((dead >> s) & 1) || zero_all) { v[0] = 0.f; v[1] = 0.f; v[2] = 0.f; v[3] = 0.f; }
            if constexpr (RS) rs[s] += (v[0] + v[1]) + (v[2] + v[3]);
            *(floatx4 *)(lds + (r0 + 32 * s) * LDF + kq) = v;
        }
    }
    // one slot of a tile without masked rows (dead == 0, not zero_all)
    template <bool RS>
    __device__ __forceinline__ void store_slot(const floatx4 (&reg)[SLOTS], float *lds, float (&rs)[SLOTS], int s) const
    {
        const floatx4 v = reg[s];
        if constexpr (RS) rs[s] += (v[0] + v[1]) + (v[2] + v[3]);
        *(floatx4 *)(lds + (r0 + 32 * s) * LDF + kq) = v;
    }
    __device__ __forceinline__ void load_slot(floatx4 (&reg)[SLOTS], int s)
    {
        reg[s] = *(gfloat4_ptr)(base + rowoff[s] + col);
    }
    // K % 4 remainder tile (plain matrices only: hw > K): thread tid < BR fills LDS row tid
    // with the elements k4 .. kend-1 of its operand row followed by zeros; returns their sum
    __device__ __forceinline__ static float fill_remainder(const Operand &op, int tile_row0, int k4, int kend,
                                                           int tid, float *lds)
    {
        if (tid >= BR) return 0.f;
        const int row = tile_row0 + tid;
        floatx4 x = {0.f, 0.f, 0.f, 0.f};
        if (row < op.rows) {
            gfloat_ptr p = (gfloat_ptr)op.base + (long long)row * op.row_stride + k4;
            for (int e = 0; e < 3; ++e)
                if (k4 + e < kend) x[e] = p[e];
        }
        float *dst = lds + tid * LDF;
        *(floatx4 *)dst = x;
#pragma unroll
        for (int q = 1; q < 8; ++q) *(floatx4 *)(dst + 4 * q) = floatx4{0.f, 0.f, 0.f, 0.f};
        return x[0] + x[1] + x[2];
    }
};

// Finishes the border row sums of a diagonal tile: adds up the 8 lanes that share a row,
// then either stores the border entries (splits == 1) or this split's partial sums.
// Uses the first BM floats of LDS; all 256 threads call it, between barriers of its own.
template <int BM>
__device__ __forceinline__ void finish_row_sums(const GemmProblem &P, float *lds, int tm, int tile, int split,
                                                int tid, float (&rs)[BM / 32], float rs_rem)
{
#pragma unroll
    for (int s = 0; s < BM / 32; ++s) {
        float v = rs[s];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 4);
        rs[s] = v;
    }
    __syncthreads();   // the operand stages are dead
    if ((tid & 7) == 0) {
#pragma unroll
        for (int s = 0; s < BM / 32; ++s) lds[(tid >> 3) + 32 * s] = rs[s];
    }
    __syncthreads();
    if (tid < BM) {
        const float total = lds[tid] + rs_rem;
        const int row = tm * BM + tid;
        if (P.splits > 1) P.partial_rs[((long long)tm * P.splits + split) * BM + tid] = total;
        else if (row < P.M) store_border(P, row, total);
    }
    if (tile == 0 && tid == 0 && P.splits == 1) store_corner(P);
    __syncthreads();
}

// ------------------------------------------------------------------ fp32 kernel
// Software pipeline over the K tiles, two LDS stages, one barrier per tile.  While the matrix
// instructions of tile `it` run out of stage it & 1, the same wavefront
//   - stores tile it + 1 (held in registers since the previous iteration) into the other stage,
//   - issues the global loads of tile it + 2 into those registers,
//   - reads its operand fragments a quarter tile ahead of the matrix instructions,
// so that no wavefront depends on another one sharing its SIMD to keep the matrix pipe busy.
// The barrier sits before the last quarter: after it every wavefront has finished reading
// stage it & 1 up to the fragments it already holds, and has stored its part of tile it + 1,
// whose first fragments are read during the last quarter.
// RS: the row sums of the a-operand tile are accumulated on the side (rs: rows r0 + 32*s of
// the vector-loaded part, rs_rem: row tid of the K % 4 remainder).
template <int TM, int TN>
struct FragF32 {
    floatx4 a[TM], b[TN];
};

template <int TM, int TN>
__device__ __forceinline__ void read_frag(FragF32<TM, TN> &f, const float *pa, const float *pb, int q)
{
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = *(const floatx4 *)(pa + i * 32 * LDF + 4 * q);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = *(const floatx4 *)(pb + j * 32 * LDF + 4 * q);
}

template <int TM, int TN>
__device__ __forceinline__ void mma_frag(const FragF32<TM, TN> &f, floatx16 (&acc)[TM][TN])
{
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[i][e], f.b[j][e], acc[i][j], 0, 0, 0);
}

template <int TM, int TN, bool LIVE, bool RS>
__device__ __forceinline__ void gemm_f32_mainloop(const GemmProblem &P, int tm, int tn, int tid,
                                                  LoaderF32<64 * TM> &la, LoaderF32<64 * TN> &lb, float *lds,
                                                  int k0, int k1, int wave_m, int wave_n, int l32, int half,
                                                  floatx16 (&acc)[TM][TN], float (&rs)[2 * TM], float &rs_rem)
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
    if (nk == 0) return;
    floatx4 ra[BM / 32], rb[BN / 32];

    // global loads of tile `it` into the staging registers (nothing beyond the vector tiles)
    auto load_tile = [&](int it) {
        if (it < nfull) {
            if (it > 0) { la.advance(); lb.advance(); }
            la.load_full(ra); lb.load_full(rb);
        } else if (it < nvec) {
            if (careful) {
                la.load_careful(ra, k0 + klen4); lb.load_careful(rb, k0 + klen4);
            } else {
                la.seek(k0 + klen4 - KT); lb.seek(k0 + klen4 - KT);
                la.load_full(ra); lb.load_full(rb);
                la.zero_below(k0 + nfull * KT);
            }
        }
    };
    // tile `it` (< nk) into its LDS stage: from the staging registers, or the K % 4 remainder
    auto store_tile = [&](int it) {
        float *sa = lds + (it & 1) * STAGE, *sb = sa + BM * LDF;
        if (it < nvec) {
            float unused[BN / 32];
            la.template store_lds<RS>(ra, sa, rs);
            lb.template store_lds<false>(rb, sb, unused);
        } else {
            rs_rem = LoaderF32<BM>::fill_remainder(P.a, tm * BM, k0 + klen4, k1, tid, sa);
            LoaderF32<BN>::fill_remainder(P.b, tn * BN, k0 + klen4, k1, tid, sb);
        }
    };
    // each half-wave takes 16 consecutive k of the tile (the same 16 for both operands)
    const int off_a = (wave_m * 32 * TM + l32) * LDF + half * 16;
    const int off_b = BM * LDF + (wave_n * 32 * TN + l32) * LDF + half * 16;

    la.seek(k0); lb.seek(k0);
    load_tile(0);
    store_tile(0);
    load_tile(1);
    __syncthreads();
    FragF32<TM, TN> f0, f1;
    if constexpr (LIVE) read_frag<TM, TN>(f0, lds + off_a, lds + off_b, 0);

    // One iteration of the general form: any kind of tile, stores and loads as blocks.
    auto step = [&](int it) {
        const float *cur = lds + (it & 1) * STAGE;
        const float *nxt = lds + ((it + 1) & 1) * STAGE;
        if constexpr (LIVE) read_frag<TM, TN>(f1, cur + off_a, cur + off_b, 1);
        if (it + 1 < nk) store_tile(it + 1);
        if constexpr (LIVE) mma_frag<TM, TN>(f0, acc);
        if constexpr (LIVE) read_frag<TM, TN>(f0, cur + off_a, cur + off_b, 2);
        load_tile(it + 2);
        if constexpr (LIVE) mma_frag<TM, TN>(f1, acc);
        if constexpr (LIVE) read_frag<TM, TN>(f1, cur + off_a, cur + off_b, 3);
        if constexpr (LIVE) mma_frag<TM, TN>(f0, acc);
        __syncthreads();
        if constexpr (LIVE) {
            if (it + 1 < nk) read_frag<TM, TN>(f0, nxt + off_a, nxt + off_b, 0);
            mma_frag<TM, TN>(f1, acc);
        }
    };
    // The steady state: tile it + 1 is a vector tile without masked rows and tile it + 2 a full
    // one reached by a single wrap of the position.  Straight-line code in a fixed order (the
    // scheduling barriers keep the compiler from regrouping it): the stores of tile it + 1 and
    // the loads of tile it + 2 are dealt out one by one behind the matrix instructions of the
    // first quarter, in whose shadow they issue; the loads then have the rest of the tile to
    // arrive, and every fragment read has a quarter.
    auto fast_step = [&](int it) {
        const float *cur = lds + (it & 1) * STAGE;
        float *nxt = lds + ((it + 1) & 1) * STAGE;
        constexpr int SA = BM / 32, SB = BN / 32, NOPS = 2 * (SA + SB);
        constexpr int NMMA = LIVE ? 4 * TM * TN : 1;
        constexpr int PER = (NOPS + NMMA - 1) / NMMA;
        auto side_op = [&](int k) {   // k-th of: stores of a, stores of b, loads of a, loads of b
            if (k < SA) {
                la.template store_slot<RS>(ra, nxt, rs, k);
            } else if (k < SA + SB) {
                float unused[SB];
                lb.template store_slot<false>(rb, nxt + BM * LDF, unused, k - SA);
            } else if (k < 2 * SA + SB) {
                if (k == SA + SB) { la.advance_once(); lb.advance_once(); }
                la.load_slot(ra, k - SA - SB);
            } else if (k < NOPS) {
                lb.load_slot(rb, k - 2 * SA - SB);
            }
        };
        if constexpr (LIVE) {
            read_frag<TM, TN>(f1, cur + off_a, cur + off_b, 1);
            __builtin_amdgcn_sched_barrier(0);
            int n = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f0.a[i][e], f0.b[j][e], acc[i][j], 0, 0, 0);
#pragma unroll
                        for (int u = 0; u < PER; ++u) side_op(n * PER + u);
                        ++n;
                        __builtin_amdgcn_sched_barrier(0);
                    }
            read_frag<TM, TN>(f0, cur + off_a, cur + off_b, 2);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag<TM, TN>(f1, acc);
            __builtin_amdgcn_sched_barrier(0);
            read_frag<TM, TN>(f1, cur + off_a, cur + off_b, 3);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag<TM, TN>(f0, acc);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            read_frag<TM, TN>(f0, nxt + off_a, nxt + off_b, 0);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag<TM, TN>(f1, acc);
        } else {
#pragma unroll
            for (int k = 0; k < NOPS; ++k) side_op(k);
            __syncthreads();
        }
    };
    int it = 0;
    // (a condition the whole workgroup agrees on: every row of both operand tiles exists)
    if (la.hw >= KT && lb.hw >= KT && (tm + 1) * BM <= P.a.rows && (tn + 1) * BN <= P.b.rows)
        for (; it + 2 < nfull; ++it) fast_step(it);
    for (; it < nk; ++it) step(it);
}

// ------------------------------------------------------------------ fp32 through three bf16 planes
// The bf16 matrix instruction runs at 16 times the rate of the fp32 one.  An fp32 value is the
// exact sum of three bf16 values (8 + 8 + 8 significant bits: x = h + m + l by two truncations
// and two exact subtractions), and a product of two bf16 values is exact in fp32, so
//     x y  =  h h' + (h m' + m h') + (h l' + m m' + l h')  +  terms below 2^-23 |x y|
// with fp32 accumulation inside the matrix unit: six bf16 instructions give the product to
// fp32 accuracy in 6 x 32 cycles per 32x32x16 block instead of 8 x 64.  The operands stay fp32 in
// HBM; the loader of the fp32 kernel brings a K tile of 32 into registers and the split happens
// on the way into LDS, which holds one stage of three planes (two barriers per tile; the second
// workgroup of the compute unit computes while this one stores).
constexpr int LDQ = 40;     // LDS row length in bf16 (32 + 8 pad: 80-byte rows, conflict-free 16-byte reads)
// Rows of a group of 8 are stored in the order 0 4 1 5 2 6 3 7: the 8-byte stores of 16 lanes cover two
// rows, and rows 80 bytes apart share 4 of their 16 banks while rows 4 apart (320 bytes) share none.  The
// fragment reads take the same 8 rows per group of lanes as before.
__device__ __forceinline__ int lds_row(int r) { return (r & ~7) | ((r & 1) << 2) | ((r >> 1) & 3); }

// the staged tile of one operand into its rows of the three planes (plane stride in bf16 units)
template <int BR, bool RS>
__device__ __forceinline__ void store_split(const LoaderF32<BR> &ld, const floatx4 (&reg)[BR / 32], unsigned short *rows,
                                            int plane, float (&rs)[BR / 32])
{
#pragma unroll
    for (int s = 0; s < BR / 32; ++s) {
        floatx4 v = reg[s];
        if (((ld.dead >> s) & 1) || ld.zero_all) { v[0] = 0.f; v[1] = 0.f; v[2] = 0.f; v[3] = 0.f; }
        if constexpr (RS) rs[s] += (v[0] + v[1]) + (v[2] + v[3]);
        uint2 h, m, l;
        split_pair(v[0], v[1], h.x, m.x, l.x);
        split_pair(v[2], v[3], h.y, m.y, l.y);
        unsigned short *dst = rows + (lds_row(ld.r0) + 32 * s) * LDQ + ld.kq;
        *(uint2 *)dst = h;
        *(uint2 *)(dst + plane) = m;
        *(uint2 *)(dst + 2 * plane) = l;
    }
}

// K % 4 remainder tile: thread tid < BR fills row tid of the three planes with the elements
// k4 .. kend-1 of its operand row followed by zeros; returns their sum
template <int BR>
__device__ __forceinline__ float fill_remainder_split(const Operand &op, int tile_row0, int k4, int kend, int tid,
                                                      unsigned short *rows, int plane)
{
    if (tid >= BR) return 0.f;
    const int row = tile_row0 + tid;
    float x[4] = {0.f, 0.f, 0.f, 0.f};
    if (row < op.rows) {
        gfloat_ptr p = (gfloat_ptr)op.base + (long long)row * op.row_stride + k4;
        for (int e = 0; e < 3; ++e)
            if (k4 + e < kend) x[e] = p[e];
    }
    uint2 v[3];
    split_pair(x[0], x[1], v[0].x, v[1].x, v[2].x);
    split_pair(x[2], x[3], v[0].y, v[1].y, v[2].y);
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        unsigned short *dst = rows + q * plane + lds_row(tid) * LDQ;
        *(uint4 *)dst = uint4{v[q].x, v[q].y, 0u, 0u};
#pragma unroll
        for (int w = 1; w < 4; ++w) *(uint4 *)(dst + 8 * w) = uint4{0u, 0u, 0u, 0u};
    }
    return x[0] + x[1] + x[2];
}

// SAME: a and b are the same operand tile (a diagonal tile of a Gram matrix): it is loaded, split and stored
// once, and the fragments of b are read from the rows of a.
template <int TM, int TN, bool LIVE, bool RS, bool SAME>
__device__ __forceinline__ void gemm_split_mainloop(const GemmProblem &P, int tm, int tn, int tid,
                                                    LoaderF32<64 * TM> &la, LoaderF32<64 * TN> &lb, unsigned short *lds,
                                                    int k0, int k1, int wave_m, int wave_n, int l32, int half,
                                                    floatx16 (&acc)[TM][TN], float (&rs)[2 * TM], float &rs_rem)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int PLANE = (BM + BN) * LDQ;
    const int klen = max(k1 - k0, 0);
    const int klen4 = klen & ~3;
    const int nfull = klen4 / KT;
    const bool shifted = nfull > 0 && klen4 > nfull * KT;
    const bool careful = nfull == 0 && klen4 > 0;
    const int nvec = nfull + ((shifted || careful) ? 1 : 0);
    const int nk = nvec + (klen4 < klen ? 1 : 0);
    if (nk == 0) return;
    // two tiles in flight in registers: the loads of tile it + 2 are issued when tile it has gone
    // into LDS, and have two tile times to arrive
    floatx4 ra0[BM / 32], rb0[BN / 32], ra1[BM / 32], rb1[BN / 32];
    bool za0 = false, zb0 = false, za1 = false, zb1 = false;   // the loaders' zero_all of the tile held

    auto load_tile = [&](int it, auto &ra, auto &rb, bool &za, bool &zb) {
        if (it < nfull) {
            if constexpr (SAME) {
                if (it > 0) la.advance();
                la.load_full(ra);
            } else {
                if (it > 0) { la.advance(); lb.advance(); }
                la.load_full(ra); lb.load_full(rb);
            }
        } else if (it < nvec) {
            if (careful) {
                la.load_careful(ra, k0 + klen4);
                if constexpr (!SAME) lb.load_careful(rb, k0 + klen4);
            } else if constexpr (SAME) {
                la.seek(k0 + klen4 - KT);
                la.load_full(ra);
                la.zero_below(k0 + nfull * KT);
            } else {
                la.seek(k0 + klen4 - KT); lb.seek(k0 + klen4 - KT);
                la.load_full(ra); lb.load_full(rb);
                la.zero_below(k0 + nfull * KT);
            }
        }
        za = la.zero_all; zb = lb.zero_all;
    };
    auto store_tile = [&](int it, const auto &ra, const auto &rb, bool za, bool zb) {
        if (it < nvec) {
            float unused[BN / 32];
            la.zero_all = za; lb.zero_all = zb;
            store_split<BM, RS>(la, ra, lds, PLANE, rs);
            if constexpr (!SAME) store_split<BN, false>(lb, rb, lds + BM * LDQ, PLANE, unused);
        } else {
            rs_rem = fill_remainder_split<BM>(P.a, tm * BM, k0 + klen4, k1, tid, lds, PLANE);
            if constexpr (!SAME) fill_remainder_split<BN>(P.b, tn * BN, k0 + klen4, k1, tid, lds + BM * LDQ, PLANE);
        }
    };
    // v_mfma_f32_32x32x16_bf16: a lane supplies 8 consecutive k of row lane % 32, the half-waves
    // two different groups of 8; step u of a tile uses k = 16u + 8*half + 0..7 for both operands
    const int off_a = (wave_m * 32 * TM + lds_row(l32)) * LDQ + 8 * half;
    const int off_b = (SAME ? 0 : BM * LDQ) + (wave_n * 32 * TN + lds_row(l32)) * LDQ + 8 * half;
    // One step: the fragments of the h and m planes and of l' are requested up front, the l
    // fragments of the a operand take over the registers of h once its products are issued (their
    // latency lies under the m products).  Fixed order (the scheduling barriers keep the compiler
    // from hoisting the next step's reads, which would cost the second workgroup of the compute
    // unit its registers).
    auto compute = [&]() {
        if constexpr (LIVE) {
            auto rd = [&](int q, int off, int u) {
                return __builtin_bit_cast(bf16x8, *(const ushortx8 *)(lds + q * PLANE + off + 16 * u));
            };
            auto mm = [&](const bf16x8 (&x)[TM], const bf16x8 (&y)[TN]) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[i], y[j], acc[i][j], 0, 0, 0);
            };
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 ah[TM], am[TM], bh[TN], bm[TN], bl[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) ah[i] = rd(0, off_a + i * 32 * LDQ, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bh[j] = rd(0, off_b + j * 32 * LDQ, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bm[j] = rd(1, off_b + j * 32 * LDQ, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bl[j] = rd(2, off_b + j * 32 * LDQ, u);
#pragma unroll
                for (int i = 0; i < TM; ++i) am[i] = rd(1, off_a + i * 32 * LDQ, u);
                __builtin_amdgcn_sched_barrier(0);
                mm(ah, bh);
                mm(ah, bm);
                mm(ah, bl);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TM; ++i) ah[i] = rd(2, off_a + i * 32 * LDQ, u);   // the l plane of a
                __builtin_amdgcn_sched_barrier(0);
                mm(am, bh);
                mm(am, bm);
                mm(ah, bh);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    if constexpr (SAME) la.seek(k0);
    else { la.seek(k0); lb.seek(k0); }
    load_tile(0, ra0, rb0, za0, zb0);
    load_tile(1, ra1, rb1, za1, zb1);
    for (int it = 0; it < nk; it += 2) {
        if (it > 0) __syncthreads();   // every wavefront has read the tile before
        store_tile(it, ra0, rb0, za0, zb0);
        load_tile(it + 2, ra0, rb0, za0, zb0);
        __syncthreads();
        compute();
        if (it + 1 < nk) {
            __syncthreads();
            store_tile(it + 1, ra1, rb1, za1, zb1);
            load_tile(it + 3, ra1, rb1, za1, zb1);
            __syncthreads();
            compute();
        }
    }
}

// ------------------------------------------------------------------ transposed operands (NHWC in place)
// Element (r, m) of the operand lives at base + m * ld + r: the rows are the contiguous direction.  A thread
// loads 16 bytes = four adjacent rows at one m (lanes along the rows: 512 contiguous bytes per 32 lanes), splits
// them and stores 8 bytes per plane into an LDS tile that keeps this order, [m][row]; the fragments of the
// matrix instruction (8 consecutive m of one row per lane) come out of that tile through the transposing LDS
// read of gfx950 (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i % 4 of the four 8-byte groups
// addressed by lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12).  Every m of the range is read where it is: no
// shifted tile, no remainder tile; loads beyond the range are clamped and zeroed by value.
template <int BR>
struct LoaderF32T {
    static constexpr int SLOTS = BR / 32;
    static constexpr int CG = BR / 4;          // row chunks of the tile
    static constexpr int MSTEP = 256 / CG;     // m positions covered by one slot of all threads
    static constexpr int RS = BR + 16;         // LDS row (one m) in bf16: four rows of a read 32 bytes apart in banks
    gfloat_ptr base;
    long long ld;
    int c_local, c_load, mk, K;
    bool dead;

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int tid, int K_)
    {
        base = (gfloat_ptr)op.base;
        ld = op.row_stride;
        c_local = 4 * (tid % CG);
        mk = tid / CG;
        const int c = tile_row0 + c_local;
        dead = c >= op.rows;                         // rows % 4 == 0: a chunk is inside or outside as a whole
        c_load = min(c, op.rows - 4);
        K = K_;
    }
    __device__ __forceinline__ void load(floatx4 (&reg)[SLOTS], int tile_m0) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int m = min(tile_m0 + mk + MSTEP * s, K - 1);
            reg[s] = *(gfloat4_ptr)(base + (long long)m * ld + c_load);
        }
    }
    // mend: end of the workgroup's range; rs: running sums of the thread's four rows
    template <bool RSUM>
    __device__ __forceinline__ void store(const floatx4 (&reg)[SLOTS], unsigned short *rows, int plane, int tile_m0,
                                          int mend, float (&rs)[4]) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            floatx4 v = reg[s];
            const int ml = mk + MSTEP * s;
            if (dead || tile_m0 + ml >= mend) { v[0] = 0.f; v[1] = 0.f; v[2] = 0.f; v[3] = 0.f; }
            if constexpr (RSUM) { rs[0] += v[0]; rs[1] += v[1]; rs[2] += v[2]; rs[3] += v[3]; }
            uint2 h, m, l;
            split_pair(v[0], v[1], h.x, m.x, l.x);
            split_pair(v[2], v[3], h.y, m.y, l.y);
            unsigned short *dst = rows + ml * RS + c_local;
            *(uint2 *)dst = h;
            *(uint2 *)(dst + plane) = m;
            *(uint2 *)(dst + 2 * plane) = l;
        }
    }
};

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) shortx4 *lds_shortx4_ptr;

template <int TM, int TN, bool LIVE, bool RSUM>
__device__ __forceinline__ void gemm_split_mainloop_trans(const GemmProblem &P, int tm, int tn, int tid,
                                                          unsigned short *lds, int k0, int k1, int wave_m, int wave_n,
                                                          int lane, floatx16 (&acc)[TM][TN], float (&rs)[4])
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int RSA = LoaderF32T<BM>::RS, RSB = LoaderF32T<BN>::RS;
    constexpr int PLANE_A = KT * RSA, PLANE_B = KT * RSB;
    unsigned short *lds_b = lds + 3 * PLANE_A;
    LoaderF32T<BM> la;
    LoaderF32T<BN> lb;
    la.init(P.a, tm * BM, tid, P.K);
    lb.init(P.b, tn * BN, tid, P.K);
    const int nk = (max(k1 - k0, 0) + KT - 1) / KT;
    if (nk == 0) return;
    floatx4 ra0[BM / 32], rb0[BN / 32], ra1[BM / 32], rb1[BN / 32];
    // fragment addressing of the transposing read: lane -> (m within the 16-wide step, first of four rows)
    const int frag_m = 8 * (lane >> 5) + ((lane & 15) >> 2);
    const int frag_r = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int off_a = frag_m * RSA + wave_m * 32 * TM + frag_r;
    const int off_b = frag_m * RSB + wave_n * 32 * TN + frag_r;
    auto compute = [&]() {
        if constexpr (LIVE) {
            auto rd = [&](const unsigned short *plane, int rs_, int off, int u) {
                const unsigned short *p = plane + off + 16 * u * rs_;
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_ptr)p);
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_ptr)(p + 4 * rs_));
                typedef short shortx8 __attribute__((ext_vector_type(8)));
                return __builtin_bit_cast(bf16x8, shortx8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
            };
            auto mm = [&](const bf16x8 (&x)[TM], const bf16x8 (&y)[TN]) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[i], y[j], acc[i][j], 0, 0, 0);
            };
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 ah[TM], am[TM], bh[TN], bm[TN], bl[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) ah[i] = rd(lds, RSA, off_a + i * 32, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bh[j] = rd(lds_b, RSB, off_b + j * 32, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bm[j] = rd(lds_b + PLANE_B, RSB, off_b + j * 32, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) bl[j] = rd(lds_b + 2 * PLANE_B, RSB, off_b + j * 32, u);
#pragma unroll
                for (int i = 0; i < TM; ++i) am[i] = rd(lds + PLANE_A, RSA, off_a + i * 32, u);
                __builtin_amdgcn_sched_barrier(0);
                mm(ah, bh);
                mm(ah, bm);
                mm(ah, bl);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TM; ++i) ah[i] = rd(lds + 2 * PLANE_A, RSA, off_a + i * 32, u);   // the l plane of a
                __builtin_amdgcn_sched_barrier(0);
                mm(am, bh);
                mm(am, bm);
                mm(ah, bh);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    float unused[4] = {0.f, 0.f, 0.f, 0.f};
    la.load(ra0, k0); lb.load(rb0, k0);
    la.load(ra1, k0 + KT); lb.load(rb1, k0 + KT);
    for (int it = 0; it < nk; it += 2) {
        if (it > 0) __syncthreads();   // every wavefront has read the tile before
        la.template store<RSUM>(ra0, lds, PLANE_A, k0 + it * KT, k1, rs);
        lb.template store<false>(rb0, lds_b, PLANE_B, k0 + it * KT, k1, unused);
        la.load(ra0, k0 + (it + 2) * KT); lb.load(rb0, k0 + (it + 2) * KT);
        __syncthreads();
        compute();
        if (it + 1 < nk) {
            __syncthreads();
            la.template store<RSUM>(ra1, lds, PLANE_A, k0 + (it + 1) * KT, k1, rs);
            lb.template store<false>(rb1, lds_b, PLANE_B, k0 + (it + 1) * KT, k1, unused);
            la.load(ra1, k0 + (it + 3) * KT); lb.load(rb1, k0 + (it + 3) * KT);
            __syncthreads();
            compute();
        }
    }
}

// Row sums of a diagonal tile whose operand is stored transposed: a thread holds the sums of its four rows over
// the m positions it loaded; the 256 / (BM / 4) threads that share a row chunk are added up through LDS.
template <int BM, int E>
__device__ __forceinline__ void finish_row_sums_trans(const GemmProblem &P, float *lds, int tm, int tile, int split,
                                                      int tid, const float (&rs)[E])
{
    constexpr int CG = BM / E, PARTS = 256 / CG;
    __syncthreads();   // the operand stages are dead
#pragma unroll
    for (int e = 0; e < E; ++e) lds[(tid / CG) * BM + E * (tid % CG) + e] = rs[e];
    __syncthreads();
    if (tid < BM) {
        float total = 0.f;
#pragma unroll
        for (int q = 0; q < PARTS; ++q) total += lds[q * BM + tid];
        const int row = tm * BM + tid;
        if (P.splits > 1) P.partial_rs[((long long)tm * P.splits + split) * BM + tid] = total;
        else if (row < P.M) store_border(P, row, total);
    }
    if (tile == 0 && tid == 0 && P.splits == 1) store_corner(P);
    __syncthreads();
}

template <int TM, int TN, bool SPLIT, bool TRANS = false>
__device__ __forceinline__ void gemm_nt_f32_body(const GemmProblem *__restrict__ probs,
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
    decode_tile(P, tile, tm, tn);
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

    // The diagonal tiles of a bordered problem also take the row sums of their operand rows.
    const bool border = diag_tile && (P.flags & GEMM_BORDER);
    float rs[BM / 32], rs_rem = 0.f;
#pragma unroll
    for (int s = 0; s < BM / 32; ++s) rs[s] = 0.f;
    // a diagonal tile of a Gram matrix (a and b the same operand) stages its operand tile once (64 x 64 tiles
    // only: the large tile has no registers to spare for one more copy of the main loop)
    constexpr bool CAN_SHARE = SPLIT && TM == 1 && TN == 1;
    const bool same = CAN_SHARE && tm == tn && P.a.base == P.b.base && P.a.row_stride == P.b.row_stride &&
                      P.a.batch_stride == P.b.batch_stride && P.a.hw == P.b.hw && P.a.rows == P.b.rows;
    auto mainloop = [&](auto live_c, auto rs_c) {
        constexpr bool LV = decltype(live_c)::value, RSUM = decltype(rs_c)::value;
        if constexpr (SPLIT) {
            if (CAN_SHARE && same)
                gemm_split_mainloop<TM, TN, LV, RSUM, CAN_SHARE>(P, tm, tn, tid, la, lb, (unsigned short *)lds, k0, k1,
                                                                 wave_m, wave_n, l32, half, acc, rs, rs_rem);
            else
                gemm_split_mainloop<TM, TN, LV, RSUM, false>(P, tm, tn, tid, la, lb, (unsigned short *)lds, k0, k1, wave_m,
                                                             wave_n, l32, half, acc, rs, rs_rem);
        } else
            gemm_f32_mainloop<TM, TN, LV, RSUM>(P, tm, tn, tid, la, lb, lds, k0, k1, wave_m, wave_n, l32, half, acc, rs,
                                                rs_rem);
    };
    if constexpr (TRANS) {   // both operands stored with the rows contiguous (a launch of its own)
        static_assert(SPLIT, "transposed operands: product mode of three bf16 planes only");
        float rst[4] = {0.f, 0.f, 0.f, 0.f};
        unsigned short *l16 = (unsigned short *)lds;
        if (border) {
            if (live) gemm_split_mainloop_trans<TM, TN, true, true>(P, tm, tn, tid, l16, k0, k1, wave_m, wave_n, lane, acc, rst);
            else      gemm_split_mainloop_trans<TM, TN, false, true>(P, tm, tn, tid, l16, k0, k1, wave_m, wave_n, lane, acc, rst);
            finish_row_sums_trans<BM, 4>(P, lds, tm, tile, split, tid, rst);
        } else {
            if (live) gemm_split_mainloop_trans<TM, TN, true, false>(P, tm, tn, tid, l16, k0, k1, wave_m, wave_n, lane, acc, rst);
            else      gemm_split_mainloop_trans<TM, TN, false, false>(P, tm, tn, tid, l16, k0, k1, wave_m, wave_n, lane, acc, rst);
        }
    } else if (border) {
        if (live) mainloop(std::true_type{}, std::true_type{});
        else      mainloop(std::false_type{}, std::true_type{});
        finish_row_sums<BM>(P, lds, tm, tile, split, tid, rs, rs_rem);
    } else {
        if (live) mainloop(std::true_type{}, std::false_type{});
        else      mainloop(std::false_type{}, std::false_type{});
    }

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

template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(const GemmProblem *__restrict__ probs,
                                                          const int *__restrict__ tile_start, int n_probs)
{
    gemm_nt_f32_body<TM, TN, false>(probs, tile_start, n_probs);
}

// the same for problems whose operands are stored transposed (GEMM_TRANS)
template <int TM, int TN>
__global__ __launch_bounds__(256, 2) void gemm_nt_f32_split_trans_kernel(const GemmProblem *__restrict__ probs,
                                                                         const int *__restrict__ tile_start, int n_probs)
{
    gemm_nt_f32_body<TM, TN, true, true>(probs, tile_start, n_probs);
}

// (two wavefronts per SIMD: the register allocation is held to 256)
template <int TM, int TN>
__global__ __launch_bounds__(256, 2) void gemm_nt_f32_split_kernel(const GemmProblem *__restrict__ probs,
                                                                   const int *__restrict__ tile_start, int n_probs)
{
    gemm_nt_f32_body<TM, TN, true>(probs, tile_start, n_probs);
}

// ------------------------------------------------------------------ bf16 operand loader
// Same scheme as the fp32 loader with 64-wide K tiles: a thread owns one chunk of 8 bf16
// (16 bytes, 16-byte aligned: the host only contracts NCHW tensors in place when
// hw % 8 == 0 and the base is aligned; everything else goes through the repack kernel,
// whose rows are padded) of the rows r0 + 32*s.
constexpr int KTH = 64;     // contraction tile of the bf16 kernel
constexpr int LDH = 72;     // LDS row length in bf16 (64 + 8 pad: 144-byte rows, conflict-free 16-byte reads)
typedef const unsigned short __attribute__((address_space(1))) *gushort_ptr;
typedef const ushortx8 __attribute__((address_space(1))) *gushort8_ptr;

template <int BR, bool TAIL = false>
struct LoaderBF16 {
    static constexpr int SLOTS = BR / 32;
    gushort_ptr base;
    long long rowoff[SLOTS];
    unsigned dead;
    long long batch_stride;
    long long col;             // offset of the thread's chunk within a row: n * batch_stride + t
    int hw, kq, r0, m, n, t;
    int tail;                  // see Operand
    int n_last;                // TAIL: index of the last run of a row
    unsigned lastrow;          // TAIL: bit s set if slot s reads the last row of the operand
    bool zero_all;

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int tid, int K = 0)
    {
        base = (gushort_ptr)op.base;
        batch_stride = op.batch_stride;
        hw = op.hw;
        tail = op.tail;
        kq = (tid & 7) * 8; r0 = tid >> 3;
        dead = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int row = tile_row0 + r0 + 32 * s;
            if (row >= op.rows) dead |= 1u << s;
            rowoff[s] = (long long)min(row, op.rows - 1) * op.row_stride;
        }
        m = n = t = 0;
        col = 0;
        zero_all = false;
        n_last = 0;
        lastrow = 0;
        if constexpr (TAIL) {
            n_last = K / hw - 1;
#pragma unroll
            for (int s = 0; s < SLOTS; ++s)
                if (tile_row0 + r0 + 32 * s >= op.rows - 1) lastrow |= 1u << s;
        }
    }
    __device__ __forceinline__ void seek(int tile_k0)
    {
        m = tile_k0 + kq;
        n = m / hw;
        t = m - n * hw;
        col = (long long)n * batch_stride + t;
    }
    __device__ __forceinline__ void advance()
    {
        m += KTH; t += KTH; col += KTH;
        while (t >= hw) {
            t -= hw; col += batch_stride - hw;
            if constexpr (TAIL) ++n;
        }
    }
    // the same for runs of at least one tile (hw >= KTH): at most one wrap, no branch
    __device__ __forceinline__ void advance_once()
    {
        m += KTH; t += KTH; col += KTH;
        const bool wrap = t >= hw;
        t -= wrap ? hw : 0;
        col += wrap ? batch_stride - hw : 0;
        if constexpr (TAIL) n += wrap ? 1 : 0;
    }
    // The thread's chunk of row slot s.  Runs with a tail: the last chunk of a run is loaded whole as well (its
    // upper half lies in the next row of the tensor) and the upper half set to zero; only behind the last run
    // of the last row there is no next row, so that one chunk is loaded four elements lower and moved up.
    __device__ __forceinline__ ushortx8 fetch(int s) const
    {
        const long long off = rowoff[s] + col;
        if constexpr (!TAIL) return *(gushort8_ptr)(base + off);
        typedef unsigned short ushortx8_a8 __attribute__((ext_vector_type(8), aligned(8)));
        typedef const ushortx8_a8 __attribute__((address_space(1))) *gushort8a8_ptr;
        const bool last = tail != 0 && t + 8 == hw;
        const bool edge = last && n == n_last && ((lastrow >> s) & 1);
        const ushortx8_a8 v = *(gushort8a8_ptr)(base + off - (edge ? 4 : 0));
        ushortx8 r = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
        if (edge) { r[0] = v[4]; r[1] = v[5]; r[2] = v[6]; r[3] = v[7]; }
        if (last) { r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0; }
        return r;
    }
    __device__ __forceinline__ void load_full(ushortx8 (&reg)[SLOTS])
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) reg[s] = fetch(s);
        zero_all = false;
    }
    __device__ __forceinline__ void zero_below(int mlo) { zero_all = m < mlo; }
    __device__ __forceinline__ void load_careful(ushortx8 (&reg)[SLOTS], int kend8)
    {
        const bool in = m < kend8;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            ushortx8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (in) v = fetch(s);
            reg[s] = v;
        }
        zero_all = !in;
    }
    static __device__ __forceinline__ float widen(unsigned short h) { return __uint_as_float((unsigned)h << 16); }
    template <bool RS>
    __device__ __forceinline__ void store_lds(const ushortx8 (&reg)[SLOTS], unsigned short *lds, float (&rs)[SLOTS]) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            ushortx8 v = reg[s];
            if (((dead >> s) & 1) || zero_all) v = ushortx8{0, 0, 0, 0, 0, 0, 0, 0};
            if constexpr (RS)
                rs[s] += ((widen(v[0]) + widen(v[1])) + (widen(v[2]) + widen(v[3]))) +
                         ((widen(v[4]) + widen(v[5])) + (widen(v[6]) + widen(v[7])));
            *(ushortx8 *)(lds + (r0 + 32 * s) * LDH + kq) = v;
        }
    }
    // one slot of a tile without masked rows (dead == 0, not zero_all)
    template <bool RS>
    __device__ __forceinline__ void store_slot(const ushortx8 (&reg)[SLOTS], unsigned short *lds, float (&rs)[SLOTS], int s) const
    {
        const ushortx8 v = reg[s];
        if constexpr (RS)
            rs[s] += ((widen(v[0]) + widen(v[1])) + (widen(v[2]) + widen(v[3]))) +
                     ((widen(v[4]) + widen(v[5])) + (widen(v[6]) + widen(v[7])));
        *(ushortx8 *)(lds + (r0 + 32 * s) * LDH + kq) = v;
    }
    __device__ __forceinline__ void load_slot(ushortx8 (&reg)[SLOTS], int s)
    {
        reg[s] = fetch(s);
    }
    // K % 8 remainder tile (repacked operands only): thread tid < BR fills LDS row tid
    __device__ __forceinline__ static float fill_remainder(const Operand &op, int tile_row0, int k8, int kend,
                                                           int tid, unsigned short *lds)
    {
        if (tid >= BR) return 0.f;
        const int row = tile_row0 + tid;
        ushortx8 x = {0, 0, 0, 0, 0, 0, 0, 0};
        if (row < op.rows) {
            gushort_ptr p = (gushort_ptr)op.base + (long long)row * op.row_stride + k8;
            for (int e = 0; e < 7; ++e)
                if (k8 + e < kend) x[e] = p[e];
        }
        unsigned short *dst = lds + tid * LDH;
        *(ushortx8 *)dst = x;
#pragma unroll
        for (int q = 1; q < 8; ++q) *(ushortx8 *)(dst + 8 * q) = ushortx8{0, 0, 0, 0, 0, 0, 0, 0};
        float sum = 0.f;
        for (int e = 0; e < 7; ++e) sum += widen(x[e]);
        return sum;
    }
};

// ------------------------------------------------------------------ bf16 kernel
// The software pipeline of the fp32 kernel with 64-wide K tiles.  v_mfma_f32_32x32x16_bf16: a
// lane supplies 8 consecutive k of row lane % 32, the two half-waves supply two different k
// groups; step u (0..3) of a tile uses k = 16u + 8*half + 0..7, identically for both operands.
// A matrix instruction takes a quarter of the time of the fp32 one while a tile moves the same
// number of bytes, so the stores and loads are dealt out over the first three steps.
template <int TM, int TN>
struct FragBF16 {
    ushortx8 a[TM], b[TN];
};

template <int TM, int TN>
__device__ __forceinline__ void read_frag16(FragBF16<TM, TN> &f, const unsigned short *pa, const unsigned short *pb, int u)
{
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = *(const ushortx8 *)(pa + i * 32 * LDH + 16 * u);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = *(const ushortx8 *)(pb + j * 32 * LDH + 16 * u);
}

template <int TM, int TN>
__device__ __forceinline__ void mma_frag16(const FragBF16<TM, TN> &f, floatx16 (&acc)[TM][TN])
{
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]),
                                                                __builtin_bit_cast(bf16x8, f.b[j]), acc[i][j], 0, 0, 0);
}

// SAME: as in gemm_split_mainloop (a diagonal tile of a Gram matrix stages its operand tile once).
template <int TM, int TN, bool LIVE, bool RS, bool TAIL, bool SAME>
__device__ __forceinline__ void gemm_bf16_mainloop(const GemmProblem &P, int tm, int tn, int tid,
                                                   LoaderBF16<64 * TM, TAIL> &la, LoaderBF16<64 * TN, TAIL> &lb,
                                                   unsigned short *lds, int k0, int k1, int wave_m, int wave_n,
                                                   int l32, int half, floatx16 (&acc)[TM][TN], float (&rs)[2 * TM],
                                                   float &rs_rem)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int STAGE = (BM + BN) * LDH;
    const int klen = max(k1 - k0, 0);
    const int klen8 = klen & ~7;
    const int nfull = klen8 / KTH;
    const bool shifted = nfull > 0 && klen8 > nfull * KTH;
    const bool careful = nfull == 0 && klen8 > 0;
    const int nvec = nfull + ((shifted || careful) ? 1 : 0);
    const int nk = nvec + (klen8 < klen ? 1 : 0);
    if (nk == 0) return;
    ushortx8 ra[BM / 32], rb[BN / 32];

    auto load_tile = [&](int it) {
        if (it < nfull) {
            if constexpr (SAME) {
                if (it > 0) la.advance();
                la.load_full(ra);
            } else {
                if (it > 0) { la.advance(); lb.advance(); }
                la.load_full(ra); lb.load_full(rb);
            }
        } else if (it < nvec) {
            if (careful) {
                la.load_careful(ra, k0 + klen8);
                if constexpr (!SAME) lb.load_careful(rb, k0 + klen8);
            } else if constexpr (SAME) {
                la.seek(k0 + klen8 - KTH);
                la.load_full(ra);
                la.zero_below(k0 + nfull * KTH);
            } else {
                la.seek(k0 + klen8 - KTH); lb.seek(k0 + klen8 - KTH);
                la.load_full(ra); lb.load_full(rb);
                la.zero_below(k0 + nfull * KTH);
            }
        }
    };
    auto store_tile = [&](int it) {
        unsigned short *sa = lds + (it & 1) * STAGE, *sb = sa + BM * LDH;
        if (it < nvec) {
            float unused[BN / 32];
            la.template store_lds<RS>(ra, sa, rs);
            if constexpr (!SAME) lb.template store_lds<false>(rb, sb, unused);
        } else {
            rs_rem = LoaderBF16<BM>::fill_remainder(P.a, tm * BM, k0 + klen8, k1, tid, sa);
            if constexpr (!SAME) LoaderBF16<BN>::fill_remainder(P.b, tn * BN, k0 + klen8, k1, tid, sb);
        }
    };
    const int off_a = (wave_m * 32 * TM + l32) * LDH + 8 * half;
    const int off_b = (SAME ? 0 : BM * LDH) + (wave_n * 32 * TN + l32) * LDH + 8 * half;

    if constexpr (SAME) la.seek(k0);
    else { la.seek(k0); lb.seek(k0); }
    load_tile(0);
    store_tile(0);
    load_tile(1);
    __syncthreads();
    FragBF16<TM, TN> f0, f1;
    if constexpr (LIVE) read_frag16<TM, TN>(f0, lds + off_a, lds + off_b, 0);

    auto step = [&](int it) {
        const unsigned short *cur = lds + (it & 1) * STAGE;
        const unsigned short *nxt = lds + ((it + 1) & 1) * STAGE;
        if constexpr (LIVE) read_frag16<TM, TN>(f1, cur + off_a, cur + off_b, 1);
        if (it + 1 < nk) store_tile(it + 1);
        if constexpr (LIVE) mma_frag16<TM, TN>(f0, acc);
        if constexpr (LIVE) read_frag16<TM, TN>(f0, cur + off_a, cur + off_b, 2);
        load_tile(it + 2);
        if constexpr (LIVE) mma_frag16<TM, TN>(f1, acc);
        if constexpr (LIVE) read_frag16<TM, TN>(f1, cur + off_a, cur + off_b, 3);
        if constexpr (LIVE) mma_frag16<TM, TN>(f0, acc);
        __syncthreads();
        if constexpr (LIVE) {
            if (it + 1 < nk) read_frag16<TM, TN>(f0, nxt + off_a, nxt + off_b, 0);
            mma_frag16<TM, TN>(f1, acc);
        }
    };
    auto fast_step = [&](int it) {
        const unsigned short *cur = lds + (it & 1) * STAGE;
        unsigned short *nxt = lds + ((it + 1) & 1) * STAGE;
        constexpr int SA = BM / 32, SB = SAME ? 0 : BN / 32, NOPS = 2 * (SA + SB);
        constexpr int NMMA = LIVE ? 3 * TM * TN : 1;   // matrix instructions ahead of the barrier
        constexpr int PER = (NOPS + NMMA - 1) / NMMA;
        auto side_op = [&](int k) {   // k-th of: stores of a, stores of b, loads of a, loads of b
            if (k < SA) {
                la.template store_slot<RS>(ra, nxt, rs, k);
            } else if (k < SA + SB) {
                if constexpr (!SAME) {
                    float unused[BN / 32];
                    lb.template store_slot<false>(rb, nxt + BM * LDH, unused, k - SA);
                }
            } else if (k < 2 * SA + SB) {
                if (k == SA + SB) {
                    if constexpr (SAME) la.advance_once();
                    else { la.advance_once(); lb.advance_once(); }
                }
                la.load_slot(ra, k - SA - SB);
            } else if (k < NOPS) {
                if constexpr (!SAME) lb.load_slot(rb, k - 2 * SA - SB);
            }
        };
        if constexpr (LIVE) {
            int n = 0;
            // step u multiplies the fragments read during step u - 1 and reads those of step u + 1
            auto group = [&](FragBF16<TM, TN> &use, FragBF16<TM, TN> &fill, int u_fill) {
                read_frag16<TM, TN>(fill, cur + off_a, cur + off_b, u_fill);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, use.a[i]),
                                                                            __builtin_bit_cast(bf16x8, use.b[j]),
                                                                            acc[i][j], 0, 0, 0);
#pragma unroll
                        for (int q = 0; q < PER; ++q) side_op(n * PER + q);
                        ++n;
                        __builtin_amdgcn_sched_barrier(0);
                    }
            };
            group(f0, f1, 1);
            group(f1, f0, 2);
            group(f0, f1, 3);
            __syncthreads();
            read_frag16<TM, TN>(f0, nxt + off_a, nxt + off_b, 0);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag16<TM, TN>(f1, acc);
        } else {
#pragma unroll
            for (int k = 0; k < NOPS; ++k) side_op(k);
            __syncthreads();
        }
    };
    int it = 0;
    // (a condition the whole workgroup agrees on: every row of both operand tiles exists)
    if (la.hw >= KTH && lb.hw >= KTH && (tm + 1) * BM <= P.a.rows && (tn + 1) * BN <= P.b.rows)
        for (; it + 2 < nfull; ++it) fast_step(it);
    for (; it < nk; ++it) step(it);
}

// ------------------------------------------------------------------ bf16 operands stored transposed
// As LoaderF32T / gemm_split_mainloop_trans with one plane and no conversion: a thread loads 16 bytes = eight
// adjacent rows at one m and stores them as they are into the [m][row] tile; rows % 8 == 0, 16-byte aligned base.
template <int BR>
struct LoaderBF16T {
    static constexpr int CG = BR / 8;
    static constexpr int MSTEP = 256 / CG;
    static constexpr int SLOTS = KT / MSTEP;   // K tiles of 32 here
    static constexpr int RS = BR + 16;
    gushort_ptr base;
    long long ld;
    int c_local, c_load, mk, K;
    bool dead;

    __device__ __forceinline__ void init(const Operand &op, int tile_row0, int tid, int K_)
    {
        base = (gushort_ptr)op.base;
        ld = op.row_stride;
        c_local = 8 * (tid % CG);
        mk = tid / CG;
        const int c = tile_row0 + c_local;
        dead = c >= op.rows;
        c_load = min(c, op.rows - 8);
        K = K_;
    }
    __device__ __forceinline__ void load(ushortx8 (&reg)[SLOTS], int tile_m0) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int m = min(tile_m0 + mk + MSTEP * s, K - 1);
            reg[s] = *(gushort8_ptr)(base + (long long)m * ld + c_load);
        }
    }
    template <bool RSUM>
    __device__ __forceinline__ void store(const ushortx8 (&reg)[SLOTS], unsigned short *rows, int tile_m0, int mend,
                                          float (&rs)[8]) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            ushortx8 v = reg[s];
            const int ml = mk + MSTEP * s;
            if (dead || tile_m0 + ml >= mend) v = ushortx8{0, 0, 0, 0, 0, 0, 0, 0};
            if constexpr (RSUM) {
#pragma unroll
                for (int e = 0; e < 8; ++e) rs[e] += __uint_as_float((unsigned)v[e] << 16);
            }
            *(ushortx8 *)(rows + ml * RS + c_local) = v;
        }
    }
};

template <int TM, int TN, bool LIVE, bool RSUM>
__device__ __forceinline__ void gemm_bf16_mainloop_trans(const GemmProblem &P, int tm, int tn, int tid,
                                                         unsigned short *lds, int k0, int k1, int wave_m, int wave_n,
                                                         int lane, floatx16 (&acc)[TM][TN], float (&rs)[8])
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int RSA = LoaderBF16T<BM>::RS, RSB = LoaderBF16T<BN>::RS;
    unsigned short *lds_b = lds + KT * RSA;
    LoaderBF16T<BM> la;
    LoaderBF16T<BN> lb;
    la.init(P.a, tm * BM, tid, P.K);
    lb.init(P.b, tn * BN, tid, P.K);
    const int nk = (max(k1 - k0, 0) + KT - 1) / KT;
    if (nk == 0) return;
    ushortx8 ra0[LoaderBF16T<BM>::SLOTS], rb0[LoaderBF16T<BN>::SLOTS], ra1[LoaderBF16T<BM>::SLOTS], rb1[LoaderBF16T<BN>::SLOTS];
    const int frag_m = 8 * (lane >> 5) + ((lane & 15) >> 2);
    const int frag_r = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int off_a = frag_m * RSA + wave_m * 32 * TM + frag_r;
    const int off_b = frag_m * RSB + wave_n * 32 * TN + frag_r;
    auto compute = [&]() {
        if constexpr (LIVE) {
            auto rd = [&](const unsigned short *tile, int rs_, int off, int u) {
                const unsigned short *p = tile + off + 16 * u * rs_;
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_ptr)p);
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4_ptr)(p + 4 * rs_));
                typedef short shortx8 __attribute__((ext_vector_type(8)));
                return __builtin_bit_cast(bf16x8, shortx8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
            };
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) a[i] = rd(lds, RSA, off_a + i * 32, u);
#pragma unroll
                for (int j = 0; j < TN; ++j) b[j] = rd(lds_b, RSB, off_b + j * 32, u);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
            }
        }
    };
    float unused[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    la.load(ra0, k0); lb.load(rb0, k0);
    la.load(ra1, k0 + KT); lb.load(rb1, k0 + KT);
    for (int it = 0; it < nk; it += 2) {
        if (it > 0) __syncthreads();
        la.template store<RSUM>(ra0, lds, k0 + it * KT, k1, rs);
        lb.template store<false>(rb0, lds_b, k0 + it * KT, k1, unused);
        la.load(ra0, k0 + (it + 2) * KT); lb.load(rb0, k0 + (it + 2) * KT);
        __syncthreads();
        compute();
        if (it + 1 < nk) {
            __syncthreads();
            la.template store<RSUM>(ra1, lds, k0 + (it + 1) * KT, k1, rs);
            lb.template store<false>(rb1, lds_b, k0 + (it + 1) * KT, k1, unused);
            la.load(ra1, k0 + (it + 3) * KT); lb.load(rb1, k0 + (it + 3) * KT);
            __syncthreads();
            compute();
        }
    }
}

// TAIL: an operand of the problem has runs with a four-element tail (Operand::tail); a variant of its
// own, so that the loads of all other problems stay single 16-byte loads without a branch.
template <int TM, int TN, bool TAIL, bool TRANS = false>
__device__ __forceinline__ void gemm_nt_bf16_body(const GemmProblem &P, int local, float *lds)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const int split = local / P.n_tiles;
    const int tile = local - split * P.n_tiles;
    int tm, tn;
    decode_tile(P, tile, tm, tn);
    const int k0 = split * P.k_per_split;
    const int k1 = min(P.K, k0 + P.k_per_split);
    const int tid = threadIdx.x;

    LoaderBF16<BM, TAIL> la;
    LoaderBF16<BN, TAIL> lb;
    la.init(P.a, tm * BM, tid, P.K);
    lb.init(P.b, tn * BN, tid, P.K);

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
    const bool diag_tile = (P.flags & GEMM_SYM) && tm == tn;
    const int wave_r0 = tm * BM + wave_m * 32 * TM, wave_c0 = tn * BN + wave_n * 32 * TN;
    const bool live = wave_r0 < P.M && wave_c0 < P.N && !(diag_tile && wave_c0 >= wave_r0 + 32 * TM);

    unsigned short *lds16 = (unsigned short *)lds;
    const bool border = diag_tile && (P.flags & GEMM_BORDER);
    float rs[BM / 32], rs_rem = 0.f;
#pragma unroll
    for (int s = 0; s < BM / 32; ++s) rs[s] = 0.f;
    if constexpr (TRANS) {
        float rst[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (border) {
            if (live) gemm_bf16_mainloop_trans<TM, TN, true, true>(P, tm, tn, tid, lds16, k0, k1, wave_m, wave_n, lane, acc, rst);
            else      gemm_bf16_mainloop_trans<TM, TN, false, true>(P, tm, tn, tid, lds16, k0, k1, wave_m, wave_n, lane, acc, rst);
            finish_row_sums_trans<BM, 8>(P, lds, tm, tile, split, tid, rst);
        } else {
            if (live) gemm_bf16_mainloop_trans<TM, TN, true, false>(P, tm, tn, tid, lds16, k0, k1, wave_m, wave_n, lane, acc, rst);
            else      gemm_bf16_mainloop_trans<TM, TN, false, false>(P, tm, tn, tid, lds16, k0, k1, wave_m, wave_n, lane, acc, rst);
        }
    } else {
        // a diagonal tile of a Gram matrix (a and b the same operand) stages its operand tile once (64 x 64 tiles
        // only: the large tile has no registers to spare for one more copy of the main loop)
        constexpr bool CAN_SHARE = TM == 1 && TN == 1;
        const bool same = CAN_SHARE && tm == tn && P.a.base == P.b.base && P.a.row_stride == P.b.row_stride &&
                          P.a.batch_stride == P.b.batch_stride && P.a.hw == P.b.hw && P.a.rows == P.b.rows;
        auto mainloop = [&](auto live_c, auto rs_c) {
            constexpr bool LV = decltype(live_c)::value, RSUM = decltype(rs_c)::value;
            if (CAN_SHARE && same)
                gemm_bf16_mainloop<TM, TN, LV, RSUM, TAIL, CAN_SHARE>(P, tm, tn, tid, la, lb, lds16, k0, k1, wave_m, wave_n, l32, half, acc, rs, rs_rem);
            else
                gemm_bf16_mainloop<TM, TN, LV, RSUM, TAIL, false>(P, tm, tn, tid, la, lb, lds16, k0, k1, wave_m, wave_n, l32, half, acc, rs, rs_rem);
        };
        if (border) {
            if (live) mainloop(std::true_type{}, std::true_type{});
            else      mainloop(std::false_type{}, std::true_type{});
            finish_row_sums<BM>(P, lds, tm, tile, split, tid, rs, rs_rem);
        } else {
            if (live) mainloop(std::true_type{}, std::false_type{});
            else      mainloop(std::false_type{}, std::false_type{});
        }
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

// ------------------------------------------------------------------ split-K reduction + epilogue
// One workgroup per 32-row slab of a partial tile: sums the partial tiles in split order
// (fixed order, so results are reproducible bit for bit) into LDS and applies the same
// row-wise epilogue.  red_start counts slabs.
template <int B>
__device__ __forceinline__ void reduce_slab(const GemmProblem &P, int tile, int slab, int tm, int tn, float *T)
{
    const bool diag_tile = (P.flags & GEMM_SYM) && tm == tn;
    const float *part = P.partial + (long long)tile * P.splits * (B * B) + slab * 32 * B;
    // 32 * B elements, 4 per thread per pass.  Split q goes into partial sum q % 4 of its element;
    // the four are combined in a fixed order: as reproducible as one running sum, with the loads
    // of four splits and all passes in flight at once (the partial tiles are read exactly once)
    constexpr int PASSES = 32 * B / 1024;
    floatx4 acc[PASSES][4];
#pragma unroll
    for (int p = 0; p < PASSES; ++p)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[p][k] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int q = 0; q < P.splits; q += 4) {
        floatx4 v[PASSES][4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                v[p][k] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (q + k < P.splits)
                    v[p][k] = __builtin_nontemporal_load((const floatx4 *)(part + (long long)(q + k) * (B * B) + threadIdx.x * 4 + p * 1024));
            }
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int p = 0; p < PASSES; ++p)
                if (q + k < P.splits) acc[p][k] += v[p][k];
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const floatx4 s = (acc[p][0] + acc[p][1]) + (acc[p][2] + acc[p][3]);
        const int e = threadIdx.x * 4 + p * 1024;
        const int r = e / B, c = e - r * B;
        float *t = T + r * (B + 1) + c;
        t[0] = s[0]; t[1] = s[1]; t[2] = s[2]; t[3] = s[3];
    }
    __syncthreads();
    store_slab<32, B>(P, T, tm * B + slab * 32, tn * B, diag_tile, threadIdx.x);
    if (diag_tile && (P.flags & GEMM_BORDER)) {
        const int row = tm * B + slab * 32 + threadIdx.x;
        if (threadIdx.x < 32 && row < P.M) {
            const float *prs = P.partial_rs + (long long)tm * P.splits * B + slab * 32 + threadIdx.x;
            float sum = 0.f;
            for (int q = 0; q < P.splits; ++q) sum += prs[(long long)q * B];
            store_border(P, row, sum);
        }
        if (tile == 0 && slab == 0 && threadIdx.x == 0) store_corner(P);
    }
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
    decode_tile(P, tile, tm, tn);
    if (tm * B + slab * 32 >= P.M) return;
    if (B == 128) reduce_slab<128>(P, tile, slab, tm, tn, T);
    else          reduce_slab<64>(P, tile, slab, tm, tn, T);
}

// LDS per workgroup: two operand stages, reused for the (BM x BN+1) fp32 output tile.

template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(const GemmProblem *__restrict__ probs,
                                                           const int *__restrict__ tile_start, int n_probs)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];   // operand stages, then the output tile

    const int wg = blockIdx.x;
    const int pi = find_problem(tile_start, n_probs, wg);
    const GemmProblem &P = probs[pi];
    const int n_local = P.n_tiles * P.splits;
    const int local = xcd_remap(wg - tile_start[pi], (n_local + 7) & ~7);
    if (local >= n_local) return;
    if (P.a.tail | P.b.tail) gemm_nt_bf16_body<TM, TN, true>(P, local, lds);
    else                     gemm_nt_bf16_body<TM, TN, false>(P, local, lds);
}
template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_bf16_trans_kernel(const GemmProblem *__restrict__ probs,
                                                                 const int *__restrict__ tile_start, int n_probs)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int wg = blockIdx.x;
    const int pi = find_problem(tile_start, n_probs, wg);
    const GemmProblem &P = probs[pi];
    const int n_local = P.n_tiles * P.splits;
    const int local = xcd_remap(wg - tile_start[pi], (n_local + 7) & ~7);
    if (local >= n_local) return;
    gemm_nt_bf16_body<TM, TN, false, true>(P, local, lds);
}

template <int TM, int TN>
constexpr size_t gemm_lds_bytes()
{
    const size_t stages = 2 * (64 * TM + 64 * TN) * LDF * sizeof(float);   // same size for LDH bf16 rows
    const size_t tile = (size_t)(64 * TM) * (64 * TN + 1) * sizeof(float);
    return stages > tile ? stages : tile;
}

template <int TM, int TN, int DT>
static hipError_t launch_one(const GemmProblem *probs_dev, const int *tile_start_dev, int n_probs, int total_wgs,
                             hipStream_t s)
{
    static_assert(2 * LDH == 4 * LDF, "bf16 and fp32 stages have the same size");
    constexpr size_t lds_bytes = gemm_lds_bytes<TM, TN>();
    static_assert(3 * (64 * TM + 64 * TN) * LDQ * sizeof(unsigned short) <= gemm_lds_bytes<TM, TN>(), "the three planes fit");
    static_assert(3 * KT * (64 * TM + 16 + 64 * TN + 16) * sizeof(unsigned short) <= gemm_lds_bytes<TM, TN>(), "and so do the transposed ones");
    auto kernel = DT == 0 ? gemm_nt_f32_kernel<TM, TN> : DT == 2 ? gemm_nt_f32_split_kernel<TM, TN>
                  : DT == 3 ? gemm_nt_f32_split_trans_kernel<TM, TN> : DT == 4 ? gemm_nt_bf16_trans_kernel<TM, TN>
                  : gemm_nt_bf16_kernel<TM, TN>;
    static bool configured = false;   // the attribute is per function, set once per process
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kernel<<<dim3(total_wgs), dim3(256), lds_bytes, s>>>(probs_dev, tile_start_dev, n_probs);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmProblem *probs_dev, const int *tile_start_dev, int n_probs,
                       int total_wgs, int tile_cfg, int dtype, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    if (dtype == 0) {
        if (tile_cfg == 0) return launch_one<2, 2, 0>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
        return launch_one<1, 1, 0>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    }
    if (dtype == 4) {   // bf16 operands stored transposed
        if (tile_cfg == 0) return launch_one<2, 2, 4>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
        return launch_one<1, 1, 4>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    }
    if (dtype == 3) {   // the same on operands stored transposed
        if (tile_cfg == 0) return launch_one<2, 2, 3>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
        return launch_one<1, 1, 3>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    }
    if (dtype == 2) {   // fp32 operands, products through three bf16 planes
        if (tile_cfg == 0) return launch_one<2, 2, 2>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
        return launch_one<1, 1, 2>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    }
    if (tile_cfg == 0) return launch_one<2, 2, 1>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
    return launch_one<1, 1, 1>(probs_dev, tile_start_dev, n_probs, total_wgs, s);
}

hipError_t launch_gemm_reduce(const GemmProblem *probs_dev, const int *red_start_dev, int n_probs,
                              int total_wgs, hipStream_t s)
{
    if (total_wgs <= 0) return hipSuccess;
    gemm_reduce_kernel<<<dim3(total_wgs), dim3(256), 0, s>>>(probs_dev, red_start_dev, n_probs);
    return hipGetLastError();
}

}  // namespace kfac
