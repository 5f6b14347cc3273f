/*
 * kfac.h -- C ABI of the MI355X (gfx950) K-FAC hot path.
 *
 * One natural-gradient step of SP-NGD (arXiv 2002.06015) for the layers that
 * live on one GPU: Kronecker factors A and G of every Conv/FC layer (Sec. 3.3),
 * their running averages, the pi-split damped inverses (Eq. 12), the
 * preconditioned gradient G^-1 dW A^-1 (Eq. 6 with Eq. 7), and the unit-wise
 * 2x2 Fisher of BatchNorm scale/shift (Sec. 4.2).
 *
 * General rules for every entry point
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host"
 *     pointers are ordinary host memory, read during the call only.
 *   - Every entry point that takes a layer list processes all listed layers in
 *     a few grouped launches; per-layer device pointers are passed as HOST
 *     arrays of device pointers.
 *   - All work is enqueued on the HIP stream given to kfac_create (internal streams
 *     are joined into it before a call returns); calls return without waiting for
 *     their own work (see kfac_create for the bounded run-ahead of the host).  A
 *     context is used by one host thread at a time.
 *   - The library allocates no device memory: scratch comes from the caller's
 *     workspace (size from kfac_workspace_bytes for the same layer list).  What
 *     kfac_create allocates besides is listed there.
 *   - Matrices are dense, row-major, leading dimension = number of columns.
 *     Factors and inverses are stored in full (both triangles, exactly symmetric).
 *   - Argument errors are found before anything is launched and leave all
 *     buffers untouched.  Numerical failure (a non-positive pivot) is reported
 *     through the device array `info`, never by aborting.
 *   - Outputs must not overlap inputs unless stated.
 *   - Arithmetic of the dense contractions on fp32 operands (factors, Schur
 *     products of the inversion, preconditioning): fp32 accumulation of products
 *     that are exact to fp32 rounding.  By default an fp32 operand is split
 *     exactly into three bf16 planes and each block product is formed by six bf16
 *     matrix instructions (every term above 2^-23 of the product kept); a context
 *     created with kfac_options.fp32_products = KFAC_PRODUCTS_FP32_MFMA uses the
 *     fp32 matrix instruction instead.  Range of the default mode: operands of
 *     magnitude 2^-110 and above keep every bit; smaller ones lose low bits step by
 *     step (2^-120: about 4e-5 relative) and fp32 subnormals are lost; an infinite
 *     operand gives NaN where the fp32 instruction gives infinity.  Results of the two agree to fp32
 *     rounding of the accumulation.  bf16 operands (kfac_dtype KFAC_BF16) are
 *     multiplied as they are.
 */
#ifndef KFAC_H
#define KFAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KFAC_OK = 0,
    KFAC_ERR_INVALID = 1,    /* null pointer, bad dimension, bad scalar */
    KFAC_ERR_WORKSPACE = 2,  /* caller's workspace is too small for this call */
    KFAC_ERR_NOT_PD = 3,     /* reserved for host-side reporting by callers that read `info` */
    KFAC_ERR_DEVICE = 4      /* a HIP runtime call failed */
} kfac_status;

typedef enum {
    KFAC_F32 = 0,            /* activations / output gradients are float32 */
    KFAC_BF16 = 1            /* ... are bfloat16 (products exact in fp32, fp32 accumulation) */
} kfac_dtype;

/*
 * One Conv or FC layer (Sec. 3.3).  A fully-connected layer is k=1, stride=1,
 * pad=0, h_in=w_in=1.  Square kernels, zero padding, dilation 1, output size
 * h = floor((h_in + 2 pad - k)/stride) + 1.  dA = c_in*k*k + bias, dG = c_out.
 * bias != 0 appends a constant-one row LAST to the patch matrix (the paper
 * drops the bias; this is the homogeneous-coordinate extension), so A gains a
 * row/column and the last column of grad_W is the bias gradient.
 */
typedef struct {
    int32_t N;        /* samples in the local mini-batch */
    int32_t c_in, c_out;
    int32_t k, stride, pad;
    int32_t h_in, w_in;
    int32_t bias;     /* 0 or 1 */
} kfac_layer;

typedef struct kfac_ctx kfac_ctx;

/*
 * How the fp32 contractions are formed and how a context schedules its launches.  None of
 * this changes what is computed (results of different settings agree to fp32 rounding of the
 * accumulations).  kfac_options_default fills in the defaults; a NULL options pointer means
 * the defaults.  The library reads no environment variables and keeps no state outside a context.
 */
typedef enum {
    KFAC_PRODUCTS_SPLIT_BF16 = 0, /* fp32 operands split exactly into three bf16 planes, six bf16 matrix
                                     instructions per block product, fp32 accumulation (default) */
    KFAC_PRODUCTS_FP32_MFMA = 1   /* the fp32 matrix instruction */
} kfac_products;

typedef struct {
    int32_t struct_size;          /* sizeof(kfac_options); any other value is rejected */
    int32_t fp32_products;        /* kfac_products */
    int32_t streams;              /* 1..4: HIP streams a call may use at once (the context's + internal ones); 4 */
    int32_t staging_slots;        /* 2..8: calls the host may run ahead of the device; 2 */
    int32_t correlation_form;     /* A factor of 3x3 / stride 1 / pad 1 layers from displaced image correlations; 1 */
    int32_t pipeline_phases;      /* kfac_step: factor phases spread over the streams; 1 */
    int32_t early_n;              /* kfac_step: layers with a factor at least this large are built and inverted first; 2048 */
    int32_t target_workgroups;    /* split along K until a product has this many workgroups; 128 */
    int32_t min_k_per_split;      /* ... but no part shorter than this; 512 */
    int32_t max_k_per_workgroup;  /* ... and none longer than this; 4096 */
    int32_t recursion_leaf;       /* 32..288: the blocked inversion recurses down to blocks of this size; 288 */
    int32_t force_tile;           /* 0: chosen per product; 64 / 128: every product with that tile */
    int32_t group_by_depth;       /* kfac_invert: layers share a stream with layers whose chains are as long (1) or
                                     the streams get equal sums of n^3 (0); 1 */
    float chunk_gflop;            /* kfac_step: factor launches beside long inversion chains in parts of this size; 48 */
} kfac_options;

void kfac_options_default(kfac_options *opt);

const char *kfac_status_string(kfac_status s);

/* Validates a layer and returns its derived sizes (any out pointer may be NULL). Host only. */
kfac_status kfac_layer_dims(const kfac_layer *L, int32_t *dA, int32_t *dG, int32_t *h, int32_t *w);

/*
 * Bytes of device workspace that any single call below needs for the layer list
 * L[0..n_layers) with inputs of type `in`.  Returns 0 on invalid arguments.  Host only.
 */
size_t kfac_workspace_bytes(const kfac_layer *L, int32_t n_layers, kfac_dtype in);
/* The same for a context that will be created with `opt` (the options change the scratch layout). */
size_t kfac_workspace_bytes_opt(const kfac_layer *L, int32_t n_layers, kfac_dtype in, const kfac_options *opt);

/*
 * Exactly what one kfac_step call with this invert_mask (host uint8 [n_layers] or NULL = all)
 * takes from the workspace.  kfac_workspace_bytes is sized for the separate calls exactly and
 * for kfac_step with a margin over every mask tried (the scratch of a masked plan varies by a
 * few percent with the mask); a caller that changes the mask from step to step (Algorithm 1)
 * can check a mask here.  Every call checks its own plan and returns KFAC_ERR_WORKSPACE before
 * launching anything if the workspace is too small.  Host only; 0 on invalid arguments.
 */
size_t kfac_step_workspace_bytes(const kfac_layer *L, int32_t n_layers, kfac_dtype in, const uint8_t *invert_mask,
                                 const kfac_options *opt);

/*
 * Creates a context bound to a HIP stream (hipStream_t passed as void*, NULL =
 * the default stream) and a caller-owned device workspace (256-byte aligned), on the
 * current device.  kfac_create also creates what the context needs beyond the workspace:
 * three internal streams (default priority), the events that order them, and a ring of
 * `staging_slots` pinned host buffers of 1 MiB through which a call's tables (its layer
 * list turned into kernel arguments) reach the device.  Nothing is allocated after that,
 * with one exception: a call whose tables exceed 1 MiB (layer lists of several thousand
 * layers) re-allocates its staging buffer.  On a machine without a GPU the context is
 * created without these (argument validation needs none).
 * Host blocking: a call enqueues its work and returns, but it first waits until the device
 * has started the call made `staging_slots` calls earlier on this context (its staging
 * buffer is reused); with the default of 2 the host runs at most two calls ahead.
 * kfac_create_opt: the same with explicit options (NULL = defaults).
 */
kfac_status kfac_create(kfac_ctx **out, void *hip_stream, void *workspace_dev, size_t workspace_bytes);
kfac_status kfac_create_opt(kfac_ctx **out, void *hip_stream, void *workspace_dev, size_t workspace_bytes,
                            const kfac_options *opt);
void kfac_destroy(kfac_ctx *ctx);

/*
 * Patch extraction, Sec. 3.3 Eq. 10:  M_A = im2col(A) in R^{c_in k^2 x h w}.
 * act: dev [N, c_in, h_in, w_in] (NCHW) of type `dt`.  patches: dev, same type,
 * [c_in*k*k, ld] row-major; row r = (c*k + ky)*k + kx, column m = n*h*w + y*w + x
 * holds act[n, c, y*stride+ky-pad, x*stride+kx-pad] (0 outside the image).
 * ld >= N*h*w; columns [N*h*w, ld) are left untouched.  The bias row is not
 * materialised (kfac_stats supplies it on the fly).
 */
kfac_status kfac_im2col(kfac_ctx *ctx, const kfac_layer *L, kfac_dtype dt,
                        const void *act, void *patches, int64_t ld);

/*
 * Factor construction + running average, Sec. 3.3 Eq. 9 (FC) and Eq. 11 (Conv):
 *   A_batch = 1/(N h w) sum_n M_A(n) M_A(n)^T     (with the bias row if L.bias)
 *   G_batch = 1/N sum_n D_n D_n^T,  D_n = grad_out[n] as a c_out x hw matrix
 *             (also divided by h*w if g_spatial_mean != 0; the paper does not)
 *   X_ema  <- decay * X_ema + (1 - decay) * X_batch         (0 <= decay < 1;
 *             decay == 0 overwrites and never reads the old contents)
 * act[l]:      dev [N, c_in, h_in, w_in] of type `in`, or NULL to skip A of layer l
 *              (act == NULL skips A for all layers).
 * grad_out[l]: dev [N, c_out, h, w] of type `in`: PER-SAMPLE gradient of log p
 *              w.r.t. the layer output (unscaled by 1/N); NULL skips G.
 * A_ema[l]:    dev in/out [dA, dA] fp32;  G_ema[l]: dev in/out [dG, dG] fp32.
 * E[.] is the mean over the N local samples.
 */
kfac_status kfac_stats(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                       const void *const *act, const void *const *grad_out,
                       float decay, int32_t g_spatial_mean,
                       float *const *A_ema, float *const *G_ema);

/*
 * Damped inversion of both factors, Sec. 3.3 Eq. 12 (right-hand side):
 *   pi^2 = (tr A_ema / dA) / (tr G_ema / dG)   (pi = 1 if a trace is not positive)
 *   A_inv = (A_ema + pi*gamma I)^-1,   G_inv = (G_ema + gamma/pi I)^-1,
 * gamma = sqrt(lambda) >= 0.  The stored running averages are not modified.
 * A_inv[l], G_inv[l]: dev out, full symmetric.  pi_out: dev [n_layers] or NULL.
 * info: dev int32 [2*n_layers] or NULL; info[2l] (A) / info[2l+1] (G) is 0, or
 * the 1-based index of a non-positive pivot (the matrix was not positive
 * definite; its inverse is then meaningless).
 * Passing a subset of the layers refreshes only their inverses (Algorithm 1).
 */
kfac_status kfac_invert(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L,
                        const float *const *A_ema, const float *const *G_ema, float gamma,
                        float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info);

/*
 * Natural-gradient direction, Eq. 6 with F = G (x) A (Eq. 7) and Eq. 12, in
 * matrix form for W in R^{dG x dA} (row = output channel):
 *   out = G_inv * grad_W * A_inv .
 * G_inv[l]: dev [dG, dG], A_inv[l]: dev [dA, dA], both symmetric (as kfac_invert
 * writes them; the products read them along rows, so a non-symmetric matrix
 * would enter transposed).  grad_W[l], out[l]: dev [dG, dA]; out[l] may equal
 * grad_W[l].
 */
kfac_status kfac_precondition(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L,
                              const float *const *G_inv, const float *const *A_inv,
                              const float *const *grad_W, float *const *out);

/*
 * One whole step for a layer list (Algorithm 1, one iteration on one GPU): exactly
 *   kfac_stats(all layers) -> kfac_invert(layers with invert_mask[l] != 0)
 *   -> kfac_precondition(all layers, with the inverses then stored in A_inv / G_inv)
 * with the same arguments and the same results up to the rounding order of the
 * contractions, but planned as one dependency graph: the factors of the layers
 * with the largest matrices are built first and their inversions (long chains of
 * small launches) run on internal streams underneath the remaining factor
 * contractions.  Use it when nothing else has to happen between the three stages
 * (a multi-GPU caller that reduces the factors between stages uses the separate
 * calls).  invert_mask: host uint8 [n_layers] or NULL (invert every layer); layers
 * not inverted keep the inverses their buffers hold (stale statistics, Sec. 4.3).
 * pi_out: dev [n_layers] or NULL, info: dev int32 [2*n_layers] or NULL, both
 * indexed by position in the layer list; entries of layers not inverted: pi_out
 * untouched, info 0.  No argument may be NULL otherwise.  On return every stream
 * the call used internally has been joined into the context's stream.
 */
kfac_status kfac_step(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                      const void *const *act, const void *const *grad_out,
                      float decay, int32_t g_spatial_mean,
                      float *const *A_ema, float *const *G_ema,
                      const uint8_t *invert_mask, float gamma,
                      float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info,
                      const float *const *grad_W, float *const *out);

/*
 * Unit-wise natural gradient for BatchNorm, Sec. 4.2 Eq. 15-17.  Per layer l
 * and channel i, with per-sample gradients gg = g_gamma[l][n, i], gb = g_beta[l][n, i]:
 *   F_batch = mean_n (gg^2, gg*gb, gb^2);  F_ema[l][i, 0..2] <- decay F_ema + (1-decay) F_batch
 *   [out_gamma, out_beta] = (F + lambda I)^-1 [mean_n gg, mean_n gb]   (2x2 closed form)
 * g_gamma[l], g_beta[l]: dev [N, C[l]];  F_ema[l]: dev in/out [C[l], 3];
 * out_gamma[l], out_beta[l]: dev [C[l]].  C: host array.  lambda >= 0 is used as is.
 */
kfac_status bn_unitwise_precondition(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                     const float *const *g_gamma, const float *const *g_beta,
                                     float decay, float lambda, float *const *F_ema,
                                     float *const *out_gamma, float *const *out_beta);

/*
 * Natural gradient for BatchNorm with the Fisher block of the whole layer (Sec. 4.2, the
 * 2c x 2c matrix that the unit-wise approximation replaces; "fullBN" in Sec. 7).  With
 * g_n = (g_gamma[n,0], g_beta[n,0], ..., g_gamma[n,c-1], g_beta[n,c-1]) the per-sample
 * gradient in the order of the layer's parameter vector:
 *   F_ema[l] <- decay F_ema[l] + (1-decay) (1/N) sum_n g_n g_n^T      (decay == 0: F_ema is not read)
 *   F_inv[l] <- (F_ema[l] + lambda I)^-1      for layers with invert_mask[l] != 0
 *   (out_gamma[l][i], out_beta[l][i]) = rows 2i, 2i+1 of F_inv[l] mean_n g_n
 * g_gamma[l], g_beta[l]: dev [N, C[l]];  F_ema[l]: dev in/out [2C, 2C];  F_inv[l]: dev
 * [2C, 2C], out for inverted layers and in otherwise (stale inverse, Sec. 4.3), must
 * not be F_ema[l];  out_gamma[l], out_beta[l]: dev [C[l]].  invert_mask: host uint8
 * [n_layers] or NULL (all).  info: dev int32 [n_layers] or NULL, 0 or the first
 * non-positive pivot (1-based) as for kfac_invert.  C: host, 1 <= C[l] <= 32768.
 * Scratch comes from the context's workspace: bn_full_workspace_bytes reports the size
 * (0 for invalid arguments) that serves every layer inverted and any one layer alone;
 * KFAC_ERR_WORKSPACE before any launch if a call needs more than the context has.
 */
size_t bn_full_workspace_bytes(int32_t n_layers, int32_t N, const int32_t *C);
kfac_status bn_full_precondition(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                 const float *const *g_gamma, const float *const *g_beta,
                                 float decay, float lambda, float *const *F_ema,
                                 const uint8_t *invert_mask, float *const *F_inv, int32_t *info,
                                 float *const *out_gamma, float *const *out_beta);

/*
 * Producer of the per-sample BatchNorm gradients used above (Sec. 4.2): for
 * y = gamma*xhat + beta,  g_gamma[n, c] = sum_t dy[n,c,t]*xhat[n,c,t],
 * g_beta[n, c] = sum_t dy[n,c,t].  dy[l], xhat[l]: dev fp32 [N, C[l], HW[l]];
 * g_gamma[l], g_beta[l]: dev out [N, C[l]].
 */
kfac_status bn_unitwise_reduce_nchw(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                    const int32_t *HW, const float *const *dy, const float *const *xhat,
                                    float *const *g_gamma, float *const *g_beta);
/* The same from tensors kept in NHWC (Sec. 5.2): dy[l], xhat[l]: dev fp32 [N, HW[l], C[l]]. */
kfac_status bn_unitwise_reduce_nhwc(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                    const int32_t *HW, const float *const *dy, const float *const *xhat,
                                    float *const *g_gamma, float *const *g_beta);

/*
 * Staleness of statistics, Sec. 4.3 (the similarity criterion under Algorithm 2).
 * For each of n dense matrices X[i] of dims[i] x dims[i] floats (a Kronecker factor,
 * an inverse, any statistic the caller refreshes) and its two predecessors:
 *   ratios[2i]     = ||X[i] - X_m1[i]||_F / ||X_m1[i]||_F
 *   ratios[2i + 1] = ||X[i] - X_m2[i]||_F / ||X_m2[i]||_F
 * X[i] is "similar to" a predecessor when the ratio is below the threshold alpha
 * (0.1 in the paper's experiments).  A predecessor that does not exist yet is passed
 * as NULL (the array itself may be NULL: none exists) and gives +infinity; a
 * predecessor of norm 0 gives 0 if X[i] equals it and +infinity otherwise.
 * dims, X, X_m1, X_m2: host arrays (X, X_m1, X_m2 of device pointers);
 * ratios: dev out [2 n] doubles.  Sums are accumulated in double in a fixed order
 * (the same inputs give the same bits).  Uses 32 bytes of the workspace per 4096
 * matrix elements (KFAC_ERR_WORKSPACE if it does not fit).
 */
kfac_status kfac_staleness(kfac_ctx *ctx, int32_t n, const int32_t *dims, const float *const *X,
                           const float *const *X_m1, const float *const *X_m2, double *ratios);

/*
 * kfac_staleness for callers that cannot allocate: code under HIP graph capture, tight
 * serving or training loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * (the same kernels' arithmetic in the same order), but no context and no workspace: the
 * per-chunk sums go to a fixed 512 KiB device array inside the library (one copy per GPU,
 * held until the process ends) and the job table travels in the kernel arguments.  The call
 * allocates nothing (no hipMalloc / hipFree / hipHostMalloc, no events or streams); work is
 * enqueued on `hip_stream` (hipStream_t as void*, NULL = the default stream) of the current
 * device and the call returns without waiting.
 * Limit: one matrix may have at most 2^26 elements (dims[i] <= 8192); a larger one gives
 * KFAC_ERR_WORKSPACE before anything is launched.  Any number of matrices: they are
 * processed in successive launches that reuse the array in stream order.
 * All calls on one GPU share that GPU's array: two calls that may run at the same time on
 * one GPU (different streams, different host threads) race on it and must be ordered by the
 * caller.  Nothing in the array has to start at zero (every sum is written before it is read).
 */
kfac_status kfac_staleness_static(void *hip_stream, int32_t n, const int32_t *dims, const float *const *X,
                                  const float *const *X_m1, const float *const *X_m2, double *ratios);

/*
 * Learning rate and momentum schedules, Sec. 6.2 (host only, no GPU work):
 *   kfac_lr_polynomial:    eta(e) = eta0 (1 - (e - e_start) / (e_end - e_start))^p_decay  for
 *                          e_start <= e <= e_end; eta0 before e_start, 0 after e_end
 *   kfac_momentum_coupled: m(e) = m0 / eta0 * eta(e)   (the ratio m / eta stays fixed)
 * NaN for e_end <= e_start or eta0 == 0 respectively.
 */
double kfac_lr_polynomial(double eta0, double e, double e_start, double e_end, double p_decay);
double kfac_momentum_coupled(double m0, double eta0, double eta);

/*
 * Parameter update and weight rescaling, Sec. 6.2 Eq. "paramupdate" and Sec. 6.3.
 * Per layer l, with the preconditioned gradient U[l] (as kfac_precondition writes it):
 *   w' = W[l] - eta U[l] + momentum (W[l] - W_prev[l]);   W_prev[l] <- W[l];   W[l] <- w'
 * and, if rescale != 0,  W[l] <- sqrt(2 c_out) W[l] / (||W[l]||_F + eps)  (the paper uses
 * eps = 1e-9).  W[l], W_prev[l]: dev in/out, U[l]: dev in, all [dG, dA] floats
 * (the layer's weights as a matrix, bias column last if it has one); the three must
 * not overlap.  Arithmetic in fp32 (fused multiply-adds), the norm accumulated in
 * double in a fixed order.  Uses 8 bytes of the workspace per 4096 weights plus 4 per
 * layer when rescaling.
 */
kfac_status kfac_update_weights(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, const float *const *U,
                                float eta, float momentum, int32_t rescale, float eps, float *const *W,
                                float *const *W_prev);

/*
 * Convolution inputs kept in NHWC (Sec. 5.2 names that layout for the tensors around
 * convolution layers): converts them to the NCHW layout kfac_stats, kfac_step and kfac_im2col
 * read.  which = 0: activations, src[l] dev [N, h_in, w_in, c_in] -> dst[l] dev [N, c_in, h_in, w_in];
 * which = 1: output gradients, src[l] dev [N, h, w, c_out] -> dst[l] dev [N, c_out, h, w].
 * type: element type of both (fp32 or bf16); bits are copied unchanged.  src[l] == NULL skips
 * layer l (dst[l] is not touched); src[l] and dst[l] must not overlap.  For fully-connected
 * layers (h = w = 1) the two layouts coincide and the call copies.
 */
kfac_status kfac_nhwc_to_nchw(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, int32_t which, kfac_dtype type,
                              const void *const *src, void *const *dst);

/*
 * kfac_stats and kfac_step on tensors kept in NHWC (Sec. 5.2): act[l] dev [N, h_in, w_in, c_in],
 * grad_out[l] dev [N, h, w, c_out]; every other argument, every result and every error as for
 * kfac_stats / kfac_step (the statistics of Sec. 3.3 do not depend on the storage order).
 * Tensors of pointwise layers (1 x 1, stride 1, no padding, fully connected) and all output
 * gradients are contracted where they are if their channel count is a whole number of 16-byte
 * chunks (fp32: a multiple of 4, and the context forms products in its default mode
 * KFAC_PRODUCTS_SPLIT_BF16; bf16: a multiple of 8 and a 16-byte aligned pointer); all other
 * tensors are first brought into NCHW order inside the workspace (the conversion of
 * kfac_nhwc_to_nchw, the scratch is part of kfac_workspace_bytes).
 */
kfac_status kfac_stats_nhwc(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                            const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                            float *const *A_ema, float *const *G_ema);
kfac_status kfac_step_nhwc(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                           const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                           float *const *A_ema, float *const *G_ema, const uint8_t *invert_mask, float gamma,
                           float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info,
                           const float *const *grad_W, float *const *out);

/*
 * Symmetry-aware packing of the statistics, Sec. 5.2: a symmetric d x d matrix is
 * communicated as its upper triangle, d (d + 1) / 2 elements.  Layout of `packed`
 * (the paper fixes only the count): matrix i starts at element sum_{j<i} d_j (d_j + 1) / 2;
 * inside it row r contributes X[r][r], X[r][r+1], ..., X[r][d-1], rows in order.
 * kfac_packed_elems: the total number of elements (0 for invalid arguments).
 * kfac_pack_upper: X[i] (dev, dense d_i x d_i floats; only the upper triangle is read)
 * -> packed (dev, type floats or, for KFAC_BF16, bfloat16 rounded to nearest, ties to
 * even).  kfac_unpack_upper: packed -> X[i], both triangles written (exactly symmetric).
 * dims, X: host arrays.  X[i] must not overlap `packed`.  fp32 packing is a bit-exact copy.
 */
size_t kfac_packed_elems(int32_t n, const int32_t *dims);
kfac_status kfac_pack_upper(kfac_ctx *ctx, int32_t n, const int32_t *dims, const float *const *X,
                            kfac_dtype type, void *packed);
kfac_status kfac_unpack_upper(kfac_ctx *ctx, int32_t n, const int32_t *dims, kfac_dtype type,
                              const void *packed, float *const *X);

/*
 * Algorithm 2 (Sec. 4.3): the acceptable interval, in steps, until a statistic is
 * refreshed next.  delta_m1: its last interval, delta_m2: the one before (both >= 1).
 *   not similar to the last value:                       max(1, delta_m1 / 2)
 *   similar to the last, not to the one before the last: delta_m1
 *   similar to both:                                     delta_m1 + delta_m2
 * Host only, no GPU work.  Returns 0 for an interval argument below 1.
 */
int32_t kfac_next_interval(int32_t similar_to_last, int32_t similar_to_before_last, int32_t delta_m1,
                           int32_t delta_m2);

/*
 * What Algorithm 1 (Sec. 4.3) keeps per statistic: the step t_X of its next refresh
 * and its two most recent intervals.  kfac_refresh_init: t_X = 1 and both intervals 1
 * (the paper leaves the initial intervals open).  kfac_refresh_due: t == t_X.
 * kfac_refresh_advance, called after the statistic has been recomputed at step t_X and
 * compared with its predecessors (ratios as kfac_staleness writes them, alpha > 0):
 * the interval of Algorithm 2 becomes the last interval and t_X moves on by it.
 * Host only; all three ignore a NULL state.
 */
typedef struct {
    int32_t t_next;    /* t_X */
    int32_t delta;     /* the last interval */
    int32_t delta_m1;  /* the interval before the last */
} kfac_refresh_state;
void kfac_refresh_init(kfac_refresh_state *s, int32_t n);
int32_t kfac_refresh_due(const kfac_refresh_state *s, int32_t t);
void kfac_refresh_advance(kfac_refresh_state *s, double ratio_m1, double ratio_m2, double alpha);

/*
 * Optional per-launch timing for benchmarks (not part of the method).  While enabled,
 * every kernel launch of this context is bracketed by HIP events on the context's stream.
 * kfac_profile_read waits for the stream, copies up to max_entries records (in launch
 * order) to the host array `out`, clears the log and returns the number of launches
 * that were recorded (which may exceed max_entries), or -1 on error.
 * flops / bytes are the algorithmic counts of the launch: K*M*(M+1) for a symmetric
 * product, 2*M*N*K for a general one; bytes read + written for the copy-like kernels.
 */
typedef enum {
    KFAC_K_GEMM_F32 = 0, KFAC_K_GEMM_BF16 = 1, KFAC_K_GEMM_REDUCE = 2, KFAC_K_PATCH = 3, KFAC_K_TRACE = 4,
    KFAC_K_COPY_DAMP = 5, KFAC_K_LEAF_INVERSE = 6, KFAC_K_ZERO = 7, KFAC_K_BN_UNIT = 8, KFAC_K_BN_REDUCE = 9,
    KFAC_K_PAD = 10, KFAC_K_ASSEMBLE = 11, KFAC_K_BORDER = 12, KFAC_K_STALENESS = 13, KFAC_K_PACK = 14, KFAC_K_UPDATE = 15, KFAC_K_BN_FULL = 16, KFAC_K_LAYOUT = 17, KFAC_K_GEMM_F32_SPLIT = 18
} kfac_kernel;

typedef struct {
    int32_t kernel;    /* kfac_kernel */
    int32_t variant;   /* GEMM: 0 = 128x128 tiles, 1 = 64x64 tiles; leaf inverse: size class */
    int32_t workgroups;
    float ms;
    double flops;
    double bytes;
    float start_ms;    /* start of the launch, measured from the start of the first recorded launch */
    int32_t stream;    /* 0: the context's stream, 1..3: internal streams */
} kfac_profile_entry;

kfac_status kfac_profile_enable(kfac_ctx *ctx, int32_t on);
int32_t kfac_profile_read(kfac_ctx *ctx, kfac_profile_entry *out, int32_t max_entries);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H */
