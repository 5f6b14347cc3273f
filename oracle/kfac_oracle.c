/*
 * kfac_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, float64 CPU statement of what one K-FAC-style natural-gradient
 * step computes for one layer (SP-NGD, arXiv 2002.06015).  It exists so that the
 * GPU library can be checked against something that can be read side by side
 * with the paper.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper
 * with the GPU path; it takes host pointers to doubles only.
 *
 * Every loop below is the definition written out: no blocking, no fusion, no
 * reordering beyond "row i of the result is independent of row j" (which is
 * where the OpenMP pragmas sit).
 *
 * Conventions (readings of points the paper leaves open are marked READING):
 *   - E[.] is the mean over the N samples of the local mini-batch
 *     (Sec. 3.1 "Mini-batch Stochastic Learning").
 *   - im2col rows are ordered (c, ky, kx), i.e. the flattening of an
 *     [c_out, c_in, k, k] weight into W in R^{c_out x c_in k^2} (Sec. 3.3,
 *     the convolution forward equation, Eq. 10).  READING: zero padding,
 *     dilation 1, floor output size.
 *   - READING (bias): the paper drops the bias for simplicity; with bias=1 a
 *     constant-one row is appended LAST to every patch matrix, so A gains one
 *     row/column and grad_W's last column is the bias gradient.
 *   - READING (running average): X_ema <- decay*X_ema + (1-decay)*X_batch.
 *   - READING (average eigenvalue): trace / dimension of the undamped
 *     running-average factor; pi := 1 if either trace is not positive.
 *
 * Return codes: 0 ok, 1 invalid argument, 3 matrix not positive definite.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_INVALID 1
#define ORC_NOT_PD 3

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Output spatial size of a convolution: floor((in + 2 pad - k)/stride) + 1. */
int oracle_out_size(int in, int k, int stride, int pad)
{
    if (in < 1 || k < 1 || stride < 1 || pad < 0) return -1;
    int num = in + 2 * pad - k;
    if (num < 0) return -1;
    return num / stride + 1;
}

/*
 * Patch matrix of ONE sample (Sec. 3.3, Eq. 10: M_A = im2col(A) in
 * R^{c_in k^2 x h w}).  act_n: [c_in, h_in, w_in]; P: [dA, h*w] row-major with
 * dA = c_in k^2 + bias.  Row r = (c*k + ky)*k + kx, column t = y*w + x.
 */
static void im2col_one(int c_in, int k, int s, int p, int h_in, int w_in, int bias,
                       int h, int w, const double *act_n, double *P)
{
    const int hw = h * w;
    for (int c = 0; c < c_in; ++c)
        for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
                const int r = (c * k + ky) * k + kx;
                for (int y = 0; y < h; ++y)
                    for (int x = 0; x < w; ++x) {
                        const int iy = y * s + ky - p;
                        const int ix = x * s + kx - p;
                        double v = 0.0;
                        if (iy >= 0 && iy < h_in && ix >= 0 && ix < w_in)
                            v = act_n[((size_t)c * h_in + iy) * w_in + ix];
                        P[(size_t)r * hw + y * w + x] = v;
                    }
            }
    if (bias)
        for (int t = 0; t < hw; ++t) P[(size_t)(c_in * k * k) * hw + t] = 1.0;
}

/* All samples: P is [N, dA, h*w]. Exposed for the tests. */
int oracle_im2col(int N, int c_in, int k, int s, int p, int h_in, int w_in, int bias,
                  const double *act, double *P)
{
    const int h = oracle_out_size(h_in, k, s, p), w = oracle_out_size(w_in, k, s, p);
    if (N < 1 || c_in < 1 || h < 1 || w < 1 || !act || !P) return ORC_INVALID;
    const size_t dA = (size_t)c_in * k * k + (bias ? 1 : 0);
    for (int n = 0; n < N; ++n)
        im2col_one(c_in, k, s, p, h_in, w_in, bias, h, w,
                   act + (size_t)n * c_in * h_in * w_in, P + (size_t)n * dA * h * w);
    return ORC_OK;
}

/*
 * Activation factor of one mini-batch (Sec. 3.3, Eq. 11, and Eq. 9 for a
 * fully-connected layer, which is the case k=1, h=w=1):
 *     A = 1/(h w) * (1/N) sum_n  M_A(n) M_A(n)^T .
 * A_batch: [dA, dA] row-major.
 */
int oracle_factor_A(int N, int c_in, int k, int s, int p, int h_in, int w_in, int bias,
                    const double *act, double *A_batch)
{
    const int h = oracle_out_size(h_in, k, s, p), w = oracle_out_size(w_in, k, s, p);
    if (N < 1 || c_in < 1 || h < 1 || w < 1 || !act || !A_batch) return ORC_INVALID;
    const int hw = h * w;
    const int dA = c_in * k * k + (bias ? 1 : 0);
    double *P = (double *)malloc((size_t)dA * hw * sizeof(double));
    if (!P) return ORC_INVALID;
    memset(A_batch, 0, (size_t)dA * dA * sizeof(double));
    for (int n = 0; n < N; ++n) {
        im2col_one(c_in, k, s, p, h_in, w_in, bias, h, w,
                   act + (size_t)n * c_in * h_in * w_in, P);
#pragma omp parallel for schedule(dynamic, 4)
        for (int i = 0; i < dA; ++i)
            for (int j = 0; j < dA; ++j) {
                double acc = 0.0;
                for (int t = 0; t < hw; ++t) acc += P[(size_t)i * hw + t] * P[(size_t)j * hw + t];
                A_batch[(size_t)i * dA + j] += acc;
            }
    }
    const double scale = 1.0 / ((double)N * (double)hw);
    for (size_t e = 0; e < (size_t)dA * dA; ++e) A_batch[e] *= scale;
    free(P);
    return ORC_OK;
}

/*
 * Output-gradient factor of one mini-batch (Sec. 3.3, Eq. 11 / Eq. 9):
 *     G = (1/N) sum_n  D_n D_n^T ,   D_n = grad_out[n] in R^{c_out x h w}
 * (per-sample gradient of log p w.r.t. the layer output, as a c_out x hw
 * matrix).  The paper puts no 1/(hw) on G; READING: spatial_mean != 0 divides
 * by h*w as well (the benchmark configurations ask for gradients "averaged
 * over spatial positions").
 */
int oracle_factor_G(int N, int c_out, int hw, int spatial_mean, const double *grad_out,
                    double *G_batch)
{
    if (N < 1 || c_out < 1 || hw < 1 || !grad_out || !G_batch) return ORC_INVALID;
    memset(G_batch, 0, (size_t)c_out * c_out * sizeof(double));
    for (int n = 0; n < N; ++n) {
        const double *D = grad_out + (size_t)n * c_out * hw;
#pragma omp parallel for schedule(dynamic, 4)
        for (int i = 0; i < c_out; ++i)
            for (int j = 0; j < c_out; ++j) {
                double acc = 0.0;
                for (int t = 0; t < hw; ++t) acc += D[(size_t)i * hw + t] * D[(size_t)j * hw + t];
                G_batch[(size_t)i * c_out + j] += acc;
            }
    }
    double scale = 1.0 / (double)N;
    if (spatial_mean) scale /= (double)hw;
    for (size_t e = 0; e < (size_t)c_out * c_out; ++e) G_batch[e] *= scale;
    return ORC_OK;
}

/*
 * Single entries of the two factors, each computed on its own straight from
 * the definition (no patch matrix is formed): used to spot-check factors that
 * are too large to rebuild in full.
 */
int oracle_factor_A_entries(int N, int c_in, int k, int s, int p, int h_in, int w_in, int bias,
                            const double *act, int n_pairs, const int32_t *I, const int32_t *J,
                            double *out)
{
    const int h = oracle_out_size(h_in, k, s, p), w = oracle_out_size(w_in, k, s, p);
    if (N < 1 || c_in < 1 || h < 1 || w < 1 || !act || !I || !J || !out) return ORC_INVALID;
    const int d0 = c_in * k * k;
    const int dA = d0 + (bias ? 1 : 0);
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < n_pairs; ++q) {
        const int r[2] = {I[q], J[q]};
        if (r[0] < 0 || r[0] >= dA || r[1] < 0 || r[1] >= dA) { out[q] = NAN; continue; }
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int y = 0; y < h; ++y)
                for (int x = 0; x < w; ++x) {
                    double v[2];
                    for (int e = 0; e < 2; ++e) {
                        if (r[e] == d0) { v[e] = 1.0; continue; }   /* bias row */
                        const int c = r[e] / (k * k), ky = (r[e] / k) % k, kx = r[e] % k;
                        const int iy = y * s + ky - p, ix = x * s + kx - p;
                        v[e] = (iy >= 0 && iy < h_in && ix >= 0 && ix < w_in)
                                   ? act[(((size_t)n * c_in + c) * h_in + iy) * w_in + ix] : 0.0;
                    }
                    acc += v[0] * v[1];
                }
        out[q] = acc / ((double)N * (double)(h * w));
    }
    return ORC_OK;
}

int oracle_factor_G_entries(int N, int c_out, int hw, int spatial_mean, const double *grad_out,
                            int n_pairs, const int32_t *I, const int32_t *J, double *out)
{
    if (N < 1 || c_out < 1 || hw < 1 || !grad_out || !I || !J || !out) return ORC_INVALID;
    for (int q = 0; q < n_pairs; ++q) {
        const int i = I[q], j = J[q];
        if (i < 0 || i >= c_out || j < 0 || j >= c_out) { out[q] = NAN; continue; }
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int t = 0; t < hw; ++t)
                acc += grad_out[((size_t)n * c_out + i) * hw + t] * grad_out[((size_t)n * c_out + j) * hw + t];
        out[q] = acc / (double)N / (spatial_mean ? (double)hw : 1.0);
    }
    return ORC_OK;
}

/* READING (running average; not in the paper): X_ema <- decay X_ema + (1-decay) X_batch. */
int oracle_ema(size_t n_elem, double decay, const double *X_batch, double *X_ema)
{
    if (!X_batch || !X_ema || !(decay >= 0.0 && decay < 1.0)) return ORC_INVALID;
    for (size_t e = 0; e < n_elem; ++e) X_ema[e] = decay * X_ema[e] + (1.0 - decay) * X_batch[e];
    return ORC_OK;
}

/*
 * The first of the four calls: factors of one mini-batch folded into the
 * running averages.  act may be NULL (skip A) and grad_out may be NULL (skip
 * G): in Algorithm 3 A is built in the forward pass and G in the backward pass.
 */
int oracle_kfac_stats(int N, int c_in, int c_out, int k, int s, int p, int h_in, int w_in, int bias,
                      const double *act, const double *grad_out, double decay, int g_spatial_mean,
                      double *A_ema, double *G_ema)
{
    const int h = oracle_out_size(h_in, k, s, p), w = oracle_out_size(w_in, k, s, p);
    if (N < 1 || c_in < 1 || c_out < 1 || h < 1 || w < 1) return ORC_INVALID;
    if (!(decay >= 0.0 && decay < 1.0)) return ORC_INVALID;
    if (act) {
        if (!A_ema) return ORC_INVALID;
        const size_t dA = (size_t)c_in * k * k + (bias ? 1 : 0);
        double *Ab = (double *)malloc(dA * dA * sizeof(double));
        if (!Ab) return ORC_INVALID;
        int rc = oracle_factor_A(N, c_in, k, s, p, h_in, w_in, bias, act, Ab);
        if (rc == ORC_OK) rc = oracle_ema(dA * dA, decay, Ab, A_ema);
        free(Ab);
        if (rc) return rc;
    }
    if (grad_out) {
        if (!G_ema) return ORC_INVALID;
        const size_t dG = (size_t)c_out;
        double *Gb = (double *)malloc(dG * dG * sizeof(double));
        if (!Gb) return ORC_INVALID;
        int rc = oracle_factor_G(N, c_out, h * w, g_spatial_mean, grad_out, Gb);
        if (rc == ORC_OK) rc = oracle_ema(dG * dG, decay, Gb, G_ema);
        free(Gb);
        if (rc) return rc;
    }
    return ORC_OK;
}

/*
 * Damping split (Sec. 3.3 "Inverting Kronecker-factored FIM", Eq. 12 and the
 * sentence after it):  pi^2 = (average eigenvalue of A)/(average eigenvalue of
 * G);  A receives pi*sqrt(lambda), G receives sqrt(lambda)/pi.  gamma :=
 * sqrt(lambda).  Average eigenvalue = trace/dimension.
 */
int oracle_pi_damping(int dA, const double *A, int dG, const double *G, double gamma,
                      double *pi_out, double *damp_A, double *damp_G)
{
    if (dA < 1 || dG < 1 || !A || !G || !(gamma >= 0.0)) return ORC_INVALID;
    double trA = 0.0, trG = 0.0;
    for (int i = 0; i < dA; ++i) trA += A[(size_t)i * dA + i];
    for (int i = 0; i < dG; ++i) trG += G[(size_t)i * dG + i];
    double pi = 1.0;
    if (trA > 0.0 && trG > 0.0) pi = sqrt((trA / dA) / (trG / dG));
    *pi_out = pi;
    *damp_A = pi * gamma;
    *damp_G = gamma / pi;
    return ORC_OK;
}

/*
 * (X + damp I)^{-1} for a symmetric positive definite X + damp I.
 * Cholesky X + damp I = L L^T, then for every unit vector e_c solve
 * L y = e_c and L^T x = y; x is column c of the inverse.  The result is
 * symmetrised at the end.  info: 0, or j+1 if the j-th pivot is not positive.
 */
int oracle_spd_inverse(int n, const double *X, double damp, double *Xinv, int32_t *info)
{
    if (n < 1 || !X || !Xinv) return ORC_INVALID;
    if (info) *info = 0;
    double *L = (double *)calloc((size_t)n * n, sizeof(double));
    double *Lt = (double *)calloc((size_t)n * n, sizeof(double));
    if (!L || !Lt) { free(L); free(Lt); return ORC_INVALID; }
    for (int j = 0; j < n; ++j) {
        double d = X[(size_t)j * n + j] + damp;
        for (int q = 0; q < j; ++q) d -= L[(size_t)j * n + q] * L[(size_t)j * n + q];
        if (!(d > 0.0)) {
            if (info) *info = j + 1;
            free(L); free(Lt);
            return ORC_NOT_PD;
        }
        const double ljj = sqrt(d);
        L[(size_t)j * n + j] = ljj;
#pragma omp parallel for schedule(static)
        for (int i = j + 1; i < n; ++i) {
            /* the lower triangle of X is read; X is symmetric */
            double v = X[(size_t)i * n + j];
            for (int q = 0; q < j; ++q) v -= L[(size_t)i * n + q] * L[(size_t)j * n + q];
            L[(size_t)i * n + j] = v / ljj;
        }
    }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j <= i; ++j) Lt[(size_t)j * n + i] = L[(size_t)i * n + j];
#pragma omp parallel
    {
        double *y = (double *)malloc((size_t)n * sizeof(double));
        double *x = (double *)malloc((size_t)n * sizeof(double));
#pragma omp for schedule(dynamic, 8)
        for (int c = 0; c < n; ++c) {
            for (int i = 0; i < n; ++i) {          /* forward: L y = e_c */
                double v = (i == c) ? 1.0 : 0.0;
                for (int q = 0; q < i; ++q) v -= L[(size_t)i * n + q] * y[q];
                y[i] = v / L[(size_t)i * n + i];
            }
            for (int i = n - 1; i >= 0; --i) {     /* backward: L^T x = y */
                double v = y[i];
                for (int q = i + 1; q < n; ++q) v -= Lt[(size_t)i * n + q] * x[q];
                x[i] = v / Lt[(size_t)i * n + i];
            }
            for (int i = 0; i < n; ++i) Xinv[(size_t)i * n + c] = x[i];
        }
        free(y); free(x);
    }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < i; ++j) {
            const double m = 0.5 * (Xinv[(size_t)i * n + j] + Xinv[(size_t)j * n + i]);
            Xinv[(size_t)i * n + j] = m;
            Xinv[(size_t)j * n + i] = m;
        }
    free(L); free(Lt);
    return ORC_OK;
}

/*
 * The second call: damped inverses of both running-average factors of one
 * layer (Eq. 12, right-hand side):  A_inv = (A + pi gamma I)^{-1},
 * G_inv = (G + gamma/pi I)^{-1}.  info[0] is for A, info[1] for G.
 */
int oracle_kfac_invert(int dA, int dG, const double *A_ema, const double *G_ema, double gamma,
                       double *A_inv, double *G_inv, double *pi_out, int32_t *info)
{
    double pi, da, dg;
    int rc = oracle_pi_damping(dA, A_ema, dG, G_ema, gamma, &pi, &da, &dg);
    if (rc) return rc;
    if (pi_out) *pi_out = pi;
    int32_t ia = 0, ig = 0;
    int rca = oracle_spd_inverse(dA, A_ema, da, A_inv, &ia);
    int rcg = oracle_spd_inverse(dG, G_ema, dg, G_inv, &ig);
    if (info) { info[0] = ia; info[1] = ig; }
    return rca ? rca : rcg;
}

/*
 * The third call: the natural-gradient direction of one layer in matrix form.
 * Eq. 6 applies (F + lambda I)^{-1} to the gradient; with F = G (x) A (Eq. 7),
 * the approximation of Eq. 12 and w = row-major vec of W in R^{dG x dA},
 *     (G_inv (x) A_inv) vec(gradW) = vec(G_inv gradW A_inv)      (A_inv symmetric).
 * U = G_inv * grad_W * A_inv, all row-major; U: [dG, dA].
 */
int oracle_kfac_precondition(int dG, int dA, const double *G_inv, const double *A_inv,
                             const double *grad_W, double *U)
{
    if (dG < 1 || dA < 1 || !G_inv || !A_inv || !grad_W || !U) return ORC_INVALID;
    double *T = (double *)calloc((size_t)dG * dA, sizeof(double));
    if (!T) return ORC_INVALID;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)                   /* T = G_inv * grad_W */
        for (int q = 0; q < dG; ++q) {
            const double g = G_inv[(size_t)i * dG + q];
            for (int j = 0; j < dA; ++j) T[(size_t)i * dA + j] += g * grad_W[(size_t)q * dA + j];
        }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i) {                 /* U = T * A_inv */
        for (int j = 0; j < dA; ++j) U[(size_t)i * dA + j] = 0.0;
        for (int q = 0; q < dA; ++q) {
            const double t = T[(size_t)i * dA + q];
            for (int j = 0; j < dA; ++j) U[(size_t)i * dA + j] += t * A_inv[(size_t)q * dA + j];
        }
    }
    free(T);
    return ORC_OK;
}

/*
 * Per-sample BatchNorm scale/shift gradients from the layer's output gradient
 * dy and its normalised input xhat, both [N, C, HW]:  y = gamma*xhat + beta, so
 * d/dgamma_c = sum_t dy*xhat and d/dbeta_c = sum_t dy over the HW positions of
 * channel c of sample n.  Outputs are [N, C].
 */
int oracle_bn_reduce_nchw(int N, int C, int HW, const double *dy, const double *xhat,
                          double *g_gamma, double *g_beta)
{
    if (N < 1 || C < 1 || HW < 1 || !dy || !xhat || !g_gamma || !g_beta) return ORC_INVALID;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double sg = 0.0, sb = 0.0;
            const size_t o = ((size_t)n * C + c) * HW;
            for (int t = 0; t < HW; ++t) { sg += dy[o + t] * xhat[o + t]; sb += dy[o + t]; }
            g_gamma[(size_t)n * C + c] = sg;
            g_beta[(size_t)n * C + c] = sb;
        }
    return ORC_OK;
}

/*
 * The fourth call: unit-wise natural gradient for BatchNorm (Sec. 4.2,
 * Eq. 15-17).  Per channel i the 2x2 Fisher block is the batch mean of
 *   [ gg^2, gg*gb ; gb*gg, gb^2 ]   (gg, gb = per-sample grads of gamma_i, beta_i),
 * kept as F_ema[i] = (E gg^2, E gg gb, E gb^2) under the running average;
 * (F + lambda I)^{-1} is applied to the batch-mean gradient by the 2x2
 * closed form (Eq. 17).  lambda is used as is (no pi, no square root).
 */
int oracle_bn_unitwise_precondition(int N, int C, const double *g_gamma, const double *g_beta,
                                    double decay, double lambda, double *F_ema,
                                    double *out_gamma, double *out_beta)
{
    if (N < 1 || C < 1 || !g_gamma || !g_beta || !F_ema || !out_gamma || !out_beta) return ORC_INVALID;
    if (!(decay >= 0.0 && decay < 1.0) || !(lambda >= 0.0)) return ORC_INVALID;
    for (int i = 0; i < C; ++i) {
        double a = 0.0, b = 0.0, d = 0.0, mg = 0.0, mb = 0.0;
        for (int n = 0; n < N; ++n) {
            const double gg = g_gamma[(size_t)n * C + i], gb = g_beta[(size_t)n * C + i];
            a += gg * gg; b += gg * gb; d += gb * gb; mg += gg; mb += gb;
        }
        a /= N; b /= N; d /= N; mg /= N; mb /= N;
        double *F = F_ema + (size_t)3 * i;
        F[0] = decay * F[0] + (1.0 - decay) * a;
        F[1] = decay * F[1] + (1.0 - decay) * b;
        F[2] = decay * F[2] + (1.0 - decay) * d;
        const double fa = F[0] + lambda, fb = F[1], fd = F[2] + lambda;
        const double det = fa * fd - fb * fb;
        out_gamma[i] = (fd * mg - fb * mb) / det;
        out_beta[i] = (fa * mb - fb * mg) / det;
    }
    return ORC_OK;
}
