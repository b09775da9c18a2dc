/*
 * DarKnight masked-layer ORACLE (test infrastructure, not product code).
 *
 * Plain, slow, fp64 CPU definitions of everything the masked-layer hot path
 * computes.  Nothing here is blocked, fused or reordered: every function is
 * the definition (or the paper's steps in the paper's order) written out as
 * loops, so it can be checked against the paper by eye.  OpenMP is used only
 * across independent outputs.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * may link or load this file.  It shares no code with the HIP library.
 *
 * Storage convention (all arrays row-major, sample-major):
 *   K  private inputs per virtual batch ("group"), S = K+2 encodings
 *   (K+1 for masking, Forward Pass Eq. "DarKnight Encoding"; one more for the
 *   integrity check, section "Computational Integrity"), G groups.
 *   Group g owns inputs rows gK..gK+K-1, noise row g, encoded rows gS..gS+S-1.
 *   A[g] is S x S; A[g][i][j] = weight of source i (K inputs, then the noise
 *   vector, then an all-zero phantom source) in encoding j.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int ora_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------- */
/* Plain (unmasked) layer definitions: what the method must reproduce.     */
/* ---------------------------------------------------------------------- */

/* Dense layer, section "Forward Pass": y = <W, x> as a matrix product.
 * Y[s][o] = sum_k W[o][k] X[s][k];  W[M][N], X[R][N], Y[R][M]. */
void ora_dense_fwd(const double *W, const double *X, double *Y,
                   long R, long M, long N)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long o = 0; o < M; ++o) {
            double acc = 0.0;
            for (long k = 0; k < N; ++k)
                acc += W[o * N + k] * X[s * N + k];
            Y[s * M + o] = acc;
        }
}

/* Convolution layer, section "Forward Pass": the bilinear operator as an
 * NCHW cross-correlation without bias, zero outside the image.
 * Y[s][co][h][w] = sum_{ci,a,b} W[co][ci][a][b] X[s][ci][h*st+a-p][w*st+b-p] */
void ora_conv_fwd(const double *W, const double *X, double *Y,
                  long R, long Ci, long H, long Wd, long Co,
                  long kh, long kw, long st, long p)
{
    const long Ho = (H + 2 * p - kh) / st + 1;
    const long Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long co = 0; co < Co; ++co)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    double acc = 0.0;
                    for (long ci = 0; ci < Ci; ++ci)
                        for (long a = 0; a < kh; ++a)
                            for (long b = 0; b < kw; ++b) {
                                const long ih = h * st + a - p;
                                const long iw = w * st + b - p;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= Wd)
                                    continue;
                                acc += W[((co * Ci + ci) * kh + a) * kw + b] *
                                       X[((s * Ci + ci) * H + ih) * Wd + iw];
                            }
                    Y[((s * Co + co) * Ho + h) * Wo + w] = acc;
                }
}

/* Dense weight gradient, Backward Propagation Eq. (SGD):
 * dW[o][k] = scale * sum_s delta[s][o] X[s][k]  (scale = 1/K in the paper). */
void ora_dense_wgrad(const double *D, const double *X, double *dW,
                     long R, long M, long N, double scale)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long o = 0; o < M; ++o)
        for (long k = 0; k < N; ++k) {
            double acc = 0.0;
            for (long s = 0; s < R; ++s)
                acc += D[s * M + o] * X[s * N + k];
            dW[o * N + k] = scale * acc;
        }
}

/* Convolution weight gradient: the same bilinear pairing <delta, x>,
 * dW[co][ci][a][b] = scale * sum_{s,h,w} delta[s][co][h][w] *
 *                                        X[s][ci][h*st+a-p][w*st+b-p]. */
void ora_conv_wgrad(const double *D, const double *X, double *dW,
                    long R, long Ci, long H, long Wd, long Co,
                    long kh, long kw, long st, long p, double scale)
{
    const long Ho = (H + 2 * p - kh) / st + 1;
    const long Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long co = 0; co < Co; ++co)
        for (long ci = 0; ci < Ci; ++ci)
            for (long a = 0; a < kh; ++a)
                for (long b = 0; b < kw; ++b) {
                    double acc = 0.0;
                    for (long s = 0; s < R; ++s)
                        for (long h = 0; h < Ho; ++h)
                            for (long w = 0; w < Wo; ++w) {
                                const long ih = h * st + a - p;
                                const long iw = w * st + b - p;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= Wd)
                                    continue;
                                acc += D[((s * Co + co) * Ho + h) * Wo + w] *
                                       X[((s * Ci + ci) * H + ih) * Wd + iw];
                            }
                    dW[((co * Ci + ci) * kh + a) * kw + b] = scale * acc;
                }
}

/* ---------------------------------------------------------------------- */
/* The same definitions evaluated at chosen output coordinates only, on    */
/* the fp32 arrays the accelerator receives (promoted element by element), */
/* so that full-size tensors can be spot-checked.                          */
/* ---------------------------------------------------------------------- */

/* pts[q] = {s, o};  out[q] = sum_k W[o][k] X[s][k] */
void ora_dense_fwd_points(const float *W, const float *X, long M, long N,
                          const long *pts, long npts, double *out)
{
    (void)M;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long s = pts[2 * q], o = pts[2 * q + 1];
        double acc = 0.0;
        for (long k = 0; k < N; ++k)
            acc += (double)W[o * N + k] * (double)X[s * N + k];
        out[q] = acc;
    }
}

/* pts[q] = {o, k};  out[q] = scale * sum_s D[s][o] X[s][k] */
void ora_dense_wgrad_points(const float *D, const float *X, long R, long M,
                            long N, double scale, const long *pts, long npts,
                            double *out)
{
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long o = pts[2 * q], k = pts[2 * q + 1];
        double acc = 0.0;
        for (long s = 0; s < R; ++s)
            acc += (double)D[s * M + o] * (double)X[s * N + k];
        out[q] = scale * acc;
    }
}

/* pts[q] = {s, co, h, w} */
void ora_conv_fwd_points(const float *W, const float *X, long Ci, long H,
                         long Wd, long Co, long kh, long kw, long st, long p,
                         const long *pts, long npts, double *out)
{
    (void)Co;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long s = pts[4 * q], co = pts[4 * q + 1];
        const long h = pts[4 * q + 2], w = pts[4 * q + 3];
        double acc = 0.0;
        for (long ci = 0; ci < Ci; ++ci)
            for (long a = 0; a < kh; ++a)
                for (long b = 0; b < kw; ++b) {
                    const long ih = h * st + a - p, iw = w * st + b - p;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= Wd)
                        continue;
                    acc += (double)W[((co * Ci + ci) * kh + a) * kw + b] *
                           (double)X[((s * Ci + ci) * H + ih) * Wd + iw];
                }
        out[q] = acc;
    }
}

/* pts[q] = {co, ci, a, b} */
void ora_conv_wgrad_points(const float *D, const float *X, long R, long Ci,
                           long H, long Wd, long Co, long kh, long kw, long st,
                           long p, double scale, const long *pts, long npts,
                           double *out)
{
    const long Ho = (H + 2 * p - kh) / st + 1;
    const long Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long co = pts[4 * q], ci = pts[4 * q + 1];
        const long a = pts[4 * q + 2], b = pts[4 * q + 3];
        double acc = 0.0;
        for (long s = 0; s < R; ++s)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    const long ih = h * st + a - p, iw = w * st + b - p;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= Wd)
                        continue;
                    acc += (double)D[((s * Co + co) * Ho + h) * Wo + w] *
                           (double)X[((s * Ci + ci) * H + ih) * Wd + iw];
                }
        out[q] = scale * acc;
    }
}

/* ---------------------------------------------------------------------- */
/* The method's own steps, in the paper's order and notation.              */
/* ---------------------------------------------------------------------- */

/* Encoding, Forward Pass Eq. (DarKnight Encoding), extended by one more
 * combination for integrity (section "Computational Integrity"):
 *   xbar^(j) = alpha_{1,j} x^(1) + ... + alpha_{K,j} x^(K) + alpha_{K+1,j} r
 * for j = 1..K+2.  X[G*K][n], r[G][n], A[G][S][S] -> Xbar[G*S][n]. */
void ora_encode(const double *X, const double *r, const double *A,
                double *Xbar, long G, long K, long n)
{
    const long S = K + 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < n; ++e) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += A[(g * S + i) * S + j] * X[(g * K + i) * n + e];
                acc += A[(g * S + K) * S + j] * r[g * n + e];
                Xbar[(g * S + j) * n + e] = acc;
            }
}

/* Decoding, Forward Pass Eq. (DarKnight Decoding): Y = Ybar . A^{-1}.
 * Column i of the result is sum_j Ybar^(j) Ainv[j][i].  ncols = K gives the
 * K wanted outputs; ncols = K+1 also returns <W, r> (which the method
 * drops); ncols = K+2 also returns the phantom column that must vanish.
 * Ybar[G*S][m], Ainv[G][S][S] -> Y[G*ncols][m]. */
void ora_decode(const double *Ybar, const double *Ainv, double *Y,
                long G, long K, long m, long ncols)
{
    const long S = K + 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long i = 0; i < ncols; ++i)
            for (long e = 0; e < m; ++e) {
                double acc = 0.0;
                for (long j = 0; j < S; ++j)
                    acc += Ybar[(g * S + j) * m + e] * Ainv[(g * S + j) * S + i];
                Y[(g * ncols + i) * m + e] = acc;
            }
}

/* Integrity check, section "Computational Integrity", null-vector form.
 * K+2 equations in K+1 unknowns are consistent iff the combination with the
 * left null vector nvec of the encoding (A_ext nvec = 0) vanishes:
 *   t[e] = sum_j nvec[j] Ybar^(j)[e].
 * The group is flagged when max_e |t| exceeds tol times
 * max_e sum_j |nvec[j] Ybar^(j)[e]|, or when either maximum is not finite.
 * rho[g] receives the ratio (0 when the denominator is 0). */
void ora_verify(const double *Ybar, const double *nvec, double tol,
                int *verdict, double *rho, long G, long K, long m)
{
    const long S = K + 2;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g) {
        double tmax = 0.0, smax = 0.0;
        int bad = 0;
        for (long e = 0; e < m; ++e) {
            double t = 0.0, sc = 0.0;
            for (long j = 0; j < S; ++j) {
                const double v = nvec[g * S + j] * Ybar[(g * S + j) * m + e];
                t += v;
                sc += fabs(v);
            }
            if (!isfinite(t) || !isfinite(sc))
                bad = 1;
            if (fabs(t) > tmax) tmax = fabs(t);
            if (sc > smax) smax = sc;
        }
        const double ratio = (smax > 0.0) ? tmax / smax : 0.0;
        if (rho) rho[g] = bad ? INFINITY : ratio;
        verdict[g] = (bad || tmax > tol * smax) ? 1 : 0;
    }
}

/* Solve the (K+1)x(K+1) system  sum_j c[j][i] * M[j][q] = rhs  used by the
 * literal two-subset check below (Gaussian elimination, partial pivoting). */
static int solve_square(double *Mx, double *inv, long n)
{
    /* inv <- Mx^{-1}; Mx destroyed.  Returns 0 on success. */
    for (long i = 0; i < n; ++i)
        for (long j = 0; j < n; ++j)
            inv[i * n + j] = (i == j) ? 1.0 : 0.0;
    for (long c = 0; c < n; ++c) {
        long piv = c;
        for (long r = c + 1; r < n; ++r)
            if (fabs(Mx[r * n + c]) > fabs(Mx[piv * n + c])) piv = r;
        if (Mx[piv * n + c] == 0.0) return 1;
        if (piv != c)
            for (long j = 0; j < n; ++j) {
                double t = Mx[c * n + j]; Mx[c * n + j] = Mx[piv * n + j]; Mx[piv * n + j] = t;
                t = inv[c * n + j]; inv[c * n + j] = inv[piv * n + j]; inv[piv * n + j] = t;
            }
        const double d = Mx[c * n + c];
        for (long j = 0; j < n; ++j) { Mx[c * n + j] /= d; inv[c * n + j] /= d; }
        for (long r = 0; r < n; ++r) {
            if (r == c) continue;
            const double f = Mx[r * n + c];
            if (f == 0.0) continue;
            for (long j = 0; j < n; ++j) {
                Mx[r * n + j] -= f * Mx[c * n + j];
                inv[r * n + j] -= f * inv[c * n + j];
            }
        }
    }
    return 0;
}

/* Integrity check, section "Computational Integrity", literal form: recover
 * every y^(i) (and <W,r>) twice, once from encodings 1..K+1 and once from
 * encodings 2..K+2, each time by inverting that square sub-block of the
 * encoding matrix, and compare.  The group is flagged when the two
 * recoveries differ by more than tol relative to the larger recovered
 * magnitude.  Returns nonzero if a sub-block is singular.  Small sizes only. */
int ora_verify_two_subsets(const double *Ybar, const double *A, double tol,
                           int *verdict, double *maxdiff, long G, long K, long m)
{
    const long S = K + 2, U = K + 1;
    double *sub = (double *)malloc(sizeof(double) * U * U);
    double *inv0 = (double *)malloc(sizeof(double) * U * U);
    double *inv1 = (double *)malloc(sizeof(double) * U * U);
    int rc = 0;
    for (long g = 0; g < G && !rc; ++g) {
        /* sub-block: sources 0..K (rows of A) x encodings off..off+K */
        for (int which = 0; which < 2; ++which) {
            const long off = which;
            for (long i = 0; i < U; ++i)
                for (long j = 0; j < U; ++j)
                    sub[i * U + j] = A[(g * S + i) * S + (off + j)];
            rc |= solve_square(sub, which ? inv1 : inv0, U);
        }
        double dmax = 0.0, ymax = 0.0;
        for (long e = 0; e < m && !rc; ++e)
            for (long i = 0; i < U; ++i) {
                double y0 = 0.0, y1 = 0.0;
                for (long j = 0; j < U; ++j) {
                    y0 += Ybar[(g * S + j) * m + e] * inv0[j * U + i];
                    y1 += Ybar[(g * S + 1 + j) * m + e] * inv1[j * U + i];
                }
                if (fabs(y0 - y1) > dmax) dmax = fabs(y0 - y1);
                if (fabs(y0) > ymax) ymax = fabs(y0);
                if (fabs(y1) > ymax) ymax = fabs(y1);
            }
        if (maxdiff) maxdiff[g] = dmax;
        verdict[g] = (dmax > tol * ymax) ? 1 : 0;
    }
    free(sub); free(inv0); free(inv1);
    return rc;
}

/* Gradient mixing on the accelerator side, Backward Propagation Eq.
 * (gamma-weighted sum): deltabar^(j) = sum_i beta_{j,i} delta^(i), here
 * already multiplied by the secret gamma_j so that the contraction below
 * needs no further weights.
 * D[G*K][m], B[G][S][K], gamma[G][S] -> Dt[G*S][m]. */
void ora_delta_mix(const double *D, const double *B, const double *gamma,
                   double *Dt, long G, long K, long m)
{
    const long S = K + 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < m; ++e) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += B[(g * S + j) * K + i] * D[(g * K + i) * m + e];
                Dt[(g * S + j) * m + e] = gamma[g * S + j] * acc;
            }
}

/* Masked weight gradient of a dense layer, Backward Propagation Eq.
 * (gamma-weighted sum) and Eq. (aggregate), then summed over the virtual
 * batches of the large batch (Algorithm "parameters update"):
 *   Eq_j  = < sum_i beta_{j,i} delta^(i) , xbar^(j) >   (an outer product)
 *   gradW = scale * sum_g sum_j gamma_j Eq_j
 * D[G*K][M], Xbar[G*S][N] -> dW[M][N].  Every Eq_j is formed explicitly. */
void ora_masked_dense_wgrad(const double *D, const double *B,
                            const double *gamma, const double *Xbar,
                            double *dW, long G, long K, long M, long N,
                            double scale)
{
    const long S = K + 2;
    double *dbar = (double *)malloc(sizeof(double) * M);
    double *Eq = (double *)malloc(sizeof(double) * M * N);
    for (long q = 0; q < M * N; ++q) dW[q] = 0.0;
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j) {
            for (long o = 0; o < M; ++o) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += B[(g * S + j) * K + i] * D[(g * K + i) * M + o];
                dbar[o] = acc;
            }
#pragma omp parallel for schedule(static)
            for (long o = 0; o < M; ++o)
                for (long k = 0; k < N; ++k)
                    Eq[o * N + k] = dbar[o] * Xbar[(g * S + j) * N + k];
            const double gj = gamma[g * S + j];
#pragma omp parallel for schedule(static)
            for (long q = 0; q < M * N; ++q) dW[q] += gj * Eq[q];
        }
    for (long q = 0; q < M * N; ++q) dW[q] *= scale;
    free(dbar); free(Eq);
}

/* Masked weight gradient of a convolution layer: same steps, with Eq_j the
 * convolution weight-gradient pairing of deltabar^(j) with xbar^(j). */
void ora_masked_conv_wgrad(const double *D, const double *B,
                           const double *gamma, const double *Xbar, double *dW,
                           long G, long K, long Ci, long H, long Wd, long Co,
                           long kh, long kw, long st, long p, double scale)
{
    const long S = K + 2;
    const long Ho = (H + 2 * p - kh) / st + 1;
    const long Wo = (Wd + 2 * p - kw) / st + 1;
    const long m = Co * Ho * Wo, n = Ci * H * Wd, nw = Co * Ci * kh * kw;
    double *dbar = (double *)malloc(sizeof(double) * m);
    double *Eq = (double *)malloc(sizeof(double) * nw);
    for (long q = 0; q < nw; ++q) dW[q] = 0.0;
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j) {
            for (long e = 0; e < m; ++e) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += B[(g * S + j) * K + i] * D[(g * K + i) * m + e];
                dbar[e] = acc;
            }
            ora_conv_wgrad(dbar, Xbar + (g * S + j) * n, Eq, 1, Ci, H, Wd, Co,
                           kh, kw, st, p, 1.0);
            const double gj = gamma[g * S + j];
            for (long q = 0; q < nw; ++q) dW[q] += gj * Eq[q];
        }
    for (long q = 0; q < nw; ++q) dW[q] *= scale;
    free(dbar); free(Eq);
}

/* ---------------------------------------------------------------------- */
/* Colluding accelerators (section "Colluding GPUs"): M noise vectors.     */
/* ---------------------------------------------------------------------- */

/* Encoding with M noise vectors, Xbar = X A_1 + R A_2, plus the extra
 * integrity combination: S = K + M + 1 encodings per group.  A[g] is S x S;
 * its rows 0..K-1 are A_1, rows K..K+M-1 are A_2, its last row belongs to the
 * phantom all-zero source.  X[G*K][n], Rn[G*M][n] -> Xbar[G*S][n]. */
void ora_encode_m(const double *X, const double *Rn, const double *A, double *Xbar,
                  long G, long K, long M, long n)
{
    const long S = K + M + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < n; ++e) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += A[(g * S + i) * S + j] * X[(g * K + i) * n + e];
                for (long q = 0; q < M; ++q)
                    acc += A[(g * S + K + q) * S + j] * Rn[(g * M + q) * n + e];
                Xbar[(g * S + j) * n + e] = acc;
            }
}

/* Decoding, integrity check and gradient mixing for S encodings per group
 * (the formulas of ora_decode, ora_verify and ora_delta_mix with S free). */
void ora_decode_s(const double *Ybar, const double *Ainv, double *Y,
                  long G, long S, long m, long ncols)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long i = 0; i < ncols; ++i)
            for (long e = 0; e < m; ++e) {
                double acc = 0.0;
                for (long j = 0; j < S; ++j)
                    acc += Ybar[(g * S + j) * m + e] * Ainv[(g * S + j) * S + i];
                Y[(g * ncols + i) * m + e] = acc;
            }
}

void ora_verify_s(const double *Ybar, const double *nvec, double tol,
                  int *verdict, double *rho, long G, long S, long m)
{
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g) {
        double tmax = 0.0, smax = 0.0;
        int bad = 0;
        for (long e = 0; e < m; ++e) {
            double t = 0.0, sc = 0.0;
            for (long j = 0; j < S; ++j) {
                const double v = nvec[g * S + j] * Ybar[(g * S + j) * m + e];
                t += v;
                sc += fabs(v);
            }
            if (!isfinite(t) || !isfinite(sc))
                bad = 1;
            if (fabs(t) > tmax) tmax = fabs(t);
            if (sc > smax) smax = sc;
        }
        const double ratio = (smax > 0.0) ? tmax / smax : 0.0;
        if (rho) rho[g] = bad ? INFINITY : ratio;
        verdict[g] = (bad || tmax > tol * smax) ? 1 : 0;
    }
}

/* Eq. of the weight update with colluding accelerators:
 * Eq_j = < sum_{i<=K} beta_{j,i} delta^(i), xbar^(j) >, j = 1..S; here the
 * mixed gradient of encoding j, already times gamma_j. */
void ora_delta_mix_s(const double *D, const double *B, const double *gamma,
                     double *Dt, long G, long K, long S, long m)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < m; ++e) {
                double acc = 0.0;
                for (long i = 0; i < K; ++i)
                    acc += B[(g * S + j) * K + i] * D[(g * K + i) * m + e];
                Dt[(g * S + j) * m + e] = gamma[g * S + j] * acc;
            }
}

/* ---------------------------------------------------------------------- */
/* Noise drawn by a counter-based generator instead of being passed in.    */
/* ---------------------------------------------------------------------- */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11): a keyed bijection of a 128-bit
 * counter.  Each round multiplies two counter words by fixed odd constants
 * and mixes the high halves with the other words and the key; the key words
 * advance by Weyl constants. */
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The noise rows of the encoding (each virtual batch gets fresh noise;
 * Forward Pass, "Key Insight") drawn on the fly: elements 4b..4b+3 of noise
 * row q of group g come from one generator call with counter
 * (b mod 2^32, b div 2^32, g, q) and key (seed mod 2^32, seed div 2^32); the
 * four words become uniforms u = ((word >> 8) + 1/2) 2^-24 in (0,1) and two
 * Box-Muller pairs  sqrt(-2 ln u0) (cos, sin)(2 pi u1),  same with (u2, u3);
 * the values are sigma times these.  r[G*M][n]. */
void ora_noise_philox(double *r, long G, long M, long n, uint64_t seed, double sigma)
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for collapse(2) schedule(static)
    for (long g = 0; g < G; ++g)
        for (long q = 0; q < M; ++q)
            for (long b = 0; 4 * b < n; ++b) {
                const uint32_t ctr[4] = {(uint32_t)b, (uint32_t)((uint64_t)b >> 32), (uint32_t)g, (uint32_t)q};
                uint32_t w[4];
                ora_philox4x32_10(ctr, key, w);
                double u[4], z[4];
                for (int k = 0; k < 4; ++k) u[k] = ((double)(w[k] >> 8) + 0.5) * (1.0 / 16777216.0);
                const double m0 = sqrt(-2.0 * log(u[0])), m1 = sqrt(-2.0 * log(u[2]));
                z[0] = m0 * cos(two_pi * u[1]); z[1] = m0 * sin(two_pi * u[1]);
                z[2] = m1 * cos(two_pi * u[3]); z[3] = m1 * sin(two_pi * u[3]);
                for (int k = 0; k < 4 && 4 * b + k < n; ++k)
                    r[(g * M + q) * n + 4 * b + k] = sigma * z[k];
            }
}

/* ---------------------------------------------------------------------- */
/* Depthwise convolution (one filter per channel) and data gradients.      */
/* ---------------------------------------------------------------------- */

/* Depthwise NCHW cross-correlation, the spatial half of a depthwise-separable
 * layer: Y[s][c][h][w] = sum_{a,b} W[c][a][b] X[s][c][h*st+a-p][w*st+b-p]. */
void ora_dwconv_fwd(const double *W, const double *X, double *Y, long R, long Cc, long H,
                    long Wd, long kh, long kw, long st, long p)
{
    const long Ho = (H + 2 * p - kh) / st + 1, Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long c = 0; c < Cc; ++c)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    double acc = 0.0;
                    for (long a = 0; a < kh; ++a)
                        for (long b = 0; b < kw; ++b) {
                            const long ih = h * st + a - p, iw = w * st + b - p;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                            acc += W[(c * kh + a) * kw + b] * X[((s * Cc + c) * H + ih) * Wd + iw];
                        }
                    Y[((s * Cc + c) * Ho + h) * Wo + w] = acc;
                }
}

/* Its weight gradient, the same pairing <delta, x> per channel:
 * dW[c][a][b] = scale * sum_{s,h,w} D[s][c][h][w] X[s][c][h*st+a-p][w*st+b-p]. */
void ora_dwconv_wgrad(const double *D, const double *X, double *dW, long R, long Cc, long H,
                      long Wd, long kh, long kw, long st, long p, double scale)
{
    const long Ho = (H + 2 * p - kh) / st + 1, Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for schedule(static)
    for (long c = 0; c < Cc; ++c)
        for (long a = 0; a < kh; ++a)
            for (long b = 0; b < kw; ++b) {
                double acc = 0.0;
                for (long s = 0; s < R; ++s)
                    for (long h = 0; h < Ho; ++h)
                        for (long w = 0; w < Wo; ++w) {
                            const long ih = h * st + a - p, iw = w * st + b - p;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                            acc += D[((s * Cc + c) * Ho + h) * Wo + w] * X[((s * Cc + c) * H + ih) * Wd + iw];
                        }
                dW[(c * kh + a) * kw + b] = scale * acc;
            }
}

/* Data gradients (Backward Propagation, second linear operation: the gradient
 * with respect to the layer input; it holds no private input and runs
 * un-encoded).  Each is the transpose of the forward map:
 * dense   dX[s][k]        = sum_o D[s][o] W[o][k];
 * conv    dX[s][ci][i][j] = sum_{co,a,b} D[s][co][h][w] W[co][ci][a][b]
 *                           over the (h, w) with h*st+a-p = i, w*st+b-p = j;
 * depthwise the same with co = ci = c. */
void ora_dense_dgrad(const double *D, const double *W, double *dX, long R, long M, long N)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long k = 0; k < N; ++k) {
            double acc = 0.0;
            for (long o = 0; o < M; ++o) acc += D[s * M + o] * W[o * N + k];
            dX[s * N + k] = acc;
        }
}

void ora_conv_dgrad(const double *D, const double *W, double *dX, long R, long Ci, long H,
                    long Wd, long Co, long kh, long kw, long st, long p)
{
    const long Ho = (H + 2 * p - kh) / st + 1, Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long ci = 0; ci < Ci; ++ci)
            for (long i = 0; i < H; ++i)
                for (long j = 0; j < Wd; ++j) {
                    double acc = 0.0;
                    for (long co = 0; co < Co; ++co)
                        for (long a = 0; a < kh; ++a)
                            for (long b = 0; b < kw; ++b) {
                                const long hn = i + p - a, wn = j + p - b;
                                if (hn < 0 || wn < 0 || hn % st || wn % st) continue;
                                const long h = hn / st, w = wn / st;
                                if (h >= Ho || w >= Wo) continue;
                                acc += D[((s * Co + co) * Ho + h) * Wo + w] *
                                       W[((co * Ci + ci) * kh + a) * kw + b];
                            }
                    dX[((s * Ci + ci) * H + i) * Wd + j] = acc;
                }
}

void ora_dwconv_dgrad(const double *D, const double *W, double *dX, long R, long Cc, long H,
                      long Wd, long kh, long kw, long st, long p)
{
    const long Ho = (H + 2 * p - kh) / st + 1, Wo = (Wd + 2 * p - kw) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (long s = 0; s < R; ++s)
        for (long c = 0; c < Cc; ++c)
            for (long i = 0; i < H; ++i)
                for (long j = 0; j < Wd; ++j) {
                    double acc = 0.0;
                    for (long a = 0; a < kh; ++a)
                        for (long b = 0; b < kw; ++b) {
                            const long hn = i + p - a, wn = j + p - b;
                            if (hn < 0 || wn < 0 || hn % st || wn % st) continue;
                            const long h = hn / st, w = wn / st;
                            if (h >= Ho || w >= Wo) continue;
                            acc += D[((s * Cc + c) * Ho + h) * Wo + w] * W[(c * kh + a) * kw + b];
                        }
                    dX[((s * Cc + c) * H + i) * Wd + j] = acc;
                }
}
