/*
 * DarKnight finite-field ORACLE: test infrastructure, not product code.
 *
 * The paper's privacy guarantee is stated for a variant of the masked layer in
 * which every value lives in the prime field F_p (section "Privacy Guarantee":
 * "Quantization", "Random Numbers", and the algorithm "The pseudo-code for
 * quantization").  This file is that variant written out with one remainder
 * operation per arithmetic step: no blocking, no deferred reduction, no limb
 * tricks.  Field elements are unsigned 32-bit integers in [0, p); every
 * product is taken in 64 bits and reduced at once.
 *
 * Layout conventions equal those of the floating-point oracle: rows are
 * samples, row-major; group g owns input rows gK..gK+K-1, noise row g and
 * encoded rows gS..gS+S-1 with S = K+2; A[g][i][j] is the weight of source i
 * (K inputs, the noise, a phantom all-zero source) in encoded row j.
 *
 * Shares no code with the HIP library.
 */
#include <math.h>
#include <stdint.h>

typedef uint32_t fe;    /* field element */
typedef uint64_t u64;

static inline fe mulmod(fe a, fe b, fe p) { return (fe)(((u64)a * (u64)b) % p); }
static inline fe addmod(fe a, fe b, fe p) { return (fe)(((u64)a + (u64)b) % p); }

/* Round, then Field (algorithm "The pseudo-code for quantization", procedures
 * Round and Field).  Round takes floor(v) when the fractional part is below
 * one half and floor(v)+1 otherwise, i.e. floor(v + 1/2) for either sign.
 * The scaling by 2^l and the rounding are done in fp64, where they are exact
 * for every fp32 input of interest.  Reading where the paper is silent:
 * the rounded value is clamped to the int32 range and NaN maps to 0.
 * Field maps an integer to its least non-negative residue. */
void orf_quantize(const float *x, fe *xq, long count, int l, fe p)
{
    const double s = ldexp(1.0, l);
#pragma omp parallel for schedule(static)
    for (long i = 0; i < count; ++i) {
        double v = floor((double)x[i] * s + 0.5);
        if (v != v) v = 0.0;
        if (v > 2147483647.0) v = 2147483647.0;
        if (v < -2147483648.0) v = -2147483648.0;
        int64_t z = (int64_t)v % (int64_t)p;
        if (z < 0) z += p;
        xq[i] = (fe)z;
    }
}

/* Inverse of quantisation for a result that carries the factor 2^(2l) (a
 * product of two quantised values): lift to the centred representative
 * (subtract p from everything above p/2; section "Quantization"), then
 * Round(v * 2^-l) * 2^-l (last step of the quantisation algorithm). */
void orf_dequantize(const fe *yq, float *y, long count, int l, fe p)
{
    const double s = ldexp(1.0, -l);
#pragma omp parallel for schedule(static)
    for (long i = 0; i < count; ++i) {
        int64_t v = yq[i];
        if (v > (int64_t)(p / 2)) v -= p;
        y[i] = (float)(floor((double)v * s + 0.5) * s);
    }
}

/* Encoding in the field (Forward Pass, "DarKnight Encoding", with the extra
 * integrity combination): xbar[gS+j] = sum_i A[g][i][j] xq[gK+i] + A[g][K][j] r[g]. */
void orf_encode(const fe *xq, const fe *r, const fe *A, fe *xbar,
                long G, long K, long n, fe p)
{
    const long S = K + 2;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < n; ++e) {
                fe acc = 0;
                for (long i = 0; i < K; ++i)
                    acc = addmod(acc, mulmod(A[(g * S + i) * S + j], xq[(g * K + i) * n + e], p), p);
                acc = addmod(acc, mulmod(A[(g * S + K) * S + j], r[g * n + e], p), p);
                xbar[(g * S + j) * n + e] = acc;
            }
}

/* The linear operation the accelerator performs on encoded rows, over the
 * field: Y[s][o] = sum_k W[o][k] X[s][k]  (mod p). */
void orf_dense_fwd(const fe *W, const fe *X, fe *Y, long R, long M, long N, fe p)
{
#pragma omp parallel for schedule(static) collapse(2)
    for (long s = 0; s < R; ++s)
        for (long o = 0; o < M; ++o) {
            fe acc = 0;
            for (long k = 0; k < N; ++k)
                acc = addmod(acc, mulmod(W[o * N + k], X[s * N + k], p), p);
            Y[s * M + o] = acc;
        }
}

/* Same, for a list of (s, o) output positions only. */
void orf_dense_fwd_points(const fe *W, const fe *X, long M, long N, const long *pts,
                          long npts, fe *out, fe p)
{
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long s = pts[2 * q], o = pts[2 * q + 1];
        fe acc = 0;
        for (long k = 0; k < N; ++k)
            acc = addmod(acc, mulmod(W[o * N + k], X[s * N + k], p), p);
        out[q] = acc;
    }
}

/* Decoding in the field (Forward Pass, "DarKnight Decoding"; the quantisation
 * algorithm applies it to the field values): yq[gK+i] = sum_j Ainv[g][j][i] ybar[gS+j]
 * for i < ncols (ncols = K gives the outputs, K+2 every column). */
void orf_decode(const fe *ybar, const fe *Ainv, fe *yq, long G, long K, long m,
                long ncols, fe p)
{
    const long S = K + 2;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long i = 0; i < ncols; ++i)
            for (long e = 0; e < m; ++e) {
                fe acc = 0;
                for (long j = 0; j < S; ++j)
                    acc = addmod(acc, mulmod(Ainv[(g * S + j) * S + i], ybar[(g * S + j) * m + e], p), p);
                yq[(g * ncols + i) * m + e] = acc;
            }
}

/* Integrity check (section "Computational Integrity"): the extra combination
 * makes the system overdetermined; with nvec the last column of A^{-1},
 * sum_j nvec[g][j] ybar[gS+j] must vanish in the field.  verdict[g] = 1 if any
 * element's combination is non-zero or any ybar entry is not a field element. */
void orf_verify(const fe *ybar, const fe *nvec, int *verdict, long G, long K, long m, fe p)
{
    const long S = K + 2;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g) {
        int bad = 0;
        for (long e = 0; e < m; ++e) {
            fe acc = 0;
            for (long j = 0; j < S; ++j) {
                const fe v = ybar[(g * S + j) * m + e];
                if (v >= p) bad = 1;
                acc = addmod(acc, mulmod(nvec[g * S + j], v % p, p), p);
            }
            if (acc != 0) bad = 1;
        }
        verdict[g] = bad;
    }
}

/* Gradient mixing (Backward Propagation: the accelerators see delta B^T, the
 * enclave's gamma_j scales combination j):
 * dtilde[gS+j] = gamma[g][j] * sum_i B[g][j][i] dq[gK+i]. */
void orf_delta_mix(const fe *dq, const fe *B, const fe *gamma, fe *dtilde,
                   long G, long K, long m, fe p)
{
    const long S = K + 2;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < m; ++e) {
                fe acc = 0;
                for (long i = 0; i < K; ++i)
                    acc = addmod(acc, mulmod(B[(g * S + j) * K + i], dq[(g * K + i) * m + e], p), p);
                dtilde[(g * S + j) * m + e] = mulmod(gamma[g * S + j], acc, p);
            }
}

/* Weight-gradient contraction over encoded rows, over the field:
 * dWq[o][k] = sum_rho D[rho][o] X[rho][k]. */
void orf_dense_wgrad(const fe *D, const fe *X, fe *dWq, long R, long M, long N, fe p)
{
#pragma omp parallel for schedule(static) collapse(2)
    for (long o = 0; o < M; ++o)
        for (long k = 0; k < N; ++k) {
            fe acc = 0;
            for (long s = 0; s < R; ++s)
                acc = addmod(acc, mulmod(D[s * M + o], X[s * N + k], p), p);
            dWq[o * N + k] = acc;
        }
}

void orf_dense_wgrad_points(const fe *D, const fe *X, long R, long M, long N,
                            const long *pts, long npts, fe *out, fe p)
{
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long o = pts[2 * q], k = pts[2 * q + 1];
        fe acc = 0;
        for (long s = 0; s < R; ++s)
            acc = addmod(acc, mulmod(D[s * M + o], X[s * N + k], p), p);
        out[q] = acc;
    }
}

/* NCHW cross-correlation over the field, no bias (the linear operation of a
 * convolution layer on encoded rows):
 * Y[s][co][h][w] = sum_{ci,a,b} W[co][ci][a][b] X[s][ci][h*st+a-pad][w*st+b-pad]  (mod p),
 * zero outside the image. */
void orf_conv_fwd(const fe *W, const fe *X, fe *Y, long R, long Ci, long H, long Wd,
                  long Co, long kh, long kw, long st, long pad, fe p)
{
    const long Ho = (H + 2 * pad - kh) / st + 1, Wo = (Wd + 2 * pad - kw) / st + 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (long s = 0; s < R; ++s)
        for (long co = 0; co < Co; ++co)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    fe acc = 0;
                    for (long ci = 0; ci < Ci; ++ci)
                        for (long a = 0; a < kh; ++a)
                            for (long b = 0; b < kw; ++b) {
                                const long ih = h * st + a - pad, iw = w * st + b - pad;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                                acc = addmod(acc, mulmod(W[((co * Ci + ci) * kh + a) * kw + b],
                                                         X[((s * Ci + ci) * H + ih) * Wd + iw], p), p);
                            }
                    Y[((s * Co + co) * Ho + h) * Wo + w] = acc;
                }
}

/* Same, for a list of (s, co, h, w) output positions only. */
void orf_conv_fwd_points(const fe *W, const fe *X, long Ci, long H, long Wd, long Co,
                         long kh, long kw, long st, long pad, const long *pts, long npts,
                         fe *out, fe p)
{
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long s = pts[4 * q], co = pts[4 * q + 1], h = pts[4 * q + 2], w = pts[4 * q + 3];
        fe acc = 0;
        for (long ci = 0; ci < Ci; ++ci)
            for (long a = 0; a < kh; ++a)
                for (long b = 0; b < kw; ++b) {
                    const long ih = h * st + a - pad, iw = w * st + b - pad;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                    acc = addmod(acc, mulmod(W[((co * Ci + ci) * kh + a) * kw + b],
                                             X[((s * Ci + ci) * H + ih) * Wd + iw], p), p);
                }
        out[q] = acc;
    }
}

/* Weight-gradient correlation over the field:
 * dWq[co][ci][a][b] = sum_{s,h,w} D[s][co][h][w] X[s][ci][h*st+a-pad][w*st+b-pad]  (mod p). */
void orf_conv_wgrad(const fe *D, const fe *X, fe *dWq, long R, long Ci, long H, long Wd,
                    long Co, long kh, long kw, long st, long pad, fe p)
{
    const long Ho = (H + 2 * pad - kh) / st + 1, Wo = (Wd + 2 * pad - kw) / st + 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (long co = 0; co < Co; ++co)
        for (long ci = 0; ci < Ci; ++ci)
            for (long a = 0; a < kh; ++a)
                for (long b = 0; b < kw; ++b) {
                    fe acc = 0;
                    for (long s = 0; s < R; ++s)
                        for (long h = 0; h < Ho; ++h)
                            for (long w = 0; w < Wo; ++w) {
                                const long ih = h * st + a - pad, iw = w * st + b - pad;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                                acc = addmod(acc, mulmod(D[((s * Co + co) * Ho + h) * Wo + w],
                                                         X[((s * Ci + ci) * H + ih) * Wd + iw], p), p);
                            }
                    dWq[((co * Ci + ci) * kh + a) * kw + b] = acc;
                }
}

/* Same, for a list of (co, ci, a, b) positions only. */
void orf_conv_wgrad_points(const fe *D, const fe *X, long R, long Ci, long H, long Wd,
                           long Co, long kh, long kw, long st, long pad, const long *pts,
                           long npts, fe *out, fe p)
{
    const long Ho = (H + 2 * pad - kh) / st + 1, Wo = (Wd + 2 * pad - kw) / st + 1;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < npts; ++q) {
        const long co = pts[4 * q], ci = pts[4 * q + 1], a = pts[4 * q + 2], b = pts[4 * q + 3];
        fe acc = 0;
        for (long s = 0; s < R; ++s)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    const long ih = h * st + a - pad, iw = w * st + b - pad;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                    acc = addmod(acc, mulmod(D[((s * Co + co) * Ho + h) * Wo + w],
                                             X[((s * Ci + ci) * H + ih) * Wd + iw], p), p);
                }
        out[q] = acc;
    }
}

/* Depthwise cross-correlation over the field (one filter per channel,
 * W[C][kh][kw]): the linear operation of the spatial half of a
 * depthwise-separable layer on encoded rows.
 * Y[s][c][h][w] = sum_{a,b} W[c][a][b] X[s][c][h*st+a-pad][w*st+b-pad]  (mod p). */
void orf_dwconv_fwd(const fe *W, const fe *X, fe *Y, long R, long C, long H, long Wd,
                    long kh, long kw, long st, long pad, fe p)
{
    const long Ho = (H + 2 * pad - kh) / st + 1, Wo = (Wd + 2 * pad - kw) / st + 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (long s = 0; s < R; ++s)
        for (long c = 0; c < C; ++c)
            for (long h = 0; h < Ho; ++h)
                for (long w = 0; w < Wo; ++w) {
                    fe acc = 0;
                    for (long a = 0; a < kh; ++a)
                        for (long b = 0; b < kw; ++b) {
                            const long ih = h * st + a - pad, iw = w * st + b - pad;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                            acc = addmod(acc, mulmod(W[(c * kh + a) * kw + b],
                                                     X[((s * C + c) * H + ih) * Wd + iw], p), p);
                        }
                    Y[((s * C + c) * Ho + h) * Wo + w] = acc;
                }
}

/* dWq[c][a][b] = sum_{s,h,w} D[s][c][h][w] X[s][c][h*st+a-pad][w*st+b-pad]  (mod p). */
void orf_dwconv_wgrad(const fe *D, const fe *X, fe *dWq, long R, long C, long H, long Wd,
                      long kh, long kw, long st, long pad, fe p)
{
    const long Ho = (H + 2 * pad - kh) / st + 1, Wo = (Wd + 2 * pad - kw) / st + 1;
#pragma omp parallel for schedule(static)
    for (long c = 0; c < C; ++c)
        for (long a = 0; a < kh; ++a)
            for (long b = 0; b < kw; ++b) {
                fe acc = 0;
                for (long s = 0; s < R; ++s)
                    for (long h = 0; h < Ho; ++h)
                        for (long w = 0; w < Wo; ++w) {
                            const long ih = h * st + a - pad, iw = w * st + b - pad;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                            acc = addmod(acc, mulmod(D[((s * C + c) * Ho + h) * Wo + w],
                                                     X[((s * C + c) * H + ih) * Wd + iw], p), p);
                        }
                dWq[(c * kh + a) * kw + b] = acc;
            }
}

/* The layer's bias in the field (quantisation algorithm: b_q = Field(Round(b 2^{2l})),
 * two factors of 2^l because it joins products of two quantised values).  It is
 * added to the decoded field values, entry e of every row taking bias[e / per]:
 * yq[row][e] <- yq[row][e] + b_q[e / per]  (mod p). */
void orf_add_bias(fe *yq, const float *bias, long rows, long m, long per, int l, fe p)
{
    const double s = ldexp(1.0, 2 * l);
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r)
        for (long e = 0; e < m; ++e) {
            double v = floor((double)bias[e / per] * s + 0.5);
            if (v != v) v = 0.0;
            if (v > 2147483647.0) v = 2147483647.0;
            if (v < -2147483648.0) v = -2147483648.0;
            long long z = (long long)v % (long long)p;
            if (z < 0) z += p;
            yq[r * m + e] = addmod(yq[r * m + e], (fe)z, p);
        }
}

/* ----------------------------------------------------------------------
 * Several colluding accelerators over the field (section "Colluding GPUs",
 * and the paragraph of "Privacy Guarantee" on it: M noise vectors uniform
 * over F_p, A_2 of full rank): S = K + M + 1 encodings per group, sources are
 * the K inputs, then the M noise vectors, then the phantom zero source.
 * ---------------------------------------------------------------------- */

/* xbar[gS+j] = sum_{i<K} A[g][i][j] xq[gK+i] + sum_{q<M} A[g][K+q][j] r[gM+q]. */
void orf_encode_m(const fe *xq, const fe *r, const fe *A, fe *xbar,
                  long G, long K, long M, long n, fe p)
{
    const long S = K + M + 1;
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < n; ++e) {
                fe acc = 0;
                for (long i = 0; i < K; ++i)
                    acc = addmod(acc, mulmod(A[(g * S + i) * S + j], xq[(g * K + i) * n + e], p), p);
                for (long q = 0; q < M; ++q)
                    acc = addmod(acc, mulmod(A[(g * S + K + q) * S + j], r[(g * M + q) * n + e], p), p);
                xbar[(g * S + j) * n + e] = acc;
            }
}

/* yq[g*ncols+i] = sum_{j<S} Ainv[g][j][i] ybar[gS+j], i < ncols. */
void orf_decode_s(const fe *ybar, const fe *Ainv, fe *yq, long G, long S, long m,
                  long ncols, fe p)
{
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long i = 0; i < ncols; ++i)
            for (long e = 0; e < m; ++e) {
                fe acc = 0;
                for (long j = 0; j < S; ++j)
                    acc = addmod(acc, mulmod(Ainv[(g * S + j) * S + i], ybar[(g * S + j) * m + e], p), p);
                yq[(g * ncols + i) * m + e] = acc;
            }
}

/* verdict[g] = 1 if sum_{j<S} nvec[g][j] ybar[gS+j] is non-zero anywhere or an
 * entry of ybar is not a field element. */
void orf_verify_s(const fe *ybar, const fe *nvec, int *verdict, long G, long S, long m, fe p)
{
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g) {
        int bad = 0;
        for (long e = 0; e < m; ++e) {
            fe acc = 0;
            for (long j = 0; j < S; ++j) {
                const fe v = ybar[(g * S + j) * m + e];
                if (v >= p) bad = 1;
                acc = addmod(acc, mulmod(nvec[g * S + j], v % p, p), p);
            }
            if (acc != 0) bad = 1;
        }
        verdict[g] = bad;
    }
}

/* dtilde[gS+j] = gamma[g][j] * sum_{i<K} B[g][j][i] dq[gK+i], j < S. */
void orf_delta_mix_s(const fe *dq, const fe *B, const fe *gamma, fe *dtilde,
                     long G, long K, long S, long m, fe p)
{
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long j = 0; j < S; ++j)
            for (long e = 0; e < m; ++e) {
                fe acc = 0;
                for (long i = 0; i < K; ++i)
                    acc = addmod(acc, mulmod(B[(g * S + j) * K + i], dq[(g * K + i) * m + e], p), p);
                dtilde[(g * S + j) * m + e] = mulmod(gamma[g * S + j], acc, p);
            }
}

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11), as in the
 * real-valued oracle. */
static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const u64 p0 = (u64)0xD2511F53u * c0, p1 = (u64)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform field noise drawn on the fly ("Random Numbers": the noise is uniform
 * over F_p): elements 2t, 2t+1 of the noise row of group g come from one
 * generator call with counter (t mod 2^32, t div 2^32, g, 0) and key
 * (seed mod 2^32, seed div 2^32); each element is a 64-bit word
 * (first word high) reduced mod p, which is uniform up to 2^-39.  r[G][n]. */
void orf_noise_philox(fe *r, long G, long n, uint64_t seed, fe p)
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
#pragma omp parallel for schedule(static)
    for (long g = 0; g < G; ++g)
        for (long t = 0; 2 * t < n; ++t) {
            const uint32_t ctr[4] = {(uint32_t)t, (uint32_t)((u64)t >> 32), (uint32_t)g, 0u};
            uint32_t w[4];
            philox4x32_10(ctr, key, w);
            r[g * n + 2 * t] = (fe)((((u64)w[0] << 32) | w[1]) % p);
            if (2 * t + 1 < n) r[g * n + 2 * t + 1] = (fe)((((u64)w[2] << 32) | w[3]) % p);
        }
}
