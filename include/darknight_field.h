/*
 * darknight_field.h -- C ABI of the finite-field variant of the masked layer
 * (MI355X / gfx950), dense layers and NCHW convolutions.
 *
 * The paper's privacy statement holds for a version of the scheme in which
 * every value is an element of the prime field F_p, p = 2^25 - 39 (section
 * "Privacy Guarantee", paragraphs "Quantization" and "Random Numbers", and the
 * algorithm "The pseudo-code for quantization"): inputs, weights and output
 * gradients are turned into fixed point with l fractional bits
 * (Round(v * 2^l): floor when the fractional part is below one half, floor + 1
 * otherwise) and mapped to their least non-negative residue (Field); the
 * noise, the matrices A and B and the scalars gamma are uniform field
 * elements; encoding, the layer's linear operation, decoding and the
 * integrity check are exact arithmetic modulo p.  Decoded values are lifted
 * to the centred representative (subtract p above p/2) and brought back to
 * floating point by Round(v * 2^-l) * 2^-l.
 *
 * All conventions of darknight.h hold (K, S = K+2, G, R = G*S, row layout,
 * meaning of A, "device" and "host" pointers, streams, error channel,
 * `dk_layer`).  Field elements are uint32_t in [0, DKF_P).  Readings where the
 * paper is silent: a rounded value is clamped to the int32 range before Field
 * and NaN becomes 0; an encoded result that is not a field element (>= p)
 * counts as corrupted.
 *
 * Results are exact, so they do not depend on launch configuration.
 */
#ifndef DARKNIGHT_FIELD_H
#define DARKNIGHT_FIELD_H

#include <stddef.h>
#include <stdint.h>
#include "darknight.h"

#ifdef __cplusplus
extern "C" {
#endif

#define DKF_P 33554393u      /* 2^25 - 39 */
#define DKF_MAX_L 12         /* largest number of fractional bits accepted */

/* Trusted-side coefficient derivation over the field (host arithmetic).
 * From uniform draws A[G][S][S] and gamma[G][S] (host, gamma non-zero):
 *   Ainv = A^{-1} mod p            [G][S][S]  (decoding, Forward Pass);
 *   nvec = last column of Ainv     [G][S]     (the combination of the K+2
 *                                             results that must vanish,
 *                                             section Computational Integrity);
 *   B[j][i] = Ainv[j][i]/gamma[j]  [G][S][K]  (B^T Gamma A^T = [I|0],
 *                                             Backward Propagation).
 * Outputs may be NULL to skip them.  DK_ERR_SINGULAR if some A[g] is singular
 * modulo p or a gamma is 0; DK_ERR_SHAPE if an entry is not below p. */
dk_status dkf_coeffs(const uint32_t *A, const uint32_t *gamma, int G, int K,
                     uint32_t *Ainv, uint32_t *nvec, uint32_t *B);

/* Field(Round(x * 2^l)) for `count` floats (quantisation algorithm, lines for
 * W_q and X_q).  x, xq device.  Used for the weights; dkf_encode and dkf_wgrad
 * quantise their float operand themselves. */
dk_status dkf_quantize(const float *x, uint32_t *xq, long long count, int l, void *stream);

/* Centred lift, then Round(v * 2^-l) * 2^-l (last step of the quantisation
 * algorithm), for `count` field elements.  yq, y device. */
dk_status dkf_dequantize(const uint32_t *yq, float *y, long long count, int l, void *stream);

/* Quantise and encode (quantisation algorithm, X_q then Encode; Forward Pass
 * encoding equation with the extra integrity combination), over the field:
 *   xbar[gS+j][e] = sum_{i<K} A[g][i][j] Xq[gK+i][e] + A[g][K][j] r[g][e]  mod p
 * with Xq = Field(Round(x * 2^l)).  x[G*K][n] float, r[G][n], A[G][S][S] field
 * elements (all device) -> xbar[G*S][n] (device). */
dk_status dkf_encode(const float *x, const uint32_t *r, const uint32_t *A, uint32_t *xbar,
                     int G, int K, long long n, int l, void *stream);

/* Uniform field noise from a counter-based generator ("Random Numbers": the
 * noise is uniform over F_p; it is fresh for every virtual batch and cancels
 * in decoding, so a 64-bit seed can stand for it).  Philox4x32, 10 rounds:
 * elements 2t, 2t+1 of the noise row of group g come from one call with
 * counter (t mod 2^32, t div 2^32, g, 0) and key (seed mod 2^32, seed div
 * 2^32); an element is the 64-bit word (first word high) mod p, uniform up to
 * 2^-39.  dkf_noise_rng writes the rows r[G][n] (device); dkf_encode_rng is
 * dkf_encode with r generated on the fly (same result, r never in memory). */
dk_status dkf_noise_rng(uint32_t *r, int G, long long n, unsigned long long seed, void *stream);
dk_status dkf_encode_rng(const float *x, const uint32_t *A, uint32_t *xbar, int G, int K,
                         long long n, int l, unsigned long long seed, void *stream);

/* The accelerator's linear operation on encoded rows, over the field
 * (quantisation algorithm, the step in which the accelerators apply W_q to
 * the encodings):
 *   ybar[rho][o] = sum_k Wq[o][k] xbar[rho][k]  mod p.
 * Wq[M][N], xbar[R][N] -> ybar[R][M], all device, any R >= 1.  Workspace:
 * dkf_fwd_workspace_bytes(M, N, R), 256-byte aligned.
 * Cost depends on the size of the weights, the result does not: operands are
 * multiplied as four base-128 digits each, all-zero digit planes are found on
 * the device and skipped, so weights with |Round(w 2^l)| < 2^13 cost half of
 * arbitrary field elements and weights with |Round(w 2^l)| <= 127 a quarter (the same
 * holds for dkf_conv_fwd with a contraction Ci kh kw of at least 512, unless
 * the last 128 output channels are at most 64). */
dk_status dkf_linear_fwd(const uint32_t *Wq, const uint32_t *xbar, uint32_t *ybar,
                         int M, int N, int R, void *ws, size_t ws_bytes, void *stream);

/* The same with the weights given as real values W[M][N] (float, device):
 * W_q = Field(Round(W 2^l)) of the quantisation algorithm is formed where the
 * weights are split into digits, so the quantised matrix is never written
 * (for a weight matrix that changes with every step this saves its round trip
 * through memory).  Same result as dkf_quantize followed by dkf_linear_fwd,
 * same workspace. */
dk_status dkf_linear_fwd_w(const float *W, int l, const uint32_t *xbar, uint32_t *ybar,
                           int M, int N, int R, void *ws, size_t ws_bytes, void *stream);

/* The same step for a convolution layer (kind DK_CONV2D): NCHW
 * cross-correlation without bias over the field,
 *   ybar[rho][co][h][w] = sum_{ci,a,b} Wq[co][ci][a][b]
 *                         * xbar[rho][ci][h*stride+a-pad][w*stride+b-pad]  mod p
 * (zero outside the image).  Wq[Co][Ci][kh][kw], xbar[R][Ci][H][W] ->
 * ybar[R][Co][Ho][Wo], all device.  DK_ERR_UNSUPPORTED for a dense layer.
 * Workspace: dkf_conv_fwd_workspace_bytes(L, R), 256-byte aligned. */
dk_status dkf_conv_fwd(const dk_layer *L, const uint32_t *Wq, const uint32_t *xbar,
                       uint32_t *ybar, int R, void *ws, size_t ws_bytes, void *stream);

/* Integrity check and decoding of the forward results in one pass over ybar
 * (section Computational Integrity; quantisation algorithm, Y_q and Y):
 *   t[e]      = sum_j nvec[g][j] ybar[gS+j][e]  mod p;
 *   verdict[g] = 1 if some t[e] != 0 or some ybar entry of the group is >= p,
 *                else 0  (exact: no tolerance);
 *   Yq[gK+i][e] = sum_j Ainv[g][j][i] ybar[gS+j][e]  mod p,  i < K;
 *   y = Round(lift(Yq) * 2^-l) * 2^-l.
 * ybar[G*S][m], Ainv[G][S][S], nvec[G][S] -> y[G*K][m] float, verdict[G] int
 * (all device); yq[G*K][m] (device) receives the field values if not NULL. */
dk_status dkf_decode_verify(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                            float *y, uint32_t *yq, int *verdict,
                            int G, int K, long long m, int l, void *stream);

/* Masked weight gradient over the field (Backward Propagation: the
 * accelerator forms delta-bar = delta B^T and the per-encoding products with
 * the stored xbar; gamma_j weights term j):
 *   Dq = Field(Round(delta * 2^l));
 *   dtilde[gS+j] = gamma[g][j] * sum_{i<K} B[g][j][i] Dq[gK+i]   mod p;
 *   dense: dWq[o][k] = sum_rho dtilde[rho][o] xbar[rho][k]        mod p;
 *   conv:  dWq[co][ci][a][b] = sum_{rho,h,w} dtilde[rho][co][h][w]
 *                              * xbar[rho][ci][h*stride+a-pad][w*stride+b-pad]  mod p;
 *   dW = (accumulate ? dW : 0) + scale * Round(lift(dWq) * 2^-l) * 2^-l.
 * delta[G*K][m] float, B[G][S][K], gamma[G][S], xbar[G*S][n] -> dW (shape of
 * the layer's weights) float, all device.  dwq (same shape, device) receives
 * the field values if not NULL.  Workspace: dkf_wgrad_workspace_bytes(L, G, K),
 * 256-byte aligned. */
dk_status dkf_wgrad(const dk_layer *L, const float *delta, const uint32_t *B,
                    const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                    int G, int K, int l, float scale, int accumulate,
                    void *ws, size_t ws_bytes, void *stream);

/* ---- Dynamic normalisation ("Quantization": networks without normalisation
 * layers divide a vector whose values pass the limits by its largest absolute
 * entry before quantisation).
 *
 * Readings where the paper is silent.  A vector is one row: one sample's
 * features, or the whole weight tensor given as a single row.  It passes the
 * limit when its largest absolute entry m (NaN entries skipped) exceeds
 * `limit`; its factor is then the fp32 value nearest to 1/m, and 1 otherwise
 * (also for m = infinity: the quantiser's clamp deals with that row).  The
 * factors are applied and taken back as follows, every step defined so that
 * the result is one fixed bit pattern:
 *   forward   Xq[i] = Field(Round(x[i] * xscale[i] * 2^l)) (the scaled value is
 *             exact in fp64), Wq likewise with wscale[0];
 *   decode    y[i] = fp32(fp64(Round(lift(Yq[i]) 2^-l) 2^-l)
 *                         * (1 / (xscale[i] * wscale[0])))   (fp64 reciprocal);
 *   backward  the stored encodings hold s_i x_i, and sum_i delta_i (x) x_i =
 *             sum_i (delta_i / s_i) (x) (s_i x_i), so
 *             Dq[i] = Field(Round(fp64(delta[i] * (1 / xscale[i])) * 2^l))
 *             and dW needs no factor afterwards.
 * With all factors equal to 1 every _norm call returns exactly what the call
 * without the suffix returns. */

/* scale[row] from x[rows][len] (both device) as defined above.  rows <= 65535,
 * 0 < limit < infinity.  Three short launches on `stream`, no workspace. */
dk_status dkf_norm_scales(const float *x, float *scale, long long rows, long long len,
                          float limit, void *stream);

/* dkf_quantize of x[rows][len] with row i multiplied by scale[i] first
 * (device pointers; rows = 1 for a weight tensor). */
dk_status dkf_quantize_norm(const float *x, const float *scale, uint32_t *xq, long long rows,
                            long long len, int l, void *stream);

/* dkf_encode / dkf_encode_rng with input row gK+i multiplied by xscale[gK+i]
 * before quantisation.  xscale[G*K] device. */
dk_status dkf_encode_norm(const float *x, const float *xscale, const uint32_t *r, const uint32_t *A,
                          uint32_t *xbar, int G, int K, long long n, int l, void *stream);
dk_status dkf_encode_rng_norm(const float *x, const float *xscale, const uint32_t *A, uint32_t *xbar,
                              int G, int K, long long n, int l, unsigned long long seed,
                              void *stream);

/* dkf_decode_verify whose float rows are brought back to the units of the
 * un-normalised layer.  xscale[G*K], wscale[1] device; yq, verdict unaffected. */
dk_status dkf_decode_verify_norm(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                                 const float *xscale, const float *wscale, float *y, uint32_t *yq,
                                 int *verdict, int G, int K, long long m, int l, void *stream);

/* dkf_wgrad for encodings made by dkf_encode_norm with the same xscale[G*K]
 * (device): row i of delta is divided by xscale[i] before quantisation.  Same
 * workspace as dkf_wgrad. */
dk_status dkf_wgrad_norm(const dk_layer *L, const float *delta, const float *xscale,
                         const uint32_t *B, const uint32_t *gamma, const uint32_t *xbar, float *dW,
                         uint32_t *dwq, int G, int K, int l, float scale, int accumulate,
                         void *ws, size_t ws_bytes, void *stream);

/* Workspace sizes in bytes (0 for invalid arguments). */
/* The layer's bias (quantisation algorithm: b_q = Field(Round(b 2^{2l})), two
 * factors of 2^l because it joins products of two quantised values).  Adding b
 * to every encoded result would not decode to Y + b, so it is added on the
 * trusted side, to the decoded field values:
 *   yq[row][e] <- yq[row][e] + b_q[e / per]  mod p;   y = Round(lift(yq) 2^-l) 2^-l
 * with per = 1 for a dense layer (bias[m]) and Ho*Wo for a convolution
 * (bias[Co]).  yq[rows][m] in place, bias[m / per] float (device); y[rows][m]
 * float (device) receives the de-quantised sums if not NULL. */
dk_status dkf_add_bias(uint32_t *yq, float *y, const float *bias, long long rows, long long m,
                       long long per, int l, void *stream);

/* Depthwise layers (dk_layer.kind = DK_DWCONV2D, W[C][kh][kw]): dkf_conv_fwd,
 * dkf_wgrad and their workspace queries take them too; a few multiply-adds per
 * element moved, so they run on the vector ALUs, exact modulo p like the rest. */

/* ---- Several colluding accelerators over the field (section "Colluding
 * GPUs"; "Privacy Guarantee", the paragraph on colluding accelerators: with M
 * noise vectors uniform over F_p and A_2 of full rank, any M encodings are
 * uniform whatever the inputs).  S = K + M + 1 encodings per group: A[g] is
 * S x S over the field with rows A_1 (the K inputs), A_2 (the M noise vectors)
 * and the phantom zero source; r[G*M][n].  Everything else as in the entry
 * points above, which are the case M = 1; the forward entry points take
 * R = G*S rows unchanged.  Requires K + M - 1 <= DK_MAX_K. ---- */

/* dkf_coeffs for S = K+M+1: Ainv[G][S][S], nvec[G][S] (last column of Ainv),
 * B[G][S][K] = Ainv[j][i] * gamma_j^{-1}.  Host pointers. */
dk_status dkf_coeffs_m(const uint32_t *A, const uint32_t *gamma, int G, int K, int M,
                       uint32_t *Ainv, uint32_t *nvec, uint32_t *B);

/* xbar[gS+j] = sum_{i<K} A[g][i][j] Xq[gK+i] + sum_{q<M} A[g][K+q][j] r[gM+q]  mod p,
 * Xq = Field(Round(x 2^l)).  x[G*K][n] float, r[G*M][n], A[G][S][S] ->
 * xbar[G*S][n], all device. */
dk_status dkf_encode_m(const float *x, const uint32_t *r, const uint32_t *A, uint32_t *xbar,
                       int G, int K, int M, long long n, int l, void *stream);

/* dkf_decode_verify for S = K+M+1: the first K columns of ybar A^{-1} are
 * decoded (the M columns <W_q, r_q> are not produced), the verdict tests the
 * combination nvec. */
dk_status dkf_decode_verify_m(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                              float *y, uint32_t *yq, int *verdict,
                              int G, int K, int M, long long m, int l, void *stream);

/* dkf_wgrad for S = K+M+1.  Workspace: dkf_wgrad_workspace_bytes_m(L, G, K, M). */
dk_status dkf_wgrad_m(const dk_layer *L, const float *delta, const uint32_t *B,
                      const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                      int G, int K, int M, int l, float scale, int accumulate,
                      void *ws, size_t ws_bytes, void *stream);
size_t dkf_wgrad_workspace_bytes_m(const dk_layer *L, int G, int K, int M);

size_t dkf_fwd_workspace_bytes(int M, int N, int R);
size_t dkf_conv_fwd_workspace_bytes(const dk_layer *L, int R);
size_t dkf_wgrad_workspace_bytes(const dk_layer *L, int G, int K);

/* Diagnostic (for the roofline discussion, not part of the path): launches a
 * kernel that does nothing but int8 matrix instructions, `iterations` x 16 per
 * wave on one wave per SIMD of 256 compute units, with constant operands
 * (random_operands = 0), pseudo-random bytes (1) or pseudo-random balanced
 * base-128 digits, i.e. bytes in [-64, 63] as the digit planes hold them (2),
 * in registers, and stores the
 * number of int8 operations of the launch in *int8_ops (host, may be NULL).
 * Time it with events on `stream`: operations / time is what the matrix pipe
 * sustains for such operands when nothing else limits it. */
dk_status dkf_probe_mfma_rate(int random_operands, int iterations, double *int8_ops, void *stream);

#ifdef __cplusplus
}
#endif
#endif
