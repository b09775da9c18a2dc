/*
 * darknight.h -- C ABI of the MI355X (gfx950) masked-layer library.
 *
 * The library implements the data-parallel hot path of DarKnight's matrix
 * masking: encode K private inputs plus a noise input into K+2 obfuscated
 * inputs, run the layer's bilinear operation (dense product or NCHW
 * convolution) and its weight gradient on the obfuscated inputs only, decode
 * with the inverse of the encoding matrix and check the redundant
 * combination for integrity.
 *
 * Conventions
 *   K  private inputs per virtual batch ("group"); S = K+2 encodings per
 *      group (K+1 mask the inputs, one more is the integrity redundancy);
 *      G groups; R = G*S encoded rows.  1 <= K <= DK_MAX_K.
 *   All tensors are fp32, row-major and sample-major: a sample (or encoding)
 *   is one contiguous row of n (input) or m (output) floats; convolution
 *   rows are CHW images.  Group g owns input rows gK..gK+K-1, noise row g and
 *   encoded rows gS..gS+S-1.
 *   A[g] is S x S, A[g][i][j] = weight of source i in encoding j; sources are
 *   the K inputs, then the noise vector, then a phantom all-zero source, so
 *   the last row of A[g] is never read by dk_encode.
 *   "device" pointers are HIP device memory owned by the caller; the library
 *   never allocates, frees or keeps them.  "host" pointers are ordinary host
 *   memory.  Kernels are enqueued on `stream` (a hipStream_t passed as
 *   void*, NULL = default stream) and the call returns without waiting;
 *   results, verdicts included, are in device memory once the stream has
 *   drained.
 *   The return value is the only error channel.  Argument errors are found
 *   on the host before anything is launched; DK_ERR_HIP reports a failed
 *   launch.  Nothing is written on error.
 */
#ifndef DARKNIGHT_H
#define DARKNIGHT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DK_MAX_K 16

typedef enum {
    DK_OK = 0,
    DK_ERR_NULL = 1,        /* a required pointer is NULL                      */
    DK_ERR_SHAPE = 2,       /* a size is non-positive, too large or K invalid  */
    DK_ERR_UNSUPPORTED = 3, /* layer geometry the kernels do not cover         */
    DK_ERR_ALIGN = 4,       /* a device pointer is not 4-byte aligned (the
                               integrity check's workspace: 16-byte)           */
    DK_ERR_WORKSPACE = 5,   /* workspace missing or smaller than required      */
    DK_ERR_HIP = 6,         /* the HIP runtime refused a launch                */
    DK_ERR_SINGULAR = 7,    /* dk_coeffs: A[g] is singular or gamma has a zero */
    DK_ERR_STATIC_LIMIT = 8 /* dk_decode_verify_static: more groups than its
                               built-in scratch array serves                   */
} dk_status;

/* Layer descriptor.  kind 0: dense y = W x with W[M][N].  kind 1: NCHW
 * cross-correlation without bias, W[Co][Ci][kh][kw], zero padding, output
 * Ho = (H + 2 pad - kh)/stride + 1 (same for Wo).  kind 2: depthwise
 * cross-correlation, one filter per channel, W[Ci][kh][kw], Co == Ci, filter
 * edges up to 7 (the spatial half of a depthwise-separable layer; the
 * entry points that take a convolution layer take this kind too). */
typedef struct dk_layer {
    int kind;
    int M, N;
    int Ci, Co, H, W, kh, kw, stride, pad;
} dk_layer;

enum { DK_LINEAR = 0, DK_CONV2D = 1, DK_DWCONV2D = 2 };
enum { DK_OP_FWD = 0, DK_OP_WGRAD = 1, DK_OP_VERIFY = 2 };

const char *dk_status_str(int status);
int dk_version(void);

/* Flat per-sample input length n and output length m of a layer (0 if the
 * descriptor is invalid). */
long long dk_layer_in_len(const dk_layer *L);
long long dk_layer_out_len(const dk_layer *L);

/* Bytes of device workspace that dk_linear_fwd / dk_conv_fwd (DK_OP_FWD),
 * dk_wgrad (DK_OP_WGRAD) or dk_verify (DK_OP_VERIFY) need for this layer,
 * G groups of K inputs.  For DK_OP_VERIFY the layer may be NULL.  Returns 0
 * for invalid arguments (every valid case needs a non-zero workspace). */
size_t dk_workspace_bytes(const dk_layer *L, int op, int G, int K);

/* The DK_OP_FWD workspace for exactly R encoded rows (R need not be a
 * multiple of K+2: the forward entry points take any row count). */
size_t dk_fwd_workspace_bytes(const dk_layer *L, long long R);

/* Trusted-side coefficient derivation (host arithmetic, fp64 internally).
 * From the random draws A[G][S][S] and gamma[G][S] (host) derive, per group:
 *   Ainv = A^{-1}                 [G][S][S]  (Forward Pass, decoding relation
 *                                             Y = Ybar A^{-1});
 *   nvec = last column of Ainv    [G][S]     (the combination of the K+2
 *                                             results that must vanish,
 *                                             section Computational Integrity);
 *   B[j][i] = Ainv[j][i]/gamma[j] [G][S][K]  (so that B^T Gamma A^T = [I|0],
 *                                             Backward Propagation matrix
 *                                             relation).
 * All pointers are host memory; outputs may be NULL to skip them. */
dk_status dk_coeffs(const float *A, const float *gamma, int G, int K,
                    float *Ainv, float *nvec, float *B);

/* Encoding (Forward Pass, DarKnight Encoding equation, plus the extra
 * combination of section Computational Integrity):
 *   xbar[gS+j][e] = sum_{i<K} A[g][i][j] x[gK+i][e] + A[g][K][j] r[g][e]
 * x[G*K][n], r[G][n], A[G][S][S] (all device) -> xbar[G*S][n] (device). */
dk_status dk_encode(const float *x, const float *r, const float *A,
                    float *xbar, int G, int K, long long n, void *stream);

/* The bilinear operation on encoded rows, dense case (Forward Pass):
 *   ybar[R][M] = xbar[R][N] . W[M][N]^T.
 * ws: device workspace of at least dk_workspace_bytes(L, DK_OP_FWD, ..). */
dk_status dk_linear_fwd(const float *W, const float *xbar, float *ybar,
                        int M, int N, int R, void *ws, size_t ws_bytes,
                        void *stream);

/* The bilinear operation on encoded rows, convolution case: R encoded CHW
 * images xbar[R][Ci][H][W] -> ybar[R][Co][Ho][Wo]. */
dk_status dk_conv_fwd(const dk_layer *L, const float *W, const float *xbar,
                      float *ybar, int R, void *ws, size_t ws_bytes,
                      void *stream);

/* Masked weight gradient (Backward Propagation, gamma-weighted sum of the
 * per-encoding products Eq_j, summed over all G virtual batches as in the
 * large-batch aggregation):
 *   dtilde[gS+j] = gamma[g][j] * sum_{i<K} B[g][j][i] delta[gK+i]
 *   dW = (accumulate ? dW : 0) + scale * sum_rows <dtilde[row], xbar[row]>
 * where <.,.> is the outer product (dense) or the convolution weight-gradient
 * pairing.  xbar is the buffer dk_encode wrote at forward time.
 * delta[G*K][m], B[G][S][K], gamma[G][S], xbar[G*S][n] (device) -> dW with
 * the shape of W (device).  scale = 1/K gives the paper's average. */
dk_status dk_wgrad(const dk_layer *L, const float *delta, const float *B,
                   const float *gamma, const float *xbar, float *dW, int G,
                   int K, float scale, int accumulate, void *ws,
                   size_t ws_bytes, void *stream);

/* Decoding (Forward Pass, DarKnight Decoding): the K wanted columns of
 * Ybar . A^{-1}; the <W, r> column is not produced.
 *   y[gK+i][e] = sum_j ybar[gS+j][e] Ainv[g][j][i],  i < K
 * ybar[G*S][m], Ainv[G][S][S] (device) -> y[G*K][m] (device). */
dk_status dk_decode(const float *ybar, const float *Ainv, float *y, int G,
                    int K, long long m, void *stream);

/* Integrity check (section Computational Integrity).  Per group,
 *   t[e] = sum_j nvec[g][j] ybar[gS+j][e],  s[e] = sum_j |nvec[g][j] ybar[gS+j][e]|
 *   resid[g] = max_e |t| / max_e s   (0 if the denominator is 0, +inf if any
 *                                     t or s is not finite)
 *   verdict[g] = 1 if resid[g] > tol or not finite, else 0.
 * ybar[G*S][m], nvec[G][S] (device) -> verdict[G] int32, resid[G] (device;
 * resid may be NULL).  ws: at least dk_workspace_bytes(NULL, DK_OP_VERIFY, G, K),
 * 16-byte aligned, contents arbitrary: the workgroups that share a group
 * publish their maxima there under a tag drawn for the call, and the one that
 * finds all of them present writes the verdict, so the check is one launch.
 * Calls that overlap in time need workspaces of their own. */
dk_status dk_verify(const float *ybar, const float *nvec, float tol,
                    int *verdict, float *resid, int G, int K, long long m,
                    void *ws, size_t ws_bytes, void *stream);

/* dk_decode and dk_verify in one sweep over ybar (both read every encoded row
 * once): same arguments, same results as the two calls, one workspace of
 * dk_workspace_bytes(NULL, DK_OP_VERIFY, G, K). */
dk_status dk_decode_verify(const float *ybar, const float *Ainv,
                           const float *nvec, float tol, float *y,
                           int *verdict, float *resid, int G, int K,
                           long long m, void *ws, size_t ws_bytes,
                           void *stream);

/* ------------------------------------------------------------------------
 * Fused forms (the paper's pipelined mode keeps the encodings of the forward
 * pass for the backward pass and overlaps the trusted side's work with the
 * accelerators'; on one GPU the counterpart is to stop round trips through
 * memory between the mixing steps and the bilinear operation).
 * ------------------------------------------------------------------------ */

/* dk_conv_fwd followed by dk_decode_verify as one call:
 *   ybar = <W, xbar> on all G*(K+2) encoded images, y = first K columns of
 *   ybar A^{-1}, verdict/resid as in dk_verify.
 * For 1x1 filters with stride 1 and no padding and K in {2, 4, 8} the encoded
 * results never reach memory: a workgroup runs a virtual batch's K+2 products
 * one after the other and folds each result tile into the decoded tiles and
 * the integrity sums it keeps in registers.  Every other layer runs the two
 * steps one after the other with ybar in the workspace.
 * W, xbar[G*(K+2)] images, Ainv[G][S][S], nvec[G][S] (device) -> y[G*K] images,
 * verdict[G], resid[G] (device; resid may be NULL).
 * ws: dk_conv_fwd_decode_verify_workspace_bytes(L, G, K), 256-byte aligned,
 * contents arbitrary. */
dk_status dk_conv_fwd_decode_verify(const dk_layer *L, const float *W, const float *xbar,
                                    const float *Ainv, const float *nvec, float tol, float *y,
                                    int *verdict, float *resid, int G, int K, void *ws,
                                    size_t ws_bytes, void *stream);
size_t dk_conv_fwd_decode_verify_workspace_bytes(const dk_layer *L, int G, int K);

/* Switches between the fused and the separate kernels where both exist.
 *   DK_OPT_FUSE_FWD    dk_conv_fwd_decode_verify on eligible 1x1 layers;
 *   DK_OPT_FUSE_WGRAD  dk_wgrad on 1x1 stride-1 layers (K in {2, 4, 8}, images
 *                      of a multiple of 16 pixels, 16-byte aligned tensors):
 *                      the gradient mixing runs inside the contraction's
 *                      operand loader and dtilde is never written.
 * value: DK_FUSE_NEVER, DK_FUSE_ALWAYS (whenever eligible) or DK_FUSE_AUTO
 * (the library's own choice by layer shape; the default).  Process-wide. */
enum { DK_OPT_FUSE_FWD = 0, DK_OPT_FUSE_WGRAD = 1, DK_OPT_COUNT = 2 };
enum { DK_FUSE_NEVER = 0, DK_FUSE_ALWAYS = 1, DK_FUSE_AUTO = 2 };
dk_status dk_set_option(int which, int value);
int dk_get_option(int which);

/* dk_decode_verify for callers that cannot allocate device memory and so
 * have no workspace to pass: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments (minus ws), same
 * kernels and bit-identical results; the per-workgroup maxima of the
 * integrity check go to an array of DK_STATIC_SCRATCH_BYTES bytes built into the
 * library's device code (each GPU the library runs on holds it until the
 * process ends), whose address is looked up once per device on the first
 * call there.  The call allocates and frees nothing.
 * Limit: G <= DK_STATIC_MAX_G, else DK_ERR_STATIC_LIMIT and nothing is
 * launched.  All calls on one GPU share the array: calls that overlap there
 * (different streams, or graphs replayed concurrently) race on it and give
 * undefined verdicts; calls that follow each other on one stream are safe,
 * and nothing needs clearing between them (a slot of the array counts only
 * if it carries the call's own tag, and a call resets the tags it set). */
#define DK_STATIC_SCRATCH_BYTES (4u << 20)
#define DK_STATIC_MAX_G 4096
dk_status dk_decode_verify_static(const float *ybar, const float *Ainv,
                                  const float *nvec, float tol, float *y,
                                  int *verdict, float *resid, int G, int K,
                                  long long m, void *stream);
size_t dk_static_scratch_bytes(void);

/* Optional per-kernel timing for benchmarks (not part of the method).  While
 * enabled (on = 1 also clears earlier records) every kernel the library
 * launches is bracketed by two HIP events on its launch stream; the library
 * creates and keeps those events (up to 8192 launches are recorded, later ones
 * are not timed).  Not thread-safe. */
dk_status dk_profile_enable(int on);

/* Diagnostic (for the roofline discussion, not part of the path): launches a
 * kernel that does nothing but fp32 matrix instructions, `iterations` x 16 per
 * wave on one wave per SIMD of 256 compute units, with constant operands
 * (random_operands = 0) or pseudo-random ones (1) in registers, and stores the
 * FLOP of the launch in *flop (host, may be NULL).  Timed with events on
 * `stream`, FLOP / time is what the matrix pipe sustains for such operands
 * when nothing else limits it. */
dk_status dk_probe_mfma_rate(int random_operands, int iterations, double *flop, void *stream);

/* Waits for the recorded events and returns the number of distinct kernel
 * labels; for 0 <= index < that number also writes the label (host buffer of
 * name_cap bytes), its average launch duration in milliseconds and its launch
 * count.  Any output pointer may be NULL. */
int dk_profile_read(int index, char *name, int name_cap, double *avg_ms,
                    int *launches);

/* ------------------------------------------------------------------------
 * Several colluding accelerators (section "Colluding GPUs").  To keep the
 * inputs private from any M accelerators that pool what they see, a group is
 * encoded with M independent noise vectors: Xbar = X A_1 + R A_2 with
 * S = K + M encodings, plus the one redundant encoding of section
 * "Computational Integrity", so S = K + M + 1 here.  A[g] is S x S: rows
 * 0..K-1 are A_1, rows K..K+M-1 are A_2, the last row belongs to the phantom
 * all-zero source.  Everything else is as in the entry points above, which
 * are the case M = 1; the forward entry points take R = G*S rows unchanged.
 * Requires K + M - 1 <= DK_MAX_K.
 * ------------------------------------------------------------------------ */

/* dk_coeffs for S = K+M+1: Ainv[G][S][S], nvec[G][S] (last column of Ainv),
 * B[G][S][K] with B[j][i] = Ainv[j][i]/gamma[j], which satisfies the
 * section's relation B^T Gamma A = [I_K | 0] over the K+M real sources.
 * Host pointers. */
dk_status dk_coeffs_m(const float *A, const float *gamma, int G, int K, int M,
                      float *Ainv, float *nvec, float *B);

/* xbar[gS+j] = sum_{i<K} A[g][i][j] x[gK+i] + sum_{q<M} A[g][K+q][j] r[gM+q].
 * x[G*K][n], r[G*M][n], A[G][S][S] -> xbar[G*S][n], all device. */
dk_status dk_encode_m(const float *x, const float *r, const float *A, float *xbar,
                      int G, int K, int M, long long n, void *stream);

/* dk_decode_verify for S = K+M+1 encodings per group: y[G*K][m] are the first
 * K columns of ybar A^{-1} (the M columns <W, r_q> are dropped), the verdict
 * tests the combination nvec as in dk_verify. */
dk_status dk_decode_verify_m(const float *ybar, const float *Ainv, const float *nvec, float tol,
                             float *y, int *verdict, float *resid, int G, int K, int M,
                             long long m, void *ws, size_t ws_bytes, void *stream);

/* dk_wgrad for S = K+M+1: Eq_j = < sum_{i<K} beta_{j,i} delta_i, xbar_j >,
 * dW = (accumulate ? dW : 0) + scale * sum_g sum_{j<S} gamma_j Eq_j.
 * delta[G*K][m], B[G][S][K], gamma[G][S], xbar[G*S][n] -> dW, all device.
 * Workspace: dk_workspace_bytes_m(L, DK_OP_WGRAD, G, K, M). */
dk_status dk_wgrad_m(const dk_layer *L, const float *delta, const float *B, const float *gamma,
                     const float *xbar, float *dW, int G, int K, int M, float scale,
                     int accumulate, void *ws, size_t ws_bytes, void *stream);

/* dk_workspace_bytes for S = K+M+1. */
size_t dk_workspace_bytes_m(const dk_layer *L, int op, int G, int K, int M);

/* ------------------------------------------------------------------------
 * Noise drawn inside the encoding kernel.  The noise vector of a virtual batch
 * is random and only ever used for that batch's encodings (Forward Pass, text
 * after the encoding equation: scalars and noise are generated at random, anew
 * for each virtual batch; it cancels in decoding and is never needed again), so
 * it does not have to exist in memory: a 64-bit seed stands for it.
 * Generator: Philox4x32, 10 rounds.  Elements 4b..4b+3 of noise row q of group
 * g come from one call with counter (b mod 2^32, b div 2^32, g, q) and key
 * (seed mod 2^32, seed div 2^32): the four words w give uniforms
 * u = ((w >> 8) + 1/2) 2^-24 and the two Box-Muller pairs
 * sqrt(-2 ln u0) (cos, sin)(2 pi u1), sqrt(-2 ln u2) (cos, sin)(2 pi u3),
 * times noise_std.  Use a fresh seed for every layer and step.
 * ------------------------------------------------------------------------ */

/* The noise rows a seed stands for, written out: r[G*M][n] (device).  For
 * tests and for callers that want the rows; dk_encode_rng does not need it. */
dk_status dk_noise_rng(float *r, int G, int M, long long n, unsigned long long seed,
                       float noise_std, void *stream);

/* dk_encode_m (M = 1: dk_encode) with r = dk_noise_rng(seed, noise_std)
 * generated on the fly; the result equals dk_encode_m on those rows bit for
 * bit.  x[G*K][n], A[G][S][S] -> xbar[G*S][n], S = K+M+1, all device. */
dk_status dk_encode_rng(const float *x, const float *A, float *xbar, int G, int K, int M,
                        long long n, unsigned long long seed, float noise_std, void *stream);

/* ------------------------------------------------------------------------
 * Data gradient (Backward Propagation, second linear operation: the gradient
 * with respect to a layer's input is computed from the next layer's gradient
 * and the weights only; it holds no private input and runs un-encoded).  Not
 * part of the masked path; provided so that a whole backward pass can run on
 * the library.  It is the transpose of the layer's forward map:
 *   dense      dx[r][k]        = sum_o delta[r][o] W[o][k];
 *   conv       dx[r][ci][i][j] = sum_{co,a,b} delta[r][co][h][w] W[co][ci][a][b]
 *                                over the (h, w) with h*stride+a-pad = i,
 *                                w*stride+b-pad = j;
 *   depthwise  the same with co = ci.
 * W (shape of the layer's weights), delta[R][m] -> dx[R][n], all device.
 * Stride-1 convolutions with square filters run as a forward convolution with
 * transposed, flipped filters; other convolution geometries gather delta
 * through the generic contraction engine.  Workspace: dk_dgrad_workspace_bytes(L, R), 256-byte aligned.
 * ------------------------------------------------------------------------ */
dk_status dk_dgrad(const dk_layer *L, const float *W, const float *delta, float *dx, int R,
                   void *ws, size_t ws_bytes, void *stream);
size_t dk_dgrad_workspace_bytes(const dk_layer *L, int R);

#ifdef __cplusplus
}
#endif
#endif /* DARKNIGHT_H */
