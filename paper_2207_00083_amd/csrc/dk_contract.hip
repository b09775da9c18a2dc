// The contractions of the masked layer on fp32 MFMA tiles: the layer's
// forward on encoded rows (dense product, convolution as implicit GEMM) and
// the weight gradient as one contraction of the mixed gradients with the
// stored encodings.
//
// One engine serves all four: a workgroup of 64-lane waves owns a BM x BN
// output tile and walks the contraction axis in steps of BK.  Both operands
// are staged through LDS "k-major" (As[k][row], Bs[k][col]) so that the
// v_mfma_f32_32x32x2_f32 operand fetch (lane l supplies row l%32 of k-slice
// l/32) is one conflict-free ds_read_b32 per operand block.  Global loads for
// step t+1 are issued before the MFMA loop of step t and land in the other
// LDS buffer after it (register-staged double buffering, one barrier per
// step).  What differs per operation is only how an operand tile is fetched
// from HBM (the loader) and where an output element lives (the epilogue).
#include "dk_internal.h"
#include "dk_patch.h"

namespace {

#include "dk_contract_tiles.h"

struct ConvParams {
    const float *p;       // xbar[R][Ci][H][W] or dtilde[R][Co][Ho][Wo]
    int Ci, Co, H, W, kh, kw, stride, pad, Ho, Wo;
    int HoWo, Kg;         // Ho*Wo, Ci*kh*kw
    int Q;                // R*Ho*Wo output pixels over all encoded rows
    long long img;        // Ci*H*W
};

// Convolution forward, B operand: rows = output pixels q = (r, ho, wo),
// contraction k = (ci, a, b); element = xbar[r][ci][ho*s+a-p][wo*s+b-p].
template <int ROWS, int BK, int NT, int LD>
struct LoadIm2colFwd {
    using Params = ConvParams;
    static constexpr int KSTEP = NT / ROWS;
    static constexpr int NE = BK / KSTEP;
    static_assert(NT % ROWS == 0 && BK % KSTEP == 0, "tile/threads");
    float st[NE];
    const float *base; int H, W, kh, kw, Kg, ih0, iw0, pcol, ksub; bool valid;

    __device__ __forceinline__ void init(const Params &a, int q0, int tid)
    {
        pcol = tid % ROWS; ksub = tid / ROWS;
        H = a.H; W = a.W; kh = a.kh; kw = a.kw; Kg = a.Kg;
        const int q = q0 + pcol;
        valid = q < a.Q;
        const int r = valid ? q / a.HoWo : 0;
        const int pix = valid ? q - r * a.HoWo : 0;
        const int ho = pix / a.Wo, wo = pix - ho * a.Wo;
        ih0 = ho * a.stride - a.pad;
        iw0 = wo * a.stride - a.pad;
        base = a.p + (long long)r * a.img;
    }

    __device__ __forceinline__ void load(int kt)
    {
        int k = kt * BK + ksub;
        int ci = k / (kh * kw);
        int rem = k - ci * (kh * kw);
        int fa = rem / kw, fb = rem - fa * kw;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int ih = ih0 + fa, iw = iw0 + fb;
            const bool ok = valid && k < Kg && (unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W;
            st[e] = ok ? base[((long long)ci * H + ih) * W + iw] : 0.0f;
            k += KSTEP; fb += KSTEP;
            while (fb >= kw) { fb -= kw; ++fa; }
            while (fa >= kh) { fa -= kh; ++ci; }
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < NE; ++e) buf[(ksub + e * KSTEP) * LD + pcol] = st[e];
    }
};

// Convolution data gradient, B operand: rows = input pixels q = (r, i, j),
// contraction k = (co, a, b); element = delta[r][co][(i+p-a)/s][(j+p-b)/s] when
// both quotients are whole and inside the output, else 0.  ConvParams are those
// of the layer with p pointing at delta; Q = R*H*W, HoWo stands for H*W here.
template <int ROWS, int BK, int NT, int LD>
struct LoadIm2colDgrad {
    using Params = ConvParams;
    static constexpr int KSTEP = NT / ROWS;
    static constexpr int NE = BK / KSTEP;
    static_assert(NT % ROWS == 0 && BK % KSTEP == 0, "tile/threads");
    float st[NE];
    const float *base; int Ho, Wo, kh, kw, Kg, stride, ip, jp, pcol, ksub; bool valid;

    __device__ __forceinline__ void init(const Params &a, int q0, int tid)
    {
        pcol = tid % ROWS; ksub = tid / ROWS;
        Ho = a.Ho; Wo = a.Wo; kh = a.kh; kw = a.kw; Kg = a.Co * a.kh * a.kw; stride = a.stride;
        const int q = q0 + pcol;
        const int HW = a.H * a.W;
        valid = q < a.Q;
        const int r = valid ? q / HW : 0;
        const int pix = valid ? q - r * HW : 0;
        const int i = pix / a.W, j = pix - i * a.W;
        ip = i + a.pad; jp = j + a.pad;
        base = a.p + (long long)r * a.Co * a.Ho * a.Wo;
    }

    __device__ __forceinline__ void load(int kt)
    {
        int k = kt * BK + ksub;
        int co = k / (kh * kw);
        int rem = k - co * (kh * kw);
        int fa = rem / kw, fb = rem - fa * kw;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int hn = ip - fa, wn = jp - fb;
            const int h = hn / stride, w = wn / stride;
            const bool ok = valid && k < Kg && hn >= 0 && wn >= 0 && h * stride == hn && w * stride == wn &&
                            h < Ho && w < Wo;
            st[e] = ok ? base[((long long)co * Ho + h) * Wo + w] : 0.0f;
            k += KSTEP; fb += KSTEP;
            while (fb >= kw) { fb -= kw; ++fa; }
            while (fa >= kh) { fa -= kh; ++co; }
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < NE; ++e) buf[(ksub + e * KSTEP) * LD + pcol] = st[e];
    }
};

// Data gradient of a strided convolution, one class of input pixels at a time.
// With stride s, an input pixel (i, j) receives only the filter taps
// a = (i + pad) mod s, + s, + 2s, ... (likewise b), so the pixels of one
// residue class (i mod s, j mod s) = (pi, pj) all use the same sub-filter of
// na x nb taps a = a0 + s a', b = b0 + s b', and for pixel i = s u + pi the
// gradient row it meets is h = u + bh - a' with bh = (pi + pad - a0) / s: a
// stride-1 correlation without the structural zeros of the full gather.
struct DgradClassParams {
    const float *p;       // delta[R][Co][Ho][Wo]
    int Co, Ho, Wo;
    int U, V;             // pixels of the class per image: rows, columns
    int na, nb, bh, bw;
    int Kc;               // Co*na*nb
    int Q;                // R*U*V
};

// B operand: rows = class pixels q = (r, u, v), contraction k = (co, a', b').
// When the class's tap count divides the step (1, 2 or 4 taps of a 3x3 or 1x1
// filter), a lane's elements of a step are the same taps of consecutive channel
// groups in every step: their offsets are computed once, a step only moves a
// scalar offset on, and taps outside the gradient image read as zero through
// the buffer's range check.
template <int ROWS, int BK, int NT, int LD>
struct LoadDgradClass {
    using Params = DgradClassParams;
    static constexpr int KSTEP = NT / ROWS;
    static constexpr int NE = BK / KSTEP;
    static_assert(NT % ROWS == 0 && BK % KSTEP == 0, "tile/threads");
    float st[NE];
    const float *base; int Ho, Wo, na, nb, Kc, h0, w0, pcol, ksub; bool valid;
    __amdgpu_buffer_rsrc_t rs; unsigned voff[NE]; unsigned step_bytes; bool fast;

    __device__ __forceinline__ void init(const Params &a, int q0, int tid)
    {
        pcol = tid % ROWS; ksub = tid / ROWS;
        Ho = a.Ho; Wo = a.Wo; na = a.na; nb = a.nb; Kc = a.Kc;
        const int q = q0 + pcol;
        const int UV = a.U * a.V;
        valid = q < a.Q;
        const int r = valid ? q / UV : 0;
        const int pix = valid ? q - r * UV : 0;
        const int u = pix / a.V, v = pix - u * a.V;
        h0 = u + a.bh; w0 = v + a.bw;
        base = a.p + (long long)r * a.Co * a.Ho * a.Wo;
        const int tn = na * nb;
        const long long bytes = (long long)(a.Q / UV) * a.Co * a.Ho * a.Wo * 4;
        fast = BK % tn == 0 && bytes <= DK_RSRC_MAX;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
        step_bytes = 4u * (unsigned)(BK / tn) * (unsigned)(a.Ho * a.Wo);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int k = ksub + e * KSTEP;          // position within a step
            const int co = k / tn, rem = k - co * tn;
            const int fa = rem / nb, fb = rem - fa * nb;
            const int h = h0 - fa, w = w0 - fb;
            const bool ok = valid && (unsigned)h < (unsigned)Ho && (unsigned)w < (unsigned)Wo;
            voff[e] = ok ? 4u * (unsigned)(((r * a.Co + co) * a.Ho + h) * a.Wo + w) : DK_OOB;
        }
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= Kc) {
            const unsigned soff = (unsigned)kt * step_bytes;
#pragma unroll
            for (int e = 0; e < NE; ++e)
                st[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)voff[e], (int)soff, 0));
            return;
        }
        int k = kt * BK + ksub;
        int co = k / (na * nb);
        int rem = k - co * (na * nb);
        int fa = rem / nb, fb = rem - fa * nb;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int h = h0 - fa, w = w0 - fb;
            const bool ok = valid && k < Kc && (unsigned)h < (unsigned)Ho && (unsigned)w < (unsigned)Wo;
            st[e] = ok ? base[((long long)co * Ho + h) * Wo + w] : 0.0f;
            k += KSTEP; fb += KSTEP;
            while (fb >= nb) { fb -= nb; ++fa; }
            while (fa >= na) { fa -= na; ++co; }
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < NE; ++e) buf[(ksub + e * KSTEP) * LD + pcol] = st[e];
    }
};

// Convolution weight gradient, A operand: rows = co, contraction q = (r, pix);
// element = dtilde[r][co][pix].
template <int ROWS, int BK, int NT, int LD>
struct LoadDeltaQ {
    using Params = ConvParams;
    static constexpr int RSTEP = NT / BK;
    static constexpr int NE = ROWS / RSTEP;
    static_assert(NT % BK == 0 && ROWS % RSTEP == 0, "tile/threads");
    float st[NE];
    const float *p; int Co, HoWo, Q, row0, kq, rsub;
    // fast path (whole steps): the lane's pixel as a cursor (pixel within its
    // image, byte offset of the image) that moves on by BK pixels per step, one
    // precomputed byte offset per row, buffer loads
    __amdgpu_buffer_rsrc_t rs; unsigned coff[NE]; bool fast;
    int cur_kt, cur_pix; unsigned cur_img;

    __device__ __forceinline__ void init(const Params &a, int row0_, int tid)
    {
        p = a.p; Co = a.Co; HoWo = a.HoWo; Q = a.Q; row0 = row0_; kq = tid % BK; rsub = tid / BK;
        const long long bytes = (long long)(a.Q / a.HoWo) * a.Co * a.HoWo * 4;
        fast = bytes <= DK_RSRC_MAX && HoWo >= BK;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int co = row0 + rsub + e * RSTEP;
            coff[e] = co < Co ? 4u * (unsigned)co * (unsigned)HoWo : DK_OOB;
        }
        cur_kt = -2; cur_pix = 0; cur_img = 0;
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= Q) {
            if (cur_kt + 1 == kt) {
                cur_pix += BK;
                if (cur_pix >= HoWo) { cur_pix -= HoWo; cur_img += 4u * (unsigned)Co * (unsigned)HoWo; }
            } else {
                const int q = kt * BK + kq;
                const int r = q / HoWo;
                cur_pix = q - r * HoWo;
                cur_img = 4u * (unsigned)r * (unsigned)Co * (unsigned)HoWo;
            }
            cur_kt = kt;
            const unsigned base = cur_img + 4u * (unsigned)cur_pix;
#pragma unroll
            for (int e = 0; e < NE; ++e)
                st[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(base + coff[e]), 0, 0));
            return;
        }
        cur_kt = -2;
        const int q = kt * BK + kq;
        const bool ok = q < Q;
        const int r = ok ? q / HoWo : 0;
        const int pix = ok ? q - r * HoWo : 0;
        const float *s = p + (long long)r * Co * HoWo + pix;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int co = row0 + rsub + e * RSTEP;
            st[e] = (ok && co < Co) ? s[(long long)co * HoWo] : 0.0f;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < NE; ++e) buf[kq * LD + rsub + e * RSTEP] = st[e];
    }
};

// Convolution weight gradient, B operand: rows = j = (ci, a, b), contraction
// q = (r, ho, wo); element = xbar[r][ci][ho*s+a-p][wo*s+b-p].
template <int ROWS, int BK, int NT, int LD>
struct LoadIm2colQ {
    using Params = ConvParams;
    static constexpr int RSTEP = NT / BK;
    static constexpr int NE = ROWS / RSTEP;
    static_assert(NT % BK == 0 && ROWS % RSTEP == 0, "tile/threads");
    float st[NE];
    int joff[NE];          // (ci*H + a)*W + b
    short fa[NE], fb[NE];  // filter tap; fa = -20000 marks a row beyond Kg
    const float *p; int H, W, Wo, HoWo, Q, stride, pad, kq, rsub; long long img;
    // fast path (whole steps): pixel cursor as in LoadDeltaQ; the output row of
    // the pixel comes from a multiplication by ceil(2^32 / Wo) (exact below 2^16)
    __amdgpu_buffer_rsrc_t rs; bool fast;
    int cur_kt, cur_pix; unsigned cur_img, wo_magic;

    __device__ __forceinline__ void init(const Params &a, int row0, int tid)
    {
        p = a.p; H = a.H; W = a.W; Wo = a.Wo; HoWo = a.HoWo; Q = a.Q;
        stride = a.stride; pad = a.pad; img = a.img;
        kq = tid % BK; rsub = tid / BK;
        const long long bytes = (long long)(a.Q / a.HoWo) * a.img * 4;
        fast = bytes <= DK_RSRC_MAX && HoWo >= BK && HoWo < 65536 && Wo > 1;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
        wo_magic = (unsigned)((0x100000000ull + (unsigned)Wo - 1) / (unsigned)Wo);
        cur_kt = -2; cur_pix = 0; cur_img = 0;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int j = row0 + rsub + e * RSTEP;
            const int ci = j / (a.kh * a.kw);
            const int rem = j - ci * (a.kh * a.kw);
            const int ta = rem / a.kw, tb = rem - ta * a.kw;
            const bool ok = j < a.Kg;
            joff[e] = ok ? (ci * H + ta) * W + tb : 0;
            fa[e] = ok ? (short)ta : (short)-20000;
            fb[e] = (short)tb;
        }
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= Q) {
            if (cur_kt + 1 == kt) {
                cur_pix += BK;
                if (cur_pix >= HoWo) { cur_pix -= HoWo; cur_img += 4u * (unsigned)img; }
            } else {
                const int q = kt * BK + kq;
                const int r = q / HoWo;
                cur_pix = q - r * HoWo;
                cur_img = 4u * (unsigned)r * (unsigned)img;
            }
            cur_kt = kt;
            const int ho = (int)__umulhi((unsigned)cur_pix, wo_magic), wo = cur_pix - ho * Wo;
            const int ih0 = ho * stride - pad, iw0 = wo * stride - pad;
            // (wraps below zero for border pixels; adding a valid tap's offset brings it back)
            const unsigned base = cur_img + 4u * (unsigned)(ih0 * W + iw0);
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const bool ok = (unsigned)(ih0 + fa[e]) < (unsigned)H && (unsigned)(iw0 + fb[e]) < (unsigned)W;
                const unsigned off = ok ? base + 4u * (unsigned)joff[e] : DK_OOB;
                st[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)off, 0, 0));
            }
            return;
        }
        cur_kt = -2;
        const int q = kt * BK + kq;
        const bool okq = q < Q;
        const int r = okq ? q / HoWo : 0;
        const int pix = okq ? q - r * HoWo : 0;
        const int ho = pix / Wo, wo = pix - ho * Wo;
        const int ih0 = ho * stride - pad, iw0 = wo * stride - pad;
        const long long b0 = (long long)r * img + (long long)ih0 * W + iw0;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int ih = ih0 + fa[e], iw = iw0 + fb[e];
            const bool ok = okq && (unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W;
            st[e] = ok ? p[b0 + joff[e]] : 0.0f;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < NE; ++e) buf[kq * LD + rsub + e * RSTEP] = st[e];
    }
};

// 1x1 convolution without padding = one product per image: no gather is
// needed, only addressing that knows where an image starts (and, with a
// stride, which pixels of the stored image the output pixels sit on).
struct ImgParams {
    const float *p;     // [R][C][chs]
    int C, HW;          // channels per image, pixels per image that take part
    int Q;              // R*HW
    int chs;            // floats between channels (= HW without a stride)
    int Wo, Wi, stride; // pixel pix = (ho, wo) is stored at (ho*stride)*Wi + wo*stride
    __device__ __forceinline__ const float *pixel(int q) const
    {
        const int r = q / HW, pix = q - r * HW;
        int off = pix;
        if (stride != 1) { const int ho = pix / Wo; off = (ho * Wi + (pix - ho * Wo)) * stride; }
        return p + (long long)r * C * chs + off;
    }
};

// Forward B operand: rows = pixels q = (r, pix), contraction = input channel;
// element = x[r][k][pix], pixels contiguous.
template <int ROWS, int BK, int NT, int LD, bool VEC>
struct LoadKMajorImg {
    using Params = ImgParams;
    static constexpr int PER_K = ROWS / 4;
    static constexpr int N4 = BK * PER_K / NT;
    static_assert(BK * PER_K % NT == 0 && NT % PER_K == 0, "tile/threads");
    float4 st[N4];
    const float *src[VEC ? 1 : 4];   // element (k = 0) of this lane's pixel(s); null = outside
    int C, chs, tid;
    __amdgpu_buffer_rsrc_t rs; unsigned voff[N4]; bool fast;
    unsigned poff[VEC ? 1 : 4];      // single pixels (rows that are not whole 16-byte vectors): byte offsets

    __device__ __forceinline__ void init(const Params &a, int q0, int tid_)
    {
        C = a.C; chs = a.chs; tid = tid_;
        const int q = q0 + (tid % PER_K) * 4;
#pragma unroll
        for (int u = 0; u < (VEC ? 1 : 4); ++u) {
            const int qq = q + u;
            src[u] = qq < a.Q ? a.pixel(qq) : nullptr;
        }
        // whole tensor as one resource: [R][C][chs]
        const long long bytes = (long long)(a.Q / a.HW) * a.C * a.chs * 4;
        fast = bytes <= DK_RSRC_MAX;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int kr = (tid + e * NT) / PER_K;
            voff[e] = VEC ? (src[0] ? 4u * (unsigned)((src[0] - a.p) + (long long)kr * chs) : DK_OOB)
                          : 4u * (unsigned)kr * (unsigned)chs;
        }
#pragma unroll
        for (int u = 0; u < (VEC ? 1 : 4); ++u)
            poff[u] = src[u] ? 4u * (unsigned)(src[u] - a.p) : DK_OOB;     // (DK_OOB + a row offset stays out of range)
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= C) {
            const unsigned soff = 4u * (unsigned)(kt * BK) * (unsigned)chs;
            if constexpr (VEC) {
#pragma unroll
                for (int e = 0; e < N4; ++e) st[e] = dk_buffer_load4(rs, voff[e], soff);
            } else {
                // four single pixels of a channel, possibly of two images
#pragma unroll
                for (int e = 0; e < N4; ++e) {
                    float v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        v[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                             rs, (int)(poff[u] + voff[e]), (int)soff, 0));
                    st[e] = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
            return;
        }
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int k = kt * BK + (tid + e * NT) / PER_K;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < C) {
                const long long ko = (long long)k * chs;
                if constexpr (VEC) {
                    if (src[0]) v = *reinterpret_cast<const float4 *>(src[0] + ko);
                } else {
                    if (src[0]) v.x = src[0][ko];
                    if (src[1]) v.y = src[1][ko];
                    if (src[2]) v.z = src[2][ko];
                    if (src[3]) v.w = src[3][ko];
                }
            }
            st[e] = v;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            *reinterpret_cast<float4 *>(buf + (idx / PER_K) * LD + (idx % PER_K) * 4) = st[e];
        }
    }
};

// Weight-gradient operands: rows = channel, contraction = pixels q = (r, pix);
// element = t[r][row][pix].
template <int ROWS, int BK, int NT, int LD, bool VEC>
struct LoadRowMajorKImg {
    using Params = ImgParams;
    static constexpr int PER_ROW = BK / 4;
    static constexpr int N4 = ROWS * PER_ROW / NT;
    static_assert(ROWS * PER_ROW % NT == 0 && NT % PER_ROW == 0, "tile/threads");
    float4 st[N4];
    const float *p; int C, HW, Q, row0, tid;
    // fast path: the lane's pixel quad as a cursor (pixel within its image, byte
    // offset of (image, channel 0, pixel)) that moves on by BK pixels per step
    __amdgpu_buffer_rsrc_t rs; unsigned roff[N4]; bool fast;
    int cur_kt, cur_pix; unsigned cur_off;

    // (stride-1 layers only: chs == HW)
    __device__ __forceinline__ void init(const Params &a, int row0_, int tid_)
    {
        p = a.p; C = a.C; HW = a.HW; Q = a.Q; row0 = row0_; tid = tid_;
        const long long bytes = (long long)(a.Q / a.HW) * a.C * a.HW * 4;
        fast = bytes <= DK_RSRC_MAX && HW >= BK;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int row = row0 + (tid + e * NT) / PER_ROW;
            roff[e] = row < C ? 4u * (unsigned)row * (unsigned)HW : DK_OOB;
        }
        cur_kt = -2; cur_pix = 0; cur_off = 0;      // no step fetched yet
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= Q) {
            if (cur_kt + 1 == kt) {              // the usual case: one step on
                cur_pix += BK; cur_off += 4u * BK;
                if (cur_pix >= HW) { cur_pix -= HW; cur_off += 4u * (unsigned)(C - 1) * (unsigned)HW; }
            } else {
                const int q = kt * BK + (tid % PER_ROW) * 4;
                const int r = q / HW;
                cur_pix = q - r * HW;
                cur_off = 4u * ((unsigned)r * (unsigned)C * (unsigned)HW + (unsigned)cur_pix);
            }
            cur_kt = kt;
            if constexpr (VEC) {
#pragma unroll
                for (int e = 0; e < N4; ++e) st[e] = dk_buffer_load4(rs, roff[e] + cur_off, 0u);
            } else {
                // four single pixels; one that runs past its image is the next image's first
                unsigned po[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    po[u] = cur_off + 4u * u + (cur_pix + u >= HW ? 4u * (unsigned)(C - 1) * (unsigned)HW : 0u);
#pragma unroll
                for (int e = 0; e < N4; ++e) {
                    float v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        v[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(roff[e] + po[u]), 0, 0));
                    st[e] = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
            return;
        }
        cur_kt = -2;
        const int q = kt * BK + (tid % PER_ROW) * 4;
        const float *s[VEC ? 1 : 4];
#pragma unroll
        for (int u = 0; u < (VEC ? 1 : 4); ++u) {
            const int qq = q + u;
            const int r = qq / HW, pix = qq - r * HW;
            s[u] = qq < Q ? p + (long long)r * C * HW + pix : nullptr;
        }
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int row = row0 + (tid + e * NT) / PER_ROW;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < C) {
                const long long ro = (long long)row * HW;
                if constexpr (VEC) {
                    if (s[0]) v = *reinterpret_cast<const float4 *>(s[0] + ro);
                } else {
                    if (s[0]) v.x = s[0][ro];
                    if (s[1]) v.y = s[1][ro];
                    if (s[2]) v.z = s[2][ro];
                    if (s[3]) v.w = s[3][ro];
                }
            }
            st[e] = v;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int row = idx / PER_ROW, kc = idx % PER_ROW;
            float *d = buf + (kc * 4) * LD + row;
            d[0 * LD] = st[e].x;
            d[1 * LD] = st[e].y;
            d[2 * LD] = st[e].z;
            d[3 * LD] = st[e].w;
        }
    }
};

// ---------------------------------------------------------------------------
// Epilogues: where output element (row, col) lives.
// ---------------------------------------------------------------------------

struct EpiDense {            // C[row][col], leading dimension ld
    long long ld; int rows, cols;
    __device__ __forceinline__ bool col_ok(int col) const { return col < cols; }
    __device__ __forceinline__ long long col_off(int col) const { return col; }
    __device__ __forceinline__ long long row_off(int row) const { return (long long)row * ld; }
};

struct EpiConvFwd {          // ybar[r][co][pix]; row = co, col = q = r*HoWo + pix
    int rows, cols, HoWo; long long chw;   // chw = Co*HoWo
    __device__ __forceinline__ bool col_ok(int col) const { return col < cols; }
    __device__ __forceinline__ long long col_off(int col) const
    { const int r = col / HoWo; return (long long)r * chw + (col - r * HoWo); }
    __device__ __forceinline__ long long row_off(int row) const { return (long long)row * HoWo; }
};

struct EpiDgradClass {       // dx[r][ci][s u + pi][s v + pj]; row = ci, col = q = (r, u, v)
    int rows, cols, U, V, stride, pi, pj, Wd; long long hw, chw;   // hw = H*W, chw = Ci*H*W
    __device__ __forceinline__ bool col_ok(int col) const { return col < cols; }
    __device__ __forceinline__ long long col_off(int col) const
    {
        const int UV = U * V;
        const int r = col / UV, pix = col - r * UV;
        const int u = pix / V, v = pix - u * V;
        return (long long)r * chw + (long long)(u * stride + pi) * Wd + v * stride + pj;
    }
    __device__ __forceinline__ long long row_off(int row) const { return (long long)row * hw; }
};

// ---------------------------------------------------------------------------
// The engine.
// ---------------------------------------------------------------------------

struct RunParams {
    int tiles_m, tiles_n;     // output tiles
    int ktiles, per_split;    // contraction steps in total / per K slice
    int splits;
    float alpha; int accumulate;
    float *out;               // final output (splits == 1) ...
    float *part;              // ... or partial sums [splits][out_elems]
    long long out_elems;
};

// One workgroup's share: tile `bid` of the run's tiles_m x tiles_n x splits.
template <class C, class LA, class LB, class EP>
__device__ __forceinline__ void contract_tile(const typename LA::Params &pa, const typename LB::Params &pb,
                                              const EP &ep, const RunParams &rp, const int bid)
{
    __shared__ __attribute__((aligned(16))) float lds[C::LDS_FLOATS];
    constexpr int A_BUF = C::BK * C::LDA, B_BUF = C::BK * C::LDB;
    float *const As = lds;                 // two buffers of A_BUF floats
    float *const Bs = lds + 2 * A_BUF;     // two buffers of B_BUF floats

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % C::WM) * (C::BM / C::WM);
    const int wn0 = (wave / C::WM) * (C::BN / C::WN);

    const int tiles = rp.tiles_m * rp.tiles_n;
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    // Tiles that run at the same time should share operand panels in both
    // directions: walk the output in bands of 8 tile rows, column by column
    // inside a band, so that the ~100 tiles resident on an XCD form a block of
    // about 8 x 12 instead of one or two whole tile columns.
    int tile_m, tile_n;
    {
        constexpr int GM = 8;
        const int band = t / (GM * rp.tiles_n);
        const int in_band = t - band * (GM * rp.tiles_n);
        const int rows_here = rp.tiles_m - band * GM < GM ? rp.tiles_m - band * GM : GM;
        tile_n = in_band / rows_here;
        tile_m = band * GM + (in_band - tile_n * rows_here);
    }
    const int row0 = tile_m * C::BM, col0 = tile_n * C::BN;

    LA la; LB lb;
    la.init(pa, row0, tid);
    lb.init(pb, col0, tid);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::TN; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const int kt0 = split * rp.per_split;
    int kt1 = kt0 + rp.per_split;
    if (kt1 > rp.ktiles) kt1 = rp.ktiles;

    const int li = lane & 31, lh = lane >> 5;
    if (kt0 < kt1) {
        la.load(kt0); lb.load(kt0);
        la.store(As); lb.store(Bs);
        __syncthreads();
        for (int kt = kt0; kt < kt1; ++kt) {
            const int cur = (kt - kt0) & 1;
            const bool more = kt + 1 < kt1;
            if (more) {
                // the next step's loads go out ahead of the MFMAs of the other waves
                // on this SIMD (their address arithmetic would queue behind them):
                // 8 % on the gather loaders, 0-4 % elsewhere; the same around the LDS
                // stores measured worse
                __builtin_amdgcn_s_setprio(3);
                la.load(kt + 1); lb.load(kt + 1);
                __builtin_amdgcn_s_setprio(0);
            }
            const float *a_s = As + cur * A_BUF + lh * C::LDA + wm0 + li;
            const float *b_s = Bs + cur * B_BUF + lh * C::LDB + wn0 + li;
#pragma unroll
            for (int kk = 0; kk < C::BK; kk += 2) {
                float a[C::TM], b[C::TN];
#pragma unroll
                for (int mi = 0; mi < C::TM; ++mi) a[mi] = a_s[kk * C::LDA + mi * 32];
#pragma unroll
                for (int ni = 0; ni < C::TN; ++ni) b[ni] = b_s[kk * C::LDB + ni * 32];
#pragma unroll
                for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < C::TN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
            }
            if (more) { la.store(As + (cur ^ 1) * A_BUF); lb.store(Bs + (cur ^ 1) * B_BUF); }
            __syncthreads();
        }
    }

    // 32x32 accumulator block: lane holds column li, rows 8*(v/4) + 4*lh + v%4.
    float *dst = rp.splits > 1 ? rp.part + (long long)split * rp.out_elems : rp.out;
    const bool direct = rp.splits == 1;
#pragma unroll
    for (int ni = 0; ni < C::TN; ++ni) {
        const int col = col0 + wn0 + ni * 32 + li;
        if (!ep.col_ok(col)) continue;
        const long long coff = ep.col_off(col);
#pragma unroll
        for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm0 + mi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (row >= ep.rows) continue;
                float *d = dst + ep.row_off(row) + coff;
                float val = acc[mi][ni][v];
                if (direct) {
                    val *= rp.alpha;
                    if (rp.accumulate) val += *d;
                }
                *d = val;
            }
    }
}

template <class C, class LA, class LB, class EP>
__global__ __launch_bounds__(C::NT) void contract_kernel(typename LA::Params pa,
                                                          typename LB::Params pb, EP ep,
                                                          RunParams rp)
{
    contract_tile<C, LA, LB, EP>(pa, pb, ep, rp, dk_xcd_block());
}

// Several independent contractions of the same kind in one launch (each too
// small to fill the chip alone).  The hardware deals workgroups to the eight
// XCDs in turn, so workgroup b is slot b / 8 of XCD b % 8; every XCD walks the
// runs in the order given (longest tiles first) and takes a contiguous eighth
// of each run's tiles (neighbours share operand panels in its L2): run c owns
// slots first[c] .. first[c + 1] - 1 of every XCD, slot s of XCD x being tile
// x (first[c + 1] - first[c]) + s - first[c]; slots past the run's last tile
// do nothing.  (One contiguous range of workgroups per run put all the long
// tiles on the first XCDs: twice the time for the strided data gradient.)
constexpr int DK_MAX_BATCH = 9;
template <class LA, class LB, class EP>
struct ContractBatch {
    typename LA::Params pa[DK_MAX_BATCH];
    typename LB::Params pb[DK_MAX_BATCH];
    EP ep[DK_MAX_BATCH];
    RunParams rp[DK_MAX_BATCH];
    int first[DK_MAX_BATCH + 1];
    int count;
};

template <class C, class LA, class LB, class EP>
__global__ __launch_bounds__(C::NT) void contract_batch_kernel(ContractBatch<LA, LB, EP> b)
{
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int c = 0;
    while (c + 1 < b.count && slot >= b.first[c + 1]) ++c;
    // wave-uniform, and the compiler has to know: taken for divergent, the run's parameters
    // land in vector registers and every buffer load is wrapped in a loop over the distinct
    // resource descriptors of the wave
    c = __builtin_amdgcn_readfirstlane(c);
    const int tile = xcd * (b.first[c + 1] - b.first[c]) + slot - b.first[c];
    if (tile >= b.rp[c].tiles_m * b.rp[c].tiles_n * b.rp[c].splits) return;
    contract_tile<C, LA, LB, EP>(b.pa[c], b.pb[c], b.ep[c], b.rp[c], tile);
}

// out[i] = (accumulate ? out[i] : 0) + alpha * sum_s part[s][i].  The order of
// the additions depends only on (splits, kernel variant), so reruns are bitwise
// identical.
//
// Few slices over a large output: one thread per 16 bytes of output walks the
// slices (bandwidth-bound, every byte read once).
template <bool VEC>
__global__ __launch_bounds__(256) void fold_wide_kernel(const float *__restrict__ part,
                                                        float *__restrict__ out, long long out_elems,
                                                        int splits, float alpha, int accumulate)
{
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * (VEC ? 4 : 1);
    if (i >= out_elems) return;
    if constexpr (VEC) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        int k = 0;
        for (; k + 4 <= splits; k += 4) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = *reinterpret_cast<const float4 *>(part + (long long)(k + u) * out_elems + i);
#pragma unroll
            for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
        }
        for (; k < splits; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(part + (long long)k * out_elems + i);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
        float4 *d = reinterpret_cast<float4 *>(out + i);
        if (accumulate) { const float4 o = *d; s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w; }
        *d = s;
    } else {
        float s = 0.0f;
        for (int k = 0; k < splits; ++k) s += part[(long long)k * out_elems + i];
        s *= alpha;
        if (accumulate) s += out[i];
        out[i] = s;
    }
}

// Many slices over a small output: a workgroup folds 64 consecutive elements,
// wave w of its SG waves sums slices w, w+SG, ... (loads batched eight deep)
// and the SG sub-sums are added in wave order.
template <int SG>
__global__ __launch_bounds__(64 * SG) void fold_deep_kernel(const float *__restrict__ part,
                                                            float *__restrict__ out, long long out_elems,
                                                            int splits, float alpha, int accumulate)
{
    __shared__ float red[SG][64];
    const int io = threadIdx.x & 63, sg = threadIdx.x >> 6;
    const long long i = (long long)blockIdx.x * 64 + io;
    float s = 0.0f;
    if (i < out_elems) {
        const float *src = part + i;
        int k = sg;
        for (; k + 7 * SG < splits; k += 8 * SG) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(long long)(k + SG * u) * out_elems];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; k < splits; k += SG) s += src[(long long)k * out_elems];
    }
    red[sg][io] = s;
    __syncthreads();
    if (sg != 0 || i >= out_elems) return;
    s = red[0][io];
#pragma unroll
    for (int w = 1; w < SG; ++w) s += red[w][io];
    s *= alpha;
    if (accumulate) s += out[i];
    out[i] = s;
}

} // namespace

dk_status dk_fold_slices(const float *part, float *out, long long out_elems, int splits, float alpha,
                         int accumulate, hipStream_t st)
{
    dk_prof_scope ps("splitk_reduce", st);
    // enough 16-byte columns to fill the chip: stream them; else spread the
    // slices of each column over the waves of a workgroup
    const bool vec = out_elems % 4 == 0 && dk_aligned(part, 16) && dk_aligned(out, 16);
    const long long cols = vec ? out_elems / 4 : out_elems;
    if (cols >= 256 * 1024 || splits <= 4) {
        const unsigned blocks = (unsigned)((cols + 255) / 256);
        if (vec) fold_wide_kernel<true><<<dim3(blocks), dim3(256), 0, st>>>(part, out, out_elems, splits, alpha, accumulate);
        else fold_wide_kernel<false><<<dim3(blocks), dim3(256), 0, st>>>(part, out, out_elems, splits, alpha, accumulate);
    } else {
        const unsigned blocks = (unsigned)((out_elems + 63) / 64);
        if (splits >= 64 && blocks < 2048)
            fold_deep_kernel<16><<<dim3(blocks), dim3(1024), 0, st>>>(part, out, out_elems, splits, alpha, accumulate);
        else
            fold_deep_kernel<4><<<dim3(blocks), dim3(256), 0, st>>>(part, out, out_elems, splits, alpha, accumulate);
    }
    return dk_launch_status();
}

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

template <class C, class LA, class LB, class EP>
dk_status run(const typename LA::Params &pa, const typename LB::Params &pb, const EP &ep,
              int rows, int cols, long long kdim, float alpha, int accumulate, float *out,
              long long out_elems, float *part, size_t part_bytes, hipStream_t st,
              const char *label, bool may_slice = true)
{
    RunParams rp;
    rp.tiles_m = (rows + C::BM - 1) / C::BM;
    rp.tiles_n = (cols + C::BN - 1) / C::BN;
    rp.ktiles = (int)((kdim + C::BK - 1) / C::BK);
    const long long tiles = (long long)rp.tiles_m * rp.tiles_n;
    // (an epilogue that scatters into a larger tensor cannot go through the
    // partial sums, which are laid out like the output: such callers do not slice)
    const dk_split_plan sp = may_slice ? dk_plan_split(tiles, rp.ktiles, out_elems, C::STEP_US)
                                       : dk_split_plan{1, rp.ktiles};
    rp.splits = sp.splits;
    rp.per_split = sp.ktiles_per_split;
    rp.alpha = alpha;
    rp.accumulate = accumulate;
    rp.out = out;
    rp.part = part;
    rp.out_elems = out_elems;
    DK_REQUIRE(tiles * rp.splits <= 0x7fffffffll, DK_ERR_SHAPE);
    if (rp.splits > 1)
        DK_REQUIRE(part && part_bytes >= (size_t)rp.splits * out_elems * sizeof(float), DK_ERR_WORKSPACE);
    {
        dk_prof_scope ps(label, st);
        contract_kernel<C, LA, LB, EP><<<dim3((unsigned)(tiles * rp.splits)), dim3(C::NT), 0, st>>>(pa, pb, ep, rp);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    if (rp.splits > 1) return dk_fold_slices(part, out, out_elems, rp.splits, alpha, accumulate, st);
    return DK_OK;
}

template <class C>
size_t split_bytes(long long rows, long long cols, long long kdim, long long out_elems)
{
    const long long tiles = ((rows + C::BM - 1) / C::BM) * ((cols + C::BN - 1) / C::BN);
    const long long ktiles = (kdim + C::BK - 1) / C::BK;
    const dk_split_plan sp = dk_plan_split(tiles, ktiles, out_elems, C::STEP_US);
    return sp.splits > 1 ? (size_t)sp.splits * out_elems * sizeof(float) : 0;
}

// Tile shapes.  Dense layers and wide convolutions use a square 128x128 tile
// (four waves, 64x64 each); convolutions with at most 64 output channels use
// a 64-row tile so that no MFMA row is wasted.
using CfgSq = Cfg<128, 128, 16, 2, 2>;
using CfgFlat = Cfg<64, 256, 16, 1, 4>;
using CfgWg64 = Cfg<64, 128, 16, 2, 2>;
using CfgTall = Cfg<128, 64, 16, 2, 2>;
using CfgSmall = Cfg<64, 64, 16, 2, 2>;

// Weight gradients have small outputs (rows = output channels, columns = input
// channels or filter elements): pick the tile that wastes no MFMA rows or
// columns on a 64-wide side.
template <class Fn>
auto with_wgrad_cfg(long long rows, long long cols, Fn fn)
{
    if (rows <= 64 && cols <= 64) return fn(CfgSmall{});
    if (rows <= 64) return fn(CfgWg64{});
    if (cols <= 64) return fn(CfgTall{});
    return fn(CfgSq{});
}

ConvParams conv_params(const dk_geom &g, const float *p, long long R)
{
    ConvParams c;
    c.p = p;
    c.Ci = g.Ci; c.Co = g.Co; c.H = g.H; c.W = g.W; c.kh = g.kh; c.kw = g.kw;
    c.stride = g.stride; c.pad = g.pad; c.Ho = g.Ho; c.Wo = g.Wo;
    c.HoWo = g.Ho * g.Wo;
    c.Kg = (int)g.Kg;
    c.Q = (int)(R * c.HoWo);
    c.img = g.n;
    return c;
}

template <class C, bool VA, bool VB>
dk_status run_dense_nt(const float *A, const float *B, float *Cout, int rows, int cols, int kdim,
                       float *part, size_t part_bytes, hipStream_t st,
                       const char *label = "contract_dense_fwd")
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VA>;
    using LB = LoadRowMajorK<C::BN, C::BK, C::NT, C::LDB, VB>;
    MatParams pa = {A, kdim, rows, kdim}, pb = {B, kdim, cols, kdim};
    EpiDense ep = {cols, rows, cols};
    return run<C, LA, LB, EpiDense>(pa, pb, ep, rows, cols, kdim, 1.0f, 0, Cout,
                                    (long long)rows * cols, part, part_bytes, st, label);
}

// C[rows][cols] = A[rows][k] . B[k][cols]  (A contiguous along k, B along cols)
template <class C, bool VA, bool VB>
dk_status run_dense_nn(const float *A, const float *B, float *Cout, int rows, int cols, int kdim,
                       float *part, size_t part_bytes, hipStream_t st)
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VA>;
    using LB = LoadKMajor<C::BN, C::BK, C::NT, C::LDB, VB>;
    MatParams pa = {A, kdim, rows, kdim}, pb = {B, cols, cols, kdim};
    EpiDense ep = {cols, rows, cols};
    return run<C, LA, LB, EpiDense>(pa, pb, ep, rows, cols, kdim, 1.0f, 0, Cout,
                                    (long long)rows * cols, part, part_bytes, st, "contract_dense_dgrad");
}

template <class C, bool VEC>
dk_status run_dense_tn(const float *A, const float *B, float *Cout, int rows, int cols, int kdim,
                       float alpha, int accumulate, float *part, size_t part_bytes, hipStream_t st,
                       const char *label = "contract_dense_wgrad")
{
    using LA = LoadKMajor<C::BM, C::BK, C::NT, C::LDA, VEC>;
    using LB = LoadKMajor<C::BN, C::BK, C::NT, C::LDB, VEC>;
    MatParams pa = {A, rows, rows, kdim}, pb = {B, cols, cols, kdim};
    EpiDense ep = {cols, rows, cols};
    return run<C, LA, LB, EpiDense>(pa, pb, ep, rows, cols, kdim, alpha, accumulate, Cout,
                                    (long long)rows * cols, part, part_bytes, st, label);
}

template <class C, bool VW>
dk_status run_conv_fwd(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                       float *part, size_t part_bytes, hipStream_t st)
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VW>;
    using LB = LoadIm2colFwd<C::BN, C::BK, C::NT, C::LDB>;
    const ConvParams cp = conv_params(g, xbar, R);
    MatParams pa = {W, g.Kg, g.Co, (int)g.Kg};
    EpiConvFwd ep = {g.Co, cp.Q, cp.HoWo, (long long)g.Co * cp.HoWo};
    return run<C, LA, LB, EpiConvFwd>(pa, cp, ep, g.Co, cp.Q, g.Kg, 1.0f, 0, ybar, R * g.m, part,
                                      part_bytes, st, "contract_conv_fwd_gather");
}

// dx[r][ci][pix] = sum_k Wt[ci][k] * gathered delta, k = (co, a, b); Wt is the
// filter bank regrouped as [ci][co][a][b].
template <class C, bool VW>
dk_status run_conv_dgrad(const dk_geom &g, const float *Wt, const float *delta, float *dx, long long R,
                         float *part, size_t part_bytes, hipStream_t st)
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VW>;
    using LB = LoadIm2colDgrad<C::BN, C::BK, C::NT, C::LDB>;
    ConvParams cp = conv_params(g, delta, R);
    const int HW = g.H * g.W, Kd = g.Co * g.kh * g.kw;
    cp.Q = (int)(R * HW);
    MatParams pa = {Wt, Kd, g.Ci, Kd};
    EpiConvFwd ep = {g.Ci, cp.Q, HW, (long long)g.Ci * HW};
    return run<C, LA, LB, EpiConvFwd>(pa, cp, ep, g.Ci, cp.Q, Kd, 1.0f, 0, dx, R * g.n, part, part_bytes,
                                      st, "contract_conv_dgrad_gather");
}

template <class C>
dk_status run_conv_wgrad(const dk_geom &g, const float *dtilde, const float *xbar, float *dW,
                         long long R, float alpha, int accumulate, float *part, size_t part_bytes,
                         hipStream_t st)
{
    using LB = LoadIm2colQ<C::BN, C::BK, C::NT, C::LDB>;
    const ConvParams ca = conv_params(g, dtilde, R);
    const ConvParams cb = conv_params(g, xbar, R);
    EpiDense ep = {g.Kg, g.Co, (int)g.Kg};
    if (ca.HoWo % 4 == 0 && dk_aligned(dtilde, 16)) {
        // the mixed gradients are plain [R][Co][Ho*Wo] images whatever the filter: whole
        // 16-byte vectors along the pixels instead of single floats
        using LA = LoadRowMajorKImg<C::BM, C::BK, C::NT, C::LDA, true>;
        ImgParams pa = {dtilde, g.Co, ca.HoWo, ca.Q, ca.HoWo, g.Wo, g.Wo, 1};
        return run<C, LA, LB, EpiDense>(pa, cb, ep, g.Co, (int)g.Kg, ca.Q, alpha, accumulate, dW,
                                        (long long)g.Co * g.Kg, part, part_bytes, st, "contract_conv_wgrad_gather");
    }
    using LA = LoadDeltaQ<C::BM, C::BK, C::NT, C::LDA>;
    return run<C, LA, LB, EpiDense>(ca, cb, ep, g.Co, (int)g.Kg, ca.Q, alpha, accumulate, dW,
                                    (long long)g.Co * g.Kg, part, part_bytes, st, "contract_conv_wgrad_gather");
}

// 1x1 pad-0 convolution (any stride) through the image-aware loaders.
template <class C, bool VW, bool VX>
dk_status run_conv1x1_fwd(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                          float *part, size_t part_bytes, hipStream_t st)
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VW>;
    using LB = LoadKMajorImg<C::BN, C::BK, C::NT, C::LDB, VX>;
    const int HW = g.Ho * g.Wo, Q = (int)(R * HW);
    MatParams pa = {W, g.Ci, g.Co, g.Ci};
    ImgParams pb = {xbar, g.Ci, HW, Q, g.H * g.W, g.Wo, g.W, g.stride};
    EpiConvFwd ep = {g.Co, Q, HW, (long long)g.Co * HW};
    return run<C, LA, LB, EpiConvFwd>(pa, pb, ep, g.Co, Q, g.Ci, 1.0f, 0, ybar, R * g.m, part, part_bytes,
                                      st, "contract_conv1x1_fwd");
}

template <class C, bool VD, bool VX>
dk_status run_conv1x1_wgrad(const dk_geom &g, const float *dtilde, const float *xbar, float *dW,
                            long long R, float alpha, int accumulate, float *part, size_t part_bytes,
                            hipStream_t st)
{
    using LA = LoadRowMajorKImg<C::BM, C::BK, C::NT, C::LDA, VD>;
    using LB = LoadRowMajorKImg<C::BN, C::BK, C::NT, C::LDB, VX>;
    const int HW = g.H * g.W, Q = (int)(R * HW);          // stride 1
    ImgParams pa = {dtilde, g.Co, HW, Q, HW, g.W, g.W, 1};
    ImgParams pb = {xbar, g.Ci, HW, Q, HW, g.W, g.W, 1};
    EpiDense ep = {g.Ci, g.Co, g.Ci};
    return run<C, LA, LB, EpiDense>(pa, pb, ep, g.Co, g.Ci, Q, alpha, accumulate, dW,
                                    (long long)g.Co * g.Ci, part, part_bytes, st, "contract_conv1x1_wgrad");
}

// A convolution over images of at most 2x2 pixels is a small dense layer: every
// output pixel sees the whole image, and most taps of the im2col form fall on
// padding.  Its matrix is
//   Wd[(co, oh, ow)][(ci, ih, iw)] = W[co][ci][ih - oh*s + p][iw - ow*s + p]   (0 outside the filter)
// so ybar[r] = Wd . xbar[r] in the NCHW flattening both sides already have, and
// the weight gradient is the dense one folded back over the pixel pairs.
bool conv_as_dense(const dk_geom &g)
{
    return g.conv && !g.dw && g.H * g.W <= 4 && g.Ho * g.Wo <= 4 &&
           (long long)g.Co * g.Ho * g.Wo * g.Ci * g.H * g.W <= (16ll << 20);
}

size_t conv_dense_matrix_bytes(const dk_geom &g)
{
    return align_up((size_t)g.Co * g.Ho * g.Wo * g.Ci * g.H * g.W * sizeof(float), 256);
}

// One thread per (matrix row, input channel): the H*W <= 4 entries of that
// channel are consecutive in the row.
__global__ __launch_bounds__(256) void conv_unfold_filters_kernel(const float *__restrict__ W,
                                                                  float *__restrict__ Wd, int Ci, int H,
                                                                  int Wi, int Ho, int Wo, int kh, int kw,
                                                                  int stride, int pad, long long total)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int HW = H * Wi, HoWo = Ho * Wo;
    const int ci = (int)(e % Ci);
    const long long row = e / Ci;
    const int po = (int)(row % HoWo);
    const long long co = row / HoWo;
    const float *w = W + (co * Ci + ci) * kh * kw;
    const int a0 = pad - (po / Wo) * stride, b0 = pad - (po % Wo) * stride;
    float v[4];
#pragma unroll
    for (int pi = 0; pi < 4; ++pi) {
        const int a = pi / Wi + a0, b = pi % Wi + b0;
        v[pi] = (pi < HW && a >= 0 && a < kh && b >= 0 && b < kw) ? w[a * kw + b] : 0.0f;
    }
    float *d = Wd + (row * Ci + ci) * HW;
    if (HW == 4) {
        *reinterpret_cast<float4 *>(d) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int pi = 0; pi < 4; ++pi)
            if (pi < HW) d[pi] = v[pi];
    }
}

// dW[co][ci][a][b] = (accumulate ? dW : 0) + scale * sum over output pixels (oh, ow) whose
// tap (a, b) lies inside the image of dWd[(co, oh, ow)][(ci, oh*s + a - p, ow*s + b - p)].
// One thread per (co, ci): it reads its block of at most 4 x 4 dense entries
// (consecutive threads read consecutive 16-byte pieces) and writes the kh*kw
// consecutive taps.
__global__ __launch_bounds__(256) void conv_refold_wgrad_kernel(const float *__restrict__ dWd,
                                                                float *__restrict__ dW, int Ci, int H,
                                                                int Wi, int Ho, int Wo, int kh, int kw,
                                                                int stride, int pad, float scale,
                                                                int accumulate, long long total)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int ci = (int)(e % Ci);
    const long long co = e / Ci;
    const int HW = H * Wi, HoWo = Ho * Wo;
    const long long ncol = (long long)Ci * HW;
    float blk[4][4];
#pragma unroll
    for (int po = 0; po < 4; ++po) {
        const float *src = dWd + (co * HoWo + po) * ncol + (long long)ci * HW;
        if (po < HoWo && HW == 4) {
            const float4 v = *reinterpret_cast<const float4 *>(src);
            blk[po][0] = v.x; blk[po][1] = v.y; blk[po][2] = v.z; blk[po][3] = v.w;
        } else {
#pragma unroll
            for (int pi = 0; pi < 4; ++pi) blk[po][pi] = (po < HoWo && pi < HW) ? src[pi] : 0.0f;
        }
    }
    float *d = dW + (co * Ci + ci) * kh * kw;
    for (int a = 0; a < kh; ++a)
        for (int b = 0; b < kw; ++b) {
            float s = 0.0f;
#pragma unroll
            for (int po = 0; po < 4; ++po)
#pragma unroll
                for (int pi = 0; pi < 4; ++pi) {
                    // entry (po, pi) belongs to tap (pi/W - (po/Wo)*s + p, pi%W - (po%Wo)*s + p)
                    const bool hit = po < HoWo && pi < HW && pi / Wi - (po / Wo) * stride + pad == a &&
                                     pi % Wi - (po % Wo) * stride + pad == b;
                    s += hit ? blk[po][pi] : 0.0f;
                }
            s *= scale;
            if (accumulate) s += d[a * kw + b];
            d[a * kw + b] = s;
        }
}

bool conv_is_1x1(const dk_geom &g) { return g.kh == 1 && g.kw == 1 && g.pad == 0; }

bool conv_flat(const dk_geom &g) { return g.Co <= 64; }

} // namespace

size_t dk_ws_fwd_bytes(const dk_geom &g, long long R)
{
    if (g.dw) return 256;
    if (conv_as_dense(g)) {
        const long long Md = (long long)g.Co * g.Ho * g.Wo, Nd = (long long)g.Ci * g.H * g.W;
        return conv_dense_matrix_bytes(g) + split_bytes<CfgSq>(R, Md, Nd, R * Md);
    }
    size_t b;
    if (!g.conv)
        b = split_bytes<CfgSq>(R, g.M, g.N, R * g.m);
    else if (conv_flat(g))
        b = split_bytes<CfgFlat>(g.Co, R * g.Ho * g.Wo, g.Kg, R * g.m);
    else
        b = split_bytes<CfgSq>(g.Co, R * g.Ho * g.Wo, g.Kg, R * g.m);
    if (g.conv) {
        // whichever kernel family the entry point picks (it depends on the
        // alignment of xbar too), the workspace must be large enough
        dk_patch_plan pl;
        for (int aligned = 0; aligned < 2; ++aligned)
            if (dk_patch_fwd_plan(g, R, aligned != 0, &pl)) {
                const size_t pb = dk_patch_wp_bytes(pl) + pl.part_bytes;
                if (pb > b) b = pb;
            }
    }
    return b < 256 ? 256 : b;
}

size_t dk_ws_wgrad_bytes(const dk_geom &g, long long R)
{
    // mixed gradients dtilde[R][m] first, then the partial sums
    if (g.dw) return align_up((size_t)R * g.m * sizeof(float), 256) + dk_dw_wgrad_part_bytes(g, R);
    size_t part;
    if (conv_as_dense(g)) {
        const long long Md = (long long)g.Co * g.Ho * g.Wo, Nd = (long long)g.Ci * g.H * g.W;
        part = conv_dense_matrix_bytes(g) + with_wgrad_cfg(Md, Nd, [&](auto c) {
            return split_bytes<decltype(c)>(Md, Nd, R, Md * Nd); });
    } else if (!g.conv)
        part = with_wgrad_cfg(g.M, g.N, [&](auto c) {
            return split_bytes<decltype(c)>(g.M, g.N, R, (long long)g.M * g.N); });
    else
        part = with_wgrad_cfg(g.Co, g.Kg, [&](auto c) {
            return split_bytes<decltype(c)>(g.Co, g.Kg, R * g.Ho * g.Wo, g.Co * g.Kg); });
    if (g.conv && !conv_as_dense(g)) {
        dk_wgpatch_plan pl;
        for (int aligned = 0; aligned < 2; ++aligned)
            if (dk_patch_wgrad_plan(g, R, aligned != 0, &pl) && pl.part_bytes > part) part = pl.part_bytes;
        const size_t fb = dk_fused1x1_wgrad_part_bytes(g, R);
        if (fb > part) part = fb;
        const size_t sb = dk_smallci_wgrad_part_bytes(g, R);
        if (sb > part) part = sb;
    }
    return align_up((size_t)R * g.m * sizeof(float), 256) + part;
}

DK_EXPORT dk_status dk_linear_fwd(const float *W, const float *xbar, float *ybar, int M, int N, int R,
                                  void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(W && xbar && ybar, DK_ERR_NULL);
    DK_REQUIRE(M >= 1 && N >= 1 && R >= 1, DK_ERR_SHAPE);
    DK_REQUIRE((long long)R * M < (1ll << 40) && (long long)M * N < (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(W, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
    dk_geom g = {};
    g.M = M; g.N = N; g.n = N; g.m = M;
    DK_REQUIRE(ws && ws_bytes >= dk_ws_fwd_bytes(g, R), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const bool va = (N % 4 == 0) && dk_aligned(xbar, 16);
    const bool vb = (N % 4 == 0) && dk_aligned(W, 16);
    if (va && vb)
        return run_dense_nt<CfgSq, true, true>(xbar, W, ybar, R, M, N, (float *)ws, ws_bytes, st);
    return run_dense_nt<CfgSq, false, false>(xbar, W, ybar, R, M, N, (float *)ws, ws_bytes, st);
}

// The convolution forward dispatch for a validated geometry (also the engine
// behind the stride-1 data gradient, which is a forward convolution with
// transposed, flipped filters).
static dk_status conv_fwd_impl(const dk_geom &g, const float *W, const float *xbar, float *ybar, int R,
                               void *ws, size_t ws_bytes, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (g.dw) return dk_dw_fwd_run(g, W, xbar, ybar, R, st);
    if (conv_as_dense(g)) {
        const int Md = g.Co * g.Ho * g.Wo, Nd = g.Ci * g.H * g.W;
        float *Wd = (float *)ws;
        const size_t wd_bytes = conv_dense_matrix_bytes(g);
        const long long total = (long long)Md * g.Ci;
        {
            dk_prof_scope ps("unfold_filters", st);
            conv_unfold_filters_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
                W, Wd, g.Ci, g.H, g.W, g.Ho, g.Wo, g.kh, g.kw, g.stride, g.pad, total);
        }
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        float *part = (float *)((char *)ws + wd_bytes);
        const bool v = (Nd % 4 == 0) && dk_aligned(xbar, 16);
        if (v) return run_dense_nt<CfgSq, true, true>(xbar, Wd, ybar, R, Md, Nd, part, ws_bytes - wd_bytes, st, "contract_conv_dense_fwd");
        return run_dense_nt<CfgSq, false, false>(xbar, Wd, ybar, R, Md, Nd, part, ws_bytes - wd_bytes, st, "contract_conv_dense_fwd");
    }
    // at most four input channels: bound by writing the results, not by the matrix cores
    if (dk_smallci_ok(g, R, xbar, ybar)) return dk_smallci_fwd_run(g, W, xbar, ybar, R, st);
    dk_patch_plan pl;
    if (dk_patch_fwd_plan(g, R, dk_aligned(xbar, 16) && dk_aligned(ybar, 16), &pl))
        return dk_patch_fwd_run(g, pl, W, xbar, ybar, (float *)ws, st);
    const bool vw = (g.Kg % 4 == 0) && dk_aligned(W, 16);
    if (conv_is_1x1(g)) {
        const bool vx = g.stride == 1 && (g.H * g.W) % 4 == 0 && dk_aligned(xbar, 16);
        float *pw = (float *)ws;
        if (conv_flat(g)) {
            if (vw && vx) return run_conv1x1_fwd<CfgFlat, true, true>(g, W, xbar, ybar, R, pw, ws_bytes, st);
            if (vw) return run_conv1x1_fwd<CfgFlat, true, false>(g, W, xbar, ybar, R, pw, ws_bytes, st);
            return run_conv1x1_fwd<CfgFlat, false, false>(g, W, xbar, ybar, R, pw, ws_bytes, st);
        }
        if (vw && vx) return run_conv1x1_fwd<CfgSq, true, true>(g, W, xbar, ybar, R, pw, ws_bytes, st);
        if (vw) return run_conv1x1_fwd<CfgSq, true, false>(g, W, xbar, ybar, R, pw, ws_bytes, st);
        return run_conv1x1_fwd<CfgSq, false, false>(g, W, xbar, ybar, R, pw, ws_bytes, st);
    }
    if (conv_flat(g))
        return vw ? run_conv_fwd<CfgFlat, true>(g, W, xbar, ybar, R, (float *)ws, ws_bytes, st)
                  : run_conv_fwd<CfgFlat, false>(g, W, xbar, ybar, R, (float *)ws, ws_bytes, st);
    return vw ? run_conv_fwd<CfgSq, true>(g, W, xbar, ybar, R, (float *)ws, ws_bytes, st)
              : run_conv_fwd<CfgSq, false>(g, W, xbar, ybar, R, (float *)ws, ws_bytes, st);
}

DK_EXPORT dk_status dk_conv_fwd(const dk_layer *L, const float *W, const float *xbar, float *ybar,
                                int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && W && xbar && ybar, DK_ERR_NULL);
    dk_geom g;
    dk_status s = dk_layer_geom(L, &g);
    if (s != DK_OK) return s;
    DK_REQUIRE(g.conv, DK_ERR_UNSUPPORTED);
    DK_REQUIRE(R >= 1 && (long long)R * g.Ho * g.Wo < (1ll << 31) - 512, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(W, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_ws_fwd_bytes(g, R), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    return conv_fwd_impl(g, W, xbar, ybar, R, ws, ws_bytes, stream);
}

// Where the fused forms measured faster than the separate kernels (the twelve
// 1x1 stride-1 shapes of ResNet-50 at K = 8, batch 64).
// Weight gradient with the mixing in its loader: ahead on the 56x56 layers
// (64->64: 0.060 ms against 0.073; 64->256: 0.148 / 0.184; 256->64: 0.119 /
// 0.128; 256->128: 0.200 / 0.205), behind from 28x28 down (128->512: 0.133 /
// 0.127; 512->128: 0.127 / 0.101): the mixed gradients saved are Co x pixels per
// image, the K loads and multiply-adds per operand element are paid per step.
static bool fused_wgrad_pays(const dk_geom &g, int K)
{
    (void)K;
    return (long long)g.H * g.W >= 1600;
}
// Forward + decode + verify: one accumulator block per wave is all the K
// decoded tiles leave room for, so the product itself runs at half the rate of
// the 128x128 tiles; ahead only where the product is short (64 input channels:
// 64->64 0.051 ms against 0.074, 64->256 0.185 / 0.195), behind from 128
// channels on (128->512 @28x28 0.156 / 0.144, 256->64 @56x56 0.173 / 0.123).
static bool fused_fwd_pays(const dk_geom &g, int K)
{
    (void)K;
    return g.Ci <= 64;
}

// Layout of the workspace of dk_conv_fwd_decode_verify when the two steps run
// one after the other: ybar, the forward's own workspace, the integrity slots.
struct fwd_dv_ws {
    size_t ybar, fwd, slots, total;
};

static fwd_dv_ws fwd_dv_layout(const dk_geom &g, int G, int K)
{
    const long long R = (long long)G * (K + 2);
    fwd_dv_ws w;
    w.ybar = align_up((size_t)R * g.m * sizeof(float), 256);
    w.fwd = align_up(dk_ws_fwd_bytes(g, R), 256);
    w.slots = align_up(dk_ws_verify_bytes(G), 256);
    const size_t fused = dk_fused1x1_fwd_ok(g, K) ? align_up(dk_fused1x1_fwd_slot_bytes(g, G), 256) : 0;
    w.total = w.ybar + w.fwd + w.slots;
    if (fused > w.total) w.total = fused;
    return w;
}

DK_EXPORT size_t dk_conv_fwd_decode_verify_workspace_bytes(const dk_layer *L, int G, int K)
{
    dk_geom g;
    if (G < 1 || K < 1 || K > DK_MAX_K || dk_layer_geom(L, &g) != DK_OK || !g.conv) return 0;
    return fwd_dv_layout(g, G, K).total;
}

DK_EXPORT dk_status dk_conv_fwd_decode_verify(const dk_layer *L, const float *W, const float *xbar,
                                              const float *Ainv, const float *nvec, float tol, float *y,
                                              int *verdict, float *resid, int G, int K, void *ws,
                                              size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && W && xbar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && tol >= 0.0f, DK_ERR_SHAPE);
    dk_geom g;
    dk_status s = dk_layer_geom(L, &g);
    if (s != DK_OK) return s;
    DK_REQUIRE(g.conv, DK_ERR_UNSUPPORTED);
    const long long R = (long long)G * (K + 2);
    DK_REQUIRE(R * g.Ho * g.Wo < (1ll << 31) - 512, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(W, 4) && dk_aligned(xbar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) &&
                   dk_aligned(y, 4) && dk_aligned(verdict, 4) && (!resid || dk_aligned(resid, 4)), DK_ERR_ALIGN);
    const fwd_dv_ws w = fwd_dv_layout(g, G, K);
    DK_REQUIRE(ws && ws_bytes >= w.total, DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    const int opt = dk_option(DK_OPT_FUSE_FWD);
    if (opt != DK_FUSE_NEVER && dk_fused1x1_fwd_ok(g, K) && (opt == DK_FUSE_ALWAYS || fused_fwd_pays(g, K)))
        return dk_fused1x1_fwd_run(g, W, xbar, Ainv, nvec, tol, y, verdict, resid, G, K, ws, (hipStream_t)stream);
    float *ybar = (float *)ws;
    s = conv_fwd_impl(g, W, xbar, ybar, (int)R, (char *)ws + w.ybar, w.fwd, stream);
    if (s != DK_OK) return s;
    return dk_decode_verify(ybar, Ainv, nvec, tol, y, verdict, resid, G, K, g.m, (char *)ws + w.ybar + w.fwd,
                            w.slots, stream);
}

// dk_wgrad for K private inputs and M noise rows per group (S = K + M + 1).
static dk_status wgrad_impl(const dk_layer *L, const float *delta, const float *B, const float *gamma,
                            const float *xbar, float *dW, int G, int K, int M, float scale,
                            int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && delta && B && gamma && xbar && dW, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && M >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    dk_geom g;
    dk_status s = dk_layer_geom(L, &g);
    if (s != DK_OK) return s;
    const long long R = (long long)G * (K + M + 1);
    DK_REQUIRE(R < (1ll << 31), DK_ERR_SHAPE);
    if (g.conv) DK_REQUIRE(R * g.Ho * g.Wo < (1ll << 31) - 512, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(delta, 4) && dk_aligned(B, 4) && dk_aligned(gamma, 4) &&
                   dk_aligned(xbar, 4) && dk_aligned(dW, 4), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_ws_wgrad_bytes(g, R), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;

    float *dtilde = (float *)ws;
    const size_t dt_bytes = align_up((size_t)R * g.m * sizeof(float), 256);
    float *part = (float *)((char *)ws + dt_bytes);
    const size_t part_bytes = ws_bytes - dt_bytes;

    // 1x1 layers: the mixing can run inside the contraction's operand loader
    if (dk_option(DK_OPT_FUSE_WGRAD) != DK_FUSE_NEVER && dk_fused1x1_wgrad_ok(g, G, K, M, delta, xbar) &&
        (dk_option(DK_OPT_FUSE_WGRAD) == DK_FUSE_ALWAYS || fused_wgrad_pays(g, K)))
        return dk_fused1x1_wgrad_run(g, delta, B, gamma, xbar, dW, G, K, scale, accumulate, part, part_bytes, st);

    s = dk_delta_mix(delta, B, gamma, dtilde, G, K, M, g.m, st);
    if (s != DK_OK) return s;

    if (g.dw) return dk_dw_wgrad_run(g, dtilde, xbar, dW, R, scale, accumulate, part, st);
    if (!g.conv) {
        const bool vec = (g.M % 4 == 0) && (g.N % 4 == 0) && dk_aligned(xbar, 16);
        return with_wgrad_cfg(g.M, g.N, [&](auto c) {
            using C = decltype(c);
            return vec ? run_dense_tn<C, true>(dtilde, xbar, dW, g.M, g.N, (int)R, scale, accumulate, part, part_bytes, st)
                       : run_dense_tn<C, false>(dtilde, xbar, dW, g.M, g.N, (int)R, scale, accumulate, part, part_bytes, st);
        });
    }
    if (conv_as_dense(g)) {
        const int Md = g.Co * g.Ho * g.Wo, Nd = g.Ci * g.H * g.W;
        float *dWd = part;
        const size_t wd_bytes = conv_dense_matrix_bytes(g);
        float *part2 = (float *)((char *)part + wd_bytes);
        const bool vec = (Md % 4 == 0) && (Nd % 4 == 0) && dk_aligned(xbar, 16);
        s = with_wgrad_cfg(Md, Nd, [&](auto c) {
            using C = decltype(c);
            return vec ? run_dense_tn<C, true>(dtilde, xbar, dWd, Md, Nd, (int)R, 1.0f, 0, part2, part_bytes - wd_bytes, st, "contract_conv_dense_wgrad")
                       : run_dense_tn<C, false>(dtilde, xbar, dWd, Md, Nd, (int)R, 1.0f, 0, part2, part_bytes - wd_bytes, st, "contract_conv_dense_wgrad");
        });
        if (s != DK_OK) return s;
        const long long total = (long long)g.Co * g.Ci;
        dk_prof_scope ps("refold_wgrad", st);
        conv_refold_wgrad_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
            dWd, dW, g.Ci, g.H, g.W, g.Ho, g.Wo, g.kh, g.kw, g.stride, g.pad, scale, accumulate, total);
        return dk_launch_status();
    }
    if (dk_smallci_ok(g, R, xbar, dtilde))
        return dk_smallci_wgrad_run(g, dtilde, xbar, dW, R, scale, accumulate, part, part_bytes, st);
    dk_wgpatch_plan pl;
    if (dk_patch_wgrad_plan(g, R, dk_aligned(xbar, 16), &pl)) {
        DK_REQUIRE(part_bytes >= pl.part_bytes, DK_ERR_WORKSPACE);
        return dk_patch_wgrad_run(g, pl, dtilde, xbar, dW, scale, accumulate, part, st);
    }
    // (with a stride the scalar image loads of xbar measured slower here than the gather engine)
    if (conv_is_1x1(g) && g.stride == 1) {
        const bool vd = (g.Ho * g.Wo) % 4 == 0;           // dtilde rows (the workspace is aligned)
        const bool vx = vd && dk_aligned(xbar, 16);
        return with_wgrad_cfg(g.Co, g.Kg, [&](auto c) {
            using C = decltype(c);
            if (vx) return run_conv1x1_wgrad<C, true, true>(g, dtilde, xbar, dW, R, scale, accumulate, part, part_bytes, st);
            if (vd) return run_conv1x1_wgrad<C, true, false>(g, dtilde, xbar, dW, R, scale, accumulate, part, part_bytes, st);
            return run_conv1x1_wgrad<C, false, false>(g, dtilde, xbar, dW, R, scale, accumulate, part, part_bytes, st);
        });
    }
    return with_wgrad_cfg(g.Co, g.Kg, [&](auto c) {
        return run_conv_wgrad<decltype(c)>(g, dtilde, xbar, dW, R, scale, accumulate, part, part_bytes, st);
    });
}

DK_EXPORT dk_status dk_wgrad(const dk_layer *L, const float *delta, const float *B, const float *gamma,
                             const float *xbar, float *dW, int G, int K, float scale, int accumulate,
                             void *ws, size_t ws_bytes, void *stream)
{
    return wgrad_impl(L, delta, B, gamma, xbar, dW, G, K, 1, scale, accumulate, ws, ws_bytes, stream);
}

DK_EXPORT dk_status dk_wgrad_m(const dk_layer *L, const float *delta, const float *B, const float *gamma,
                               const float *xbar, float *dW, int G, int K, int M, float scale,
                               int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    return wgrad_impl(L, delta, B, gamma, xbar, dW, G, K, M, scale, accumulate, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------
// Data gradients (un-encoded: they hold no private input).
// ---------------------------------------------------------------------------
namespace {

// Wt[ci][co][a][b] = W[co][ci][kh-1-a][kw-1-b] (flip) or W[co][ci][a][b]
__global__ __launch_bounds__(256) void dgrad_filter_kernel(const float *__restrict__ W, float *__restrict__ Wt,
                                                           int Co, int Ci, int kh, int kw, int flip)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= Co * Ci * kh * kw) return;
    const int khw = kh * kw;
    const int ci = e / (Co * khw);
    int rem = e - ci * (Co * khw);
    const int co = rem / khw;
    rem -= co * khw;
    const int a = rem / kw, b = rem - a * kw;
    Wt[e] = flip ? W[((long long)(co * Ci + ci) * kh + (kh - 1 - a)) * kw + (kw - 1 - b)]
                 : W[((long long)(co * Ci + ci) * kh + a) * kw + b];
}

// Any geometry, one thread per input element:
// dx[r][ci][i][j] = sum_{co,a,b} d[r][co][(i+pad-a)/stride][(j+pad-b)/stride] W[co][ci][a][b]
// over the taps whose quotients are whole and inside the output.
__global__ __launch_bounds__(256) void conv_dgrad_direct_kernel(const float *__restrict__ W,
                                                                const float *__restrict__ d,
                                                                float *__restrict__ dx, long long total, int Ci,
                                                                int Co, int H, int Wd, int kh, int kw,
                                                                int stride, int pad, int Ho, int Wo)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int HW = H * Wd;
    const long long rc = idx / HW;
    const int px = (int)(idx - rc * HW);
    const int i = px / Wd, j = px - i * Wd;
    const long long r = rc / Ci;
    const int ci = (int)(rc - r * Ci);
    float acc = 0.0f;
    for (int a = 0; a < kh; ++a) {
        const int hn = i + pad - a;
        if (hn < 0 || hn % stride) continue;
        const int h = hn / stride;
        if (h >= Ho) continue;
        for (int b = 0; b < kw; ++b) {
            const int wn = j + pad - b;
            if (wn < 0 || wn % stride) continue;
            const int w = wn / stride;
            if (w >= Wo) continue;
            const float *dp = d + ((long long)r * Co * Ho + h) * Wo + w;
            const float *wp = W + ((long long)ci * kh + a) * kw + b;
            for (int co = 0; co < Co; ++co)
                acc = fmaf(dp[(long long)co * Ho * Wo], wp[(long long)co * Ci * kh * kw], acc);
        }
    }
    dx[idx] = acc;
}

bool conv_flat_dgrad(const dk_geom &g) { return g.Ci <= 64; }

// One residue class of a strided data gradient.
struct dgrad_class {
    int pi, pj, a0, b0, na, nb, bh, bw, U, V;
    size_t wt_off;     // floats, start of the class's filter matrix in the workspace
};

int dgrad_classes(const dk_geom &g, dgrad_class *cl)
{
    const int s = g.stride;
    size_t off = 0;
    int n = 0;
    for (int pi = 0; pi < s; ++pi)
        for (int pj = 0; pj < s; ++pj) {
            dgrad_class c;
            c.pi = pi; c.pj = pj;
            c.a0 = (pi + g.pad) % s; c.b0 = (pj + g.pad) % s;
            c.na = c.a0 < g.kh ? (g.kh - c.a0 + s - 1) / s : 0;
            c.nb = c.b0 < g.kw ? (g.kw - c.b0 + s - 1) / s : 0;
            c.bh = (pi + g.pad - c.a0) / s; c.bw = (pj + g.pad - c.b0) / s;
            c.U = pi < g.H ? (g.H - pi + s - 1) / s : 0;
            c.V = pj < g.W ? (g.W - pj + s - 1) / s : 0;
            c.wt_off = off;
            off += ((size_t)g.Ci * g.Co * c.na * c.nb + 63) / 64 * 64;      // 256-byte steps
            cl[n++] = c;
        }
    return n;
}

size_t dgrad_class_filter_bytes(const dk_geom &g)
{
    return ((size_t)g.Ci * g.Co * g.kh * g.kw + 64 * (size_t)g.stride * g.stride) * sizeof(float);
}

// The sub-filter matrices of all classes in one launch:
// Wt_c[ci][(co, a', b')] = W[co][ci][a0 + s a'][b0 + s b'], class c at Wt + off[c].
struct dgrad_filter_batch {
    int count;
    int a0[9], b0[9], na[9], nb[9];
    int first[10];           // running element counts
    long long off[9];
};

__global__ __launch_bounds__(256) void dgrad_class_filter_kernel(const float *__restrict__ W, float *__restrict__ Wt,
                                                                 int Co, int Ci, int kh, int kw, int stride,
                                                                 dgrad_filter_batch fb)
{
    const int e0 = blockIdx.x * 256 + threadIdx.x;
    if (e0 >= fb.first[fb.count]) return;
    int c = 0;
    while (c + 1 < fb.count && e0 >= fb.first[c + 1]) ++c;
    const int e = e0 - fb.first[c];
    const int nb = fb.nb[c], tn = fb.na[c] * nb;
    const int ci = e / (Co * tn);
    int rem = e - ci * (Co * tn);
    const int co = rem / tn;
    rem -= co * tn;
    const int ap = rem / nb, bp = rem - ap * nb;
    Wt[fb.off[c] + e] = W[((long long)(co * Ci + ci) * kh + (fb.a0[c] + stride * ap)) * kw + (fb.b0[c] + stride * bp)];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ p, long long count)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0.0f;
}

// All non-empty classes in one launch: alone, a class of a 14x14 or 7x7 image
// has fewer tiles than the chip has compute units.
template <class C, bool VW>
dk_status run_dgrad_classes(const dk_geom &g, const dgrad_class *cl, int ncl, const float *Wt, const float *delta,
                            float *dx, long long R, hipStream_t st)
{
    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VW>;
    using LB = LoadDgradClass<C::BN, C::BK, C::NT, C::LDB>;
    ContractBatch<LA, LB, EpiDgradClass> b;
    b.count = 0;
    long long slots = 0;
    // classes with the most taps first: their tiles take longest and must not start last
    int order[9];
    for (int i = 0; i < ncl; ++i) order[i] = i;
    for (int i = 1; i < ncl; ++i)
        for (int j = i; j > 0 && cl[order[j]].na * cl[order[j]].nb > cl[order[j - 1]].na * cl[order[j - 1]].nb; --j) {
            const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t;
        }
    for (int oi = 0; oi < ncl; ++oi) {
        const dgrad_class &c = cl[order[oi]];
        if (c.na == 0 || c.nb == 0 || c.U == 0 || c.V == 0) continue;
        const int Kc = g.Co * c.na * c.nb;
        const int k = b.count++;
        b.pb[k] = {delta, g.Co, g.Ho, g.Wo, c.U, c.V, c.na, c.nb, c.bh, c.bw, Kc, (int)(R * c.U * c.V)};
        b.pa[k] = {Wt + c.wt_off, Kc, g.Ci, Kc};
        b.ep[k] = {g.Ci, b.pb[k].Q, c.U, c.V, g.stride, c.pi, c.pj, g.W, (long long)g.H * g.W, g.n};
        RunParams &rp = b.rp[k];
        rp.tiles_m = (g.Ci + C::BM - 1) / C::BM;
        rp.tiles_n = (b.pb[k].Q + C::BN - 1) / C::BN;
        rp.ktiles = (Kc + C::BK - 1) / C::BK;
        rp.per_split = rp.ktiles;
        rp.splits = 1;          // the epilogue scatters into dx: no partial sums
        rp.alpha = 1.0f; rp.accumulate = 0;
        rp.out = dx; rp.part = nullptr; rp.out_elems = R * g.n;
        b.first[k] = (int)slots;
        slots += ((long long)rp.tiles_m * rp.tiles_n + 7) / 8;       // per XCD
    }
    if (b.count == 0) return DK_OK;
    DK_REQUIRE(slots * 8 <= 0x7fffffffll, DK_ERR_SHAPE);
    for (int k = b.count; k <= DK_MAX_BATCH; ++k) b.first[k] = (int)slots;
    dk_prof_scope ps("contract_conv_dgrad_classes", st);
    contract_batch_kernel<C, LA, LB, EpiDgradClass><<<dim3((unsigned)(slots * 8)), dim3(C::NT), 0, st>>>(b);
    return dk_launch_status();
}

// stride 1 with pad <= k-1 and a square filter: a forward convolution of delta
bool dgrad_as_forward(const dk_geom &g, dk_geom *t)
{
    if (g.dw || g.stride != 1 || g.kh != g.kw || g.pad > g.kh - 1) return false;
    *t = g;
    t->Ci = g.Co; t->Co = g.Ci; t->H = g.Ho; t->W = g.Wo; t->pad = g.kh - 1 - g.pad;
    t->Ho = g.H; t->Wo = g.W;
    t->n = (long long)t->Ci * t->H * t->W;
    t->m = (long long)t->Co * t->Ho * t->Wo;
    t->Kg = (long long)t->Ci * t->kh * t->kw;
    return t->pad <= 16;
}

} // namespace

DK_EXPORT size_t dk_dgrad_workspace_bytes(const dk_layer *L, int R)
{
    dk_geom g, t;
    if (R < 1 || dk_layer_geom(L, &g) != DK_OK) return 0;
    if (!g.conv) {
        dk_geom d = {};
        d.M = g.N; d.N = g.M; d.n = g.M; d.m = g.N;          // C[R][N] over k = M
        return dk_ws_fwd_bytes(d, R);
    }
    const size_t wt = align_up((size_t)g.Co * g.Ci * g.kh * g.kw * sizeof(float), 256);
    if (g.dw) return 256;
    if (dgrad_as_forward(g, &t)) return wt + dk_ws_fwd_bytes(t, R);
    if (g.stride >= 2 && g.stride <= 3) return align_up(dgrad_class_filter_bytes(g), 256);
    // gather engine: C[Ci][R*H*W] over k = Co*kh*kw
    const long long Kd = (long long)g.Co * g.kh * g.kw;
    const size_t part = conv_flat_dgrad(g) ? split_bytes<CfgFlat>(g.Ci, (long long)R * g.H * g.W, Kd, R * g.n)
                                           : split_bytes<CfgSq>(g.Ci, (long long)R * g.H * g.W, Kd, R * g.n);
    return wt + (part < 256 ? 256 : part);
}

DK_EXPORT dk_status dk_dgrad(const dk_layer *L, const float *W, const float *delta, float *dx, int R,
                             void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && W && delta && dx, DK_ERR_NULL);
    dk_geom g, t;
    dk_status s = dk_layer_geom(L, &g);
    if (s != DK_OK) return s;
    DK_REQUIRE(R >= 1 && (long long)R * g.n < (1ll << 40) && (long long)R * g.m < (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(W, 4) && dk_aligned(delta, 4) && dk_aligned(dx, 4), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_dgrad_workspace_bytes(L, R), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    if (!g.conv) {
        const bool vec = (g.M % 4 == 0) && (g.N % 4 == 0) && dk_aligned(W, 16) && dk_aligned(delta, 16);
        if (vec)
            return run_dense_nn<CfgSq, true, true>(delta, W, dx, R, g.N, g.M, (float *)ws, ws_bytes, st);
        return run_dense_nn<CfgSq, false, false>(delta, W, dx, R, g.N, g.M, (float *)ws, ws_bytes, st);
    }
    if (g.dw) return dk_dw_dgrad_run(g, W, delta, dx, R, st);
    if (dgrad_as_forward(g, &t)) {
        DK_REQUIRE((long long)R * t.Ho * t.Wo < (1ll << 31) - 512, DK_ERR_SHAPE);
        float *Wt = (float *)ws;
        const size_t wt_bytes = align_up((size_t)g.Co * g.Ci * g.kh * g.kw * sizeof(float), 256);
        const int count = g.Co * g.Ci * g.kh * g.kw;
        {
            dk_prof_scope ps("dgrad_filter", st);
            dgrad_filter_kernel<<<dim3((count + 255) / 256), dim3(256), 0, st>>>(W, Wt, g.Co, g.Ci, g.kh, g.kw, 1);
        }
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        return conv_fwd_impl(t, Wt, delta, dx, R, (char *)ws + wt_bytes, ws_bytes - wt_bytes, stream);
    }
    if (g.stride >= 2 && g.stride <= 3 && (long long)R * g.H * g.W < (1ll << 31) - 512) {
        // strided: one dense sub-convolution per residue class of input pixels
        dgrad_class cl[9];
        const int ncl = dgrad_classes(g, cl);
        float *Wt = (float *)ws;
        bool any_empty = false;
        for (int c = 0; c < ncl; ++c) any_empty |= cl[c].na == 0 || cl[c].nb == 0;
        if (any_empty) {
            // pixels no filter tap reaches (a 1x1 filter with stride 2 skips three of four)
            const long long total = (long long)R * g.n;
            DK_REQUIRE((total + 255) / 256 <= 0x7fffffffll, DK_ERR_SHAPE);
            dk_prof_scope ps("dgrad_fill", st);
            fill_zero_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(dx, total);
            DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        }
        bool vw = true;
        dgrad_filter_batch fb;
        fb.count = 0;
        fb.first[0] = 0;
        for (int c = 0; c < ncl; ++c) {
            const dgrad_class &k = cl[c];
            if (k.na == 0 || k.nb == 0 || k.U == 0 || k.V == 0) continue;
            const int q = fb.count++;
            fb.a0[q] = k.a0; fb.b0[q] = k.b0; fb.na[q] = k.na; fb.nb[q] = k.nb;
            fb.off[q] = (long long)k.wt_off;
            fb.first[q + 1] = fb.first[q] + g.Co * g.Ci * k.na * k.nb;
            vw &= (g.Co * k.na * k.nb) % 4 == 0;    // rows of whole vectors (the matrices are 256-byte aligned)
        }
        if (fb.count) {
            dk_prof_scope ps("dgrad_filter", st);
            dgrad_class_filter_kernel<<<dim3((fb.first[fb.count] + 255) / 256), dim3(256), 0, st>>>(
                W, Wt, g.Co, g.Ci, g.kh, g.kw, g.stride, fb);
            DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        }
        if (conv_flat_dgrad(g))
            return vw ? run_dgrad_classes<CfgFlat, true>(g, cl, ncl, Wt, delta, dx, R, st)
                      : run_dgrad_classes<CfgFlat, false>(g, cl, ncl, Wt, delta, dx, R, st);
        return vw ? run_dgrad_classes<CfgSq, true>(g, cl, ncl, Wt, delta, dx, R, st)
                  : run_dgrad_classes<CfgSq, false>(g, cl, ncl, Wt, delta, dx, R, st);
    }
    if ((long long)R * g.H * g.W < (1ll << 31) - 512) {
        // any other geometry: gather loader on the generic contraction engine
        float *Wt = (float *)ws;
        const size_t wt_bytes = align_up((size_t)g.Co * g.Ci * g.kh * g.kw * sizeof(float), 256);
        const int count = g.Co * g.Ci * g.kh * g.kw;
        {
            dk_prof_scope ps("dgrad_filter", st);
            dgrad_filter_kernel<<<dim3((count + 255) / 256), dim3(256), 0, st>>>(W, Wt, g.Co, g.Ci, g.kh, g.kw, 0);
        }
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        float *part = (float *)((char *)ws + wt_bytes);
        const size_t part_bytes = ws_bytes - wt_bytes;
        const bool vw = ((g.Co * g.kh * g.kw) % 4 == 0);
        if (conv_flat_dgrad(g))
            return vw ? run_conv_dgrad<CfgFlat, true>(g, Wt, delta, dx, R, part, part_bytes, st)
                      : run_conv_dgrad<CfgFlat, false>(g, Wt, delta, dx, R, part, part_bytes, st);
        return vw ? run_conv_dgrad<CfgSq, true>(g, Wt, delta, dx, R, part, part_bytes, st)
                  : run_conv_dgrad<CfgSq, false>(g, Wt, delta, dx, R, part, part_bytes, st);
    }
    const long long total = (long long)R * g.n;
    DK_REQUIRE((total + 255) / 256 <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("conv_dgrad_direct", st);
    conv_dgrad_direct_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
        W, delta, dx, total, g.Ci, g.Co, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    return dk_launch_status();
}

// ---------------------------------------------------------------------------
// Diagnostic: what the fp32 matrix pipe sustains when nothing else limits it.
// ---------------------------------------------------------------------------
namespace {

// One wave per SIMD, eight independent accumulator blocks, operands in registers:
// 16 MFMAs per iteration and nothing else.
__global__ __launch_bounds__(256) void mfma_rate_kernel(int random_operands, int iterations, float *out)
{
    const unsigned seed = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    float a[2], b[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const unsigned h = (seed ^ (0x9e3779b9u * (unsigned)(x + 1))) * 2246822519u;
        // random: uniform in [1, 2) with a random sign (all mantissa bits toggle, no overflow)
        a[x] = random_operands ? __uint_as_float(0x3f800000u | ((h ^ (h >> 15)) & 0x807fffffu)) : 1.0f;
        b[x] = random_operands ? __uint_as_float(0x3f800000u | (((h * 3266489917u) ^ (h >> 13)) & 0x807fffffu)) : 1.0f;
    }
    f32x16 acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.0f;
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int q = 0; q < 8; ++q)
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q & 1], b[(q >> 1) & 1], acc[q], 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[q][v];
    if (out && sum == 1.2345e-30f) out[threadIdx.x] = sum;     // keeps the loop; practically never true
}

} // namespace

DK_EXPORT dk_status dk_probe_mfma_rate(int random_operands, int iterations, double *flop, void *stream)
{
    DK_REQUIRE(iterations >= 1 && iterations <= (1 << 24) && random_operands >= 0 && random_operands <= 1,
               DK_ERR_SHAPE);
    const int blocks = 256;
    dk_prof_scope ps(random_operands ? "mfma_rate_random" : "mfma_rate_constant", (hipStream_t)stream);
    mfma_rate_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>(random_operands, iterations, nullptr);
    if (flop) *flop = (double)blocks * 4.0 * (double)iterations * 16.0 * 4096.0;
    return dk_launch_status();
}
