// Finite-field variant: the dense contractions  C[i][j] = sum_k A[i][k] B[j][k]
// (mod p) on the int8 matrix cores.
//
// A field element is first lifted to its centred representative in
// (-p/2, p/2) and written as four balanced base-128 digits,
//     v = e0 + 128 e1 + 128^2 e2 + 128^3 e3,   e0..e2 in [-64, 63], |e3| <= 8,
// one int8 plane per digit (a lift within [-127, 127] stays one digit e0 = v).  A product of two elements is then the sum of 16
// digit products weighted by 128^(a+b).  The digits of each operand are taken
// in two halves ("low" = digits 0,1; "high" = digits 2,3); one part of a launch
// multiplies one half of A with one half of B and keeps one int32 accumulator
// per weight 128^s, s = 0..2 (more accumulators than that do not fit the 256
// accumulation registers of a wave with a 64 x 64 tile).  An accumulator holds
// at most two digit products per k, each at most 2^12 in magnitude, or one of
// two single-digit elements, at most 127^2: 2^17 values of k fit.  The epilogue recombines the three
// accumulators in 64 bits, reduces modulo p and applies the part's weight
// 128^(2 (ha + hb)).  A workgroup runs the four parts of its tile one after the
// other and adds their residues in registers; a part that involves a high half
// whose digits are all zero (quantised weights of ordinary magnitude) is
// skipped: the digit kernels record that in device flags, so nothing is read
// back to the host.  With more than one k slice the slices are residues too and
// are folded by modular addition.  All of it is exact: the result is the field
// product whatever the tiling.
//
// When both operands have non-zero high halves (the weight gradient: masked
// values are uniform over the field) the four parts become three: with
// L, H the halves and S = L + H taken digit by digit (e0 + e2 in [-128, 126],
// e1 + e3 in [-72, 71]: still int8),
//     A B = L_A L_B (1 - 128^2) + S_A S_B 128^2 + H_A H_B (128^4 - 128^2),
// so a third pair of planes holding S replaces a quarter of the MFMAs, of the
// LDS traffic and of the operand fetches.  A sum-half accumulator grows by at
// most 2 * 128 * 72 per k, so 2^16 values of k fit an int32.
//
// The contraction index has to be contiguous for both operands; digit planes
// are written k-major by the digit kernels (straight for row-major operands,
// through an LDS transpose for the weight gradient, whose contraction index is
// the encoded-row index).
#include <type_traits>
#include "dk_field.h"

namespace {

constexpr int BI = 128, BJ = 128;      // workgroup tile
constexpr int KT = 128;                // k bytes per LDS tile
constexpr int PITCH = 144;             // LDS row pitch in bytes: 16 (mod 32) keeps 16-byte reads conflict-free
constexpr int B_PLANE = BJ * PITCH;
constexpr int LDS_BYTES = 2 * (2 * BI * PITCH + 2 * B_PLANE);   // 147456: two buffers of the 128-row tile
constexpr int MAX_KSPLIT = 1 << 17;    // k values per slice (int32 accumulators)
constexpr int MAX_KSPLIT_SUMS = 1 << 16;   // ... when the digit-sum planes are multiplied
constexpr int RSRC_FLAGS = 0x00020000;  // raw buffer resource, gfx9 family
constexpr int MAX_SPLITS = 256;        // k slices per output tile (the fold adds their residues in 64 bits)

struct fgemm_params {
    const int8_t *Ap;      // [4 or 6][I_pad][Kp]
    const int8_t *Bp;      // [4 or 6][J_pad][Kp]
    uint32_t *out_q;       // residues [splits][I][J] (a slice per k split), or NULL
    float *out_f;          // de-quantised result [I][J] (only with one split), or NULL
    const int *flags;      // [0]: A, [1]: B; bit 0: non-zero high digits (planes 2, 3), bit 1: non-zero plane 1 (device)
    long long a_plane, b_plane;   // bytes per plane
    int I, J, Kp;
    int tiles_i, tiles_j, splits, ktiles_per_split, ktiles;
    // implicit convolution operand (B read from channels-last digit planes [R][H][W][cp])
    int cp, cH, cW, ckh, ckw, cstride, cpad, cWo, cHoWo;
    // padded-rows operand (B of a stride-1 convolution's weight gradient, see f_digits_rows_kernel):
    // with it cp = Ci, ckh, ckw = filter size, cWo = row pitch Wp of the contraction index
    int sRow;              // bytes per channel row of a plane: R * Hp * Wpp
    int sImgK;             // contraction indices per image: Ho * Wp
    int sImgP;             // plane bytes per image: Hp * Wpp
    int sWpp;              // row pitch of the planes
    int sK;                // contraction length R * Ho * Wp
    int out_hw;            // 0: C[i][j] at i*J + j;  hw > 0: j = (image, pixel), C at ((image*I + i)*hw + pixel
    double s_inv;          // 2^-l for out_f
    int lq;                // l
    float scale;
    int accumulate;
    int sums;              // planes 4, 5 of both operands hold the digit sums of the halves
    int single_mask;       // bit 0: a SINGLE = 1 launch accompanies this one, bit 1: a SINGLE = 2 launch
};

// Four base-128 digits of the centred lift of q, packed one per byte: balanced
// digits in [-64, 63], except that a lift within [-127, 127] is its own single
// digit (a byte holds it, and ordinary quantised weights then occupy one plane
// up to twice the magnitude).  Either way the lift is sum_i e_i 128^i with
// |e_0| <= 127, |e_i| <= 64 above it, and e_0 beyond [-64, 63] only next to
// zero higher digits: a digit product is at most 127^2 where both factors are
// such single digits (127^2 2^17 < 2^31) and at most 127 * 64 < 2^13 otherwise,
// and a digit sum of the halves is the digit itself.
__device__ __forceinline__ uint32_t digits_of(uint32_t q)
{
    int w = (int)q;
    if (q > DKF_P / 2) w -= (int)DKF_P;
    // With 64 added to each of the three low digits they are the plain 7-bit fields of
    // u = w + 64 (1 + 128 + 128^2), and what lies above them is e3 (arithmetic shifts keep
    // this true for negative u).  The fields are spread to one per byte, 64 is taken off
    // again by flipping bit 6, and bit 7 becomes a copy of bit 6 (the sign of a value in
    // [-64, 63]).
    const int u = w + 64 * (1 + 128 + 128 * 128);
    uint32_t x = ((uint32_t)u & 0x7fu) | (((uint32_t)u << 1) & 0x7f00u) | (((uint32_t)u << 2) & 0x7f0000u);
    x ^= 0x404040u;
    x |= (x & 0x404040u) << 1;
    x |= (uint32_t)(u >> 21) << 24;
    return (uint32_t)(w + 127) <= 254u ? (uint32_t)(w & 255) : x;
}

// (e0 + e2, e1 + e3) of a packed-digit word in its two low bytes: a byte-wise
// add of the two half-words (no carry from one byte into the next)
__device__ __forceinline__ uint32_t half_sums(uint32_t d)
{
    const uint32_t lo = d & 0xffffu, hi = d >> 16;
    return ((lo & 0x7f7fu) + (hi & 0x7f7fu)) ^ ((lo ^ hi) & 0x8080u);
}

// byte `a` of four packed-digit words -> one word of plane a
__device__ __forceinline__ uint32_t gather_byte(const uint32_t (&d)[4], int a)
{
    // byte permutes: (byte a of d0, byte a of d1), the same of d2, d3, then the two pairs
    const uint32_t sel = 0x0c0c0000u | (uint32_t)a | (uint32_t)(4 + a) << 8;
    const uint32_t p01 = __builtin_amdgcn_perm(d[1], d[0], sel);
    const uint32_t p23 = __builtin_amdgcn_perm(d[3], d[2], sel);
    return __builtin_amdgcn_perm(p23, p01, 0x05040100u);
}

// Sixteen packed-digit words -> one 16-byte piece of each plane at `dst`
// (plane a at dst + a * plane); with `sums` planes 4, 5 get the digit sums of
// the halves.  Returns the OR of the high-half words; `mid` gets the OR of
// the words of plane 1.
__device__ __forceinline__ uint32_t store_pieces(const uint32_t (&d)[16], int8_t *dst, long long plane, int sums,
                                                 uint32_t &mid)
{
    uint32_t hi = 0;
    mid = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        u32x4 w;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t dq[4] = {d[4 * q], d[4 * q + 1], d[4 * q + 2], d[4 * q + 3]};
            w[q] = gather_byte(dq, a);
        }
        if (a >= 2) hi |= w.x | w.y | w.z | w.w;
        if (a == 1) mid |= w.x | w.y | w.z | w.w;
        *reinterpret_cast<u32x4 *>(dst + a * plane) = w;
    }
    if (sums) {
        uint32_t ds[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) ds[c] = half_sums(d[c]);
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            u32x4 w;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t dq[4] = {ds[4 * q], ds[4 * q + 1], ds[4 * q + 2], ds[4 * q + 3]};
                w[q] = gather_byte(dq, a);
            }
            *reinterpret_cast<u32x4 *>(dst + (4 + a) * plane) = w;
        }
    }
    return hi;
}

// Record "some high digit (planes 2, 3) is non-zero" in bit 0 and "some digit
// of plane 1 is non-zero" in bit 1.  One lane per wave looks at the flag
// first, so once it is set the other waves of the launch only read it.
__device__ __forceinline__ void raise_flag(int *flag, uint32_t hi, uint32_t mid)
{
    const int want = (__any(hi != 0) ? 1 : 0) | (__any(mid != 0) ? 2 : 0);
    if (flag && want && (threadIdx.x & 63) == 0) {
        if ((__atomic_load_n(flag, __ATOMIC_RELAXED) & want) != want) atomicOr(flag, want);
    }
}

// Row-major operand src[rows][K] -> planes[4][rows_pad][Kp].  A workgroup
// converts 4096 consecutive k of one row, a thread sixteen (four 16-byte loads
// in flight, one 16-byte store per plane); rows and k beyond the operand are
// written as zeros.  F32: the source holds real values and the field elements
// Field(Round(x scale)) are formed here, so the quantised operand never exists
// in memory.
template <bool F32>
__global__ __launch_bounds__(256) void f_digits_kernel(const void *__restrict__ src_,
                                                       int8_t *__restrict__ planes, int rows, int K,
                                                       int rows_pad, int Kp, int chunks, int vec,
                                                       double scale, int *flag)
{
    const int row = blockIdx.x / chunks;                       // workgroup-uniform
    const int k0 = ((blockIdx.x - row * chunks) * 256 + threadIdx.x) * 16;
    if (k0 >= Kp) return;
    uint32_t v[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = 0;
    if (row < rows) {
        const uint32_t *s = static_cast<const uint32_t *>(src_) + (long long)row * K + k0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (vec && k0 + 4 * q + 3 < K) {
                const u32x4 t = *reinterpret_cast<const u32x4 *>(s + 4 * q);
                v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
            } else {
#pragma unroll
                for (int c = 4 * q; c < 4 * q + 4; ++c)
                    if (k0 + c < K) v[c] = s[c];
            }
        }
        if (F32) {
#pragma unroll
            for (int c = 0; c < 16; ++c)
                if (k0 + c < K) v[c] = dkf_quant(__uint_as_float(v[c]), scale);
        }
    }
    // (the digits of 0 are 0, so absent elements need no flag of their own)
    uint32_t d[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) d[c] = digits_of(v[c]);
    const long long plane = (long long)rows_pad * Kp;
    uint32_t mid;
    const uint32_t hi = store_pieces(d, planes + (long long)row * Kp + k0, plane, 0, mid);
    raise_flag(flag, hi, mid);
}

struct fconv_geom {
    int Ci, Co, H, W, kh, kw, stride, pad, Ho, Wo, HoWo;
};

// Operands whose source is contiguous along the *row* index of the planes, not
// along k: a tile of 128 k x 64 rows goes through LDS as packed digits, read
// with consecutive lanes on consecutive rows; a thread then writes 16
// consecutive k of one row to each plane.
//   IM2COL false: src[K][cols] (operands of the dense weight gradient, whose
//                 contraction index is the encoded row);
//   IM2COL true:  row = (image r, oh, ow), k = (ci, a, b), the element is
//                 xbar[r][ci][oh*stride + a - pad][ow*stride + b - pad] or 0
//                 outside the image (forward operand of a convolution).
template <bool IM2COL>
__global__ __launch_bounds__(256) void f_digits_t_kernel(const uint32_t *__restrict__ src,
                                                         int8_t *__restrict__ planes, fconv_geom g,
                                                         int K, int cols, int cols_pad, int Kp,
                                                         int sums, int *flag)
{
    __shared__ uint32_t tile[128][65];
    const int c0 = blockIdx.x * 64, k0 = blockIdx.y * 128;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c = c0 + tx;
    long long base = 0;             // IM2COL: offset of (image, channel 0, oh*stride - pad, ow*stride - pad)
    int ih0 = 0, iw0 = 0;
    if (IM2COL && c < cols) {
        const int img = c / g.HoWo, px = c - img * g.HoWo;
        const int oh = px / g.Wo, ow = px - oh * g.Wo;
        ih0 = oh * g.stride - g.pad; iw0 = ow * g.stride - g.pad;
        base = (long long)img * g.Ci * g.H * g.W;
    }
    const int khw = g.kh * g.kw;
    // straight source with whole 16-byte vectors per row (cols % 4 == 0 and an
    // aligned base): eight vector loads per thread, all in flight at once
    const bool vec = !IM2COL && (cols & 3) == 0 && (((size_t)src) & 15) == 0;
    if (vec) {
        u32x4 t[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int item = threadIdx.x + 256 * r;
            const int k = k0 + (item >> 4), cc = c0 + (item & 15) * 4;
            t[r] = u32x4{0, 0, 0, 0};
            if (k < K && cc < cols) t[r] = *reinterpret_cast<const u32x4 *>(src + (long long)k * cols + cc);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int item = threadIdx.x + 256 * r;
            uint32_t *dst = &tile[item >> 4][(item & 15) * 4];
            dst[0] = digits_of(t[r].x); dst[1] = digits_of(t[r].y);
            dst[2] = digits_of(t[r].z); dst[3] = digits_of(t[r].w);
        }
    } else
#pragma unroll 8
    for (int r = 0; r < 32; ++r) {
        const int k = k0 + ty + 4 * r;                 // wave-uniform
        uint32_t v = 0;
        if (k < K && c < cols) {
            if (IM2COL) {
                const int ci = k / khw, ab = k - ci * khw, a = ab / g.kw, b = ab - a * g.kw;
                const int ih = ih0 + a, iw = iw0 + b;
                if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
                    v = digits_of(src[base + ((long long)ci * g.H + ih) * g.W + iw]);
            } else {
                v = digits_of(src[(long long)k * cols + c]);
            }
        }
        tile[ty + 4 * r][tx] = v;
    }
    __syncthreads();
    const long long plane = (long long)cols_pad * Kp;
    uint32_t hi = 0, mid = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int item = threadIdx.x + 256 * r;       // (row, 16 k): eight lanes write 128 contiguous bytes
        const int kq = item & 7, col = item >> 3;
        u32x4 w[6];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t d[4], ds[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                d[c] = tile[16 * kq + 4 * g + c][col];
                ds[c] = half_sums(d[c]);
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) w[a][g] = gather_byte(d, a);
            w[4][g] = gather_byte(ds, 0);
            w[5][g] = gather_byte(ds, 1);
        }
        hi |= w[2].x | w[2].y | w[2].z | w[2].w | w[3].x | w[3].y | w[3].z | w[3].w;
        mid |= w[1].x | w[1].y | w[1].z | w[1].w;
#pragma unroll
        for (int a = 0; a < 6; ++a)
            if (a < 4 || sums)
                *reinterpret_cast<u32x4 *>(planes + a * plane + (long long)(c0 + col) * Kp + k0 + 16 * kq) = w[a];
    }
    raise_flag(flag, hi, mid);
}

// Digit planes of the operands of a convolution's weight gradient, gathered
// from NCHW field tensors; the contraction index is k = (image r, oh, ow), which
// is contiguous in both sources.  A workgroup converts 4096 consecutive k of
// one row, a thread four runs of four.
//   MODE 1 (A): row = co, the element is dtilde[r][co][oh][ow];
//   MODE 2 (B): row = (ci, a, b), the element is
//               xbar[r][ci][oh*stride + a - pad][ow*stride + b - pad] or 0 outside.
// Rows beyond `rows` and k beyond K give zeros.
template <int MODE>
__global__ __launch_bounds__(256) void f_digits_conv_kernel(const uint32_t *__restrict__ src,
                                                            int8_t *__restrict__ planes, fconv_geom g,
                                                            int rows, int K, int rows_pad, int Kp,
                                                            int chunks, int sums, int *flag)
{
    const int row = blockIdx.x / chunks;                       // workgroup-uniform
    // a thread takes four groups of four k, 1024 k apart, and issues all its
    // loads before it uses the first (bytes in flight are what the kernel lives on)
    const int kb = (blockIdx.x - row * chunks) * 4096 + threadIdx.x * 4;
    int r_ci = 0, r_a = 0, r_b = 0;                            // what the row fixes
    if (MODE == 2) {
        const int khw = g.kh * g.kw;
        r_ci = row / khw;
        const int ab = row - r_ci * khw;
        r_a = ab / g.kw; r_b = ab - r_a * g.kw;
    }
    uint32_t v[4][4];
    bool ok[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int k0 = kb + q * 1024;
        // what k0 fixes; the three following k advance it like a mixed-radix counter
        int k_img = k0 / g.HoWo;
        int k_px = k0 - k_img * g.HoWo;
        int k_oh = k_px / g.Wo, k_ow = k_px - k_oh * g.Wo;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            v[q][c] = 0; ok[q][c] = false;
            if (row < rows && k0 + c < K) {
                long long idx = -1;
                if (MODE == 1) {
                    idx = ((long long)k_img * g.Co + row) * g.HoWo + k_px;
                } else {
                    const int ih = k_oh * g.stride + r_a - g.pad, iw = k_ow * g.stride + r_b - g.pad;
                    if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
                        idx = (((long long)k_img * g.Ci + r_ci) * g.H + ih) * g.W + iw;
                }
                if (idx >= 0) { v[q][c] = src[idx]; ok[q][c] = true; }
            }
            ++k_px;
            if (++k_ow == g.Wo) { k_ow = 0; if (++k_oh == g.Ho) { k_oh = 0; k_px = 0; ++k_img; } }
        }
    }
    const long long plane = (long long)rows_pad * Kp;
    uint32_t hi = 0, mid = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int k0 = kb + q * 1024;
        if (k0 >= Kp) continue;
        uint32_t d[4], ds[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            d[c] = ok[q][c] ? digits_of(v[q][c]) : 0u;
            ds[c] = half_sums(d[c]);
        }
        int8_t *dst = planes + (long long)row * Kp + k0;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint32_t w = gather_byte(d, a);
            if (a >= 2) hi |= w;
            if (a == 1) mid |= w;
            *reinterpret_cast<uint32_t *>(dst + a * plane) = w;
        }
        if (sums) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
                *reinterpret_cast<uint32_t *>(dst + (4 + a) * plane) = gather_byte(ds, a);
        }
    }
    raise_flag(flag, hi, mid);
}

// Digit planes of the operands of a stride-1 convolution's weight gradient with
// the contraction index k = (image r, row h, column wq), wq < Wp = Wo rounded up
// to 16 (so a 16-byte piece of k never leaves its row).  A workgroup converts
// 4096 consecutive k of one plane row, a thread sixteen (all in one image row).
//   SHIFTED false (A): plane row = co, h < Ho: dtilde[r][co][h][wq], zero for
//       wq >= Wo; rows beyond `rows` and k beyond R*Ho*Wp are zeros.
//   SHIFTED true (B):  plane row = ci, h < Hp = Ho + kh - 1, columns of pitch
//       Wp (here the planes' own pitch, at least Wo rounded up to 16 plus
//       kw - 1): xbar[r][ci][h - pad][wq - pad], zero outside the image.  Filter
//       tap (a, b) of channel ci is this row read from h = oh + a, b bytes on:
//       one padded copy serves all kh * kw taps.
template <bool SHIFTED>
__global__ __launch_bounds__(256) void f_digits_rows_kernel(const uint32_t *__restrict__ src,
                                                            int8_t *__restrict__ planes, fconv_geom g,
                                                            int rows, int rows_pad, int Hk, int Wp,
                                                            int len, int pitch, int chunks, int sums,
                                                            int vec, int *flag)
{
    const int row = blockIdx.x / chunks;                       // workgroup-uniform
    // all sixteen loads of a thread are issued before the first is used: the
    // kernel lives on the number of bytes in flight
    if (SHIFTED) {
        // four groups of four k, 1024 k apart: neighbouring lanes stay on
        // neighbouring 16-byte runs of the shifted source
        const int kb = (blockIdx.x - row * chunks) * 4096 + threadIdx.x * 4;
        const int ci = row;
        uint32_t v[4][4];
        bool ok[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k0 = kb + q * 1024;
#pragma unroll
            for (int c = 0; c < 4; ++c) { v[q][c] = 0; ok[q][c] = false; }
            if (row < rows && k0 < len) {
                const int img = k0 / (Hk * Wp);
                const int rem = k0 - img * (Hk * Wp);
                const int h = rem / Wp, wq = rem - h * Wp;
                const int ih = h - g.pad;
                if (ih >= 0 && ih < g.H) {
                    const uint32_t *s = src + (((long long)img * g.Ci + ci) * g.H + ih) * g.W;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int iw = wq + c - g.pad;
                        if (iw >= 0 && iw < g.W) { v[q][c] = s[iw]; ok[q][c] = true; }
                    }
                }
            }
        }
        const long long plane = (long long)rows_pad * pitch;
        uint32_t hi = 0, mid = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k0 = kb + q * 1024;
            if (k0 >= pitch) continue;
            uint32_t d[4], ds[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                d[c] = ok[q][c] ? digits_of(v[q][c]) : 0u;
                ds[c] = half_sums(d[c]);
            }
            int8_t *dst = planes + (long long)row * pitch + k0;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const uint32_t w = gather_byte(d, a);
                if (a >= 2) hi |= w;
                if (a == 1) mid |= w;
                *reinterpret_cast<uint32_t *>(dst + a * plane) = w;
            }
            if (sums) {
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    *reinterpret_cast<uint32_t *>(dst + (4 + a) * plane) = gather_byte(ds, a);
            }
        }
        raise_flag(flag, hi, mid);
        return;
    }
    const int k0 = ((blockIdx.x - row * chunks) * 256 + threadIdx.x) * 16;
    if (k0 >= pitch) return;
    uint32_t v[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = 0;
    bool ok[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) ok[c] = false;
    if (row < rows && k0 < len) {
        const int img = k0 / (Hk * Wp);
        const int rem = k0 - img * (Hk * Wp);
        const int h = rem / Wp, wq = rem - h * Wp;
        {
            const uint32_t *s = src + (((long long)img * g.Co + row) * g.Ho + h) * g.Wo;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (vec && wq + 4 * q + 3 < g.Wo) {          // vec: Wo % 4 == 0 and an aligned base
                    const u32x4 t = *reinterpret_cast<const u32x4 *>(s + wq + 4 * q);
                    v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
#pragma unroll
                    for (int c = 0; c < 4; ++c) ok[4 * q + c] = true;
                } else {
#pragma unroll
                    for (int c = 4 * q; c < 4 * q + 4; ++c)
                        if (wq + c < g.Wo) { v[c] = s[wq + c]; ok[c] = true; }
                }
            }
        }
    }
    uint32_t d[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) d[c] = ok[c] ? digits_of(v[c]) : 0u;
    const long long plane = (long long)rows_pad * pitch;
    uint32_t mid;
    const uint32_t hi = store_pieces(d, planes + (long long)row * pitch + k0, plane, sums, mid);
    raise_flag(flag, hi, mid);
}

// Encodings xbar[R][Ci][H*W] -> channels-last digit planes [4][R][H*W][cp]
// (cp = Ci, a multiple of 16): per image a tile of KC channels x 8192 / KC
// pixels (128 x 64, or 64 x 128 when there are at most 64 channels) goes
// through LDS as packed digits; a thread then writes 16 consecutive channels of
// one pixel to each plane.  Row k of the LDS tile is rotated by (k / 16) * 512 / KC
// words, so that the lanes of a wave, which read one word each from rows 16
// apart, meet distinct banks.
template <int KC>
__global__ __launch_bounds__(256) void f_digits_nhwc_kernel(const uint32_t *__restrict__ src,
                                                            int8_t *__restrict__ planes, int Ci, int HW,
                                                            int cp, long long plane, int vec, int *flag)
{
    constexpr int PX = 8192 / KC, ROT = 512 / KC, KQ = KC / 16;
    __shared__ __attribute__((aligned(16))) uint32_t tile[KC * PX];
    const int c0 = blockIdx.x * PX, k0 = blockIdx.y * KC, img = blockIdx.z;
    const uint32_t *s = src + (long long)img * Ci * HW;
    if (vec) {
        // HW % 4 == 0 and an aligned base: eight 16-byte loads per thread, all in
        // flight at once (PX / 4 lanes per channel row of the tile)
        u32x4 t[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int item = threadIdx.x + 256 * r;
            const int k = k0 + item / (PX / 4), c = c0 + (item % (PX / 4)) * 4;
            t[r] = u32x4{0, 0, 0, 0};
            if (k < Ci && c < HW) t[r] = *reinterpret_cast<const u32x4 *>(s + (long long)k * HW + c);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int item = threadIdx.x + 256 * r;
            const int kl = item / (PX / 4), c = (item % (PX / 4)) * 4;
            u32x4 d;
            d.x = digits_of(t[r].x); d.y = digits_of(t[r].y); d.z = digits_of(t[r].z); d.w = digits_of(t[r].w);
            *reinterpret_cast<u32x4 *>(&tile[kl * PX + ((c + (kl >> 4) * ROT) & (PX - 1))]) = d;
        }
    } else {
#pragma unroll 8
        for (int r = 0; r < 32; ++r) {
            const int e = threadIdx.x + 256 * r;
            const int kl = e / PX, cl = e % PX;
            const int k = k0 + kl, c = c0 + cl;
            tile[kl * PX + ((cl + (kl >> 4) * ROT) & (PX - 1))] =
                (k < Ci && c < HW) ? digits_of(s[(long long)k * HW + c]) : 0u;
        }
    }
    __syncthreads();
    uint32_t hi = 0, mid = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int item = threadIdx.x + 256 * r;       // (pixel, 16 channels)
        const int kq = item % KQ, col = item / KQ;
        if (c0 + col >= HW || k0 + 16 * kq >= cp) continue;
        const int at = (col + kq * ROT) & (PX - 1);
        u32x4 w[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t d[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) d[c] = tile[(16 * kq + 4 * g + c) * PX + at];
#pragma unroll
            for (int a = 0; a < 4; ++a) w[a][g] = gather_byte(d, a);
        }
        hi |= w[2].x | w[2].y | w[2].z | w[2].w | w[3].x | w[3].y | w[3].z | w[3].w;
        mid |= w[1].x | w[1].y | w[1].z | w[1].w;
#pragma unroll
        for (int a = 0; a < 4; ++a)
            *reinterpret_cast<u32x4 *>(planes + a * plane + ((long long)img * HW + c0 + col) * cp + k0 + 16 * kq) = w[a];
    }
    raise_flag(flag, hi, mid);
}

// Filters W[Co][Ci][kh*kw] -> digit planes [4][rows_pad][Kp] with the
// contraction index ordered k = tap * cp + ci (to match the channels-last
// operand); rows beyond Co and k beyond kh*kw*cp are zeros.
__global__ __launch_bounds__(256) void f_digits_wconv_kernel(const uint32_t *__restrict__ W,
                                                             int8_t *__restrict__ planes, int Co, int Ci,
                                                             int taps, int cp, int rows_pad, int Kp,
                                                             int chunks, int *flag)
{
    const int row = blockIdx.x / chunks;
    const int k0 = ((blockIdx.x - row * chunks) * 256 + threadIdx.x) * 4;
    if (k0 >= Kp) return;
    uint32_t d[4] = {0, 0, 0, 0};
    if (row < Co) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int k = k0 + c, tap = k / cp, ci = k - tap * cp;
            if (tap < taps && ci < Ci) d[c] = digits_of(W[((long long)row * Ci + ci) * taps + tap]);
        }
    }
    const long long plane = (long long)rows_pad * Kp;
    uint32_t hi = 0, mid = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const uint32_t w = gather_byte(d, a);
        if (a >= 2) hi |= w;
        if (a == 1) mid |= w;
        *reinterpret_cast<uint32_t *>(planes + a * plane + (long long)row * Kp + k0) = w;
    }
    raise_flag(flag, hi, mid);
}

// The same with a whole filter row staged in LDS: W[row][Ci][taps] is read as it lies in
// memory (the kernel above reads it with a stride of `taps` words per lane), and the planes
// are written in their own order.  One workgroup per plane row; Ci * taps words of LDS.
__global__ __launch_bounds__(256) void f_digits_wconv_lds_kernel(const uint32_t *__restrict__ W,
                                                                 int8_t *__restrict__ planes, int Co, int Ci,
                                                                 int taps, int cp, int rows_pad, int Kp,
                                                                 int *flag)
{
    extern __shared__ uint32_t wrow[];
    const int row = blockIdx.x, n = Ci * taps;
    if (row < Co) {
        const uint32_t *src = W + (long long)row * n;
        for (int i = threadIdx.x; i < n; i += 256) wrow[i] = digits_of(src[i]);
    }
    __syncthreads();
    const long long plane = (long long)rows_pad * Kp;
    uint32_t hi = 0, mid = 0;
    for (int k0 = threadIdx.x * 4; k0 < Kp; k0 += 1024) {
        // cp is a multiple of 16: the four k share their tap
        const int tap = k0 / cp, ci0 = k0 - tap * cp;
        uint32_t d[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            d[c] = (row < Co && tap < taps && ci0 + c < Ci) ? wrow[(ci0 + c) * taps + tap] : 0u;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint32_t w = gather_byte(d, a);
            if (a >= 2) hi |= w;
            if (a == 1) mid |= w;
            *reinterpret_cast<uint32_t *>(planes + a * plane + (long long)row * Kp + k0) = w;
        }
    }
    raise_flag(flag, hi, mid);
}

__global__ void f_flag_clear_kernel(int *flags) { if (threadIdx.x < 2) flags[threadIdx.x] = 0; }

// a0 + 2^7 a1 + 2^14 a2 (three int32 digit-class sums) as a lazily reduced
// residue below 2^25 + 2^9, in 32-bit operations only (64-bit shifts and
// multiply-adds run at a fraction of their rate): each term is split where
// its shift crosses 2^25 and the upper part comes back multiplied by 39 = 2^25 mod p
// (24-bit multiply-adds; arithmetic shifts keep the split exact for negative sums);
// 2p makes the total positive before the last fold.
__device__ __forceinline__ uint32_t fold_sum3(int a0, int a1, int a2)
{
    const int x0 = __mul24(a0 >> 25, 39) + (a0 & 0x1ffffff);                 // a0:       |.| < 2^25 + 2^12
    const int x1 = __mul24(a1 >> 18, 39) + (int)(((uint32_t)a1 << 7) & 0x1ffffffu);          // 2^7 a1:   (-2^19, 2^25 + 2^19)
    const int x2 = __mul24(a2 >> 11, 39) + (int)(((uint32_t)a2 << 14) & 0x1ffffffu);         // 2^14 a2:  (-2^26, 2^25 + 2^26)
    const uint32_t sum = (uint32_t)(x0 + x1 + x2 + 2 * (int)DKF_P);          // in (0, 2^28)
    return __umul24(sum >> 25, 39u) + (sum & 0x1ffffffu);
}

// t 2^14 mod p for t < 2^26, lazily reduced (below 2^25 + 2^21): the bits that the
// shift moves above 2^25 come back multiplied by 39.
__device__ __forceinline__ uint32_t shift14(uint32_t t)
{
    return __umul24(t >> 11, 39u) + ((t << 14) & 0x1ffffffu);
}

// One workgroup: a 128 x 128 tile of C over one k slice, all four digit-half
// parts one after the other; four waves, each a 64 x 64 quarter (2 x 2 blocks
// of 32 x 32).  Global loads of the next k tile are in flight in registers while
// the current one is multiplied out of LDS (two LDS buffers, one barrier per
// tile); the operands of the next 32-k step are read from LDS while the MFMAs
// of the current one run.
// IMPL: the B operand of a convolution forward is not a stored matrix: row
// j = (image, oh, ow) and k = (a, b, ci) address the channels-last digit planes
// of the encodings directly (16 consecutive channels per piece, zeros outside
// the image), so no patch matrix exists in memory.
// BMODE 2: the B operand of a stride-1 convolution's weight gradient: row
// j = (ci, a, b) is channel row ci of the padded-rows planes read a rows and b
// bytes further on (the 16-byte loads are then not 16-byte aligned, which
// global loads on this target allow); the contraction index k = (image, oh, wq)
// is mapped onto the planes' own pitches.  BMODE 1 is IMPL, 0 a stored matrix.
// NBI: 32-row blocks of A per wave; the workgroup tile is (64 NBI) x 128 (a
// 64-row tile keeps operands with at most 64 rows from wasting half the MFMAs).
// SINGLE: an operand whose elements all fit one digit (ordinary quantised
// weights: |Round(w 2^l)| <= 127) has an all-zero plane 1 as well; the SINGLE = 1
// (A is such) and SINGLE = 2 (B is) variants move and multiply one plane of it
// instead of two, half the MFMAs of a step.  The digit kernels' flags decide on
// the device which variant does the work: the host launches the general kernel
// and the variants named in p.single_mask one after the other, and the
// workgroups of all but one of them return at once.
template <int BMODE, int NBI, int SINGLE = 0>
__global__ __launch_bounds__(256) void f_gemm_kernel(fgemm_params p)
{
    constexpr bool IMPL = BMODE == 1;
    constexpr int BI = 64 * NBI, A_PLANE = BI * PITCH, BUF_BYTES = 2 * A_PLANE + 2 * B_PLANE;
    constexpr int NA = 4 * NBI;          // 16-byte pieces of A per thread and tile
    extern __shared__ __attribute__((aligned(16))) int8_t flds[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_i * p.tiles_j;
    const int bid = dk_xcd_block();
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    // Tiles are walked in bands of GI tile rows, down the band's columns: the
    // 32 workgroups an XCD runs side by side then share 8 row tiles and 4 column
    // tiles (12 operand tiles through its L2 instead of 33 for a whole column of
    // a tall output).
    constexpr int GI = 8;
    const int band = t / (GI * p.tiles_j);
    const int in_band = t - band * (GI * p.tiles_j);
    const int rows_here = p.tiles_i - band * GI < GI ? p.tiles_i - band * GI : GI;
    const int tj = in_band / rows_here;
    const int ti = band * GI + (in_band - tj * rows_here);
    const int flag_a = p.flags[0], flag_b = p.flags[1];        // workgroup-uniform
    const bool fa = (flag_a & 1) != 0, fb = (flag_b & 1) != 0;

    const int kt0 = split * p.ktiles_per_split;
    int kt1 = kt0 + p.ktiles_per_split;
    if (kt1 > p.ktiles) kt1 = p.ktiles;

    // global -> register staging: 8 + 8 sixteen-byte pieces per thread and tile.
    // A thread owns one 16-byte column of the 128-byte rows (piece tid & 7) and
    // rows (tid >> 3) + 32 q, q = 0..3, of both planes of both operands.
    // Their addresses are a workgroup-uniform base plus this 32-bit offset.
    const int srow = tid >> 3, spiece = tid & 7;
    const long long q_rows = 32ll * p.Kp;
    const unsigned s_off = (unsigned)srow * (unsigned)p.Kp + 16u * spiece;
    const int s_dst = srow * PITCH + 16 * spiece;

    // implicit operand: what this thread's four rows fix
    unsigned r_base[4];
    int r_ih[4], r_iw[4];
    bool r_ok[4];
    if (IMPL) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j = tj * BJ + srow + 32 * q;
            r_ok[q] = j < p.J;
            const int img = r_ok[q] ? j / p.cHoWo : 0;
            const int px = r_ok[q] ? j - img * p.cHoWo : 0;
            const int oh = px / p.cWo, ow = px - oh * p.cWo;
            r_ih[q] = oh * p.cstride - p.cpad;
            r_iw[q] = ow * p.cstride - p.cpad;
            r_base[q] = (unsigned)img * (unsigned)(p.cH * p.cW) * (unsigned)p.cp;
        }
    }
    if (BMODE == 2) {
        const int taps = p.ckh * p.ckw;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j = tj * BJ + srow + 32 * q;
            r_ok[q] = j < p.J;
            const int ci = r_ok[q] ? j / taps : 0;
            const int ab = r_ok[q] ? j - ci * taps : 0;
            const int fa_ = ab / p.ckw, fb_ = ab - fa_ * p.ckw;
            r_base[q] = (unsigned)ci * (unsigned)p.sRow + (unsigned)(fa_ * p.sWpp + fb_);
            r_ih[q] = r_iw[q] = 0;
        }
    }

    const int wi0 = (wave & 1) * 32 * NBI, wj0 = (wave >> 1) * 64;
    const int a_rd = (wi0 + li) * PITCH + 16 * lh;
    const int b_rd = 2 * A_PLANE + (wj0 + li) * PITCH + 16 * lh;

    uint32_t res[NBI][2][16];
#pragma unroll
    for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) res[bi][bj][v] = 0;

    i32x16 acc[NBI][2][3];
#pragma unroll
    for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[bi][bj][s][v] = 0;

    // A part is a pair of plane pairs (0 low, 1 high, 2 digit sums), A's in bits
    // 0-1 and B's in bits 2-3.  The active parts in the order (lo,lo), (hi,lo),
    // (lo,hi), (hi,hi): weights 128^0, 128^2, 128^2, 128^4, so the two middle parts
    // share accumulators (one weight group).  With the sum planes and both high
    // halves present: (lo,lo), (sum,sum), (hi,hi), a group each.
    // Steps (part, k tile) form one software-pipelined sequence.
#define DKF_PART(I) ((plist >> (4 * (I))) & 15)
#define DKF_GROUP(Q) ((Q) == 0xA ? 1 : ((Q) & 1) + ((Q) >> 2))

    i32x4 sa[NA], sb[8];
    // Stored operands are fetched with buffer loads: a resource per digit plane of the part
    // being fetched, spanning this tile's rows (rebuilt when the part changes), the lane's
    // row and piece in four precomputed offsets and the k tile in the scalar offset -- no
    // address arithmetic per load (64-bit lane addresses cost a vector instruction per load
    // and a dozen scalar ones per step, all issued by the one wave that feeds the matrix pipe).
    __amdgpu_buffer_rsrc_t rsA0, rsA1, rsB0, rsB1;
    const int8_t *bpart = p.Bp;
    unsigned voff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) voff[q] = (unsigned)(32 * q) * (unsigned)p.Kp + s_off;
#define DKF_FETCH_PART(PI) DKF_FETCH_PART_Q(DKF_PART(PI))
#define DKF_FETCH_PART_Q(Q)                                                                       \
    {                                                                                             \
        const int q_ = (Q);                                                                       \
        const int8_t *a_ = p.Ap + 2 * (q_ & 3) * p.a_plane + (long long)ti * BI * p.Kp;           \
        rsA0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a_), 0, BI * p.Kp, RSRC_FLAGS); \
        rsA1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a_ + p.a_plane), 0, BI * p.Kp, RSRC_FLAGS); \
        bpart = p.Bp + 2 * (q_ >> 2) * p.b_plane;                                                 \
        if (BMODE == 0) {                                                                         \
            const int8_t *b_ = bpart + (long long)tj * BJ * p.Kp;                                 \
            rsB0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(b_), 0, BJ * p.Kp, RSRC_FLAGS); \
            rsB1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(b_ + p.b_plane), 0, BJ * p.Kp, RSRC_FLAGS); \
        } else if (BMODE == 1) {       /* whole planes (below 2^31 bytes): a piece outside the image reads as zero */ \
            rsB0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(bpart), 0, (int)p.b_plane, RSRC_FLAGS); \
            rsB1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(bpart + p.b_plane), 0, (int)p.b_plane, RSRC_FLAGS); \
        }                                                                                         \
    }
    // What a fetch of k tile KTILE needs besides the piece number.
#define DKF_FETCH_PREP(KTILE)                                                                     \
    const int soff_ = (KTILE) * KT;                                                               \
    const int k0_ = (KTILE) * KT + 16 * spiece;                                                   \
    unsigned koff_ = 0;                                                                           \
    bool kok_ = true;                                                                             \
    int fa_ = 0, fb_ = 0;                                                                         \
    const int8_t *bp_ = bpart;                                                                    \
    if (BMODE == 2) {                                                                             \
        const int img_ = k0_ / p.sImgK;                                                           \
        const int rem_ = k0_ - img_ * p.sImgK;                                                    \
        const int oh_ = rem_ / p.cWo;                                                             \
        koff_ = (unsigned)img_ * (unsigned)p.sImgP + (unsigned)(oh_ * p.sWpp + (rem_ - oh_ * p.cWo)); \
        kok_ = k0_ < p.sK;                                                                        \
    } else if (BMODE == 1) {                                                                      \
        const int tap_ = k0_ / p.cp;                                                              \
        fa_ = tap_ / p.ckw;                                                                       \
        fb_ = tap_ - fa_ * p.ckw;                                                                 \
        kok_ = tap_ < p.ckh * p.ckw;                                                              \
        koff_ = (unsigned)(k0_ - tap_ * p.cp);                                                    \
    }
    // Pieces E0 <= e < E1 of A (of NA) and F0 <= e < F1 of B (of 8) into the staging registers.
#define DKF_FETCH_PIECES(E0, E1, F0, F1)                                                          \
    {                                                                                             \
        _Pragma("unroll") for (int e = (E0); e < (E1); ++e)                                       \
            if (e / (2 * NBI) < npa_)                                                             \
                sa[e] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(          \
                    (e / (2 * NBI)) ? rsA1 : rsA0, (int)voff[e % (2 * NBI)], soff_, 0));          \
        _Pragma("unroll") for (int e = (F0); e < (F1); ++e) {                                     \
            const int pl = e >> 2, q = e & 3;                                                     \
            if (pl >= npb_) continue;                                                             \
            if (BMODE == 0) {                                                                     \
                sb[e] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(          \
                    pl ? rsB1 : rsB0, (int)voff[q], soff_, 0));                                   \
            } else if (BMODE == 2) {                                                              \
                /* no branch between the MFMAs: a piece of a row beyond J or of a k beyond the */ \
                /* contraction only has to stay in bounds (those rows are never stored, those */  \
                /* k meet zero columns of A), so it reads the start of the plane */               \
                const unsigned off_ = (kok_ && r_ok[q]) ? r_base[q] + koff_ : 0u;                 \
                sb[e] = *reinterpret_cast<const i32x4_u *>(bp_ + pl * p.b_plane + off_);          \
            } else {                                                                              \
                const int ih_ = r_ih[q] + fa_, iw_ = r_iw[q] + fb_;                               \
                const bool ok_ = kok_ && r_ok[q] && ih_ >= 0 && ih_ < p.cH && iw_ >= 0 && iw_ < p.cW; \
                const unsigned off_ = ok_ ? r_base[q] + (unsigned)(ih_ * p.cW + iw_) * (unsigned)p.cp + koff_ \
                                          : 0x80000000u;                                          \
                sb[e] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(          \
                    pl ? rsB1 : rsB0, (int)off_, 0, 0));                                          \
            }                                                                                     \
        }                                                                                         \
    }
#define DKF_STASH_PIECES(BUF, E0, E1, F0, F1)                                                     \
    {                                                                                             \
        _Pragma("unroll") for (int e = (E0); e < (E1); ++e)                                       \
            if (e / (2 * NBI) < npa_)                                                             \
                *reinterpret_cast<i32x4 *>((BUF) + (e / (2 * NBI)) * A_PLANE + (e % (2 * NBI)) * 32 * PITCH + s_dst) = sa[e]; \
        _Pragma("unroll") for (int e = (F0); e < (F1); ++e)                                       \
            if ((e >> 2) < npb_)                                                                  \
                *reinterpret_cast<i32x4 *>((BUF) + 2 * A_PLANE + (e >> 2) * B_PLANE + (e & 3) * 32 * PITCH + s_dst) = sb[e]; \
    }
    // Quarter U of a tile's pieces: written to LDS from the staging registers, which then
    // take the same pieces of the tile two steps ahead.
#define DKF_TURN(BUF, U)                                                                          \
    DKF_STASH_PIECES(BUF, (U) * NBI, ((U) + 1) * NBI, 2 * (U), 2 * (U) + 2)                       \
    DKF_FETCH_PIECES((U) * NBI, ((U) + 1) * NBI, 2 * (U), 2 * (U) + 2)
    // in the order the MFMAs of a step consume them: A and B planes 0 first
#define DKF_READ(A, B, KS)                                                                        \
    {                                                                                             \
        _Pragma("unroll") for (int bi = 0; bi < NBI; ++bi)                                          \
            A[bi][0] = *reinterpret_cast<const i32x4 *>(cur + a_rd + bi * 32 * PITCH + (KS) * 32); \
        _Pragma("unroll") for (int bj = 0; bj < 2; ++bj)                                          \
            B[bj][0] = *reinterpret_cast<const i32x4 *>(cur + b_rd + bj * 32 * PITCH + (KS) * 32); \
        if (npb_ > 1) {                                                                           \
            _Pragma("unroll") for (int bj = 0; bj < 2; ++bj)                                      \
                B[bj][1] = *reinterpret_cast<const i32x4 *>(cur + B_PLANE + b_rd + bj * 32 * PITCH + (KS) * 32); \
        }                                                                                         \
        if (npa_ > 1) {                                                                           \
            _Pragma("unroll") for (int bi = 0; bi < NBI; ++bi)                                    \
                A[bi][1] = *reinterpret_cast<const i32x4 *>(cur + A_PLANE + a_rd + bi * 32 * PITCH + (KS) * 32); \
        }                                                                                         \
    }
    // digit pairs outermost: four independent accumulators lie between two
    // MFMAs into the same one
#define DKF_MMA(A, B)                                                                             \
    {                                                                                             \
        _Pragma("unroll") for (int pa = 0; pa < npa_; ++pa)                                       \
            _Pragma("unroll") for (int pb = 0; pb < npb_; ++pb)                                   \
                _Pragma("unroll") for (int bi = 0; bi < NBI; ++bi)                                  \
                    _Pragma("unroll") for (int bj = 0; bj < 2; ++bj)                              \
                        acc[bi][bj][pa + pb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(             \
                            A[bi][pa], B[bj][pb], acc[bi][bj][pa + pb], 0, 0, 0);                 \
    }
    // Issue order of a 32-k sub-step: its 8 NBI MFMAs with, one each, the NR LDS reads of the
    // next sub-step's operands, then the NBI + 2 (LDS write, global load) pairs of this
    // quarter of the staging registers.  Spread like this the global loads of the four waves
    // reach the vector-memory path at the rate it takes them; issued in one burst at the end
    // of a step they held the waves (and so the matrix pipes) until it had taken them all.
#define DKF_PACE(NR, U)                                                                           \
    {                                                                                             \
        constexpr int nw_ = ((U) / 2 < npa_ ? NBI : 0) + ((U) / 2 < npb_ ? 2 : 0);                \
        constexpr int nm_ = 2 * npa_ * npb_ * NBI;                                                \
        constexpr int both_ = (NR) + nw_ > nm_ ? (NR) + nw_ - nm_ : 0;                            \
        _Pragma("unroll") for (int e = 0; e < (NR) - both_; ++e) {                                \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                    \
        }                                                                                         \
        _Pragma("unroll") for (int e = 0; e < nw_; ++e) {                                         \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
            if (e < both_) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                     \
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                    \
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                    \
        }                                                                                         \
        if (nm_ - ((NR) - both_) - nw_ > 0)                                                       \
            __builtin_amdgcn_sched_group_barrier(0x008, nm_ - ((NR) - both_) - nw_, 0);           \
        __builtin_amdgcn_sched_barrier(0);                                                        \
    }
    // keep consumed operand registers live up to here, so that a read issued
    // between the MFMAs does not target a register an MFMA in flight still reads
#define DKF_KEEP(A, B)                                                                            \
    {                                                                                             \
        _Pragma("unroll") for (int x = 0; x < 2; ++x)                                             \
            _Pragma("unroll") for (int y = 0; y < 2; ++y) {                                       \
                if (x < NBI && y < npa_) asm volatile("" ::"v"(A[x][y]));                         \
                if (y < npb_) asm volatile("" ::"v"(B[x][y]));                                    \
            }                                                                                     \
    }
    // Four 32-k sub-steps with NPA planes of A and NPB of B.  The operands of sub-step
    // u+1 are read from LDS while the MFMAs of sub-step u issue; each sub-step also moves a
    // quarter of the staging registers (tile s+1) to the other LDS buffer and refills them
    // from tile s+2 (past the last step: part 0 of a valid k tile, never used).  Quarters
    // 0, 1 are the pieces of plane 0 and quarters 2, 3 those of plane 1 of both operands.
#define DKF_STEP(NPA, NPB)                                                                        \
    {                                                                                             \
        constexpr int npa_ = (NPA), npb_ = (NPB), nr_ = npa_ * NBI + npb_ * 2;                    \
        i32x4 a0[NBI][2], b0[2][2], a1[NBI][2], b1[2][2];                                         \
        DKF_READ(a0, b0, 0)                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                        \
        DKF_READ(a1, b1, 1)                                                                       \
        DKF_MMA(a0, b0)                                                                           \
        DKF_TURN(nxt, 0)                                                                          \
        DKF_PACE(nr_, 0)                                                                          \
        DKF_KEEP(a0, b0)                                                                          \
        DKF_READ(a0, b0, 2)                                                                       \
        DKF_MMA(a1, b1)                                                                           \
        DKF_TURN(nxt, 1)                                                                          \
        DKF_PACE(nr_, 1)                                                                          \
        DKF_KEEP(a1, b1)                                                                          \
        DKF_READ(a1, b1, 3)                                                                       \
        DKF_MMA(a0, b0)                                                                           \
        DKF_TURN(nxt, 2)                                                                          \
        DKF_PACE(nr_, 2)                                                                          \
        DKF_KEEP(a0, b0)                                                                          \
        DKF_MMA(a1, b1)                                                                           \
        DKF_TURN(nxt, 3)                                                                          \
        DKF_PACE(0, 3)                                                                            \
    }
    // (part index, k tile) of a step advance like a two-digit counter
#define DKF_ADVANCE(PI, KT)                                                                       \
    {                                                                                             \
        if (KT + 1 == kt1) { KT = kt0; ++PI; } else ++KT;                                         \
    }
    constexpr int npa_ = 2, npb_ = 2;     // planes per operand outside the single-digit steps
    int pi = 0, kt = kt0;                 // part index and k tile of the current step
    int pi2 = 0, kt2 = kt0;               // ... of the step the next fetch is for
    // With one-plane launches alongside, the flags name the launch that does this product
    // (uniform; the workgroups of the others leave before they touch memory).
    if (p.single_mask) {
        const int single = ((p.single_mask & 1) && flag_a == 0) ? 1 : ((p.single_mask & 2) && flag_b == 0) ? 2 : 0;
        if (single != SINGLE) return;
    } else if (SINGLE) {
        return;
    }
    // The first part is (lo,lo) whatever the flags say: its first tile is on its way before
    // the flags (a dependent scalar load) are looked at.
    if (kt1 > kt0) {
        DKF_FETCH_PART_Q(0)
        DKF_FETCH_PREP(kt0)
        DKF_FETCH_PIECES(0, NA, 0, 8)
    }
    const bool three = p.sums && fa && fb;
    int plist = 0, nparts = 0;           // four bits per active part
    if (three) {
        plist = 0x0 | 0xA << 4 | 0x5 << 8;
        nparts = 3;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (!((q & 1) && !fa) && !((q >> 1) && !fb)) plist |= ((q & 1) | (q >> 1) << 2) << (4 * nparts++);
    }
    const int nsteps = nparts * (kt1 - kt0);
    if (nsteps > 0) {
        DKF_STASH_PIECES(flds, 0, NA, 0, 8)
        DKF_ADVANCE(pi2, kt2)
        if (kt2 == kt0) DKF_FETCH_PART(pi2)
        {
            // (a tile beyond the last step is part 0 of a valid k tile: in bounds, never used)
            DKF_FETCH_PREP(kt2)
            DKF_FETCH_PIECES(0, NA, 0, 8)
        }
        DKF_ADVANCE(pi2, kt2)
        if (kt2 == kt0) DKF_FETCH_PART(pi2)
    }
    __syncthreads();

    // Outer loop: weight groups; inner loop: the steps of one group, a plain
    // pipelined MFMA loop that runs on across part and group boundaries, so only
    // the first tile of the workgroup waits for memory.  During step s the
    // staging registers hold tile s+1; quarter by quarter, one per 32-k sub-step,
    // they go to the other LDS buffer and are refilled from tile s+2, so every
    // load has a whole step to arrive.
    int step = 0;
    while (step < nsteps) {
        const int w = DKF_GROUP(DKF_PART(pi));
        const int gparts = (pi + 1 < nparts && DKF_GROUP(DKF_PART(pi + 1)) == w) ? 2 : 1;
        const int g_end = step + gparts * (kt1 - kt0);
        for (; step < g_end; ++step) {
            const int8_t *cur = flds + (step & 1) * BUF_BYTES;
            int8_t *nxt = flds + ((step + 1) & 1) * BUF_BYTES;
            DKF_FETCH_PREP(kt2)
            DKF_STEP(SINGLE == 1 ? 1 : 2, SINGLE == 2 ? 1 : 2)
            __syncthreads();
            DKF_ADVANCE(pi, kt)
            DKF_ADVANCE(pi2, kt2)
            if (kt2 == kt0) DKF_FETCH_PART(pi2)
        }

        // End of a weight group: S = a0 + 2^7 a1 + 2^14 a2 of the three accumulators
        // joins the running sums with the group's weight, which is a signed sum of
        // powers of 2^14 in every case -- 1, 2^14, 2^28 for the four-part form and
        // 1 - 2^14, 2^14, 2^28 - 2^14 for the three-part form -- so shifts, 24-bit
        // multiplies by 39 and additions do it (64-bit products with the weights took
        // three times as long).  Nothing is reduced below p here: a group adds less
        // than 2^27 to a running sum, which the epilogue reduces once.
        // One straight-line copy per weight (uniform switch), a 32 x 32 block at a time.
        auto join = [&](auto weight) {
            constexpr int WEIGHT = decltype(weight)::value;
#pragma unroll
            for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int a0, a1, a2;
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a0) : "a"(acc[bi][bj][0][v]));
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a1) : "a"(acc[bi][bj][1][v]));
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a2) : "a"(acc[bi][bj][2][v]));
                        const uint32_t t = fold_sum3(a0, a1, a2);
                        if (WEIGHT == 0) {                 // 1
                            res[bi][bj][v] += t;
                        } else if (WEIGHT == 1) {          // 1 - 2^14 (2p - u > 0 stands for -u)
                            res[bi][bj][v] += t + (2u * DKF_P - shift14(t));
                        } else if (WEIGHT == 2) {          // 2^14
                            res[bi][bj][v] += shift14(t);
                        } else if (WEIGHT == 3) {          // 2^28 - 2^14
                            const uint32_t u = shift14(t);
                            res[bi][bj][v] += shift14(u) + (2u * DKF_P - u);
                        } else {                           // 2^28
                            res[bi][bj][v] += shift14(shift14(t));
                        }
                        if (v % 4 == 3) __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int c = 0; c < 3; ++c)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[bi][bj][c][v] = 0;
                }
            __builtin_amdgcn_sched_barrier(0);
        };
        switch (three ? (w == 0 ? 1 : w == 1 ? 2 : 3) : 2 * w) {
        case 0: join(std::integral_constant<int, 0>{}); break;
        case 1: join(std::integral_constant<int, 1>{}); break;
        case 2: join(std::integral_constant<int, 2>{}); break;
        case 3: join(std::integral_constant<int, 3>{}); break;
        default: join(std::integral_constant<int, 4>{}); break;
        }
    }
#undef DKF_PART
#undef DKF_GROUP
#undef DKF_ADVANCE
#undef DKF_PACE
#undef DKF_KEEP
#undef DKF_FETCH_PART
#undef DKF_FETCH_PART_Q
#undef DKF_FETCH_PREP
#undef DKF_FETCH_PIECES
#undef DKF_STASH_PIECES
#undef DKF_TURN
#undef DKF_READ
#undef DKF_MMA
#undef DKF_STEP

    uint32_t *dst_q = p.out_q ? p.out_q + (long long)split * p.I * p.J : nullptr;   // (one slice if remapped)
    if (!p.out_hw && ti * BI + BI <= p.I && tj * BJ + BJ <= p.J) {
        // Tile inside a row-major result: no bounds tests, uniform offsets from one lane
        // address, and Round(lift(q) 2^-l) 2^-l in integers -- n = (lift(q) + 2^(l-1)) >> l is
        // the floor of lift(q) 2^-l + 1/2, n 2^-l is exact in fp32, and scale 2^-l is an exact
        // product, so n (scale 2^-l) rounds once, to the value scale (n 2^-l) rounds to.
        const long long o0 = (long long)(ti * BI + wi0 + 4 * lh) * p.J + (tj * BJ + wj0 + li);
        uint32_t *q0 = dst_q ? dst_q + o0 : nullptr;
        float *f0 = p.out_f ? p.out_f + o0 : nullptr;
        const float c = p.scale * (float)p.s_inv;
        const int half = p.lq > 0 ? 1 << (p.lq - 1) : 0;
#pragma unroll
        for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long long orow = (long long)(bi * 32 + 8 * (v / 4) + (v % 4)) * p.J;
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) {
                    const uint32_t r = res[bi][bj][v];                                 // < 2^28
                    const uint32_t u = __umul24(r >> 25, 39u) + (r & 0x1ffffffu);
                    const uint32_t q = u >= DKF_P ? u - DKF_P : u;
                    if (q0) q0[orow + bj * 32] = q;
                    if (f0) {
                        const int lift = q > DKF_P / 2 ? (int)q - (int)DKF_P : (int)q;
                        const float f = (float)((lift + half) >> p.lq) * c;
                        f0[orow + bj * 32] = p.accumulate ? f0[orow + bj * 32] + f : f;
                    }
                }
            }
        return;
    }
    if (p.out_hw && !p.out_f && dst_q && ti * BI + BI <= p.I && tj * BJ + BJ <= p.J) {
        // Tile inside an image-major result (a convolution's forward): a lane's two columns
        // are two (image, pixel) pairs, one address each; rows are uniform multiples of hw.
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int j = tj * BJ + wj0 + bj * 32 + li;
            const int jimg = j / p.out_hw, jpix = j - jimg * p.out_hw;
            uint32_t *q0 = dst_q + ((long long)jimg * p.I + (ti * BI + wi0 + 4 * lh)) * p.out_hw + jpix;
#pragma unroll
            for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t r = res[bi][bj][v];                                 // < 2^28
                    const uint32_t u = __umul24(r >> 25, 39u) + (r & 0x1ffffffu);
                    q0[(long long)(bi * 32 + 8 * (v / 4) + (v % 4)) * p.out_hw] = u >= DKF_P ? u - DKF_P : u;
                }
        }
        return;
    }
#pragma unroll
    for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int j = tj * BJ + wj0 + bj * 32 + li;
            const int jimg = p.out_hw ? j / p.out_hw : 0, jpix = p.out_hw ? j - jimg * p.out_hw : 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = ti * BI + wi0 + bi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (i < p.I && j < p.J) {
                    const long long o = p.out_hw ? ((long long)jimg * p.I + i) * p.out_hw + jpix
                                                 : (long long)i * p.J + j;
                    const uint32_t r = res[bi][bj][v];                                 // < 2^28
                    const uint32_t u = __umul24(r >> 25, 39u) + (r & 0x1ffffffu);
                    const uint32_t q = u >= DKF_P ? u - DKF_P : u;
                    if (dst_q) dst_q[o] = q;
                    if (p.out_f) {
                        const float f = p.scale * dkf_dequant(q, p.s_inv);
                        p.out_f[o] = p.accumulate ? p.out_f[o] + f : f;
                    }
                }
            }
        }
}

// Fold of the k slices: out[e] = sum_k part[k][e] (mod p).  With dW != NULL the sum is de-quantised
// (dW is never remapped: a weight gradient is [I][J] already):
// dW = (accumulate ? dW : 0) + scale * Round(lift(q) * 2^-l) * 2^-l.
__global__ __launch_bounds__(256) void f_fold_kernel(const uint32_t *__restrict__ part,
                                                     uint32_t *__restrict__ out_q, float *__restrict__ dW,
                                                     long long elems, int splits, double s_inv,
                                                     float scale, int accumulate, int I, int J, int out_hw)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= elems) return;
    uint64_t s = 0;
    for (int k = 0; k < splits; ++k) s += part[(long long)k * elems + e];
    const uint32_t q = dkf_reduce(s);
    if (out_q) {
        long long o = e;
        if (out_hw) {                         // slices are [I][J]; the result is image-major
            const int i = (int)(e / J), j = (int)(e - (long long)i * J);
            const int img = j / out_hw;
            o = ((long long)img * I + i) * out_hw + (j - img * out_hw);
        }
        out_q[o] = q;
    }
    if (dW) {
        const float v = scale * dkf_dequant(q, s_inv);
        dW[e] = accumulate ? dW[e] + v : v;
    }
}

// The same for many slices of a small result (a weight gradient of a few thousand
// elements cut into up to 256 slices): with one thread per element the launch is a few
// workgroups that each walk all slices one load after the other.  Here a workgroup takes
// 64 elements and its SG waves every SG-th slice; the SG partial sums (below 2^33 each) meet
// in LDS.  Sums of residues: any order gives the same result.
template <int SG>
__global__ __launch_bounds__(64 * SG) void f_fold_deep_kernel(const uint32_t *__restrict__ part,
                                                              uint32_t *__restrict__ out_q,
                                                              float *__restrict__ dW, long long elems,
                                                              int splits, double s_inv, float scale,
                                                              int accumulate, int I, int J, int out_hw)
{
    __shared__ uint64_t red[SG][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long e = (long long)blockIdx.x * 64 + lane;
    uint64_t s = 0;
    if (e < elems)
        for (int k = wave; k < splits; k += SG) s += part[(long long)k * elems + e];
    red[wave][lane] = s;
    __syncthreads();
    if (wave != 0 || e >= elems) return;
#pragma unroll
    for (int w = 1; w < SG; ++w) s += red[w][lane];
    const uint32_t q = dkf_reduce(s);
    if (out_q) {
        long long o = e;
        if (out_hw) {
            const int i = (int)(e / J), j = (int)(e - (long long)i * J);
            const int img = j / out_hw;
            o = ((long long)img * I + i) * out_hw + (j - img * out_hw);
        }
        out_q[o] = q;
    }
    if (dW) {
        const float v = scale * dkf_dequant(q, s_inv);
        dW[e] = accumulate ? dW[e] + v : v;
    }
}

inline int round_up(int v, int a) { return (v + a - 1) / a * a; }
inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct fgemm_plan {
    int I, J, K, I_pad, J_pad, Kp;
    int tiles_i, tiles_j, ktiles, splits, ktiles_per_split;
    int nbi;              // 1: 64-row tiles, 2: 128-row tiles
    int sums;             // the operands carry the digit-sum planes (six planes each)
    size_t a_bytes, b_bytes, part_bytes;
};

// I, J: output dimensions; K: contraction length; sums: both operands come
// with digit-sum planes (shorter k slices, see the top of the file).
bool plan_fgemm(long long I, long long J, long long K, fgemm_plan *pl, bool sums = false)
{
    const int max_kslice = sums ? MAX_KSPLIT_SUMS : MAX_KSPLIT;
    pl->sums = sums ? 1 : 0;
    // (128 rows of Kp bytes are one buffer resource and a lane's offsets in it are 32-bit: Kp < 2^24)
    if (I < 1 || J < 1 || K < 1 || I > (1 << 24) || J > (1 << 24) || K > (1 << 24) - KT) return false;
    pl->I = (int)I; pl->J = (int)J; pl->K = (int)K;
    pl->nbi = (I % 128 != 0 && I % 128 <= 64) ? 1 : 2;      // a last half-empty 128-row tile: use 64-row tiles
    pl->I_pad = round_up((int)I, 64 * pl->nbi);
    pl->J_pad = round_up((int)J, BJ);
    pl->Kp = round_up((int)K, KT);
    pl->tiles_i = pl->I_pad / (64 * pl->nbi);
    pl->tiles_j = pl->J_pad / BJ;
    pl->ktiles = pl->Kp / KT;
    const long long tiles = (long long)pl->tiles_i * pl->tiles_j;
    if (tiles > (1 << 24)) return false;
    // Number of k slices: at least what the int32 accumulators need, at most
    // MAX_SPLITS, and among those the count that wastes the
    // least of the last round of workgroups on the 256 compute units (one
    // workgroup per unit), with a small charge per extra slice for its fold.
    const long long need = ((long long)pl->Kp + max_kslice - 1) / max_kslice;
    long long splits = need;
    double best = 1e30;
    for (long long sp = need; sp <= MAX_SPLITS && sp <= pl->ktiles; ++sp) {
        const double rounds = (double)(tiles * sp) / 256.0;
        const double cost = (double)((tiles * sp + 255) / 256) / rounds * (1.0 + 0.02 * (double)(sp - 1));
        if (cost < best - 1e-9) { best = cost; splits = sp; }
        if (tiles * sp >= 256 * 8) break;          // many rounds: the tail no longer matters
    }
    if (splits > pl->ktiles) splits = pl->ktiles;
    if (splits < 1) splits = 1;
    int per = (int)((pl->ktiles + splits - 1) / splits);
    if ((long long)per * KT > max_kslice) return false;
    pl->ktiles_per_split = per;
    pl->splits = (pl->ktiles + per - 1) / per;
    const size_t nplanes = sums ? 6 : 4;
    pl->a_bytes = align256(nplanes * pl->I_pad * pl->Kp);
    pl->b_bytes = align256(nplanes * pl->J_pad * pl->Kp);
    pl->part_bytes = pl->splits > 1
        ? align256((size_t)pl->splits * (size_t)I * (size_t)J * sizeof(uint32_t)) : 0;
    return true;
}

constexpr size_t FLAG_BYTES = 256;

// Shifted-rows form of the B operand of a stride-1 convolution's weight
// gradient (f_digits_rows_kernel): sizes the GEMM needs to address it.
struct fshift {
    int Ci, kh, kw, Ho, Hp, Wp, Wpp;
    int row_bytes;          // R * Hp * Wpp
    int img_k, img_p, K;    // Ho * Wp, Hp * Wpp, R * Ho * Wp
    long long plane;        // bytes per digit plane: Ci * row_bytes
};

// C = A B^T over the field from digit planes.  out_q / out_f as in the kernel
// parameters; with more than one k slice the slices go to `part` and a fold
// kernel finishes.
dk_status run_fgemm(const fgemm_plan &pl, const int8_t *Ap, const int8_t *Bp, uint32_t *part,
                    const int *flags, uint32_t *out_q, float *out_f, int l, float scale,
                    int accumulate, int out_hw, const char *label, hipStream_t st,
                    const fconv_geom *impl = nullptr, long long impl_plane = 0,
                    const fshift *shift = nullptr, int single_mask = 0)
{
    using kernel_t = void (*)(fgemm_params);
    // [operand form][NBI - 1][SINGLE]; a null entry is a variant no caller asks for
    static const kernel_t kernels[3][2][3] = {
        {{f_gemm_kernel<0, 1, 0>, f_gemm_kernel<0, 1, 1>, f_gemm_kernel<0, 1, 2>},
         {f_gemm_kernel<0, 2, 0>, f_gemm_kernel<0, 2, 1>, f_gemm_kernel<0, 2, 2>}},
        {{f_gemm_kernel<1, 1, 0>, f_gemm_kernel<1, 1, 1>, nullptr},
         {f_gemm_kernel<1, 2, 0>, f_gemm_kernel<1, 2, 1>, nullptr}},
        {{f_gemm_kernel<2, 1, 0>, nullptr, nullptr}, {f_gemm_kernel<2, 2, 0>, nullptr, nullptr}}};
    static std::atomic<unsigned long long> allowed[3][2][3];
    const int form = shift ? 2 : impl ? 1 : 0, nb = pl.nbi == 1 ? 0 : 1;
    for (int sg = 0; sg < 3; ++sg) {
        if (sg && !(single_mask >> (sg - 1) & 1)) continue;
        DK_REQUIRE(kernels[form][nb][sg] != nullptr, DK_ERR_UNSUPPORTED);
        const dk_status as = dk_allow_dynamic_lds(reinterpret_cast<const void *>(kernels[form][nb][sg]),
                                                  LDS_BYTES, allowed[form][nb][sg]);
        if (as != DK_OK) return as;
    }
    const bool direct = pl.splits == 1;
    fgemm_params p;
    p.Ap = Ap; p.Bp = Bp; p.flags = flags;
    p.out_q = direct ? out_q : part;
    p.out_f = direct ? out_f : nullptr;
    p.a_plane = (long long)pl.I_pad * pl.Kp;
    p.b_plane = (long long)pl.J_pad * pl.Kp;
    p.I = pl.I; p.J = pl.J; p.Kp = pl.Kp;
    p.tiles_i = pl.tiles_i; p.tiles_j = pl.tiles_j; p.splits = pl.splits;
    p.ktiles_per_split = pl.ktiles_per_split; p.ktiles = pl.ktiles;
    p.s_inv = ldexp(1.0, -l); p.lq = l; p.scale = scale; p.accumulate = accumulate;
    p.sums = pl.sums;
    p.single_mask = single_mask;
    p.out_hw = direct ? out_hw : 0;
    p.cp = p.cH = p.cW = p.ckh = p.ckw = p.cstride = p.cpad = p.cWo = p.cHoWo = 0;
    if (impl) {
        p.cp = impl->Ci; p.cH = impl->H; p.cW = impl->W; p.ckh = impl->kh; p.ckw = impl->kw;
        p.cstride = impl->stride; p.cpad = impl->pad; p.cWo = impl->Wo; p.cHoWo = impl->HoWo;
        p.b_plane = impl_plane;
    }
    p.sRow = p.sImgK = p.sImgP = p.sWpp = p.sK = 0;
    if (shift) {
        p.cp = shift->Ci; p.ckh = shift->kh; p.ckw = shift->kw; p.cWo = shift->Wp;
        p.sRow = shift->row_bytes; p.sImgK = shift->img_k; p.sImgP = shift->img_p; p.sWpp = shift->Wpp;
        p.sK = shift->K;
        p.b_plane = shift->plane;
    }
    const long long blocks = (long long)pl.splits * pl.tiles_i * pl.tiles_j;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    {
        dk_prof_scope ps(label, st);
        const dim3 grid((unsigned)blocks), block(256);
        for (int sg = 0; sg < 3; ++sg)
            if (!sg || (single_mask >> (sg - 1) & 1)) kernels[form][nb][sg]<<<grid, block, LDS_BYTES, st>>>(p);
    }
    if (direct) return dk_launch_status();
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    const long long elems = (long long)pl.I * pl.J;
    dk_prof_scope ps("f_fold", st);
    if (pl.splits >= 16 && elems <= 256 * 1024)
        f_fold_deep_kernel<16><<<dim3((unsigned)((elems + 63) / 64)), dim3(1024), 0, st>>>(
            part, out_q, out_f, elems, pl.splits, p.s_inv, scale, accumulate, pl.I, pl.J, out_hw);
    else
        f_fold_kernel<<<dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st>>>(
            part, out_q, out_f, elems, pl.splits, p.s_inv, scale, accumulate, pl.I, pl.J, out_hw);
    return dk_launch_status();
}

dk_status run_digits(const uint32_t *src, int8_t *planes, int rows, int K, int rows_pad, int Kp,
                     int *flag, hipStream_t st)
{
    const int chunks = (Kp + 4095) / 4096;          // Kp is a multiple of 128
    const long long blocks = (long long)rows_pad * chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const int vec = (K % 4 == 0) && dk_aligned(src, 16);
    dk_prof_scope ps("f_digits", st);
    f_digits_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(src, planes, rows, K, rows_pad, Kp,
                                                                         chunks, vec, 1.0, flag);
    return dk_launch_status();
}

// ... of real values, quantised with l fractional bits on the way
dk_status run_digits_f32(const float *src, int l, int8_t *planes, int rows, int K, int rows_pad, int Kp,
                         int *flag, hipStream_t st)
{
    const int chunks = (Kp + 4095) / 4096;
    const long long blocks = (long long)rows_pad * chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const int vec = (K % 4 == 0) && dk_aligned(src, 16);
    dk_prof_scope ps("f_digits_quantize", st);
    f_digits_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(src, planes, rows, K, rows_pad, Kp,
                                                                        chunks, vec, ldexp(1.0, l), flag);
    return dk_launch_status();
}

dk_status run_digits_t(const uint32_t *src, int8_t *planes, int K, int cols, int cols_pad, int Kp,
                       int sums, int *flag, hipStream_t st)
{
    DK_REQUIRE(Kp / 128 <= 65535, DK_ERR_SHAPE);
    dk_prof_scope ps("f_digits_t", st);
    f_digits_t_kernel<false><<<dim3(cols_pad / 64, Kp / 128), dim3(256), 0, st>>>(src, planes, fconv_geom{},
                                                                                K, cols, cols_pad, Kp, sums, flag);
    return dk_launch_status();
}

// The gradient mixing of the backward pass written straight into the digit planes of a
// convolution's weight-gradient operand A (rows = output channels, k = (encoded row,
// output row, column of pitch Wp); Wp = Wo, or Wo rounded up to 16 for the padded-rows
// form, whose columns beyond Wo are written as zeros here):
//     dtilde[gS+j] = gamma[g][j] * (sum_i B[g][j][i] * Dq[gK+i])  (mod p),  Dq = Field(Round(delta 2^l)),
// so the mixed gradients never exist as a tensor (a write and a read of 4 bytes per element
// less).  One thread: four consecutive pixels of one channel of one virtual batch, its K
// gradient values quantised once and mixed into all S = K + 2 encoded rows; per row one
// 4-byte word to each plane.  Needs Ho*Wo % 4 == 0 (Wo % 4 == 0 when Wp > Wo: a group of
// four then stays in its row) and a 16-byte aligned delta.  Rows beyond Co and k beyond
// the contraction are zeroed by f_pad_planes_kernel.
template <int K>
__global__ __launch_bounds__(256) void f_delta_mix_digits_kernel(
    const float *__restrict__ delta, const float *__restrict__ xscale, const uint32_t *__restrict__ B,
    const uint32_t *__restrict__ gamma, int8_t *__restrict__ planes, int Ho, int Wo, int Wp, long long len,
    long long nvec, int chunks, long long span, double s, int Kp, long long plane, int sums, int *flag)
{
    const int HoWo = Ho * Wo, img_k = Ho * Wp;
    constexpr int S = K + 2;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;
    const uint32_t *Bg = B + (long long)g * S * K;
    const uint32_t *gg = gamma + (long long)g * S;
    const float *src = delta + (long long)g * K * len;
    double si[K];
#pragma unroll
    for (int i = 0; i < K; ++i) si[i] = xscale ? s * (1.0 / (double)xscale[(long long)g * K + i]) : s;
    uint32_t hi = 0, mid = 0;
    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += 256) {
        const unsigned e = (unsigned)(v * 4);                    // len < 2^31
        const unsigned co = e / (unsigned)HoWo, px = e - co * (unsigned)HoWo;
        uint32_t q[K][4];
#pragma unroll
        for (int i = 0; i < K; ++i) {
            const float4 f = *reinterpret_cast<const float4 *>(src + (long long)i * len + e);
            q[i][0] = dkf_quant(f.x, si[i]); q[i][1] = dkf_quant(f.y, si[i]);
            q[i][2] = dkf_quant(f.z, si[i]); q[i][3] = dkf_quant(f.w, si[i]);
        }
        const unsigned h = px / (unsigned)Wo, w = px - h * (unsigned)Wo;
        int8_t *row = planes + (long long)co * Kp + (long long)g * S * img_k + h * Wp + w;
        const int gutter = (Wp > Wo && (int)w + 4 == Wo) ? (Wp - Wo) / 4 : 0;     // zero words after this group
#pragma unroll
        for (int j = 0; j < S; ++j) {
            uint64_t acc[4] = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < K; ++i) {
                const uint32_t b = Bg[j * K + i];
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] += (uint64_t)b * q[i][c];
            }
            const uint32_t gj = gg[j];
            uint32_t d[4], ds[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                d[c] = digits_of(dkf_reduce((uint64_t)gj * dkf_reduce(acc[c])));
                ds[c] = half_sums(d[c]);
            }
            int8_t *dst = row + (long long)j * img_k;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const uint32_t word = gather_byte(d, a);
                if (a >= 2) hi |= word;
                if (a == 1) mid |= word;
                *reinterpret_cast<uint32_t *>(dst + a * plane) = word;
            }
            if (sums) {
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    *reinterpret_cast<uint32_t *>(dst + (4 + a) * plane) = gather_byte(ds, a);
            }
            for (int z = 1; z <= gutter; ++z)
                for (int a = 0; a < (sums ? 6 : 4); ++a)
                    *reinterpret_cast<uint32_t *>(dst + a * plane + 4 * z) = 0u;
        }
    }
    raise_flag(flag, hi, mid);
}

// Zero words of digit planes [nplanes][rows_pad][Kp] outside an operand of `rows` rows and
// K (a multiple of 4) contraction indices: k in [K, Kp) of the rows, everything of the rows
// beyond them.  One thread per word.
__global__ __launch_bounds__(256) void f_pad_planes_kernel(int8_t *__restrict__ planes, long long plane,
                                                           int rows, int rows_pad, int K, int Kp,
                                                           long long per_plane, long long total)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long pln = idx / per_plane;
    long long rem = idx - pln * per_plane;
    const long long tw = (Kp - K) / 4, tail = (long long)rows * tw;
    long long at;
    if (rem < tail) {
        const long long r = rem / tw;
        at = r * Kp + K + 4 * (rem - r * tw);
    } else {
        rem -= tail;
        const long long r = rem / (Kp / 4);
        at = (rows + r) * Kp + 4 * (rem - r * (Kp / 4));
    }
    *reinterpret_cast<uint32_t *>(planes + pln * plane + at) = 0u;
}

template <int MODE>
dk_status run_digits_conv(const uint32_t *src, int8_t *planes, const fconv_geom &cg, int rows, int K,
                          int rows_pad, int Kp, int sums, int *flag, hipStream_t st)
{
    const int chunks = (Kp + 4095) / 4096;
    const long long blocks = (long long)rows_pad * chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps(MODE == 1 ? "f_digits_dt" : "f_digits_im2col_t", st);
    f_digits_conv_kernel<MODE><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(src, planes, cg, rows, K,
                                                                             rows_pad, Kp, chunks, sums, flag);
    return dk_launch_status();
}

template <int K>
dk_status launch_mix_digits(const float *delta, const float *xscale, const uint32_t *B, const uint32_t *gamma,
                            int8_t *planes, int G, int Ho, int Wo, int Wp, long long len, int l, int Kp,
                            long long plane, int sums, int *flag, hipStream_t st)
{
    // each lane moves `iters` vectors of four; spans shrink until the launch has a few thousand workgroups
    const long long nvec = len / 4;
    long long iters = 4;
    while (iters > 1 && (long long)G * ((nvec + 256 * iters - 1) / (256 * iters)) < 4096) iters >>= 1;
    const long long span = 256 * iters;
    const int chunks = (int)((nvec + span - 1) / span);
    const long long blocks = (long long)G * chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("f_delta_mix_digits", st);
    f_delta_mix_digits_kernel<K><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
        delta, xscale, B, gamma, planes, Ho, Wo, Wp, len, nvec, chunks, span, ldexp(1.0, l), Kp, plane, sums, flag);
    return dk_launch_status();
}

// The A planes of a convolution's weight gradient from the un-mixed gradients (see the kernel).
dk_status run_mix_digits(const float *delta, const float *xscale, const uint32_t *B, const uint32_t *gamma,
                         int8_t *planes, int G, int K, int Co, int Ho, int Wo, int Wp, int l, int rows_pad,
                         int Kc, int Kp, int sums, int *flag, hipStream_t st)
{
    const long long plane = (long long)rows_pad * Kp;
    const int nplanes = sums ? 6 : 4;
    const long long per_plane = (long long)Co * ((Kp - Kc) / 4) + (long long)(rows_pad - Co) * (Kp / 4);
    if (per_plane > 0) {
        const long long total = per_plane * nplanes;
        DK_REQUIRE((total + 255) / 256 <= 0x7fffffffll, DK_ERR_SHAPE);
        dk_prof_scope ps("f_pad_planes", st);
        f_pad_planes_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
            planes, plane, Co, rows_pad, Kc, Kp, per_plane, total);
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    }
    const long long len = (long long)Co * Ho * Wo;
#define DKF_MD(KK) launch_mix_digits<KK>(delta, xscale, B, gamma, planes, G, Ho, Wo, Wp, len, l, Kp, plane, sums, flag, st)
    switch (K) {
    case 1: return DKF_MD(1);   case 2: return DKF_MD(2);   case 3: return DKF_MD(3);   case 4: return DKF_MD(4);
    case 5: return DKF_MD(5);   case 6: return DKF_MD(6);   case 7: return DKF_MD(7);   case 8: return DKF_MD(8);
    case 9: return DKF_MD(9);   case 10: return DKF_MD(10); case 11: return DKF_MD(11); case 12: return DKF_MD(12);
    case 13: return DKF_MD(13); case 14: return DKF_MD(14); case 15: return DKF_MD(15); case 16: return DKF_MD(16);
    default: return DK_ERR_SHAPE;
    }
#undef DKF_MD
}

template <bool SHIFTED>
dk_status run_digits_rows(const uint32_t *src, int8_t *planes, const fconv_geom &cg, int rows, int rows_pad,
                          int Hk, int Wp, int len, int pitch, int sums, int *flag, hipStream_t st)
{
    const int chunks = (pitch + 4095) / 4096;              // a workgroup covers 4096 k; pitch is a multiple of 16
    const long long blocks = (long long)rows_pad * chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const int vec = !SHIFTED && cg.Wo % 4 == 0 && dk_aligned(src, 16);
    dk_prof_scope ps(SHIFTED ? "f_digits_shifted" : "f_digits_dt", st);
    f_digits_rows_kernel<SHIFTED><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
        src, planes, cg, rows, rows_pad, Hk, Wp, len, pitch, chunks, sums, vec, flag);
    return dk_launch_status();
}

fconv_geom conv_geom_of(const dk_geom &g)
{
    fconv_geom c;
    c.Ci = g.Ci; c.Co = g.Co; c.H = g.H; c.W = g.W; c.kh = g.kh; c.kw = g.kw;
    c.stride = g.stride; c.pad = g.pad; c.Ho = g.Ho; c.Wo = g.Wo; c.HoWo = g.Ho * g.Wo;
    return c;
}

// Convolution forward as C[co][(r, pixel)] = W[co][(ci,a,b)] . patches: I = Co,
// J = R*Ho*Wo, K = Ci*kh*kw.  Weight gradient as C[co][(ci,a,b)] over
// k = (r, pixel): I = Co, J = Ci*kh*kw, K = R*Ho*Wo.
// Channel counts that are multiples of 16 take the implicit operand (16-byte
// pieces of the contraction never straddle two filter taps; offsets fit 32 bits).
bool conv_implicit(const dk_geom &g, long long R)
{
    return g.Ci % 16 == 0 && R * g.H * g.W * g.Ci < (1ll << 31);
}

bool plan_conv_fwd(const dk_geom &g, long long R, fgemm_plan *pl)
{
    if (!plan_fgemm(g.Co, R * g.Ho * g.Wo, g.Kg, pl)) return false;
    if (conv_implicit(g, R))        // the B operand is the channels-last planes, not a patch matrix
        pl->b_bytes = align256((size_t)4 * R * g.H * g.W * g.Ci);
    return true;
}
// The padded-rows form: stride 1, more than one tap, and an output width
// that rounding up to 16 lengthens by at most a seventh (56 -> 64).  The planes'
// rows are Wpp >= Wp + kw - 1 bytes, so a 16-byte piece read b bytes on stays
// inside its row.
bool conv_wgrad_shifted(const dk_geom &g, long long R, fshift *sh)
{
    if (g.stride != 1 || g.kh * g.kw == 1) return false;
    const int Wp = round_up(g.Wo, 16);
    if (Wp * 7 > g.Wo * 8) return false;
    const int Hp = g.Ho + g.kh - 1, Wpp = round_up(Wp + g.kw - 1, 4);
    const long long row = R * Hp * Wpp, plane = (long long)g.Ci * row;
    if (plane * 6 >= (1ll << 31) || R * g.Ho * Wp > (1 << 26)) return false;
    if (sh) {
        sh->Ci = g.Ci; sh->kh = g.kh; sh->kw = g.kw; sh->Ho = g.Ho; sh->Hp = Hp; sh->Wp = Wp; sh->Wpp = Wpp;
        sh->row_bytes = (int)row; sh->img_k = g.Ho * Wp; sh->img_p = Hp * Wpp;
        sh->K = (int)(R * g.Ho * Wp);
        sh->plane = plane;
    }
    return true;
}

bool plan_conv_wgrad(const dk_geom &g, long long R, fgemm_plan *pl)
{
    fshift sh;
    if (conv_wgrad_shifted(g, R, &sh)) {
        // one padded copy instead of kh * kw shifted ones: the digit-sum planes pay here too
        if (!plan_fgemm(g.Co, g.Kg, sh.K, pl, true)) return false;
        pl->b_bytes = align256((size_t)6 * sh.plane);
        return true;
    }
    // digit-sum planes only for 1x1 filters: otherwise every shifted copy of the
    // encodings would grow by half, which costs more than the shorter product saves
    return plan_fgemm(g.Co, g.Kg, R * g.Ho * g.Wo, pl, g.kh * g.kw == 1);
}

} // namespace

DK_EXPORT size_t dkf_conv_fwd_workspace_bytes(const dk_layer *L, int R)
{
    dk_geom g;
    if (dk_layer_geom(L, &g) != DK_OK || !g.conv || R < 1) return 0;
    if (g.dw) return 256;               // the depthwise kernel needs none
    fgemm_plan pl;
    if (!plan_conv_fwd(g, R, &pl)) return 0;
    return FLAG_BYTES + pl.a_bytes + pl.b_bytes + pl.part_bytes;
}

DK_EXPORT dk_status dkf_conv_fwd(const dk_layer *L, const uint32_t *Wq, const uint32_t *xbar,
                                 uint32_t *ybar, int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && Wq && xbar && ybar, DK_ERR_NULL);
    dk_geom g;
    const dk_status gs = dk_layer_geom(L, &g);
    if (gs != DK_OK) return gs;
    DK_REQUIRE(g.conv, DK_ERR_UNSUPPORTED);
    DK_REQUIRE(R >= 1, DK_ERR_SHAPE);
    if (g.dw) {
        DK_REQUIRE(dk_aligned(Wq, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
        return dkf_dw_fwd_run(g, Wq, xbar, ybar, R, (hipStream_t)stream);
    }
    fgemm_plan pl;
    DK_REQUIRE(plan_conv_fwd(g, R, &pl), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(Wq, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= FLAG_BYTES + pl.a_bytes + pl.b_bytes + pl.part_bytes, DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;

    char *w = (char *)ws;
    int *flag = (int *)w;                          w += FLAG_BYTES;
    int8_t *Ap = (int8_t *)w;                      w += pl.a_bytes;
    int8_t *Bp = (int8_t *)w;                      w += pl.b_bytes;
    uint32_t *part = (uint32_t *)w;
    // The one-plane steps for filters that fit one digit (A holds the filters) pay where
    // the matrix pipe bounds the product; with at most 64 output channels the gathered
    // operand does, with a short contraction the workgroups' fixed costs do, and the second
    // launch would only cost its start-up (13 us for 3 900 workgroups).
    const int filters_single = (pl.nbi == 2 && g.Kg >= 512) ? 1 : 0;

    {
        dk_prof_scope ps("f_flag_clear", st);
        f_flag_clear_kernel<<<dim3(1), dim3(64), 0, st>>>(flag);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    if (conv_implicit(g, R)) {
        const int taps = g.kh * g.kw, HW = g.H * g.W;
        const int chunks = (pl.Kp / 4 + 255) / 256;
        {
            dk_prof_scope ps("f_digits_w", st);
            if (taps > 1 && (long long)g.Ci * taps <= 12288)
                f_digits_wconv_lds_kernel<<<dim3((unsigned)pl.I_pad), dim3(256),
                                            (size_t)g.Ci * taps * sizeof(uint32_t), st>>>(
                    Wq, Ap, g.Co, g.Ci, taps, g.Ci, pl.I_pad, pl.Kp, flag);
            else
                f_digits_wconv_kernel<<<dim3((unsigned)(pl.I_pad * chunks)), dim3(256), 0, st>>>(
                    Wq, Ap, g.Co, g.Ci, taps, g.Ci, pl.I_pad, pl.Kp, chunks, flag);
        }
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        const long long plane = (long long)R * HW * g.Ci;
        DK_REQUIRE(R <= 65535 && (g.Ci + 127) / 128 <= 65535, DK_ERR_SHAPE);
        {
            dk_prof_scope ps("f_digits_nhwc", st);
            const int vec = (HW % 4 == 0) && dk_aligned(xbar, 16);
            if (g.Ci <= 64)
                f_digits_nhwc_kernel<64><<<dim3((HW + 127) / 128, 1, R), dim3(256), 0, st>>>(
                    xbar, Bp, g.Ci, HW, g.Ci, plane, vec, flag + 1);
            else
                f_digits_nhwc_kernel<128><<<dim3((HW + 63) / 64, (g.Ci + 127) / 128, R), dim3(256), 0, st>>>(
                    xbar, Bp, g.Ci, HW, g.Ci, plane, vec, flag + 1);
        }
        DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
        const fconv_geom cg = conv_geom_of(g);
        return run_fgemm(pl, Ap, Bp, part, flag, ybar, nullptr, 0, 1.0f, 0, g.Ho * g.Wo, "f_gemm_fwd", st,
                         &cg, plane, nullptr, filters_single);
    }
    dk_status s = run_digits(Wq, Ap, g.Co, (int)g.Kg, pl.I_pad, pl.Kp, flag, st);
    if (s != DK_OK) return s;
    {
        DK_REQUIRE(pl.Kp / 128 <= 65535, DK_ERR_SHAPE);
        dk_prof_scope ps("f_digits_im2col", st);
        f_digits_t_kernel<true><<<dim3(pl.J_pad / 64, pl.Kp / 128), dim3(256), 0, st>>>(
            xbar, Bp, conv_geom_of(g), (int)g.Kg, pl.J, pl.J_pad, pl.Kp, 0, flag + 1);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    return run_fgemm(pl, Ap, Bp, part, flag, ybar, nullptr, 0, 1.0f, 0, g.Ho * g.Wo, "f_gemm_fwd", st,
                     nullptr, 0, nullptr, filters_single);
}

DK_EXPORT size_t dkf_fwd_workspace_bytes(int M, int N, int R)
{
    fgemm_plan pl;
    if (!plan_fgemm(R, M, N, &pl)) return 0;
    return FLAG_BYTES + pl.a_bytes + pl.b_bytes + pl.part_bytes;
}

DK_EXPORT size_t dkf_wgrad_workspace_bytes_m(const dk_layer *L, int G, int K, int M)
{
    dk_geom g;
    if (dk_layer_geom(L, &g) != DK_OK) return 0;
    if (G < 1 || K < 1 || M < 1 || K + M - 1 > DK_MAX_K) return 0;
    const long long R = (long long)G * (K + M + 1);
    if (g.dw) return FLAG_BYTES + align256((size_t)R * g.m * sizeof(uint32_t)) + dkf_dw_wgrad_part_bytes(g, R);
    fgemm_plan pl;
    if (!(g.conv ? plan_conv_wgrad(g, R, &pl) : plan_fgemm(g.M, g.N, R, &pl, true))) return 0;
    return FLAG_BYTES + align256((size_t)R * g.m * sizeof(uint32_t)) + pl.a_bytes + pl.b_bytes + pl.part_bytes;
}

DK_EXPORT size_t dkf_wgrad_workspace_bytes(const dk_layer *L, int G, int K)
{
    return dkf_wgrad_workspace_bytes_m(L, G, K, 1);
}

namespace {

// Wq or W (real values, quantised with l fractional bits inside the digit kernel)
dk_status linear_fwd_impl(const uint32_t *Wq, const float *W, int l, const uint32_t *xbar, uint32_t *ybar,
                          int M, int N, int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE((Wq || W) && xbar && ybar, DK_ERR_NULL);
    DK_REQUIRE(M >= 1 && N >= 1 && R >= 1 && l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    fgemm_plan pl;
    DK_REQUIRE(plan_fgemm(R, M, N, &pl), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(Wq, 4) && dk_aligned(W, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= FLAG_BYTES + pl.a_bytes + pl.b_bytes + pl.part_bytes, DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;

    char *w = (char *)ws;
    int *flag = (int *)w;                          w += FLAG_BYTES;
    int8_t *Ap = (int8_t *)w;                      w += pl.a_bytes;
    int8_t *Bp = (int8_t *)w;                      w += pl.b_bytes;
    uint32_t *part = (uint32_t *)w;

    {
        dk_prof_scope ps("f_flag_clear", st);
        f_flag_clear_kernel<<<dim3(1), dim3(64), 0, st>>>(flag);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    dk_status s = run_digits(xbar, Ap, R, N, pl.I_pad, pl.Kp, flag, st);
    if (s != DK_OK) return s;
    s = Wq ? run_digits(Wq, Bp, M, N, pl.J_pad, pl.Kp, flag + 1, st)
           : run_digits_f32(W, l, Bp, M, N, pl.J_pad, pl.Kp, flag + 1, st);
    if (s != DK_OK) return s;
    return run_fgemm(pl, Ap, Bp, part, flag, ybar, nullptr, 0, 1.0f, 0, 0, "f_gemm_fwd", st,
                     nullptr, 0, nullptr, /*single_mask (B holds the weights)*/ 2);
}

} // namespace

DK_EXPORT dk_status dkf_linear_fwd(const uint32_t *Wq, const uint32_t *xbar, uint32_t *ybar,
                                   int M, int N, int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(Wq, DK_ERR_NULL);
    return linear_fwd_impl(Wq, nullptr, 0, xbar, ybar, M, N, R, ws, ws_bytes, stream);
}

DK_EXPORT dk_status dkf_linear_fwd_w(const float *W, int l, const uint32_t *xbar, uint32_t *ybar,
                                     int M, int N, int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(W, DK_ERR_NULL);
    return linear_fwd_impl(nullptr, W, l, xbar, ybar, M, N, R, ws, ws_bytes, stream);
}

namespace {

dk_status wgrad_impl(const dk_layer *L, const float *delta, const float *xscale, const uint32_t *B,
                     const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                     int G, int K, int Mn, int l, float scale, int accumulate,
                     void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && delta && B && gamma && xbar && dW, DK_ERR_NULL);
    dk_geom g;
    const dk_status gs = dk_layer_geom(L, &g);
    if (gs != DK_OK) return gs;
    DK_REQUIRE(G >= 1 && K >= 1 && Mn >= 1 && K + Mn - 1 <= DK_MAX_K && l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    const long long R = (long long)G * (K + Mn + 1);
    if (g.dw) {
        DK_REQUIRE(R < (1ll << 31), DK_ERR_SHAPE);
        DK_REQUIRE(dk_aligned(delta, 4) && dk_aligned(B, 4) && dk_aligned(gamma, 4) && dk_aligned(xbar, 4) &&
                       dk_aligned(dW, 4) && (!dwq || dk_aligned(dwq, 4)), DK_ERR_ALIGN);
        const size_t dtb = align256((size_t)R * g.m * sizeof(uint32_t));
        DK_REQUIRE(ws && ws_bytes >= FLAG_BYTES + dtb + dkf_dw_wgrad_part_bytes(g, R), DK_ERR_WORKSPACE);
        DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
        uint32_t *dt = (uint32_t *)((char *)ws + FLAG_BYTES);
        uint32_t *pt = (uint32_t *)((char *)ws + FLAG_BYTES + dtb);
        const dk_status ms = dkf_delta_mix(delta, xscale, B, gamma, dt, G, K, Mn, g.m, l, (hipStream_t)stream);
        if (ms != DK_OK) return ms;
        return dkf_dw_wgrad_run(g, dt, xbar, dW, dwq, R, l, scale, accumulate, pt, (hipStream_t)stream);
    }
    fgemm_plan pl;
    DK_REQUIRE(g.conv ? plan_conv_wgrad(g, R, &pl) : plan_fgemm(g.M, g.N, R, &pl, true), DK_ERR_SHAPE);
    DK_REQUIRE(g.conv || pl.Kp / 128 <= 65535, DK_ERR_SHAPE);   // grid.y of the transposing digit kernel
    DK_REQUIRE(dk_aligned(delta, 4) && dk_aligned(B, 4) && dk_aligned(gamma, 4) && dk_aligned(xbar, 4) &&
                   dk_aligned(dW, 4) && (!dwq || dk_aligned(dwq, 4)), DK_ERR_ALIGN);
    const size_t dt_bytes = align256((size_t)R * g.m * sizeof(uint32_t));
    DK_REQUIRE(ws && ws_bytes >= FLAG_BYTES + dt_bytes + pl.a_bytes + pl.b_bytes + pl.part_bytes, DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;

    char *w = (char *)ws;
    int *flag = (int *)w;                          w += FLAG_BYTES;
    uint32_t *dtilde = (uint32_t *)w;              w += dt_bytes;
    int8_t *Ap = (int8_t *)w;                      w += pl.a_bytes;
    int8_t *Bp = (int8_t *)w;                      w += pl.b_bytes;
    uint32_t *part = (uint32_t *)w;

    fshift sh;
    const bool shifted = g.conv && conv_wgrad_shifted(g, R, &sh);
    // whole groups of four pixels (inside a row where the rows are padded): the mixing kernel
    // writes the A planes itself
    const bool mix_to_planes = g.conv && Mn == 1 && (shifted ? g.Wo % 4 == 0 : (g.Ho * g.Wo) % 4 == 0) &&
                               dk_aligned(delta, 16) && g.m < (1ll << 31) - 4;
    dk_status s = DK_OK;
    if (!mix_to_planes) {
        s = dkf_delta_mix(delta, xscale, B, gamma, dtilde, G, K, Mn, g.m, l, st);
        if (s != DK_OK) return s;
    }
    {
        dk_prof_scope ps("f_flag_clear", st);
        f_flag_clear_kernel<<<dim3(1), dim3(64), 0, st>>>(flag);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    if (shifted) {
        // the contraction index is (encoded row, output row, column of pitch Wp)
        const fconv_geom cg = conv_geom_of(g);
        s = mix_to_planes ? run_mix_digits(delta, xscale, B, gamma, Ap, G, K, g.Co, g.Ho, g.Wo, sh.Wp, l, pl.I_pad,
                                           sh.K, pl.Kp, pl.sums, flag, st)
                          : run_digits_rows<false>(dtilde, Ap, cg, g.Co, pl.I_pad, sh.Ho, sh.Wp, sh.K, pl.Kp, pl.sums,
                                                   flag, st);
        if (s != DK_OK) return s;
        s = run_digits_rows<true>(xbar, Bp, cg, g.Ci, g.Ci, sh.Hp, sh.Wpp, sh.row_bytes, sh.row_bytes, pl.sums,
                                  flag + 1, st);
        if (s != DK_OK) return s;
        return run_fgemm(pl, Ap, Bp, part, flag, dwq, dW, l, scale, accumulate, 0, "f_gemm_wgrad", st,
                         nullptr, 0, &sh);
    }
    if (g.conv) {
        // the contraction index is (encoded row, output pixel)
        const fconv_geom cg = conv_geom_of(g);
        s = mix_to_planes ? run_mix_digits(delta, xscale, B, gamma, Ap, G, K, g.Co, g.Ho, g.Wo, g.Wo, l, pl.I_pad,
                                           pl.K, pl.Kp, pl.sums, flag, st)
                          : run_digits_conv<1>(dtilde, Ap, cg, g.Co, pl.K, pl.I_pad, pl.Kp, pl.sums, flag, st);
        if (s != DK_OK) return s;
        s = run_digits_conv<2>(xbar, Bp, cg, (int)g.Kg, pl.K, pl.J_pad, pl.Kp, pl.sums, flag + 1, st);
        if (s != DK_OK) return s;
    } else {
        // the contraction index is the encoded row: both operands are transposed
        s = run_digits_t(dtilde, Ap, (int)R, g.M, pl.I_pad, pl.Kp, pl.sums, flag, st);
        if (s != DK_OK) return s;
        s = run_digits_t(xbar, Bp, (int)R, g.N, pl.J_pad, pl.Kp, pl.sums, flag + 1, st);
        if (s != DK_OK) return s;
    }
    return run_fgemm(pl, Ap, Bp, part, flag, dwq, dW, l, scale, accumulate, 0, "f_gemm_wgrad", st);
}

} // namespace

DK_EXPORT dk_status dkf_wgrad(const dk_layer *L, const float *delta, const uint32_t *B,
                              const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                              int G, int K, int l, float scale, int accumulate,
                              void *ws, size_t ws_bytes, void *stream)
{
    return wgrad_impl(L, delta, nullptr, B, gamma, xbar, dW, dwq, G, K, 1, l, scale, accumulate, ws,
                      ws_bytes, stream);
}

DK_EXPORT dk_status dkf_wgrad_m(const dk_layer *L, const float *delta, const uint32_t *B,
                                const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                                int G, int K, int M, int l, float scale, int accumulate,
                                void *ws, size_t ws_bytes, void *stream)
{
    return wgrad_impl(L, delta, nullptr, B, gamma, xbar, dW, dwq, G, K, M, l, scale, accumulate, ws,
                      ws_bytes, stream);
}

DK_EXPORT dk_status dkf_wgrad_norm(const dk_layer *L, const float *delta, const float *xscale,
                                   const uint32_t *B, const uint32_t *gamma, const uint32_t *xbar,
                                   float *dW, uint32_t *dwq, int G, int K, int l, float scale,
                                   int accumulate, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(xscale, DK_ERR_NULL);
    DK_REQUIRE(dk_aligned(xscale, 4), DK_ERR_ALIGN);
    return wgrad_impl(L, delta, xscale, B, gamma, xbar, dW, dwq, G, K, 1, l, scale, accumulate, ws,
                      ws_bytes, stream);
}

// ---------------------------------------------------------------------------
// Diagnostic: what the int8 matrix pipe sustains when nothing else limits it.
// ---------------------------------------------------------------------------
namespace {

// One wave per SIMD (four per workgroup, one workgroup per compute unit), eight independent
// accumulator blocks, operands in registers: 16 MFMAs per iteration and nothing else.
__global__ __launch_bounds__(256) void f_mfma_rate_kernel(int random_operands, int iterations, int *out)
{
    const unsigned seed = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    i32x4 a[2], b[2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned h = (seed ^ (0x9e3779b9u * (unsigned)(4 * x + c + 1))) * 2246822519u;
            unsigned ra = h ^ (h >> 15), rb = (h * 3266489917u) ^ (h >> 13);
            if (random_operands == 2) {            // balanced base-128 digits: bytes in [-64, 63]
                ra = (ra & 0x7f7f7f7fu) | ((ra & 0x40404040u) << 1);
                rb = (rb & 0x7f7f7f7fu) | ((rb & 0x40404040u) << 1);
            }
            a[x][c] = random_operands ? (int)ra : 0x01010101;
            b[x][c] = random_operands ? (int)rb : 0x01010101;
        }
    i32x16 acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0;
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int q = 0; q < 8; ++q)
                acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[q & 1], b[(q >> 1) & 1], acc[q], 0, 0, 0);
    }
    int sum = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum ^= acc[q][v];
    if (out && sum == 0x7ffffff1) out[threadIdx.x] = sum;      // keeps the loop; practically never true
}

} // namespace

DK_EXPORT dk_status dkf_probe_mfma_rate(int random_operands, int iterations, double *int8_ops, void *stream)
{
    DK_REQUIRE(iterations >= 1 && iterations <= (1 << 24), DK_ERR_SHAPE);
    const int blocks = 256;
    DK_REQUIRE(random_operands >= 0 && random_operands <= 2, DK_ERR_SHAPE);
    dk_prof_scope ps(random_operands ? "f_mfma_rate_random" : "f_mfma_rate_constant", (hipStream_t)stream);
    f_mfma_rate_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>(random_operands, iterations, nullptr);
    if (int8_ops) *int8_ops = (double)blocks * 4.0 * (double)iterations * 16.0 * 65536.0;
    return dk_launch_status();
}
