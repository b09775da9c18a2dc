// Finite-field variant, bandwidth-bound kernels: quantisation, encoding,
// decoding with the integrity check, and gradient mixing, all exact arithmetic
// modulo p = 2^25 - 39.  Same shape as the floating-point mix kernels: one
// workgroup owns (group g, a span of the feature axis), the group's
// coefficients sit at a wave-uniform address, every input row is read once.
//
// Sums of up to K+2 <= 18 products of field elements stay below 2^55, so they
// are accumulated in 64 bits and reduced once, by folding with
// 2^25 = 39 (mod p).
#include "dk_field.h"

namespace {

constexpr int FT = 256;     // threads per workgroup

template <int VEC>
__device__ __forceinline__ void ld_u32(uint32_t (&dst)[VEC], const uint32_t *p)
{
    if constexpr (VEC == 4) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void ld_f32(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void st_u32(uint32_t *p, const uint32_t (&src)[VEC])
{
    if constexpr (VEC == 4) {
        u32x4 v; v.x = src[0]; v.y = src[1]; v.z = src[2]; v.w = src[3];
        *reinterpret_cast<u32x4 *>(p) = v;
    } else {
        *p = src[0];
    }
}

template <int VEC>
__device__ __forceinline__ void st_f32(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4) {
        f32x4 v; v.x = src[0]; v.y = src[1]; v.z = src[2]; v.w = src[3];
        *reinterpret_cast<f32x4 *>(p) = v;
    } else {
        *p = src[0];
    }
}

// One row per blockIdx.y; `scale` (one factor per row) may be null.
template <int VEC>
__global__ __launch_bounds__(FT) void quantize_kernel(const float *__restrict__ x,
                                                      const float *__restrict__ scale,
                                                      uint32_t *__restrict__ xq,
                                                      long long nvec, double s)
{
    const long long v = (long long)blockIdx.x * FT + threadIdx.x;
    if (v >= nvec) return;
    const long long row0 = (long long)blockIdx.y * nvec * VEC;
    if (scale) s *= (double)scale[blockIdx.y];      // exact: 24 bits times a power of two
    float in[VEC];
    uint32_t out[VEC];
    ld_f32<VEC>(in, x + row0 + v * VEC);
#pragma unroll
    for (int c = 0; c < VEC; ++c) out[c] = dkf_quant(in[c], s);
    st_u32<VEC>(xq + row0 + v * VEC, out);
}

// Largest absolute entry of each row, NaN skipped, gathered with an integer
// maximum on the bit patterns (non-negative floats order like their bits).
// bits[row] was cleared by the launch before this one.
template <int VEC>
__global__ __launch_bounds__(FT) void absmax_kernel(const float *__restrict__ x,
                                                    uint32_t *__restrict__ bits,
                                                    long long nvec, long long span)
{
    const long long row0 = (long long)blockIdx.y * nvec * VEC;
    const long long v0 = (long long)blockIdx.x * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    float m = 0.0f;
    for (long long v = v0 + threadIdx.x; v < v1; v += FT) {
        float in[VEC];
        ld_f32<VEC>(in, x + row0 + v * VEC);
#pragma unroll
        for (int c = 0; c < VEC; ++c) m = fmaxf(m, fabsf(in[c]));   // fmaxf drops a NaN operand
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0 && m > 0.0f) atomicMax(bits + blockIdx.y, __float_as_uint(m));
}

// bits[row] -> factor[row] in place: 1/m (nearest fp32 to the fp64 quotient)
// when limit < m < infinity, else 1.
__global__ void norm_scale_kernel(uint32_t *bits, long long rows, float limit)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    const float m = __uint_as_float(bits[i]);
    const float f = (m > limit && m < INFINITY) ? (float)(1.0 / (double)m) : 1.0f;
    bits[i] = __float_as_uint(f);
}

__global__ void f_clear_u32_kernel(uint32_t *p, long long count)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

template <int VEC>
__global__ __launch_bounds__(FT) void dequantize_kernel(const uint32_t *__restrict__ yq,
                                                        float *__restrict__ y,
                                                        long long nvec, double s)
{
    const long long v = (long long)blockIdx.x * FT + threadIdx.x;
    if (v >= nvec) return;
    uint32_t in[VEC];
    float out[VEC];
    ld_u32<VEC>(in, yq + v * VEC);
#pragma unroll
    for (int c = 0; c < VEC; ++c) out[c] = dkf_dequant(in[c], s);
    st_f32<VEC>(y + v * VEC, out);
}

// xbar[gS+j] = sum_i A[g][i][j] * Xq[gK+i] + A[g][K][j] * r[g]  (mod p),
// Xq quantised on the fly from the float rows.
// With FULL = false the group has nk <= K private inputs and K + 1 - nk noise
// rows (several colluding accelerators): the template's K counts inputs plus
// all noise rows but one, S = K + 2 stays the number of encodings, the first nk
// sources are float rows of x and the others field rows of r.  FULL = true is
// the case nk = K with every test compiled away.  The same convention holds
// for the decoding and gradient-mixing kernels below.
template <int K, int VEC, bool FULL>
__global__ __launch_bounds__(FT) void f_encode_kernel(
    const float *__restrict__ x, const float *__restrict__ xscale, const uint32_t *__restrict__ r,
    const uint32_t *__restrict__ A, uint32_t *__restrict__ xbar, long long len, long long nvec,
    int chunks, long long span, double s, int nk_rt)
{
    constexpr int S = K + 2;
    const int nk = FULL ? K : nk_rt;            // wave-uniform
    const int g = blockIdx.x / chunks;          // wave-uniform
    const int chunk = blockIdx.x - g * chunks;
    const uint32_t *Ag = A + (long long)g * S * S;
    const float *xs = x + (long long)g * nk * len;
    const uint32_t *rs = r + (long long)g * (K + 1 - nk) * len;
    uint32_t *dst = xbar + (long long)g * S * len;
    // 2^l times the row's normalisation factor, if any (exact in fp64)
    double si[K];
#pragma unroll
    for (int i = 0; i < K; ++i) si[i] = (xscale && (FULL || i < nk)) ? s * (double)xscale[(long long)g * nk + i] : s;

    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += FT) {
        const long long e = v * VEC;
        uint64_t acc[S][VEC];
#pragma unroll
        for (int j = 0; j < S; ++j)
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[j][c] = 0;
#pragma unroll
        for (int i = 0; i <= K; ++i) {
            uint32_t q[VEC];
            if (i < K && (FULL || i < nk)) {
                float f[VEC];
                ld_f32<VEC>(f, xs + (long long)i * len + e);
#pragma unroll
                for (int c = 0; c < VEC; ++c) q[c] = dkf_quant(f[c], si[i < K ? i : 0]);
            } else {
                ld_u32<VEC>(q, rs + (long long)(i - nk) * len + e);
            }
#pragma unroll
            for (int j = 0; j < S; ++j) {
                const uint32_t a = Ag[i * S + j];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[j][c] += (uint64_t)a * q[c];
            }
        }
#pragma unroll
        for (int j = 0; j < S; ++j) {
            uint32_t o[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) o[c] = dkf_reduce(acc[j][c]);
            st_u32<VEC>(dst + (long long)j * len + e, o);
        }
    }
}

// Decoding and the integrity check in one pass over a group's K+2 result rows.
template <int K, int VEC, bool FULL>
__global__ __launch_bounds__(FT) void f_decode_verify_kernel(
    const uint32_t *__restrict__ ybar, const uint32_t *__restrict__ Ainv,
    const uint32_t *__restrict__ nvec_, const float *__restrict__ xscale,
    const float *__restrict__ wscale, float *__restrict__ y, uint32_t *__restrict__ yq,
    int *__restrict__ verdict, long long len, long long nvec, int chunks, long long span, double s,
    int nk_rt)
{
    constexpr int S = K + 2;
    const int nk = FULL ? K : nk_rt;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;
    const uint32_t *Ag = Ainv + (long long)g * S * S;
    const uint32_t *ng = nvec_ + (long long)g * S;
    const uint32_t *src = ybar + (long long)g * S * len;
    // fp64 reciprocal of (input factor * weight factor): that product is exact
    double back[K];
    if (xscale) {
        const double ws = (double)wscale[0];
#pragma unroll
        for (int i = 0; i < K; ++i)
            back[i] = (FULL || i < nk) ? 1.0 / ((double)xscale[(long long)g * nk + i] * ws) : 1.0;
    }

    bool bad = false;
    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += FT) {
        const long long e = v * VEC;
        uint64_t acc[K][VEC], t[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) t[c] = 0;
#pragma unroll
        for (int i = 0; i < K; ++i)
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[i][c] = 0;
#pragma unroll
        for (int j = 0; j < S; ++j) {
            uint32_t q[VEC];
            ld_u32<VEC>(q, src + (long long)j * len + e);
#pragma unroll
            for (int c = 0; c < VEC; ++c)
                if (q[c] >= DKF_P) { bad = true; q[c] = 0; }
            const uint32_t nj = ng[j];
#pragma unroll
            for (int c = 0; c < VEC; ++c) t[c] += (uint64_t)nj * q[c];
#pragma unroll
            for (int i = 0; i < K; ++i) {
                const uint32_t a = Ag[j * S + i];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[i][c] += (uint64_t)a * q[c];
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) bad |= dkf_reduce(t[c]) != 0;
#pragma unroll
        for (int i = 0; i < K; ++i) {
            if (!FULL && i >= nk) continue;
            uint32_t o[VEC];
            float f[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                o[c] = dkf_reduce(acc[i][c]);
                f[c] = dkf_dequant(o[c], s);
                if (xscale) f[c] = (float)((double)f[c] * back[i]);
            }
            st_f32<VEC>(y + ((long long)g * nk + i) * len + e, f);
            if (yq) st_u32<VEC>(yq + ((long long)g * nk + i) * len + e, o);
        }
    }
    // verdict[g] was cleared by the launch before this one
    if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(verdict + g, 1);
}

// dtilde[gS+j] = gamma[g][j] * (sum_i B[g][j][i] * Dq[gK+i])  (mod p).
template <int K, int VEC, bool FULL>
__global__ __launch_bounds__(FT) void f_delta_mix_kernel(
    const float *__restrict__ delta, const float *__restrict__ xscale,
    const uint32_t *__restrict__ B, const uint32_t *__restrict__ gamma,
    uint32_t *__restrict__ dtilde, long long len, long long nvec, int chunks, long long span, double s,
    int nk_rt)
{
    constexpr int S = K + 2;
    const int nk = FULL ? K : nk_rt;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;
    const uint32_t *Bg = B + (long long)g * S * nk;
    const uint32_t *gg = gamma + (long long)g * S;
    const float *src = delta + (long long)g * nk * len;
    uint32_t *dst = dtilde + (long long)g * S * len;
    // 2^l over the factor of the sample's stored input: the fp64 reciprocal,
    // scaled by a power of two (so the product below rounds once, in fp64)
    double si[K];
#pragma unroll
    for (int i = 0; i < K; ++i)
        si[i] = (xscale && (FULL || i < nk)) ? s * (1.0 / (double)xscale[(long long)g * nk + i]) : s;

    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += FT) {
        const long long e = v * VEC;
        uint32_t q[K][VEC];
#pragma unroll
        for (int i = 0; i < K; ++i) {
            if (!FULL && i >= nk) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) q[i][c] = 0;
                continue;
            }
            float f[VEC];
            ld_f32<VEC>(f, src + (long long)i * len + e);
#pragma unroll
            for (int c = 0; c < VEC; ++c) q[i][c] = dkf_quant(f[c], si[i]);
        }
#pragma unroll
        for (int j = 0; j < S; ++j) {
            uint64_t acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = 0;
#pragma unroll
            for (int i = 0; i < K; ++i) {
                if (!FULL && i >= nk) continue;
                const uint32_t b = Bg[j * nk + i];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] += (uint64_t)b * q[i][c];
            }
            const uint32_t gj = gg[j];
            uint32_t o[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) o[c] = dkf_reduce((uint64_t)gj * dkf_reduce(acc[c]));
            st_u32<VEC>(dst + (long long)j * len + e, o);
        }
    }
}

__global__ void f_clear_kernel(int *p, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

struct fspan {
    long long nvec, span;
    int chunks;
};

// Each lane moves `iters` vectors; spans shrink until the launch has a few
// thousand workgroups.
fspan plan_fspan(long long len, int vec, int G)
{
    fspan p;
    p.nvec = len / vec;
    long long iters = 4;
    while (iters > 1 && (long long)G * ((p.nvec + FT * iters - 1) / (FT * iters)) < 4096) iters >>= 1;
    p.span = FT * iters;
    p.chunks = (int)((p.nvec + p.span - 1) / p.span);
    return p;
}

bool vec4_ok(long long len, std::initializer_list<const void *> ptrs)
{
    if (len % 4) return false;
    for (const void *p : ptrs)
        if (p && !dk_aligned(p, 16)) return false;
    return true;
}

dk_status check_args(int G, int K, long long len, int l)
{
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && len >= 1, DK_ERR_SHAPE);
    DK_REQUIRE(l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE((long long)G * (K + 2) <= 0x7fffffffll && len <= (1ll << 40), DK_ERR_SHAPE);
    return DK_OK;
}

#define DKF_K_SWITCH(K, CALL)                                                   \
    switch (K) {                                                                \
    case 1: return CALL(1);   case 2: return CALL(2);   case 3: return CALL(3);   \
    case 4: return CALL(4);   case 5: return CALL(5);   case 6: return CALL(6);   \
    case 7: return CALL(7);   case 8: return CALL(8);   case 9: return CALL(9);   \
    case 10: return CALL(10); case 11: return CALL(11); case 12: return CALL(12); \
    case 13: return CALL(13); case 14: return CALL(14); case 15: return CALL(15); \
    case 16: return CALL(16);                                                   \
    default: return DK_ERR_SHAPE;                                               \
    }

template <int K>
dk_status launch_encode(const float *x, const float *xscale, const uint32_t *r, const uint32_t *A,
                        uint32_t *xbar, int G, long long n, int l, hipStream_t st, int nk = K)
{
    const bool v4 = vec4_ok(n, {x, r, xbar});
    const fspan p = plan_fspan(n, v4 ? 4 : 1, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const double s = ldexp(1.0, l);
    dk_prof_scope ps("f_encode", st);
#define DKF_LAUNCH(V, F) f_encode_kernel<K, V, F><<<dim3((unsigned)blocks), dim3(FT), 0, st>>>(x, xscale, r, A, xbar, n, p.nvec, p.chunks, p.span, s, nk)
    if (nk == K) { if (v4) DKF_LAUNCH(4, true); else DKF_LAUNCH(1, true); }
    else         { if (v4) DKF_LAUNCH(4, false); else DKF_LAUNCH(1, false); }
#undef DKF_LAUNCH
    return dk_launch_status();
}

template <int K>
dk_status launch_decode_verify(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                               const float *xscale, const float *wscale, float *y, uint32_t *yq,
                               int *verdict, int G, long long m, int l, hipStream_t st, int nk = K)
{
    const bool v4 = vec4_ok(m, {ybar, y, yq});
    const fspan p = plan_fspan(m, v4 ? 4 : 1, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const double s = ldexp(1.0, -l);
    {
        dk_prof_scope ps("f_clear", st);
        f_clear_kernel<<<dim3((G + 255) / 256), dim3(256), 0, st>>>(verdict, G);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    dk_prof_scope ps("f_decode_verify", st);
#define DKF_LAUNCH(V, F) f_decode_verify_kernel<K, V, F><<<dim3((unsigned)blocks), dim3(FT), 0, st>>>( \
        ybar, Ainv, nvec, xscale, wscale, y, yq, verdict, m, p.nvec, p.chunks, p.span, s, nk)
    if (nk == K) { if (v4) DKF_LAUNCH(4, true); else DKF_LAUNCH(1, true); }
    else         { if (v4) DKF_LAUNCH(4, false); else DKF_LAUNCH(1, false); }
#undef DKF_LAUNCH
    return dk_launch_status();
}

template <int K>
dk_status launch_delta_mix(const float *delta, const float *xscale, const uint32_t *B,
                           const uint32_t *gamma, uint32_t *dtilde, int G, long long m, int l,
                           hipStream_t st, int nk = K)
{
    const bool v4 = vec4_ok(m, {delta, dtilde});
    const fspan p = plan_fspan(m, v4 ? 4 : 1, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const double s = ldexp(1.0, l);
    dk_prof_scope ps("f_delta_mix", st);
#define DKF_LAUNCH(V, F) f_delta_mix_kernel<K, V, F><<<dim3((unsigned)blocks), dim3(FT), 0, st>>>(delta, xscale, B, gamma, dtilde, m, p.nvec, p.chunks, p.span, s, nk)
    if (nk == K) { if (v4) DKF_LAUNCH(4, true); else DKF_LAUNCH(1, true); }
    else         { if (v4) DKF_LAUNCH(4, false); else DKF_LAUNCH(1, false); }
#undef DKF_LAUNCH
    return dk_launch_status();
}

} // namespace

dk_status dkf_delta_mix(const float *delta, const float *xscale, const uint32_t *B,
                        const uint32_t *gamma, uint32_t *dtilde, int G, int K, int M, long long m, int l,
                        hipStream_t st)
{
#define CALL(KK) launch_delta_mix<KK>(delta, xscale, B, gamma, dtilde, G, m, l, st, K)
    DKF_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

namespace {

dk_status quantize_rows(const float *x, const float *scale, uint32_t *xq, long long rows,
                        long long len, int l, hipStream_t st)
{
    const bool v4 = vec4_ok(len, {x, xq});
    const long long nvec = v4 ? len / 4 : len;
    const long long blocks = (nvec + FT - 1) / FT;
    DK_REQUIRE(blocks <= 0x7fffffffll && rows <= 65535, DK_ERR_SHAPE);
    const double s = ldexp(1.0, l);
    dk_prof_scope ps("f_quantize", st);
    const dim3 grid((unsigned)blocks, (unsigned)rows);
    if (v4)
        quantize_kernel<4><<<grid, dim3(FT), 0, st>>>(x, scale, xq, nvec, s);
    else
        quantize_kernel<1><<<grid, dim3(FT), 0, st>>>(x, scale, xq, nvec, s);
    return dk_launch_status();
}

} // namespace

DK_EXPORT dk_status dkf_quantize(const float *x, uint32_t *xq, long long count, int l, void *stream)
{
    DK_REQUIRE(x && xq, DK_ERR_NULL);
    DK_REQUIRE(count >= 1 && count <= (1ll << 40) && l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(xq, 4), DK_ERR_ALIGN);
    return quantize_rows(x, nullptr, xq, 1, count, l, (hipStream_t)stream);
}

DK_EXPORT dk_status dkf_quantize_norm(const float *x, const float *scale, uint32_t *xq, long long rows,
                                      long long len, int l, void *stream)
{
    DK_REQUIRE(x && scale && xq, DK_ERR_NULL);
    DK_REQUIRE(rows >= 1 && rows <= 65535 && len >= 1 && len <= (1ll << 40) && l >= 0 && l <= DKF_MAX_L,
               DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(scale, 4) && dk_aligned(xq, 4), DK_ERR_ALIGN);
    return quantize_rows(x, scale, xq, rows, len, l, (hipStream_t)stream);
}

DK_EXPORT dk_status dkf_norm_scales(const float *x, float *scale, long long rows, long long len,
                                    float limit, void *stream)
{
    DK_REQUIRE(x && scale, DK_ERR_NULL);
    DK_REQUIRE(rows >= 1 && rows <= 65535 && len >= 1 && len <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(limit > 0.0f && limit < INFINITY, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(scale, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const bool v4 = vec4_ok(len, {x});
    const long long nvec = v4 ? len / 4 : len;
    // each lane reads up to `iters` vectors; spans shrink until the launch fills the chip
    long long iters = 16;
    while (iters > 1 && rows * ((nvec + FT * iters - 1) / (FT * iters)) < 4096) iters >>= 1;
    const long long span = FT * iters;
    const long long chunks = (nvec + span - 1) / span;
    DK_REQUIRE(chunks <= 0x7fffffffll, DK_ERR_SHAPE);
    uint32_t *bits = reinterpret_cast<uint32_t *>(scale);
    {
        dk_prof_scope ps("f_clear", st);
        f_clear_u32_kernel<<<dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st>>>(bits, rows);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    {
        dk_prof_scope ps("f_absmax", st);
        const dim3 grid((unsigned)chunks, (unsigned)rows);
        if (v4)
            absmax_kernel<4><<<grid, dim3(FT), 0, st>>>(x, bits, nvec, span);
        else
            absmax_kernel<1><<<grid, dim3(FT), 0, st>>>(x, bits, nvec, span);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    dk_prof_scope ps("f_norm_scale", st);
    norm_scale_kernel<<<dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st>>>(bits, rows, limit);
    return dk_launch_status();
}

DK_EXPORT dk_status dkf_dequantize(const uint32_t *yq, float *y, long long count, int l, void *stream)
{
    DK_REQUIRE(yq && y, DK_ERR_NULL);
    DK_REQUIRE(count >= 1 && count <= (1ll << 40) && l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(yq, 4) && dk_aligned(y, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const bool v4 = vec4_ok(count, {yq, y});
    const long long nvec = v4 ? count / 4 : count;
    const long long blocks = (nvec + FT - 1) / FT;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const double s = ldexp(1.0, -l);
    dk_prof_scope ps("f_dequantize", st);
    if (v4)
        dequantize_kernel<4><<<dim3((unsigned)blocks), dim3(FT), 0, st>>>(yq, y, nvec, s);
    else
        dequantize_kernel<1><<<dim3((unsigned)blocks), dim3(FT), 0, st>>>(yq, y, nvec, s);
    return dk_launch_status();
}

DK_EXPORT dk_status dkf_encode(const float *x, const uint32_t *r, const uint32_t *A, uint32_t *xbar,
                               int G, int K, long long n, int l, void *stream)
{
    DK_REQUIRE(x && r && A && xbar, DK_ERR_NULL);
    const dk_status s = check_args(G, K, n, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_encode<KK>(x, nullptr, r, A, xbar, G, n, l, st)
    DKF_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_encode_norm(const float *x, const float *xscale, const uint32_t *r,
                                    const uint32_t *A, uint32_t *xbar, int G, int K, long long n,
                                    int l, void *stream)
{
    DK_REQUIRE(x && xscale && r && A && xbar, DK_ERR_NULL);
    const dk_status s = check_args(G, K, n, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(xscale, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) &&
                   dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_encode<KK>(x, xscale, r, A, xbar, G, n, l, st)
    DKF_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_decode_verify(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                                      float *y, uint32_t *yq, int *verdict, int G, int K,
                                      long long m, int l, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    const dk_status s = check_args(G, K, m, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(verdict, 4) && (!yq || dk_aligned(yq, 4)), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_decode_verify<KK>(ybar, Ainv, nvec, nullptr, nullptr, y, yq, verdict, G, m, l, st)
    DKF_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_decode_verify_norm(const uint32_t *ybar, const uint32_t *Ainv,
                                           const uint32_t *nvec, const float *xscale,
                                           const float *wscale, float *y, uint32_t *yq, int *verdict,
                                           int G, int K, long long m, int l, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && xscale && wscale && y && verdict, DK_ERR_NULL);
    const dk_status s = check_args(G, K, m, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(xscale, 4) && dk_aligned(wscale, 4) && dk_aligned(verdict, 4) &&
                   (!yq || dk_aligned(yq, 4)), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_decode_verify<KK>(ybar, Ainv, nvec, xscale, wscale, y, yq, verdict, G, m, l, st)
    DKF_K_SWITCH(K, CALL)
#undef CALL
}

// ---- several colluding accelerators: M noise rows per group, S = K + M + 1 ----

DK_EXPORT dk_status dkf_encode_m(const float *x, const uint32_t *r, const uint32_t *A, uint32_t *xbar,
                                 int G, int K, int M, long long n, int l, void *stream)
{
    DK_REQUIRE(x && r && A && xbar, DK_ERR_NULL);
    DK_REQUIRE(K >= 1 && M >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    const dk_status s = check_args(G, K + M - 1, n, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_encode<KK>(x, nullptr, r, A, xbar, G, n, l, st, K)
    DKF_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_decode_verify_m(const uint32_t *ybar, const uint32_t *Ainv, const uint32_t *nvec,
                                        float *y, uint32_t *yq, int *verdict, int G, int K, int M,
                                        long long m, int l, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    DK_REQUIRE(K >= 1 && M >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    const dk_status s = check_args(G, K + M - 1, m, l);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(verdict, 4) && (!yq || dk_aligned(yq, 4)), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
#define CALL(KK) launch_decode_verify<KK>(ybar, Ainv, nvec, nullptr, nullptr, y, yq, verdict, G, m, l, st, K)
    DKF_K_SWITCH(K + M - 1, CALL)
#undef CALL
}
