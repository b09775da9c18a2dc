// Encoding with the noise drawn inside the kernel by a counter-based generator,
// so that the noise rows are never written to or read from HBM: a seed stands
// for them.  Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel
// random numbers: as easy as 1, 2, 3", SC'11) is a keyed bijection of a 128-bit
// counter; the counter is (position, group, noise row), the key is the seed.
//
// Real-valued path: one call covers elements 4b..4b+3 of noise row q of group
// g, counter (b mod 2^32, b div 2^32, g, q); the four words become uniforms
// u = ((w >> 8) + 1/2) 2^-24 and two Box-Muller pairs
// sqrt(-2 ln u0) (cos, sin)(2 pi u1), same with (u2, u3), times sigma.
// Field path: one call covers elements 2t, 2t+1 of the noise row of group g,
// counter (t mod 2^32, t div 2^32, g, 0); an element is a 64-bit word (first
// word high) mod p, uniform up to 2^-39.
#include <initializer_list>
#include "dk_field.h"

namespace {

constexpr int RT = 256;

struct u32q { uint32_t v[4]; };

__device__ __forceinline__ u32q philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    u32q o;
    o.v[0] = c0; o.v[1] = c1; o.v[2] = c2; o.v[3] = c3;
    return o;
}

// four N(0, sigma^2) values for block b of noise row q of group g
__device__ __forceinline__ void gauss4(float (&z)[4], long long b, int g, int q, uint32_t k0, uint32_t k1,
                                       float sigma)
{
    const u32q w = philox4x32_10((uint32_t)b, (uint32_t)((unsigned long long)b >> 32), (uint32_t)g,
                                 (uint32_t)q, k0, k1);
    float u[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) u[k] = ((float)(w.v[k] >> 8) + 0.5f) * (1.0f / 16777216.0f);
    const float m0 = sigma * sqrtf(-2.0f * logf(u[0])), m1 = sigma * sqrtf(-2.0f * logf(u[2]));
    float s0, c0, s1, c1;
    sincospif(2.0f * u[1], &s0, &c0);
    sincospif(2.0f * u[3], &s1, &c1);
    z[0] = m0 * c0; z[1] = m0 * s0; z[2] = m1 * c1; z[3] = m1 * s1;
}

// two uniform field elements for pair t of the noise row of group g
__device__ __forceinline__ void field2(uint32_t (&r)[2], long long t, int g, uint32_t k0, uint32_t k1)
{
    const u32q w = philox4x32_10((uint32_t)t, (uint32_t)((unsigned long long)t >> 32), (uint32_t)g, 0u, k0, k1);
    // 64-bit word mod p: fold the bits above 2^25 once (2^25 = 39 mod p), then reduce
    const uint64_t a = ((uint64_t)w.v[0] << 32) | w.v[1], b = ((uint64_t)w.v[2] << 32) | w.v[3];
    r[0] = dkf_reduce((a >> 25) * 39u + (a & 0x1ffffffu));       // < 2^45
    r[1] = dkf_reduce((b >> 25) * 39u + (b & 0x1ffffffu));
}

// r[(g*M + q)][4b .. 4b+3]
__global__ __launch_bounds__(RT) void noise_kernel(float *__restrict__ r, long long len, long long nblk,
                                                   int M, uint32_t k0, uint32_t k1, float sigma)
{
    const long long b = (long long)blockIdx.x * RT + threadIdx.x;
    if (b >= nblk) return;
    const int row = blockIdx.y, g = row / M, q = row - g * M;
    float z[4];
    gauss4(z, b, g, q, k0, k1, sigma);
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (4 * b + c < len) r[(long long)row * len + 4 * b + c] = z[c];
}

__global__ __launch_bounds__(RT) void f_noise_kernel(uint32_t *__restrict__ r, long long len, long long npair,
                                                     uint32_t k0, uint32_t k1)
{
    const long long t = (long long)blockIdx.x * RT + threadIdx.x;
    if (t >= npair) return;
    const int g = blockIdx.y;
    uint32_t v[2];
    field2(v, t, g, k0, k1);
    r[(long long)g * len + 2 * t] = v[0];
    if (2 * t + 1 < len) r[(long long)g * len + 2 * t + 1] = v[1];
}

// xbar[gS+j] = sum_{i<nk} A[g][i][j] x[g nk + i] + sum_{q<M} A[g][nk+q][j] noise(g, q), with
// KT = nk + M - 1 and S = KT + 2; the sum runs in this order with fused
// multiply-adds, as in the encoding kernel that reads its noise from memory.
// A thread owns four consecutive elements (one generator block).  VEC = true:
// len is a multiple of 4 and the rows are 16-byte aligned.
template <int KT, bool VEC>
__global__ __launch_bounds__(RT) void encode_rng_kernel(const float *__restrict__ x, const float *__restrict__ A,
                                                        float *__restrict__ xbar, long long len, long long nblk,
                                                        int chunks, long long span, int nk, uint32_t k0,
                                                        uint32_t k1, float sigma)
{
    constexpr int S = KT + 2, NIN = KT + 1;
    const int g = blockIdx.x / chunks;          // wave-uniform
    const int chunk = blockIdx.x - g * chunks;
    float coef[NIN][S];
#pragma unroll
    for (int i = 0; i < NIN; ++i)
#pragma unroll
        for (int o = 0; o < S; ++o) coef[i][o] = A[((long long)g * S + i) * S + o];
    const float *src = x + (long long)g * nk * len;
    float *dst = xbar + (long long)g * S * len;

    const long long b0 = (long long)chunk * span;
    long long b1 = b0 + span;
    if (b1 > nblk) b1 = nblk;
    for (long long b = b0 + threadIdx.x; b < b1; b += RT) {
        const long long e = 4 * b;
        float v[NIN][4];
#pragma unroll
        for (int i = 0; i < NIN; ++i) {
            if (i < nk) {
                if (VEC) {
                    const f32x4 t = *reinterpret_cast<const f32x4 *>(src + (long long)i * len + e);
                    v[i][0] = t.x; v[i][1] = t.y; v[i][2] = t.z; v[i][3] = t.w;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[i][c] = e + c < len ? src[(long long)i * len + e + c] : 0.0f;
                }
            } else {
                gauss4(v[i], b, g, i - nk, k0, k1, sigma);
            }
        }
#pragma unroll
        for (int o = 0; o < S; ++o) {
            float acc[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = coef[0][o] * v[0][c];
#pragma unroll
            for (int i = 1; i < NIN; ++i)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = fmaf(coef[i][o], v[i][c], acc[c]);
            if (VEC) {
                f32x4 t; t.x = acc[0]; t.y = acc[1]; t.z = acc[2]; t.w = acc[3];
                *reinterpret_cast<f32x4 *>(dst + (long long)o * len + e) = t;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (e + c < len) dst[(long long)o * len + e + c] = acc[c];
            }
        }
    }
}

// Field version: Xq quantised on the fly, one noise row, exact arithmetic.
template <int K, bool VEC>
__global__ __launch_bounds__(RT) void f_encode_rng_kernel(const float *__restrict__ x, const float *__restrict__ xscale,
                                                          const uint32_t *__restrict__ A,
                                                          uint32_t *__restrict__ xbar, long long len,
                                                          long long nblk, int chunks, long long span, double s,
                                                          uint32_t k0, uint32_t k1)
{
    constexpr int S = K + 2;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;
    const uint32_t *Ag = A + (long long)g * S * S;
    const float *src = x + (long long)g * K * len;
    uint32_t *dst = xbar + (long long)g * S * len;
    // 2^l times the row's normalisation factor, if any (exact in fp64)
    double si[K];
#pragma unroll
    for (int i = 0; i < K; ++i) si[i] = xscale ? s * (double)xscale[(long long)g * K + i] : s;

    const long long b0 = (long long)chunk * span;
    long long b1 = b0 + span;
    if (b1 > nblk) b1 = nblk;
    for (long long b = b0 + threadIdx.x; b < b1; b += RT) {
        const long long e = 4 * b;
        uint64_t acc[S][4];
#pragma unroll
        for (int j = 0; j < S; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[j][c] = 0;
#pragma unroll
        for (int i = 0; i <= K; ++i) {
            uint32_t q[4];
            if (i < K) {
                if (VEC) {
                    const f32x4 t = *reinterpret_cast<const f32x4 *>(src + (long long)i * len + e);
                    q[0] = dkf_quant(t.x, si[i]); q[1] = dkf_quant(t.y, si[i]); q[2] = dkf_quant(t.z, si[i]); q[3] = dkf_quant(t.w, si[i]);
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) q[c] = e + c < len ? dkf_quant(src[(long long)i * len + e + c], si[i]) : 0u;
                }
            } else {
                uint32_t lo[2], hi[2];
                field2(lo, 2 * b, g, k0, k1);
                field2(hi, 2 * b + 1, g, k0, k1);
                q[0] = lo[0]; q[1] = lo[1]; q[2] = hi[0]; q[3] = hi[1];
            }
#pragma unroll
            for (int j = 0; j < S; ++j) {
                const uint32_t a = Ag[i * S + j];
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[j][c] += (uint64_t)a * q[c];
            }
        }
#pragma unroll
        for (int j = 0; j < S; ++j) {
            if (VEC) {
                u32x4 t;
                t.x = dkf_reduce(acc[j][0]); t.y = dkf_reduce(acc[j][1]);
                t.z = dkf_reduce(acc[j][2]); t.w = dkf_reduce(acc[j][3]);
                *reinterpret_cast<u32x4 *>(dst + (long long)j * len + e) = t;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (e + c < len) dst[(long long)j * len + e + c] = dkf_reduce(acc[j][c]);
            }
        }
    }
}

struct rspan {
    long long nblk, span;
    int chunks;
};

rspan plan_rspan(long long len, int G)
{
    rspan p;
    p.nblk = (len + 3) / 4;
    long long iters = 4;
    while (iters > 1 && (long long)G * ((p.nblk + RT * iters - 1) / (RT * iters)) < 4096) iters >>= 1;
    p.span = RT * iters;
    p.chunks = (int)((p.nblk + p.span - 1) / p.span);
    return p;
}

bool vec_ok(long long len, std::initializer_list<const void *> ptrs)
{
    if (len % 4) return false;
    for (const void *p : ptrs)
        if (!dk_aligned(p, 16)) return false;
    return true;
}

#define DKR_K_SWITCH(K, CALL)                                                   \
    switch (K) {                                                                \
    case 1: return CALL(1);   case 2: return CALL(2);   case 3: return CALL(3);   \
    case 4: return CALL(4);   case 5: return CALL(5);   case 6: return CALL(6);   \
    case 7: return CALL(7);   case 8: return CALL(8);   case 9: return CALL(9);   \
    case 10: return CALL(10); case 11: return CALL(11); case 12: return CALL(12); \
    case 13: return CALL(13); case 14: return CALL(14); case 15: return CALL(15); \
    case 16: return CALL(16);                                                   \
    default: return DK_ERR_SHAPE;                                               \
    }

template <int KT>
dk_status launch_encode_rng(const float *x, const float *A, float *xbar, int G, int nk, long long n,
                            uint32_t k0, uint32_t k1, float sigma, hipStream_t st)
{
    const rspan p = plan_rspan(n, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("encode_rng", st);
    if (vec_ok(n, {x, xbar}))
        encode_rng_kernel<KT, true><<<dim3((unsigned)blocks), dim3(RT), 0, st>>>(x, A, xbar, n, p.nblk, p.chunks,
                                                                               p.span, nk, k0, k1, sigma);
    else
        encode_rng_kernel<KT, false><<<dim3((unsigned)blocks), dim3(RT), 0, st>>>(x, A, xbar, n, p.nblk, p.chunks,
                                                                                p.span, nk, k0, k1, sigma);
    return dk_launch_status();
}

template <int K>
dk_status launch_f_encode_rng(const float *x, const float *xscale, const uint32_t *A, uint32_t *xbar, int G,
                              long long n, int l, uint32_t k0, uint32_t k1, hipStream_t st)
{
    const rspan p = plan_rspan(n, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const double s = ldexp(1.0, l);
    dk_prof_scope ps("f_encode_rng", st);
    if (vec_ok(n, {x, xbar}))
        f_encode_rng_kernel<K, true><<<dim3((unsigned)blocks), dim3(RT), 0, st>>>(x, xscale, A, xbar, n, p.nblk, p.chunks,
                                                                                p.span, s, k0, k1);
    else
        f_encode_rng_kernel<K, false><<<dim3((unsigned)blocks), dim3(RT), 0, st>>>(x, xscale, A, xbar, n, p.nblk, p.chunks,
                                                                                 p.span, s, k0, k1);
    return dk_launch_status();
}

} // namespace

DK_EXPORT dk_status dk_noise_rng(float *r, int G, int M, long long n, unsigned long long seed,
                                 float noise_std, void *stream)
{
    DK_REQUIRE(r, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && M >= 1 && M <= DK_MAX_K && n >= 1 && n <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE((long long)G * M <= 65535, DK_ERR_SHAPE);
    DK_REQUIRE(noise_std >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(r, 4), DK_ERR_ALIGN);
    const long long nblk = (n + 3) / 4;
    DK_REQUIRE((nblk + RT - 1) / RT <= 0x7fffffffll, DK_ERR_SHAPE);
    hipStream_t st = (hipStream_t)stream;
    dk_prof_scope ps("noise_rng", st);
    noise_kernel<<<dim3((unsigned)((nblk + RT - 1) / RT), (unsigned)(G * M)), dim3(RT), 0, st>>>(
        r, n, nblk, M, (uint32_t)seed, (uint32_t)(seed >> 32), noise_std);
    return dk_launch_status();
}

DK_EXPORT dk_status dk_encode_rng(const float *x, const float *A, float *xbar, int G, int K, int M,
                                  long long n, unsigned long long seed, float noise_std, void *stream)
{
    DK_REQUIRE(x && A && xbar, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && M >= 1 && K + M - 1 <= DK_MAX_K && n >= 1 && n <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(noise_std >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#define CALL(KK) launch_encode_rng<KK>(x, A, xbar, G, K, n, k0, k1, noise_std, st)
    DKR_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_noise_rng(uint32_t *r, int G, long long n, unsigned long long seed, void *stream)
{
    DK_REQUIRE(r, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && G <= 65535 && n >= 1 && n <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(r, 4), DK_ERR_ALIGN);
    const long long npair = (n + 1) / 2;
    DK_REQUIRE((npair + RT - 1) / RT <= 0x7fffffffll, DK_ERR_SHAPE);
    hipStream_t st = (hipStream_t)stream;
    dk_prof_scope ps("f_noise_rng", st);
    f_noise_kernel<<<dim3((unsigned)((npair + RT - 1) / RT), (unsigned)G), dim3(RT), 0, st>>>(
        r, n, npair, (uint32_t)seed, (uint32_t)(seed >> 32));
    return dk_launch_status();
}

DK_EXPORT dk_status dkf_encode_rng(const float *x, const uint32_t *A, uint32_t *xbar, int G, int K,
                                   long long n, int l, unsigned long long seed, void *stream)
{
    DK_REQUIRE(x && A && xbar, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && n >= 1 && n <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#define CALL(KK) launch_f_encode_rng<KK>(x, nullptr, A, xbar, G, n, l, k0, k1, st)
    DKR_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dkf_encode_rng_norm(const float *x, const float *xscale, const uint32_t *A,
                                        uint32_t *xbar, int G, int K, long long n, int l,
                                        unsigned long long seed, void *stream)
{
    DK_REQUIRE(x && xscale && A && xbar, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && n >= 1 && n <= (1ll << 40), DK_ERR_SHAPE);
    DK_REQUIRE(l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(xscale, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#define CALL(KK) launch_f_encode_rng<KK>(x, xscale, A, xbar, G, n, l, k0, k1, st)
    DKR_K_SWITCH(K, CALL)
#undef CALL
}
