// Bandwidth-bound kernels of the masked layer: encode, decode, gradient
// mixing and the integrity check.  Every one of them is a tiny per-group
// matrix applied along the long feature axis, so the design is the same:
// one workgroup owns (group g, a contiguous span of the feature axis), the
// group's coefficients sit at a wave-uniform address (scalar loads), each lane
// moves 16-byte vectors, and every input row is read exactly once.
#include "dk_internal.h"

static int verify_max_chunks(int G);

// Scratch memory of dk_decode_verify_static (the entry point for callers that
// cannot allocate): the partial maxima of the integrity check live here instead
// of in a caller's workspace.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[DK_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MIX_THREADS = 256;

enum MixMode { MIX_ENCODE = 0, MIX_DECODE = 1, MIX_DMIX = 2 };

template <int VEC> struct vec_t;
template <> struct vec_t<4> { using type = float4; };
template <> struct vec_t<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void vload(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = *p;
    }
}

// Streaming variants for data that is not touched again soon (the decoded
// outputs; the encoded results once they have been decoded).
template <int VEC>
__device__ __forceinline__ void vload_nt(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = __builtin_nontemporal_load(p);
    }
}

template <int VEC>
__device__ __forceinline__ void vstore_nt(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        f4 v = {src[0], src[1], src[2], src[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(p));
    } else {
        __builtin_nontemporal_store(src[0], p);
    }
}

template <int VEC>
__device__ __forceinline__ void vstore(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(src[0], src[1], src[2], src[3]);
    } else {
        *p = src[0];
    }
}

// out[o][e] = sum_i coef(i, o) * in[i][e] for one group.
//   MIX_ENCODE: in = K inputs + noise row, out = S encodings, coef = A[g][i][o]
//   MIX_DECODE: in = S results,            out = K outputs,   coef = Ainv[g][i][o]
//   MIX_DMIX:   in = K gradients,          out = S mixed,     coef = gamma[g][o] * B[g][o][i]
// With FULL = false the group has nk <= K private inputs and K + 1 - nk noise
// rows (several colluding accelerators): the template's K counts inputs plus all
// noise rows but one, S = K + 2 stays the number of encodings, the first nk
// sources come from in0 and the others from in1, and only nk outputs are decoded
// and nk gradients mixed.  FULL = true is the case nk = K with every test
// compiled away.
template <int MODE, int K, int VEC, bool FULL>
__global__ __launch_bounds__(MIX_THREADS) void mix_kernel(
    const float *__restrict__ in0, const float *__restrict__ in1,
    const float *__restrict__ c0, const float *__restrict__ c1,
    float *__restrict__ out, long long len, long long nvec, int chunks, long long span, int nk_rt)
{
    constexpr int S = K + 2;
    constexpr int NIN = MODE == MIX_ENCODE ? K + 1 : (MODE == MIX_DECODE ? S : K);
    constexpr int NOUT = MODE == MIX_DECODE ? K : S;
    const int nk = FULL ? K : nk_rt;            // wave-uniform

    const int g = blockIdx.x / chunks;          // wave-uniform
    const int chunk = blockIdx.x - g * chunks;

    float coef[NIN][NOUT];
#pragma unroll
    for (int i = 0; i < NIN; ++i)
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
            if constexpr (MODE == MIX_ENCODE)
                coef[i][o] = c0[((long long)g * S + i) * S + o];
            else if constexpr (MODE == MIX_DECODE)
                coef[i][o] = c0[((long long)g * S + i) * S + o];
            else
                coef[i][o] = (FULL || i < nk)
                                 ? c1[(long long)g * S + o] * c0[((long long)g * S + o) * nk + i] : 0.0f;
        }

    const float *src[NIN];
#pragma unroll
    for (int i = 0; i < NIN; ++i) {
        if constexpr (MODE == MIX_ENCODE)
            src[i] = (i < nk) ? in0 + ((long long)g * nk + i) * len
                              : in1 + ((long long)g * (K + 1 - nk) + (i - nk)) * len;
        else if constexpr (MODE == MIX_DECODE)
            src[i] = in0 + ((long long)g * S + i) * len;
        else
            src[i] = in0 + ((long long)g * nk + ((FULL || i < nk) ? i : 0)) * len;
    }
    float *dst = out + (long long)g * (MODE == MIX_DECODE ? nk : NOUT) * len;

    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += MIX_THREADS) {
        const long long e = v * VEC;
        float x[NIN][VEC];
#pragma unroll
        for (int i = 0; i < NIN; ++i) vload<VEC>(x[i], src[i] + e);
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
            if (!FULL && MODE == MIX_DECODE && o >= nk) continue;
            float acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = coef[0][o] * x[0][c];
#pragma unroll
            for (int i = 1; i < NIN; ++i)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = fmaf(coef[i][o], x[i][c], acc[c]);
            vstore<VEC>(dst + (long long)o * len + e, acc);
        }
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Integrity check, first pass: each workgroup reduces its span of one group's
// feature axis to (max |t|, max s) and writes the pair to part[g][chunk].
template <int K, int VEC>
__global__ __launch_bounds__(MIX_THREADS) void verify_partial_kernel(
    const float *__restrict__ ybar, const float *__restrict__ nvec_,
    float *__restrict__ part, long long len, long long nvec, int chunks, long long span)
{
    constexpr int S = K + 2;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;

    float nv[S];
#pragma unroll
    for (int j = 0; j < S; ++j) nv[j] = nvec_[(long long)g * S + j];
    const float *src = ybar + (long long)g * S * len;

    float tmax = 0.0f, smax = 0.0f;
    bool bad = false;
    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += MIX_THREADS) {
        const long long e = v * VEC;
        float t[VEC], s[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) { t[c] = 0.0f; s[c] = 0.0f; }
#pragma unroll
        for (int j = 0; j < S; ++j) {
            float y[VEC];
            vload<VEC>(y, src + (long long)j * len + e);
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const float p = nv[j] * y[c];
                t[c] += p;
                s[c] += fabsf(p);
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            // a NaN or infinity anywhere makes s non-finite (or t, via inf-inf)
            bad |= !(s[c] <= 3.402823466e+38f) || !(fabsf(t[c]) <= 3.402823466e+38f);
            tmax = fmaxf(tmax, fabsf(t[c]));
            smax = fmaxf(smax, s[c]);
        }
    }
    if (bad) tmax = __builtin_inff();

    __shared__ float red[2][MIX_THREADS / 64];
    tmax = wave_max(tmax);
    smax = wave_max(smax);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[0][wave] = tmax; red[1][wave] = smax; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < MIX_THREADS / 64; ++w) {
            tmax = fmaxf(tmax, red[0][w]);
            smax = fmaxf(smax, red[1][w]);
        }
        part[((long long)g * chunks + chunk) * 2 + 0] = tmax;
        part[((long long)g * chunks + chunk) * 2 + 1] = smax;
    }
}

// Decode and the first pass of the integrity check in one sweep over ybar:
// both need every encoded row of the group exactly once.
// (FULL = false: only the first nk of the template's K columns are outputs,
// see mix_kernel.)
template <int K, int VEC, bool FULL>
__global__ __launch_bounds__(MIX_THREADS) void decode_verify_kernel(
    const float *__restrict__ ybar, const float *__restrict__ Ainv, const float *__restrict__ nvec_,
    float *__restrict__ y, float *__restrict__ part, long long len, long long nvec, int chunks,
    long long span, int nk_rt)
{
    constexpr int S = K + 2;
    const int nk = FULL ? K : nk_rt;
    const int g = blockIdx.x / chunks;
    const int chunk = blockIdx.x - g * chunks;

    float coef[S][K], nv[S];
#pragma unroll
    for (int j = 0; j < S; ++j) {
        nv[j] = nvec_[(long long)g * S + j];
#pragma unroll
        for (int i = 0; i < K; ++i) coef[j][i] = Ainv[((long long)g * S + j) * S + i];
    }
    const float *src = ybar + (long long)g * S * len;
    float *dst = y + (long long)g * nk * len;

    float tmax = 0.0f, smax = 0.0f;
    bool bad = false;
    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += MIX_THREADS) {
        const long long e = v * VEC;
        float x[S][VEC];
#pragma unroll
        for (int j = 0; j < S; ++j) vload_nt<VEC>(x[j], src + (long long)j * len + e);
#pragma unroll
        for (int i = 0; i < K; ++i) {
            if (!FULL && i >= nk) continue;
            float acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = coef[0][i] * x[0][c];
#pragma unroll
            for (int j = 1; j < S; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = fmaf(coef[j][i], x[j][c], acc[c]);
            vstore_nt<VEC>(dst + (long long)i * len + e, acc);
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float t = 0.0f, sc = 0.0f;
#pragma unroll
            for (int j = 0; j < S; ++j) {
                const float pr = nv[j] * x[j][c];
                t += pr;
                sc += fabsf(pr);
            }
            bad |= !(sc <= 3.402823466e+38f) || !(fabsf(t) <= 3.402823466e+38f);
            tmax = fmaxf(tmax, fabsf(t));
            smax = fmaxf(smax, sc);
        }
    }
    if (bad) tmax = __builtin_inff();

    __shared__ float red[2][MIX_THREADS / 64];
    tmax = wave_max(tmax);
    smax = wave_max(smax);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[0][wave] = tmax; red[1][wave] = smax; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < MIX_THREADS / 64; ++w) {
            tmax = fmaxf(tmax, red[0][w]);
            smax = fmaxf(smax, red[1][w]);
        }
        part[((long long)g * chunks + chunk) * 2 + 0] = tmax;
        part[((long long)g * chunks + chunk) * 2 + 1] = smax;
    }
}

// Integrity check, second pass: one wave per group folds the (at most 64)
// partial pairs -- lane c holds chunk c -- and lane 0 takes the verdict.
__global__ __launch_bounds__(MIX_THREADS) void verify_final_kernel(
    const float *__restrict__ part, int chunks, float tol, int *__restrict__ verdict,
    float *__restrict__ resid, int G)
{
    const int g = blockIdx.x * (MIX_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (g >= G) return;
    float tmax = 0.0f, smax = 0.0f;
    for (int c = lane; c < chunks; c += 64) {
        tmax = fmaxf(tmax, part[((long long)g * chunks + c) * 2 + 0]);
        smax = fmaxf(smax, part[((long long)g * chunks + c) * 2 + 1]);
    }
    tmax = wave_max(tmax);
    smax = wave_max(smax);
    if (lane != 0) return;
    const bool bad = !(tmax <= 3.402823466e+38f);
    const float rho = bad ? __builtin_inff() : (smax > 0.0f ? tmax / smax : 0.0f);
    verdict[g] = (bad || rho > tol) ? 1 : 0;
    if (resid) resid[g] = rho;
}

struct span_plan {
    long long nvec;   // vectors per row
    long long span;   // vectors per workgroup (multiple of MIX_THREADS)
    int chunks;       // workgroups per group
};

// Each lane moves `iters` vectors; spans shrink until the launch has a few
// thousand workgroups (256 compute units, several resident groups each).
span_plan plan_span(long long len, int vec, int G, int max_chunks)
{
    span_plan p;
    p.nvec = len / vec;
    long long iters = 4;
    while (iters > 1 && (long long)G * ((p.nvec + MIX_THREADS * iters - 1) / (MIX_THREADS * iters)) < 4096)
        iters >>= 1;
    p.span = MIX_THREADS * iters;
    long long chunks = (p.nvec + p.span - 1) / p.span;
    if (max_chunks > 0 && chunks > max_chunks) {
        chunks = max_chunks;
        p.span = ((p.nvec + chunks - 1) / chunks + MIX_THREADS - 1) / MIX_THREADS * MIX_THREADS;
        chunks = (p.nvec + p.span - 1) / p.span;
    }
    p.chunks = (int)chunks;
    return p;
}

bool can_vec4(long long len, std::initializer_list<const void *> ptrs)
{
    if (len % 4) return false;
    for (const void *p : ptrs)
        if (p && !dk_aligned(p, 16)) return false;
    return true;
}

template <int MODE, int K>
dk_status launch_mix_k(const float *in0, const float *in1, const float *c0, const float *c1,
                       float *out, int G, long long len, bool v4, int nk, hipStream_t st)
{
    const span_plan p = plan_span(len, v4 ? 4 : 1, G, 0);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps(MODE == MIX_ENCODE ? "encode" : (MODE == MIX_DECODE ? "decode" : "delta_mix"), st);
#define DK_MIX_LAUNCH(V, F)                                                                     \
    mix_kernel<MODE, K, V, F><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(                \
        in0, in1, c0, c1, out, len, p.nvec, p.chunks, p.span, nk)
    if (nk == K) {
        if (v4) DK_MIX_LAUNCH(4, true); else DK_MIX_LAUNCH(1, true);
    } else {
        if (v4) DK_MIX_LAUNCH(4, false); else DK_MIX_LAUNCH(1, false);
    }
#undef DK_MIX_LAUNCH
    return dk_launch_status();
}

#define DK_K_SWITCH(K, CALL)                                                    \
    switch (K) {                                                                \
    case 1: return CALL(1);   case 2: return CALL(2);   case 3: return CALL(3);   \
    case 4: return CALL(4);   case 5: return CALL(5);   case 6: return CALL(6);   \
    case 7: return CALL(7);   case 8: return CALL(8);   case 9: return CALL(9);   \
    case 10: return CALL(10); case 11: return CALL(11); case 12: return CALL(12); \
    case 13: return CALL(13); case 14: return CALL(14); case 15: return CALL(15); \
    case 16: return CALL(16);                                                   \
    default: return DK_ERR_SHAPE;                                               \
    }

// K: private inputs per group; M: noise rows per group.  The kernels are
// instantiated on KT = K + M - 1 (S = KT + 2 encodings).
template <int MODE>
dk_status launch_mix(const float *in0, const float *in1, const float *c0, const float *c1,
                     float *out, int G, int K, int M, long long len, bool v4, hipStream_t st)
{
#define CALL(KK) launch_mix_k<MODE, KK>(in0, in1, c0, c1, out, G, len, v4, K, st)
    DK_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

template <int K>
dk_status launch_verify_k(const float *ybar, const float *nvec, float tol, int *verdict,
                          float *resid, int G, long long len, float *part, bool v4, hipStream_t st)
{
    const span_plan p = plan_span(len, v4 ? 4 : 1, G, verify_max_chunks(G));
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    {
    dk_prof_scope ps("verify_partial", st);
    if (v4)
        verify_partial_kernel<K, 4><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(
            ybar, nvec, part, len, p.nvec, p.chunks, p.span);
    else
        verify_partial_kernel<K, 1><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(
            ybar, nvec, part, len, p.nvec, p.chunks, p.span);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    dk_prof_scope ps("verify_final", st);
    verify_final_kernel<<<dim3((G + MIX_THREADS / 64 - 1) / (MIX_THREADS / 64)), dim3(MIX_THREADS), 0, st>>>(
        part, p.chunks, tol, verdict, resid, G);
    return dk_launch_status();
}

template <int K>
dk_status launch_decode_verify_k(const float *ybar, const float *Ainv, const float *nvec, float tol,
                                 float *y, int *verdict, float *resid, int G, long long len,
                                 float *part, bool v4, int nk, hipStream_t st)
{
    const span_plan p = plan_span(len, v4 ? 4 : 1, G, verify_max_chunks(G));
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    {
    dk_prof_scope ps("decode_verify", st);
#define DK_DV_LAUNCH(V, F)                                                                       \
    decode_verify_kernel<K, V, F><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(            \
        ybar, Ainv, nvec, y, part, len, p.nvec, p.chunks, p.span, nk)
    if (nk == K) {
        if (v4) DK_DV_LAUNCH(4, true); else DK_DV_LAUNCH(1, true);
    } else {
        if (v4) DK_DV_LAUNCH(4, false); else DK_DV_LAUNCH(1, false);
    }
#undef DK_DV_LAUNCH
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    dk_prof_scope ps("verify_final", st);
    verify_final_kernel<<<dim3((G + MIX_THREADS / 64 - 1) / (MIX_THREADS / 64)), dim3(MIX_THREADS), 0, st>>>(
        part, p.chunks, tol, verdict, resid, G);
    return dk_launch_status();
}

dk_status check_mix_args(int G, int K, long long len)
{
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && len >= 1, DK_ERR_SHAPE);
    DK_REQUIRE((long long)G * (K + 2) <= 0x7fffffffll, DK_ERR_SHAPE);
    DK_REQUIRE(len <= (1ll << 40), DK_ERR_SHAPE);
    return DK_OK;
}

} // namespace

// Workgroups per group in the integrity check's first pass: 64 when there are
// many groups, more when a few groups alone would leave most of the chip idle.
static int verify_max_chunks(int G)
{
    int c = (4096 + G - 1) / G;
    if (c < DK_VERIFY_MAX_BLOCKS) c = DK_VERIFY_MAX_BLOCKS;
    if (c > 1024) c = 1024;
    return c;
}

size_t dk_ws_verify_bytes(int G)
{
    return (size_t)G * verify_max_chunks(G) * 2 * sizeof(float);
}

DK_EXPORT dk_status dk_encode(const float *x, const float *r, const float *A, float *xbar,
                              int G, int K, long long n, void *stream)
{
    DK_REQUIRE(x && r && A && xbar, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, n);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    return launch_mix<MIX_ENCODE>(x, r, A, nullptr, xbar, G, K, 1, n, can_vec4(n, {x, r, xbar}),
                                  (hipStream_t)stream);
}

DK_EXPORT dk_status dk_encode_m(const float *x, const float *r, const float *A, float *xbar,
                                int G, int K, int M, long long n, void *stream)
{
    DK_REQUIRE(x && r && A && xbar, DK_ERR_NULL);
    DK_REQUIRE(M >= 1 && K >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    dk_status s = check_mix_args(G, K + M - 1, n);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    return launch_mix<MIX_ENCODE>(x, r, A, nullptr, xbar, G, K, M, n, can_vec4(n, {x, r, xbar}),
                                  (hipStream_t)stream);
}

DK_EXPORT dk_status dk_decode(const float *ybar, const float *Ainv, float *y, int G, int K,
                              long long m, void *stream)
{
    DK_REQUIRE(ybar && Ainv && y, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(y, 4), DK_ERR_ALIGN);
    return launch_mix<MIX_DECODE>(ybar, nullptr, Ainv, nullptr, y, G, K, 1, m, can_vec4(m, {ybar, y}),
                                  (hipStream_t)stream);
}

// Gradient mixing used by dk_wgrad: dtilde[gS+j] = gamma[g][j] sum_i B[g][j][i] delta[gK+i],
// S = K + M + 1.
dk_status dk_delta_mix(const float *delta, const float *B, const float *gamma, float *dtilde,
                       int G, int K, int M, long long m, hipStream_t st)
{
    return launch_mix<MIX_DMIX>(delta, nullptr, B, gamma, dtilde, G, K, M, m,
                                can_vec4(m, {delta, dtilde}), st);
}

DK_EXPORT dk_status dk_verify(const float *ybar, const float *nvec, float tol, int *verdict,
                              float *resid, int G, int K, long long m, void *ws, size_t ws_bytes,
                              void *stream)
{
    DK_REQUIRE(ybar && nvec && verdict, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(tol >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(nvec, 4) && dk_aligned(verdict, 4) &&
                   (!resid || dk_aligned(resid, 4)), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_ws_verify_bytes(G), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 4), DK_ERR_ALIGN);
    const bool v4 = can_vec4(m, {ybar});
#define CALL(KK) launch_verify_k<KK>(ybar, nvec, tol, verdict, resid, G, m, (float *)ws, v4, (hipStream_t)stream)
    DK_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dk_decode_verify(const float *ybar, const float *Ainv, const float *nvec, float tol,
                                     float *y, int *verdict, float *resid, int G, int K, long long m,
                                     void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(tol >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(verdict, 4) && (!resid || dk_aligned(resid, 4)), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_ws_verify_bytes(G), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 4), DK_ERR_ALIGN);
    const bool v4 = can_vec4(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, (float *)ws, v4, K, (hipStream_t)stream)
    DK_K_SWITCH(K, CALL)
#undef CALL
}

DK_EXPORT dk_status dk_decode_verify_m(const float *ybar, const float *Ainv, const float *nvec, float tol,
                                       float *y, int *verdict, float *resid, int G, int K, int M,
                                       long long m, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    DK_REQUIRE(M >= 1 && K >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    dk_status s = check_mix_args(G, K + M - 1, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(tol >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(verdict, 4) && (!resid || dk_aligned(resid, 4)), DK_ERR_ALIGN);
    DK_REQUIRE(ws && ws_bytes >= dk_ws_verify_bytes(G), DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 4), DK_ERR_ALIGN);
    const bool v4 = can_vec4(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, (float *)ws, v4, K, (hipStream_t)stream)
    DK_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<float *> scratch_ptr[MAX_DEVICES];       // device address of `scratch`, per device ordinal

// The current device's copy of the scratch array.  Looked up once per device
// (with that device current); no allocation, no stream operation.
dk_status static_scratch(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DK_ERR_HIP;
    DK_REQUIRE(dev >= 0 && dev < MAX_DEVICES, DK_ERR_UNSUPPORTED);
    float *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return DK_ERR_HIP;
        p = static_cast<float *>(q);
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return DK_OK;
}

} // namespace

DK_EXPORT size_t dk_static_scratch_bytes(void) { return DK_STATIC_SCRATCH_BYTES; }

DK_EXPORT dk_status dk_decode_verify_static(const float *ybar, const float *Ainv, const float *nvec,
                                            float tol, float *y, int *verdict, float *resid, int G,
                                            int K, long long m, void *stream)
{
    DK_REQUIRE(ybar && Ainv && nvec && y && verdict, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(tol >= 0.0f, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(nvec, 4) && dk_aligned(y, 4) &&
                   dk_aligned(verdict, 4) && (!resid || dk_aligned(resid, 4)), DK_ERR_ALIGN);
    DK_REQUIRE(G <= DK_STATIC_MAX_G && dk_ws_verify_bytes(G) <= DK_STATIC_SCRATCH_BYTES, DK_ERR_STATIC_LIMIT);
    float *part = nullptr;
    s = static_scratch(&part);
    if (s != DK_OK) return s;
    // every partial pair the second pass reads is written by the first pass of
    // the same call, so nothing of the last call's contents has to be cleared
    const bool v4 = can_vec4(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, part, v4, K, (hipStream_t)stream)
    DK_K_SWITCH(K, CALL)
#undef CALL
}
