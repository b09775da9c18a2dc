// Bandwidth-bound kernels of the masked layer: encode, decode, gradient
// mixing and the integrity check.  Every one of them is a tiny per-group
// matrix applied along the long feature axis, so the design is the same:
// one workgroup owns (group g, a contiguous span of the feature axis), the
// group's coefficients sit at a wave-uniform address (scalar loads), each lane
// moves 16-byte vectors, and every input row is read exactly once.
// Two variants of every kernel: ALIGNED (all rows start on 16-byte boundaries
// and the row length is a multiple of 4) and the general one, which moves the
// same 16-byte vectors from 4-byte-aligned addresses -- global memory accesses
// on this target need only element alignment -- and finishes the len % 4
// elements at the end of a row one by one.
#include "dk_internal.h"
#include "dk_verify_slots.h"

static int verify_max_chunks(int G);

// Scratch memory of dk_decode_verify_static (the entry point for callers that
// cannot allocate): the per-workgroup maxima of the integrity check live here instead
// of in a caller's workspace.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[DK_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MIX_THREADS = 256;

enum MixMode { MIX_ENCODE = 0, MIX_DECODE = 1, MIX_DMIX = 2 };

typedef float f4a __attribute__((ext_vector_type(4)));                 // 16-byte aligned
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));     // element aligned

// VEC = 4: one 16-byte access (AL: from a 16-byte boundary); VEC = 1: one float.
template <int VEC, bool AL>
__device__ __forceinline__ void vload(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        f4a v;
        if constexpr (AL) v = *reinterpret_cast<const f4a *>(p);
        else v = *reinterpret_cast<const f4u *>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = *p;
    }
}

// Streaming variants for data that is not touched again soon (the decoded
// outputs; the encoded results once they have been decoded).
template <int VEC, bool AL>
__device__ __forceinline__ void vload_nt(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4 && AL) {
        const f4a v = __builtin_nontemporal_load(reinterpret_cast<const f4a *>(p));
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        vload<VEC, AL>(dst, p);
    }
}

template <int VEC, bool AL>
__device__ __forceinline__ void vstore(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4) {
        const f4a v = {src[0], src[1], src[2], src[3]};
        if constexpr (AL) *reinterpret_cast<f4a *>(p) = v;
        else *reinterpret_cast<f4u *>(p) = v;
    } else {
        *p = src[0];
    }
}

template <int VEC, bool AL>
__device__ __forceinline__ void vstore_nt(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4 && AL) {
        const f4a v = {src[0], src[1], src[2], src[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<f4a *>(p));
    } else {
        vstore<VEC, AL>(p, src);
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
template <int MODE, int K, bool AL, bool FULL>
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

    // one position of the feature axis: VEC elements starting at e
    auto body = [&](auto vec_tag, long long e) {
        constexpr int VEC = decltype(vec_tag)::value;
        float x[NIN][VEC];
#pragma unroll
        for (int i = 0; i < NIN; ++i) vload<VEC, AL>(x[i], src[i] + e);
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
            vstore<VEC, AL>(dst + (long long)o * len + e, acc);
        }
    };

    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += MIX_THREADS) body(std::integral_constant<int, 4>{}, v * 4);
    if constexpr (!AL) {
        // the len % 4 elements behind the last whole vector
        const long long e = nvec * 4 + threadIdx.x;
        if (chunk == chunks - 1 && e < len) body(std::integral_constant<int, 1>{}, e);
    }
}

// One position of the feature axis in the integrity sums: updates the running
// maxima with VEC elements of t = sum_j n_j y_j and s = sum_j |n_j y_j|.
template <int S, int VEC>
__device__ __forceinline__ void verify_accumulate(const float (&nv)[S], const float (&x)[S][VEC],
                                                  float &tmax, float &smax, bool &bad)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        float t = 0.0f, sc = 0.0f;
#pragma unroll
        for (int j = 0; j < S; ++j) {
            const float pr = nv[j] * x[j][c];
            t += pr;
            sc += fabsf(pr);
        }
        // a NaN or infinity anywhere makes s non-finite (or t, via inf-inf)
        bad |= !(sc <= 3.402823466e+38f) || !(fabsf(t) <= 3.402823466e+38f);
        tmax = fmaxf(tmax, fabsf(t));
        smax = fmaxf(smax, sc);
    }
}

// The integrity check alone.
template <int K, bool AL>
__global__ __launch_bounds__(MIX_THREADS) void verify_kernel(
    const float *__restrict__ ybar, const float *__restrict__ nvec_, dk_verify_slot *__restrict__ slots,
    long long len, long long nvec, int chunks, long long span, unsigned long long tag, float tol,
    int *__restrict__ verdict, float *__restrict__ resid)
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
        float x[S][4];
#pragma unroll
        for (int j = 0; j < S; ++j) vload<4, AL>(x[j], src + (long long)j * len + v * 4);
        verify_accumulate<S, 4>(nv, x, tmax, smax, bad);
    }
    if constexpr (!AL) {
        const long long e = nvec * 4 + threadIdx.x;
        if (chunk == chunks - 1 && e < len) {
            float x[S][1];
#pragma unroll
            for (int j = 0; j < S; ++j) x[j][0] = src[(long long)j * len + e];
            verify_accumulate<S, 1>(nv, x, tmax, smax, bad);
        }
    }
    dk_verify_publish_and_finish<MIX_THREADS>(tmax, smax, bad, slots, g, chunk, chunks, tag, tol, verdict, resid);
}

// Decode and the integrity check in one sweep over ybar: both need every
// encoded row of the group exactly once.
// (FULL = false: only the first nk of the template's K columns are outputs,
// see mix_kernel.)
template <int K, bool AL, bool FULL>
__global__ __launch_bounds__(MIX_THREADS) void decode_verify_kernel(
    const float *__restrict__ ybar, const float *__restrict__ Ainv, const float *__restrict__ nvec_,
    float *__restrict__ y, dk_verify_slot *__restrict__ slots, long long len, long long nvec, int chunks,
    long long span, int nk_rt, unsigned long long tag, float tol, int *__restrict__ verdict,
    float *__restrict__ resid)
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
    auto body = [&](auto vec_tag, long long e) {
        constexpr int VEC = decltype(vec_tag)::value;
        float x[S][VEC];
#pragma unroll
        for (int j = 0; j < S; ++j) vload_nt<VEC, AL>(x[j], src + (long long)j * len + e);
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
            vstore_nt<VEC, AL>(dst + (long long)i * len + e, acc);
        }
        verify_accumulate<S, VEC>(nv, x, tmax, smax, bad);
    };
    const long long v0 = (long long)chunk * span;
    long long v1 = v0 + span;
    if (v1 > nvec) v1 = nvec;
    for (long long v = v0 + threadIdx.x; v < v1; v += MIX_THREADS) body(std::integral_constant<int, 4>{}, v * 4);
    if constexpr (!AL) {
        const long long e = nvec * 4 + threadIdx.x;
        if (chunk == chunks - 1 && e < len) body(std::integral_constant<int, 1>{}, e);
    }
    dk_verify_publish_and_finish<MIX_THREADS>(tmax, smax, bad, slots, g, chunk, chunks, tag, tol, verdict, resid);
}

struct span_plan {
    long long nvec;   // whole 16-byte vectors per row (the len % 4 elements behind them go one by one)
    long long span;   // vectors per workgroup (multiple of MIX_THREADS)
    int chunks;       // workgroups per group
};

// Each lane moves `iters` vectors; spans shrink until the launch has
// `min_blocks` workgroups: a few thousand for the plain mixing kernels (256
// compute units, several resident groups each); a thousand for the kernels that
// end with the integrity check's publish-and-look (two memory round trips per
// workgroup, which a one-vector-per-lane workgroup cannot amortise: config 2
// measured 0.0385 ms at 4096 workgroups, 0.030 ms at 1024).
span_plan plan_span(long long len, int G, int max_chunks, long long min_blocks = 4096)
{
    span_plan p;
    p.nvec = len / 4;
    long long iters = 4;
    while (iters > 1 && (long long)G * ((p.nvec + MIX_THREADS * iters - 1) / (MIX_THREADS * iters)) < min_blocks)
        iters >>= 1;
    p.span = MIX_THREADS * iters;
    long long chunks = (p.nvec + p.span - 1) / p.span;
    if (chunks < 1) chunks = 1;               // rows shorter than one vector: the tail only
    if (max_chunks > 0 && chunks > max_chunks) {
        chunks = max_chunks;
        p.span = ((p.nvec + chunks - 1) / chunks + MIX_THREADS - 1) / MIX_THREADS * MIX_THREADS;
        chunks = (p.nvec + p.span - 1) / p.span;
    }
    p.chunks = (int)chunks;
    return p;
}

// The kernels that end with the integrity check.  With many virtual batches a
// thousand workgroups of several vectors per lane amortise the in-kernel verdict
// (two memory round trips per workgroup; config 2: 0.0385 ms at 4096 workgroups,
// 0.030 ms at 1024, 0.034 ms with the verdict in a second launch).  With few
// batches that would put hundreds of workgroups on one batch: then the spans
// stay short (more, shorter workgroups balance better) and a second launch
// takes the verdict.
span_plan plan_verify_span(long long len, int G)
{
    span_plan p = plan_span(len, G, verify_max_chunks(G), 1024);
    if (p.chunks > DK_VERIFY_INLINE_MAX_CHUNKS) p = plan_span(len, G, verify_max_chunks(G), 4096);
    return p;
}

// Rows of whole 16-byte vectors, all starting on 16-byte boundaries.
bool aligned16(long long len, std::initializer_list<const void *> ptrs)
{
    if (len % 4) return false;
    for (const void *p : ptrs)
        if (p && !dk_aligned(p, 16)) return false;
    return true;
}

template <int MODE, int K>
dk_status launch_mix_k(const float *in0, const float *in1, const float *c0, const float *c1,
                       float *out, int G, long long len, bool al, int nk, hipStream_t st)
{
    const span_plan p = plan_span(len, G, 0);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps(MODE == MIX_ENCODE ? "encode" : (MODE == MIX_DECODE ? "decode" : "delta_mix"), st);
#define DK_MIX_LAUNCH(AL, F)                                                                    \
    mix_kernel<MODE, K, AL, F><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(               \
        in0, in1, c0, c1, out, len, p.nvec, p.chunks, p.span, nk)
    if (nk == K) {
        if (al) DK_MIX_LAUNCH(true, true); else DK_MIX_LAUNCH(false, true);
    } else {
        if (al) DK_MIX_LAUNCH(true, false); else DK_MIX_LAUNCH(false, false);
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
                     float *out, int G, int K, int M, long long len, bool al, hipStream_t st)
{
#define CALL(KK) launch_mix_k<MODE, KK>(in0, in1, c0, c1, out, G, len, al, K, st)
    DK_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

template <int K>
dk_status launch_verify_k(const float *ybar, const float *nvec, float tol, int *verdict,
                          float *resid, int G, long long len, dk_verify_slot *slots, bool al, hipStream_t st)
{
    const span_plan p = plan_verify_span(len, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const bool in_kernel = p.chunks <= DK_VERIFY_INLINE_MAX_CHUNKS;
    const unsigned long long tag = in_kernel ? dk_next_verify_tag() : 0ull;
    {
        dk_prof_scope ps("verify", st);
        if (al)
            verify_kernel<K, true><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(
                ybar, nvec, slots, len, p.nvec, p.chunks, p.span, tag, tol, verdict, resid);
        else
            verify_kernel<K, false><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(
                ybar, nvec, slots, len, p.nvec, p.chunks, p.span, tag, tol, verdict, resid);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    return in_kernel ? DK_OK : dk_verify_finalize(slots, p.chunks, tol, verdict, resid, G, st);
}

template <int K>
dk_status launch_decode_verify_k(const float *ybar, const float *Ainv, const float *nvec, float tol,
                                 float *y, int *verdict, float *resid, int G, long long len,
                                 dk_verify_slot *slots, bool al, int nk, hipStream_t st)
{
    const span_plan p = plan_verify_span(len, G);
    const long long blocks = (long long)G * p.chunks;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const bool in_kernel = p.chunks <= DK_VERIFY_INLINE_MAX_CHUNKS;
    const unsigned long long tag = in_kernel ? dk_next_verify_tag() : 0ull;
    {
    dk_prof_scope ps("decode_verify", st);
#define DK_DV_LAUNCH(AL, F)                                                                      \
    decode_verify_kernel<K, AL, F><<<dim3((unsigned)blocks), dim3(MIX_THREADS), 0, st>>>(           \
        ybar, Ainv, nvec, y, slots, len, p.nvec, p.chunks, p.span, nk, tag, tol, verdict, resid)
    if (nk == K) {
        if (al) DK_DV_LAUNCH(true, true); else DK_DV_LAUNCH(false, true);
    } else {
        if (al) DK_DV_LAUNCH(true, false); else DK_DV_LAUNCH(false, false);
    }
#undef DK_DV_LAUNCH
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    return in_kernel ? DK_OK : dk_verify_finalize(slots, p.chunks, tol, verdict, resid, G, st);
}

dk_status check_mix_args(int G, int K, long long len)
{
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && len >= 1, DK_ERR_SHAPE);
    DK_REQUIRE((long long)G * (K + 2) <= 0x7fffffffll, DK_ERR_SHAPE);
    DK_REQUIRE(len <= (1ll << 40), DK_ERR_SHAPE);
    return DK_OK;
}

} // namespace

// The tag of one integrity-check call: distinct from every tag this process
// drew before and never 0 (an odd multiple walked through a 64-bit mixer).
unsigned long long dk_next_verify_tag()
{
    static std::atomic<unsigned long long> counter{0x2207000830001ull};
    unsigned long long z = counter.fetch_add(0x9e3779b97f4a7c15ull, std::memory_order_relaxed);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return z | 1ull;
}

namespace {
// One wave per virtual batch folds the batch's slots -- lane c takes slots c,
// c + 64, ... -- and lane 0 takes the verdict.
__global__ __launch_bounds__(MIX_THREADS) void verify_final_kernel(
    const dk_verify_slot *__restrict__ slots, int chunks, float tol, int *__restrict__ verdict,
    float *__restrict__ resid, int G)
{
    const int g = blockIdx.x * (MIX_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (g >= G) return;
    float tmax = 0.0f, smax = 0.0f;
    for (int c = lane; c < chunks; c += 64) {
        tmax = fmaxf(tmax, __uint_as_float((unsigned)slots[(long long)g * chunks + c].t_word));
        smax = fmaxf(smax, __uint_as_float((unsigned)slots[(long long)g * chunks + c].s_word));
    }
    tmax = dk_wave_max(tmax);
    smax = dk_wave_max(smax);
    if (lane != 0) return;
    const bool bad = !(tmax <= 3.402823466e+38f);
    const float rho = bad ? __builtin_inff() : (smax > 0.0f ? tmax / smax : 0.0f);
    verdict[g] = (bad || rho > tol) ? 1 : 0;
    if (resid) resid[g] = rho;
}
} // namespace

dk_status dk_verify_finalize(const dk_verify_slot *slots, int chunks, float tol, int *verdict, float *resid,
                             int G, hipStream_t st)
{
    dk_prof_scope ps("verify_final", st);
    verify_final_kernel<<<dim3((G + MIX_THREADS / 64 - 1) / (MIX_THREADS / 64)), dim3(MIX_THREADS), 0, st>>>(
        slots, chunks, tol, verdict, resid, G);
    return dk_launch_status();
}

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
    return (size_t)G * verify_max_chunks(G) * 16;       // one dk_verify_slot per (group, workgroup)
}

DK_EXPORT dk_status dk_encode(const float *x, const float *r, const float *A, float *xbar,
                              int G, int K, long long n, void *stream)
{
    DK_REQUIRE(x && r && A && xbar, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, n);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(x, 4) && dk_aligned(r, 4) && dk_aligned(A, 4) && dk_aligned(xbar, 4), DK_ERR_ALIGN);
    return launch_mix<MIX_ENCODE>(x, r, A, nullptr, xbar, G, K, 1, n, aligned16(n, {x, r, xbar}),
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
    return launch_mix<MIX_ENCODE>(x, r, A, nullptr, xbar, G, K, M, n, aligned16(n, {x, r, xbar}),
                                  (hipStream_t)stream);
}

DK_EXPORT dk_status dk_decode(const float *ybar, const float *Ainv, float *y, int G, int K,
                              long long m, void *stream)
{
    DK_REQUIRE(ybar && Ainv && y, DK_ERR_NULL);
    dk_status s = check_mix_args(G, K, m);
    if (s != DK_OK) return s;
    DK_REQUIRE(dk_aligned(ybar, 4) && dk_aligned(Ainv, 4) && dk_aligned(y, 4), DK_ERR_ALIGN);
    return launch_mix<MIX_DECODE>(ybar, nullptr, Ainv, nullptr, y, G, K, 1, m, aligned16(m, {ybar, y}),
                                  (hipStream_t)stream);
}

// Gradient mixing used by dk_wgrad: dtilde[gS+j] = gamma[g][j] sum_i B[g][j][i] delta[gK+i],
// S = K + M + 1.
dk_status dk_delta_mix(const float *delta, const float *B, const float *gamma, float *dtilde,
                       int G, int K, int M, long long m, hipStream_t st)
{
    return launch_mix<MIX_DMIX>(delta, nullptr, B, gamma, dtilde, G, K, M, m,
                                aligned16(m, {delta, dtilde}), st);
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
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    const bool al = aligned16(m, {ybar});
#define CALL(KK) launch_verify_k<KK>(ybar, nvec, tol, verdict, resid, G, m, (dk_verify_slot *)ws, al, (hipStream_t)stream)
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
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    const bool al = aligned16(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, (dk_verify_slot *)ws, al, K, (hipStream_t)stream)
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
    DK_REQUIRE(dk_aligned(ws, 16), DK_ERR_ALIGN);
    const bool al = aligned16(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, (dk_verify_slot *)ws, al, K, (hipStream_t)stream)
    DK_K_SWITCH(K + M - 1, CALL)
#undef CALL
}

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<dk_verify_slot *> scratch_ptr[MAX_DEVICES];       // device address of `scratch`, per device ordinal

// The current device's copy of the scratch array.  Looked up once per device
// (with that device current); no allocation, no stream operation.
dk_status static_scratch(dk_verify_slot **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DK_ERR_HIP;
    DK_REQUIRE(dev >= 0 && dev < MAX_DEVICES, DK_ERR_UNSUPPORTED);
    dk_verify_slot *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return DK_ERR_HIP;
        p = static_cast<dk_verify_slot *>(q);
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
    dk_verify_slot *part = nullptr;
    s = static_scratch(&part);
    if (s != DK_OK) return s;
    // a slot counts only with this call's tag and the finishing workgroup
    // resets the tags, so nothing of the last call's contents has to be cleared
    const bool al = aligned16(m, {ybar, y});
#define CALL(KK) launch_decode_verify_k<KK>(ybar, Ainv, nvec, tol, y, verdict, resid, G, m, part, al, K, (hipStream_t)stream)
    DK_K_SWITCH(K, CALL)
#undef CALL
}
