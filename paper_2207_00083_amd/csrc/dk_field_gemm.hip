// Finite-field variant: the dense contractions  C[i][j] = sum_k A[i][k] B[j][k]
// (mod p) on the int8 matrix cores.
//
// A field element is first lifted to its centred representative in
// (-p/2, p/2) and written as four balanced base-128 digits,
//     v = e0 + 128 e1 + 128^2 e2 + 128^3 e3,   e0..e2 in [-64, 63], |e3| <= 8,
// one int8 plane per digit.  A product of two elements is then the sum of 16
// digit products weighted by 128^(a+b).  The digits of each operand are taken
// in two halves ("low" = digits 0,1; "high" = digits 2,3); one part of a launch
// multiplies one half of A with one half of B and keeps one int32 accumulator
// per weight 128^s, s = 0..2 (more accumulators than that do not fit the 256
// accumulation registers of a wave with a 64 x 64 tile).  An accumulator holds
// at most two digit products per k, each at most 2^12 in magnitude, so 2^17
// values of k fit with room to spare.  The epilogue recombines the three
// accumulators in 64 bits, reduces modulo p and applies the part's weight
// 128^(2 (ha + hb)).  The four parts are sets of workgroups of one launch; a part
// that involves a high half whose digits are all zero (quantised weights of
// ordinary magnitude) exits at once: the digit kernels record that in device
// flags, so nothing is read back to the host.  Partial results (parts, k
// slices) are residues and are folded by modular addition.  All of it is exact:
// the result is the field product whatever the tiling.
//
// The contraction index has to be contiguous for both operands; digit planes
// are written k-major by the digit kernels (straight for row-major operands,
// through an LDS transpose for the weight gradient, whose contraction index is
// the encoded-row index).
#include "dk_field.h"

namespace {

constexpr int BI = 128, BJ = 128;      // workgroup tile
constexpr int KT = 128;                // k bytes per LDS tile
constexpr int PITCH = 144;             // LDS row pitch in bytes: 16 (mod 32) keeps 16-byte reads conflict-free
constexpr int A_PLANE = BI * PITCH, B_PLANE = BJ * PITCH;
constexpr int BUF_BYTES = 2 * A_PLANE + 2 * B_PLANE;     // 73728
constexpr int LDS_BYTES = 2 * BUF_BYTES;                  // 147456
constexpr int MAX_KSPLIT = 1 << 17;    // k values per slice (int32 accumulators)
constexpr int MAX_SPLITS = 16;         // the fold adds at most 4 * 16 residues in 32 bits

struct fgemm_params {
    const int8_t *Ap;      // [4][I_pad][Kp]
    const int8_t *Bp;      // [4][J_pad][Kp]
    uint32_t *part;        // [4][splits][I][J]
    const int *flags;      // [0]: A has non-zero high digits, [1]: B has (device)
    long long a_plane, b_plane;   // bytes per plane
    int I, J, Kp;
    int tiles_i, tiles_j, splits, ktiles_per_split, ktiles;
};

// Four balanced base-128 digits of the centred lift of q, packed one per byte.
__device__ __forceinline__ uint32_t digits_of(uint32_t q)
{
    int w = (int)q;
    if (q > DKF_P / 2) w -= (int)DKF_P;
    const int e0 = ((w + 64) & 127) - 64;
    w = (w - e0) >> 7;
    const int e1 = ((w + 64) & 127) - 64;
    w = (w - e1) >> 7;
    const int e2 = ((w + 64) & 127) - 64;
    const int e3 = (w - e2) >> 7;
    return (uint32_t)(e0 & 255) | (uint32_t)(e1 & 255) << 8 | (uint32_t)(e2 & 255) << 16 |
           (uint32_t)(e3 & 255) << 24;
}

// byte `a` of four packed-digit words -> one word of plane a
__device__ __forceinline__ uint32_t gather_byte(const uint32_t (&d)[4], int a)
{
    const int sh = 8 * a;
    return ((d[0] >> sh) & 255u) | ((d[1] >> sh) & 255u) << 8 | ((d[2] >> sh) & 255u) << 16 |
           ((d[3] >> sh) & 255u) << 24;
}

// Row-major operand src[rows][K] -> planes[4][rows_pad][Kp].  One thread per
// four consecutive k; rows and k beyond the operand are written as zeros.
__global__ __launch_bounds__(256) void f_digits_kernel(const uint32_t *__restrict__ src,
                                                       int8_t *__restrict__ planes, int rows, int K,
                                                       int rows_pad, int Kp, int *flag)
{
    const int kq = Kp >> 2;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)rows_pad * kq) return;
    const int row = (int)(id / kq), k0 = (int)(id - (long long)row * kq) * 4;
    uint32_t d[4] = {0, 0, 0, 0};
    if (row < rows) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (k0 + c < K) d[c] = digits_of(src[(long long)row * K + k0 + c]);
    }
    const long long plane = (long long)rows_pad * Kp;
    uint32_t hi = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const uint32_t w = gather_byte(d, a);
        if (a >= 2) hi |= w;
        *reinterpret_cast<uint32_t *>(planes + a * plane + (long long)row * Kp + k0) = w;
    }
    if (flag && __any(hi != 0) && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}

// Operand stored with the contraction index slow, src[K][cols] ->
// planes[4][cols_pad][Kp]: a 64 x 64 tile goes through LDS as packed digits.
__global__ __launch_bounds__(256) void f_digits_t_kernel(const uint32_t *__restrict__ src,
                                                         int8_t *__restrict__ planes, int K, int cols,
                                                         int cols_pad, int Kp, int *flag)
{
    __shared__ uint32_t tile[64][65];
    const int c0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int k = k0 + ty + 4 * r, c = c0 + tx;
        tile[ty + 4 * r][tx] = (k < K && c < cols) ? digits_of(src[(long long)k * cols + c]) : 0u;
    }
    __syncthreads();
    const long long plane = (long long)cols_pad * Kp;
    uint32_t hi = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int item = threadIdx.x + 256 * r;       // (col, k group of four)
        const int kg = item & 15, col = item >> 4;
        uint32_t d[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) d[c] = tile[4 * kg + c][col];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint32_t w = gather_byte(d, a);
            if (a >= 2) hi |= w;
            *reinterpret_cast<uint32_t *>(planes + a * plane + (long long)(c0 + col) * Kp + k0 + 4 * kg) = w;
        }
    }
    if (flag && __any(hi != 0) && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}

__global__ void f_flag_clear_kernel(int *flags) { if (threadIdx.x < 2) flags[threadIdx.x] = 0; }

// |v| < 2^62 -> v mod p in [0, p)
__device__ __forceinline__ uint32_t reduce_signed(long long v)
{
    const bool neg = v < 0;
    const uint64_t m = neg ? (uint64_t)(-v) : (uint64_t)v;
    const uint64_t t = (m >> 25) * 39u + (m & 0x1ffffffu);     // < 2^43
    const uint32_t r = dkf_reduce(t);
    return (neg && r) ? DKF_P - r : r;
}

__global__ __launch_bounds__(256) void f_gemm_kernel(fgemm_params p)
{
    extern __shared__ __attribute__((aligned(16))) int8_t flds[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_i * p.tiles_j;
    int bid = dk_xcd_block();
    const int part = bid / (tiles * p.splits);
    bid -= part * tiles * p.splits;
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tj = t / p.tiles_i, ti = t - tj * p.tiles_i;
    const int ha = part & 1, hb = part >> 1;
    if ((ha && p.flags[0] == 0) || (hb && p.flags[1] == 0)) return;      // workgroup-uniform

    const int kt0 = split * p.ktiles_per_split;
    int kt1 = kt0 + p.ktiles_per_split;
    if (kt1 > p.ktiles) kt1 = p.ktiles;

    // global -> register staging: 8 + 8 sixteen-byte pieces per thread and tile.
    // A thread owns one 16-byte column of the 128-byte rows (piece tid & 7) and
    // rows (tid >> 3) + 32 q, q = 0..3, of both planes of both operands.
    const int srow = tid >> 3, spiece = tid & 7;
    const int8_t *a_src = p.Ap + 2 * ha * p.a_plane + (long long)(ti * BI + srow) * p.Kp + 16 * spiece;
    const int8_t *b_src = p.Bp + 2 * hb * p.b_plane + (long long)(tj * BJ + srow) * p.Kp + 16 * spiece;
    const long long q_rows = 32ll * p.Kp;
    const int s_dst = srow * PITCH + 16 * spiece;

    i32x16 acc[2][2][3];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[bi][bj][s][v] = 0;

    const int wi0 = (wave & 1) * 64, wj0 = (wave >> 1) * 64;
    const int a_rd = (wi0 + li) * PITCH + 16 * lh;
    const int b_rd = 2 * A_PLANE + (wj0 + li) * PITCH + 16 * lh;

    i32x4 sa[8], sb[8];
#define DKF_FETCH(KTILE)                                                                          \
    {                                                                                             \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                             \
            sa[e] = *reinterpret_cast<const i32x4 *>(a_src + (e >> 2) * p.a_plane + (e & 3) * q_rows + (long long)(KTILE) * KT); \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                             \
            sb[e] = *reinterpret_cast<const i32x4 *>(b_src + (e >> 2) * p.b_plane + (e & 3) * q_rows + (long long)(KTILE) * KT); \
    }
#define DKF_STASH(BUF)                                                                            \
    {                                                                                             \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                             \
            *reinterpret_cast<i32x4 *>((BUF) + (e >> 2) * A_PLANE + (e & 3) * 32 * PITCH + s_dst) = sa[e]; \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                             \
            *reinterpret_cast<i32x4 *>((BUF) + 2 * A_PLANE + (e >> 2) * B_PLANE + (e & 3) * 32 * PITCH + s_dst) = sb[e]; \
    }
    if (kt0 < kt1) {
        DKF_FETCH(kt0)
        DKF_STASH(flds)
    }
    __syncthreads();

    for (int kt = kt0; kt < kt1; ++kt) {
        const int8_t *cur = flds + ((kt - kt0) & 1) * BUF_BYTES;
        int8_t *nxt = flds + ((kt - kt0 + 1) & 1) * BUF_BYTES;
        const bool more = kt + 1 < kt1;
        if (more) DKF_FETCH(kt + 1)
#pragma unroll
        for (int ks = 0; ks < KT / 32; ++ks) {
            i32x4 a[2][2], b[2][2];
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl)
                    a[bi][pl] = *reinterpret_cast<const i32x4 *>(cur + pl * A_PLANE + a_rd + bi * 32 * PITCH + ks * 32);
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl)
                    b[bj][pl] = *reinterpret_cast<const i32x4 *>(cur + pl * B_PLANE + b_rd + bj * 32 * PITCH + ks * 32);
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                    for (int pa = 0; pa < 2; ++pa)
#pragma unroll
                        for (int pb = 0; pb < 2; ++pb)
                            acc[bi][bj][pa + pb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                a[bi][pa], b[bj][pb], acc[bi][bj][pa + pb], 0, 0, 0);
        }
        if (more) DKF_STASH(nxt)
        __syncthreads();
    }
#undef DKF_FETCH
#undef DKF_STASH

    // recombine the three weights in 64 bits, reduce, apply the part's weight
    uint32_t *dst = p.part + ((long long)part * p.splits + split) * p.I * p.J;
    const int wshift = 14 * (ha + hb);
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int j = tj * BJ + wj0 + bj * 32 + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = ti * BI + wi0 + bi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                long long val = 0;
#pragma unroll
                for (int s = 0; s < 3; ++s) val += (long long)acc[bi][bj][s][v] << (7 * s);
                const uint32_t r = dkf_reduce((uint64_t)reduce_signed(val) << wshift);   // < 2^53
                if (i < p.I && j < p.J) dst[(long long)i * p.J + j] = r;
            }
        }
}

// Number of residue slices to add and where they are: part q of the launch is
// present when the high halves it uses are non-zero.
__device__ __forceinline__ uint32_t fold_slices(const uint32_t *__restrict__ part,
                                                const int *__restrict__ flags, long long elems,
                                                long long e, int splits)
{
    const bool fa = flags[0] != 0, fb = flags[1] != 0;
    uint32_t s = 0;                          // at most 4 * 16 residues below 2^25
    for (int q = 0; q < 4; ++q) {
        if (((q & 1) && !fa) || ((q >> 1) && !fb)) continue;
        for (int k = 0; k < splits; ++k) s += part[((long long)q * splits + k) * elems + e];
    }
    return dkf_reduce(s);
}

__global__ __launch_bounds__(256) void f_fold_kernel(const uint32_t *__restrict__ part,
                                                     const int *__restrict__ flags,
                                                     uint32_t *__restrict__ out, long long elems,
                                                     int splits)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= elems) return;
    out[e] = fold_slices(part, flags, elems, e, splits);
}

// Same fold for the weight gradient, followed by de-quantisation:
// dW = (accumulate ? dW : 0) + scale * Round(lift(dWq) * 2^-l) * 2^-l.
__global__ __launch_bounds__(256) void f_fold_dw_kernel(const uint32_t *__restrict__ part,
                                                        const int *__restrict__ flags,
                                                        float *__restrict__ dW, uint32_t *__restrict__ dwq,
                                                        long long elems, int splits, double s_inv,
                                                        float scale, int accumulate)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= elems) return;
    const uint32_t q = fold_slices(part, flags, elems, e, splits);
    if (dwq) dwq[e] = q;
    const float v = scale * dkf_dequant(q, s_inv);
    dW[e] = accumulate ? dW[e] + v : v;
}

inline int round_up(int v, int a) { return (v + a - 1) / a * a; }
inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct fgemm_plan {
    int I, J, K, I_pad, J_pad, Kp;
    int tiles_i, tiles_j, ktiles, splits, ktiles_per_split;
    size_t a_bytes, b_bytes, part_bytes;
};

// I, J: output dimensions; K: contraction length.
bool plan_fgemm(long long I, long long J, long long K, fgemm_plan *pl)
{
    if (I < 1 || J < 1 || K < 1 || I > (1 << 24) || J > (1 << 24) || K > (1 << 28)) return false;
    pl->I = (int)I; pl->J = (int)J; pl->K = (int)K;
    pl->I_pad = round_up((int)I, BI);
    pl->J_pad = round_up((int)J, BJ);
    pl->Kp = round_up((int)K, KT);
    pl->tiles_i = pl->I_pad / BI;
    pl->tiles_j = pl->J_pad / BJ;
    pl->ktiles = pl->Kp / KT;
    const long long tiles = (long long)pl->tiles_i * pl->tiles_j;
    if (tiles > (1 << 24)) return false;
    // enough workgroups to fill 256 compute units twice over, slices short
    // enough for the int32 accumulators, not more slices than the fold sums
    long long splits = 1;
    if (tiles < 512) splits = (512 + tiles - 1) / tiles;
    const long long need = ((long long)pl->Kp + MAX_KSPLIT - 1) / MAX_KSPLIT;
    if (splits < need) splits = need;
    if (splits > pl->ktiles) splits = pl->ktiles;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    int per = (int)((pl->ktiles + splits - 1) / splits);
    if ((long long)per * KT > MAX_KSPLIT) return false;
    pl->ktiles_per_split = per;
    pl->splits = (pl->ktiles + per - 1) / per;
    pl->a_bytes = align256((size_t)4 * pl->I_pad * pl->Kp);
    pl->b_bytes = align256((size_t)4 * pl->J_pad * pl->Kp);
    pl->part_bytes = align256((size_t)4 * pl->splits * (size_t)I * (size_t)J * sizeof(uint32_t));
    return true;
}

constexpr size_t FLAG_BYTES = 256;

dk_status run_fgemm(const fgemm_plan &pl, const int8_t *Ap, const int8_t *Bp, uint32_t *part,
                    const int *flags, hipStream_t st)
{
    static bool allowed = false;
    if (!allowed) {
        DK_REQUIRE(hipFuncSetAttribute(reinterpret_cast<const void *>(f_gemm_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) == hipSuccess,
                   DK_ERR_HIP);
        allowed = true;
    }
    fgemm_params p;
    p.Ap = Ap; p.Bp = Bp; p.part = part; p.flags = flags;
    p.a_plane = (long long)pl.I_pad * pl.Kp;
    p.b_plane = (long long)pl.J_pad * pl.Kp;
    p.I = pl.I; p.J = pl.J; p.Kp = pl.Kp;
    p.tiles_i = pl.tiles_i; p.tiles_j = pl.tiles_j; p.splits = pl.splits;
    p.ktiles_per_split = pl.ktiles_per_split; p.ktiles = pl.ktiles;
    const long long blocks = 4ll * pl.splits * pl.tiles_i * pl.tiles_j;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("f_gemm", st);
    f_gemm_kernel<<<dim3((unsigned)blocks), dim3(256), LDS_BYTES, st>>>(p);
    return dk_launch_status();
}

dk_status run_digits(const uint32_t *src, int8_t *planes, int rows, int K, int rows_pad, int Kp,
                     int *flag, hipStream_t st)
{
    const long long items = (long long)rows_pad * (Kp / 4);
    dk_prof_scope ps("f_digits", st);
    f_digits_kernel<<<dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st>>>(src, planes, rows, K,
                                                                                rows_pad, Kp, flag);
    return dk_launch_status();
}

dk_status run_digits_t(const uint32_t *src, int8_t *planes, int K, int cols, int cols_pad, int Kp,
                       int *flag, hipStream_t st)
{
    dk_prof_scope ps("f_digits_t", st);
    f_digits_t_kernel<<<dim3(cols_pad / 64, Kp / 64), dim3(256), 0, st>>>(src, planes, K, cols, cols_pad,
                                                                        Kp, flag);
    return dk_launch_status();
}

} // namespace

DK_EXPORT size_t dkf_fwd_workspace_bytes(int M, int N, int R)
{
    fgemm_plan pl;
    if (!plan_fgemm(R, M, N, &pl)) return 0;
    return FLAG_BYTES + pl.a_bytes + pl.b_bytes + pl.part_bytes;
}

DK_EXPORT size_t dkf_wgrad_workspace_bytes(const dk_layer *L, int G, int K)
{
    dk_geom g;
    if (dk_layer_geom(L, &g) != DK_OK || g.conv) return 0;
    if (G < 1 || K < 1 || K > DK_MAX_K) return 0;
    const long long R = (long long)G * (K + 2);
    fgemm_plan pl;
    if (!plan_fgemm(g.M, g.N, R, &pl)) return 0;
    return FLAG_BYTES + align256((size_t)R * g.M * sizeof(uint32_t)) + pl.a_bytes + pl.b_bytes + pl.part_bytes;
}

DK_EXPORT dk_status dkf_linear_fwd(const uint32_t *Wq, const uint32_t *xbar, uint32_t *ybar,
                                   int M, int N, int R, void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(Wq && xbar && ybar, DK_ERR_NULL);
    DK_REQUIRE(M >= 1 && N >= 1 && R >= 1, DK_ERR_SHAPE);
    fgemm_plan pl;
    DK_REQUIRE(plan_fgemm(R, M, N, &pl), DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(Wq, 4) && dk_aligned(xbar, 4) && dk_aligned(ybar, 4), DK_ERR_ALIGN);
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
    s = run_digits(Wq, Bp, M, N, pl.J_pad, pl.Kp, flag + 1, st);
    if (s != DK_OK) return s;
    s = run_fgemm(pl, Ap, Bp, part, flag, st);
    if (s != DK_OK) return s;
    const long long elems = (long long)R * M;
    dk_prof_scope ps("f_fold", st);
    f_fold_kernel<<<dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st>>>(part, flag, ybar, elems, pl.splits);
    return dk_launch_status();
}

DK_EXPORT dk_status dkf_wgrad(const dk_layer *L, const float *delta, const uint32_t *B,
                              const uint32_t *gamma, const uint32_t *xbar, float *dW, uint32_t *dwq,
                              int G, int K, int l, float scale, int accumulate,
                              void *ws, size_t ws_bytes, void *stream)
{
    DK_REQUIRE(L && delta && B && gamma && xbar && dW, DK_ERR_NULL);
    dk_geom g;
    const dk_status gs = dk_layer_geom(L, &g);
    if (gs != DK_OK) return gs;
    DK_REQUIRE(!g.conv, DK_ERR_UNSUPPORTED);
    DK_REQUIRE(G >= 1 && K >= 1 && K <= DK_MAX_K && l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    const long long R = (long long)G * (K + 2);
    fgemm_plan pl;
    DK_REQUIRE(plan_fgemm(g.M, g.N, R, &pl), DK_ERR_SHAPE);
    DK_REQUIRE(pl.Kp / 64 <= 65535, DK_ERR_SHAPE);          // grid.y of the transposing digit kernel
    DK_REQUIRE(dk_aligned(delta, 4) && dk_aligned(B, 4) && dk_aligned(gamma, 4) && dk_aligned(xbar, 4) &&
                   dk_aligned(dW, 4) && (!dwq || dk_aligned(dwq, 4)), DK_ERR_ALIGN);
    const size_t dt_bytes = align256((size_t)R * g.M * sizeof(uint32_t));
    DK_REQUIRE(ws && ws_bytes >= FLAG_BYTES + dt_bytes + pl.a_bytes + pl.b_bytes + pl.part_bytes, DK_ERR_WORKSPACE);
    DK_REQUIRE(dk_aligned(ws, 256), DK_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;

    char *w = (char *)ws;
    int *flag = (int *)w;                          w += FLAG_BYTES;
    uint32_t *dtilde = (uint32_t *)w;              w += dt_bytes;
    int8_t *Ap = (int8_t *)w;                      w += pl.a_bytes;
    int8_t *Bp = (int8_t *)w;                      w += pl.b_bytes;
    uint32_t *part = (uint32_t *)w;

    dk_status s = dkf_delta_mix(delta, B, gamma, dtilde, G, K, g.M, l, st);
    if (s != DK_OK) return s;
    {
        dk_prof_scope ps("f_flag_clear", st);
        f_flag_clear_kernel<<<dim3(1), dim3(64), 0, st>>>(flag);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    // the contraction index is the encoded row: both operands are transposed
    s = run_digits_t(dtilde, Ap, (int)R, g.M, pl.I_pad, pl.Kp, flag, st);
    if (s != DK_OK) return s;
    s = run_digits_t(xbar, Bp, (int)R, g.N, pl.J_pad, pl.Kp, flag + 1, st);
    if (s != DK_OK) return s;
    s = run_fgemm(pl, Ap, Bp, part, flag, st);
    if (s != DK_OK) return s;
    const long long elems = (long long)g.M * g.N;
    dk_prof_scope ps("f_fold_dw", st);
    f_fold_dw_kernel<<<dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st>>>(
        part, flag, dW, dwq, elems, pl.splits, ldexp(1.0, -l), scale, accumulate);
    return dk_launch_status();
}
