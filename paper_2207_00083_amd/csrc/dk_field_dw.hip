// Finite-field variant of the depthwise convolution (one filter per channel:
// the spatial half of a depthwise-separable layer) and of the layer bias.
// A few multiply-adds per element moved, so these are plain bandwidth-bound
// kernels on the vector ALUs: products of two field elements are below 2^50,
// at most 49 (forward: the taps) or 32 (weight gradient: pixels between two
// reductions) of them are summed in 64 bits and reduced once by folding with
// 2^25 = 39 (mod p), which takes values below 2^56.
#include "dk_field.h"

namespace {

constexpr int DT = 256;

__device__ __forceinline__ uint32_t fe_in(uint32_t v) { return v >= DKF_P ? v % DKF_P : v; }

// y[s][c][h][w] = sum_{a,b} W[c][a][b] x[s][c][h*st+a-pad][w*st+b-pad]  (mod p);
// one thread per output element, consecutive threads along the row.
__global__ __launch_bounds__(DT) void f_dw_fwd_kernel(const uint32_t *__restrict__ W,
                                                      const uint32_t *__restrict__ x,
                                                      uint32_t *__restrict__ y, long long total, int C,
                                                      int H, int Wd, int kh, int kw, int stride, int pad,
                                                      int Ho, int Wo)
{
    const long long idx = (long long)blockIdx.x * DT + threadIdx.x;
    if (idx >= total) return;
    const int HoWo = Ho * Wo;
    const long long rc = idx / HoWo;
    const int px = (int)(idx - rc * HoWo);
    const int h = px / Wo, w = px - h * Wo;
    const int c = (int)(rc % C);
    const uint32_t *img = x + rc * H * Wd;
    const uint32_t *f = W + (long long)c * kh * kw;
    uint64_t acc = 0;                                   // at most 49 products
    for (int a = 0; a < kh; ++a) {
        const int ih = h * stride + a - pad;
        if ((unsigned)ih >= (unsigned)H) continue;
        for (int b = 0; b < kw; ++b) {
            const int iw = w * stride + b - pad;
            if ((unsigned)iw >= (unsigned)Wd) continue;
            acc += (uint64_t)fe_in(f[a * kw + b]) * fe_in(img[ih * Wd + iw]);
        }
    }
    y[idx] = dkf_reduce(acc);
}

// part[chunk][c][tap] = sum over the chunk's images and all pixels of
// dtilde[s][c][h][w] x[s][c][h*st+a-pad][w*st+b-pad]  (mod p).
// blockIdx.x = channel, blockIdx.y = chunk of images; a thread walks pixels
// DT apart and keeps one 64-bit sum per tap, reduced every 32 terms.
template <int TAPS_MAX>
__global__ __launch_bounds__(DT) void f_dw_wgrad_kernel(const uint32_t *__restrict__ d,
                                                        const uint32_t *__restrict__ x,
                                                        uint32_t *__restrict__ part, int R, int C, int H,
                                                        int Wd, int kh, int kw, int stride, int pad, int Ho,
                                                        int Wo, int imgs_per_chunk)
{
    const int c = blockIdx.x, chunk = blockIdx.y;
    const int taps = kh * kw;
    const int s0 = chunk * imgs_per_chunk;
    int s1 = s0 + imgs_per_chunk;
    if (s1 > R) s1 = R;
    const int HoWo = Ho * Wo;
    uint64_t acc[TAPS_MAX];
#pragma unroll
    for (int t = 0; t < TAPS_MAX; ++t) acc[t] = 0;
    int since = 0;
    for (int s = s0; s < s1; ++s) {
        const uint32_t *dp = d + ((long long)s * C + c) * HoWo;
        const uint32_t *img = x + ((long long)s * C + c) * H * Wd;
        for (int px = threadIdx.x; px < HoWo; px += DT) {
            const int h = px / Wo, w = px - h * Wo;
            const uint64_t dv = fe_in(dp[px]);
#pragma unroll
            for (int t = 0; t < TAPS_MAX; ++t) {
                if (t >= taps) break;
                const int a = t / kw, b = t - a * kw;
                const int ih = h * stride + a - pad, iw = w * stride + b - pad;
                if ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)Wd)
                    acc[t] += dv * fe_in(img[ih * Wd + iw]);
            }
            if (++since == 32) {
                since = 0;
#pragma unroll
                for (int t = 0; t < TAPS_MAX; ++t) acc[t] = dkf_reduce(acc[t]);
            }
        }
    }
    // 256 residues below 2^25 sum to less than 2^33: 64-bit adds, one reduction
    __shared__ uint64_t red[DT / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < TAPS_MAX; ++t) {
        if (t >= taps) break;                            // workgroup-uniform
        uint64_t v = dkf_reduce(acc[t]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        __syncthreads();
        if (lane == 0) red[wave] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t sum = 0;
#pragma unroll
            for (int wv = 0; wv < DT / 64; ++wv) sum += red[wv];
            part[((long long)chunk * C + c) * taps + t] = dkf_reduce(sum);
        }
    }
}

// ---- square filters of edge 3, 5, 7: no division per tap, none in 64 bits ----
//
// The kernels above spend their time on index arithmetic (64-bit divisions per output, a
// division per tap).  Here the filter edge is a template parameter, a pixel index splits
// into (row, column) by one multiplication with ceil(2^32 / Wo) (exact below 2^16), planes
// come from the grid, and the taps are unrolled with their offsets as constants.  One output
// (one pixel) per thread, consecutive threads on consecutive pixels: the loads of a tap are
// then coalesced, and the kernels run at about 2 TB/s, bound by the nine loads per output
// through the vector cache.  (Four outputs per thread with the input row read once per
// thread measured slower: the lanes' scalar loads are then 16 bytes apart.  The fp32 kernels'
// answer -- aligned 16-byte loads and the border columns from the neighbouring lane -- is
// not built for the field elements.)

// blockIdx.x = block of 256 consecutive (plane-local) slots, blockIdx.y + 32768 blockIdx.z =
// plane group; a group is `ppb` whole planes when a plane has fewer than 256 outputs.
template <int KS>
__global__ __launch_bounds__(DT) void f_dw_fwd_sq_kernel(const uint32_t *__restrict__ W,
                                                         const uint32_t *__restrict__ x,
                                                         uint32_t *__restrict__ y, int planes, int C, int H,
                                                         int Wd, int stride, int pad, int Ho, int Wo,
                                                         unsigned wo_magic, int ppb, unsigned howo_magic)
{
    const int HoWo = Ho * Wo;
    const int group = blockIdx.y + 32768 * blockIdx.z;
    int slot = blockIdx.x * DT + threadIdx.x;
    int plane = group * ppb;
    if (ppb > 1) {                                   // several small planes per workgroup
        const int lp = (int)__umulhi((unsigned)slot, howo_magic);
        plane += lp;
        slot -= lp * HoWo;
        if (lp >= ppb) return;
    }
    if (plane >= planes || slot >= HoWo) return;
    const int h = (int)__umulhi((unsigned)slot, wo_magic), w = slot - h * Wo;
    const int c = plane % C;
    const uint32_t *f = W + (long long)c * (KS * KS);
    const uint32_t *img = x + (long long)plane * H * Wd;
    const int ih0 = h * stride - pad, iw0 = w * stride - pad;
    uint64_t acc = 0;                                // at most 49 products below 2^50
#pragma unroll
    for (int a = 0; a < KS; ++a) {
        const int ih = ih0 + a;
        const bool rok = (unsigned)ih < (unsigned)H;
#pragma unroll
        for (int b = 0; b < KS; ++b) {
            const int iw = iw0 + b;
            const bool ok = rok && (unsigned)iw < (unsigned)Wd;
            const uint32_t xv = ok ? img[ih * Wd + iw] : 0u;
            acc += (uint64_t)f[a * KS + b] * xv;
        }
    }
    y[(long long)plane * HoWo + slot] = dkf_reduce(acc);
}

// blockIdx.x = channel, blockIdx.y = chunk of images: as f_dw_wgrad_kernel, taps unrolled.
// SMALL: planes with fewer pixels than the workgroup has threads.
template <int KS, bool SMALL>
__global__ __launch_bounds__(DT) void f_dw_wgrad_sq_kernel(const uint32_t *__restrict__ d,
                                                           const uint32_t *__restrict__ x,
                                                           uint32_t *__restrict__ part, int R, int C, int H,
                                                           int Wd, int stride, int pad, int Ho, int Wo,
                                                           unsigned wo_magic, unsigned howo_magic,
                                                           int imgs_per_chunk)
{
    constexpr int TAPS = KS * KS;
    const int c = blockIdx.x, chunk = blockIdx.y;
    const int s0 = chunk * imgs_per_chunk;
    int s1 = s0 + imgs_per_chunk;
    if (s1 > R) s1 = R;
    const int HoWo = Ho * Wo;
    uint64_t acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) acc[t] = 0;
    int since = 0;
    // planes smaller than the workgroup: its threads spread over several images at once
    const int nb = SMALL ? 65535 / HoWo : 1;             // images per pass (their pixels below 2^16)
    for (int sb = s0; sb < s1; sb += nb) {
        const int imgs = s1 - sb < nb ? s1 - sb : nb;
        for (int e = threadIdx.x; e < imgs * HoWo; e += DT) {
            const int si = SMALL ? (int)__umulhi((unsigned)e, howo_magic) : 0, px = e - si * HoWo;
            const uint32_t *dp = d + ((long long)(sb + si) * C + c) * HoWo;
            const uint32_t *img = x + ((long long)(sb + si) * C + c) * H * Wd;
            const int h = (int)__umulhi((unsigned)px, wo_magic), w = px - h * Wo;
            const int ih0 = h * stride - pad, iw0 = w * stride - pad;
            const uint64_t dv = dp[px];
#pragma unroll
            for (int a = 0; a < KS; ++a) {
                const int ih = ih0 + a;
                const bool rok = (unsigned)ih < (unsigned)H;
#pragma unroll
                for (int b = 0; b < KS; ++b) {
                    const int iw = iw0 + b;
                    const bool ok = rok && (unsigned)iw < (unsigned)Wd;
                    const uint32_t xv = ok ? img[ih * Wd + iw] : 0u;
                    acc[a * KS + b] += dv * xv;
                }
            }
            if (++since == 32) {                     // 32 products below 2^50 on top of a residue
                since = 0;
#pragma unroll
                for (int t = 0; t < TAPS; ++t) acc[t] = dkf_reduce(acc[t]);
            }
        }
    }
    __shared__ uint64_t red[DT / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
        uint64_t v = dkf_reduce(acc[t]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        __syncthreads();
        if (lane == 0) red[wave] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t sum = 0;
#pragma unroll
            for (int wv = 0; wv < DT / 64; ++wv) sum += red[wv];
            part[((long long)chunk * C + c) * TAPS + t] = dkf_reduce(sum);
        }
    }
}

// dWq[e] = sum_chunk part[chunk][e] (mod p); dW = (accumulate ? dW : 0) + scale * dequant.
__global__ __launch_bounds__(DT) void f_dw_fold_kernel(const uint32_t *__restrict__ part, int chunks, int count,
                                                       uint32_t *__restrict__ dwq, float *__restrict__ dW,
                                                       double s_inv, float scale, int accumulate)
{
    const int e = blockIdx.x * DT + threadIdx.x;
    if (e >= count) return;
    uint64_t sum = 0;
    for (int k = 0; k < chunks; ++k) {
        sum += part[(long long)k * count + e];
        if ((k & 1023) == 1023) sum = dkf_reduce(sum);
    }
    const uint32_t q = dkf_reduce(sum);
    if (dwq) dwq[e] = q;
    const float v = scale * dkf_dequant(q, s_inv);
    dW[e] = accumulate ? dW[e] + v : v;
}

// yq[row][e] += b_q[e / per] (mod p), y = dequant(yq); b_q = Field(Round(b 2^{2l})).
__global__ __launch_bounds__(DT) void f_add_bias_kernel(uint32_t *__restrict__ yq, float *__restrict__ y,
                                                        const float *__restrict__ bias, long long total,
                                                        long long m, long long per, double s2, double s_inv)
{
    const long long idx = (long long)blockIdx.x * DT + threadIdx.x;
    if (idx >= total) return;
    const long long e = idx % m;
    const uint32_t bq = dkf_quant(bias[e / per], s2);
    uint32_t v = fe_in(yq[idx]) + bq;
    if (v >= DKF_P) v -= DKF_P;
    yq[idx] = v;
    if (y) y[idx] = dkf_dequant(v, s_inv);
}

// filter edge 3, 5 or 7 on both sides and rows of at least two outputs: the unrolled kernels
bool sq_edge(const dk_geom &g) { return g.kh == g.kw && (g.kh == 3 || g.kh == 5 || g.kh == 7) && g.Wo >= 2; }

// ceil(2^32 / d) for d >= 2: x / d = umulhi(x, magic) for x < 2^16
unsigned magic(int d) { return (unsigned)((0x100000000ull + (unsigned)d - 1) / (unsigned)d); }

int dw_chunks(const dk_geom &g, long long R)
{
    // enough workgroups for the chip, whole images per chunk
    long long want = (1024 + g.Ci - 1) / g.Ci;
    if (want > R) want = R;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    const long long per = (R + want - 1) / want;
    return (int)((R + per - 1) / per);
}

} // namespace

size_t dkf_dw_wgrad_part_bytes(const dk_geom &g, long long R)
{
    return ((size_t)dw_chunks(g, R) * g.Ci * g.kh * g.kw * sizeof(uint32_t) + 255) / 256 * 256;
}

dk_status dkf_dw_fwd_run(const dk_geom &g, const uint32_t *Wq, const uint32_t *xbar, uint32_t *ybar,
                         long long R, hipStream_t st)
{
    const long long total = R * g.m;
    DK_REQUIRE((total + DT - 1) / DT <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("f_dw_fwd", st);
    const int HoWo = g.Ho * g.Wo;
    const long long planes = R * g.Ci;
    if (sq_edge(g) && HoWo < 65536 && planes < (1ll << 30)) {
        const int ppb = HoWo >= DT ? 1 : DT / HoWo;
        const long long groups = (planes + ppb - 1) / ppb;
        const dim3 grid((unsigned)(ppb > 1 ? 1 : (HoWo + DT - 1) / DT), (unsigned)(groups < 32768 ? groups : 32768),
                        (unsigned)((groups + 32767) / 32768));
        const unsigned wo_magic = magic(g.Wo), howo_magic = magic(HoWo);
#define DKF_DW_FWD(KS)                                                                                \
        f_dw_fwd_sq_kernel<KS><<<grid, dim3(DT), 0, st>>>(Wq, xbar, ybar, (int)planes, g.Ci, g.H, g.W, g.stride, \
                                                          g.pad, g.Ho, g.Wo, wo_magic, ppb, howo_magic)
        if (g.kh == 3) DKF_DW_FWD(3); else if (g.kh == 5) DKF_DW_FWD(5); else DKF_DW_FWD(7);
#undef DKF_DW_FWD
        return dk_launch_status();
    }
    f_dw_fwd_kernel<<<dim3((unsigned)((total + DT - 1) / DT)), dim3(DT), 0, st>>>(
        Wq, xbar, ybar, total, g.Ci, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    return dk_launch_status();
}

dk_status dkf_dw_wgrad_run(const dk_geom &g, const uint32_t *dtilde, const uint32_t *xbar, float *dW,
                           uint32_t *dwq, long long R, int l, float scale, int accumulate, uint32_t *part,
                           hipStream_t st)
{
    const int chunks = dw_chunks(g, R);
    const int per = (int)((R + chunks - 1) / chunks);
    const int taps = g.kh * g.kw;
    DK_REQUIRE(g.Ci <= 0x7fffffff && chunks <= 65535, DK_ERR_SHAPE);
    {
        dk_prof_scope ps("f_dw_wgrad", st);
        const dim3 grid((unsigned)g.Ci, (unsigned)chunks);
        if (sq_edge(g) && g.Ho * g.Wo < 65536) {
            const unsigned wo_magic = magic(g.Wo);
#define DKF_DW_WG(KS)                                                                                 \
            do {                                                                                      \
                if (g.Ho * g.Wo < DT)                                                                 \
                    f_dw_wgrad_sq_kernel<KS, true><<<grid, dim3(DT), 0, st>>>(                        \
                        dtilde, xbar, part, (int)R, g.Ci, g.H, g.W, g.stride, g.pad, g.Ho, g.Wo, wo_magic, \
                        magic(g.Ho * g.Wo), per);                                                     \
                else                                                                                  \
                    f_dw_wgrad_sq_kernel<KS, false><<<grid, dim3(DT), 0, st>>>(                       \
                        dtilde, xbar, part, (int)R, g.Ci, g.H, g.W, g.stride, g.pad, g.Ho, g.Wo, wo_magic, 0u, per); \
            } while (0)
            if (g.kh == 3) DKF_DW_WG(3); else if (g.kh == 5) DKF_DW_WG(5); else DKF_DW_WG(7);
#undef DKF_DW_WG
        } else if (taps <= 9)
            f_dw_wgrad_kernel<9><<<grid, dim3(DT), 0, st>>>(dtilde, xbar, part, (int)R, g.Ci, g.H, g.W, g.kh, g.kw,
                                                            g.stride, g.pad, g.Ho, g.Wo, per);
        else if (taps <= 25)
            f_dw_wgrad_kernel<25><<<grid, dim3(DT), 0, st>>>(dtilde, xbar, part, (int)R, g.Ci, g.H, g.W, g.kh, g.kw,
                                                             g.stride, g.pad, g.Ho, g.Wo, per);
        else
            f_dw_wgrad_kernel<49><<<grid, dim3(DT), 0, st>>>(dtilde, xbar, part, (int)R, g.Ci, g.H, g.W, g.kh, g.kw,
                                                             g.stride, g.pad, g.Ho, g.Wo, per);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    const int count = g.Ci * taps;
    dk_prof_scope ps("f_dw_fold", st);
    f_dw_fold_kernel<<<dim3((count + DT - 1) / DT), dim3(DT), 0, st>>>(part, chunks, count, dwq, dW,
                                                                       ldexp(1.0, -l), scale, accumulate);
    return dk_launch_status();
}

DK_EXPORT dk_status dkf_add_bias(uint32_t *yq, float *y, const float *bias, long long rows, long long m,
                                 long long per, int l, void *stream)
{
    DK_REQUIRE(yq && bias, DK_ERR_NULL);
    DK_REQUIRE(rows >= 1 && m >= 1 && per >= 1 && m % per == 0 && rows <= (1ll << 40) / m, DK_ERR_SHAPE);
    DK_REQUIRE(l >= 0 && l <= DKF_MAX_L, DK_ERR_SHAPE);
    DK_REQUIRE(dk_aligned(yq, 4) && dk_aligned(bias, 4) && (!y || dk_aligned(y, 4)), DK_ERR_ALIGN);
    const long long total = rows * m;
    DK_REQUIRE((total + DT - 1) / DT <= 0x7fffffffll, DK_ERR_SHAPE);
    hipStream_t st = (hipStream_t)stream;
    dk_prof_scope ps("f_add_bias", st);
    f_add_bias_kernel<<<dim3((unsigned)((total + DT - 1) / DT)), dim3(DT), 0, st>>>(
        yq, y, bias, total, m, per, ldexp(1.0, 2 * l), ldexp(1.0, -l));
    return dk_launch_status();
}
