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
        if (taps <= 9)
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
