// Depthwise convolution on encoded rows (one filter per channel): the spatial
// half of a depthwise-separable layer.  Nine multiply-adds per output against
// one element read and one written: bandwidth-bound, so no matrix cores and no
// LDS staging -- a thread produces four neighbouring outputs of one
// (image, channel) plane, the taps of the plane's filter sit at a wave-uniform
// address, and the overlapping input reads are served by the vector L1.
// The weight gradient reduces each plane to kh*kw partial sums with one wave
// per plane (fixed order), then sums the planes of a channel over the images.
#include "dk_internal.h"

namespace {

constexpr int DW_MAXK = 7;     // largest filter edge

__global__ __launch_bounds__(256) void dw_fwd_kernel(const float *__restrict__ Wt, const float *__restrict__ x,
                                                     float *__restrict__ y, int C, int H, int W, int kh,
                                                     int kw, int stride, int pad, int Ho, int Wo)
{
    const long long plane = blockIdx.x;                 // (image, channel), workgroup-uniform
    const int c = (int)(plane % C);
    const int HoWo = Ho * Wo;
    const int px0 = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (px0 >= HoWo) return;
    const float *wc = Wt + (long long)c * kh * kw;
    const float *xp = x + plane * H * W;
    float *yp = y + plane * HoWo;
    int oh = px0 / Wo, ow = px0 - oh * Wo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (px0 + q >= HoWo) break;
        float acc = 0.0f;
        for (int a = 0; a < kh; ++a) {
            const int ih = oh * stride + a - pad;
            if (ih < 0 || ih >= H) continue;
            for (int b = 0; b < kw; ++b) {
                const int iw = ow * stride + b - pad;
                if (iw < 0 || iw >= W) continue;
                acc = fmaf(wc[a * kw + b], xp[ih * W + iw], acc);
            }
        }
        yp[px0 + q] = acc;
        if (++ow == Wo) { ow = 0; ++oh; }
    }
}

// part[plane][tap] = sum_px dtilde[plane][px] * x[plane][px shifted by the tap]
__global__ __launch_bounds__(64) void dw_wgrad_partial_kernel(const float *__restrict__ dt,
                                                              const float *__restrict__ x,
                                                              float *__restrict__ part, int H, int W, int kh,
                                                              int kw, int stride, int pad, int Ho, int Wo)
{
    const long long plane = blockIdx.x;
    const int lane = threadIdx.x;
    const int HoWo = Ho * Wo, taps = kh * kw;
    const float *dp = dt + plane * HoWo;
    const float *xp = x + plane * H * W;
    float acc[DW_MAXK * DW_MAXK];
#pragma unroll
    for (int t = 0; t < DW_MAXK * DW_MAXK; ++t) acc[t] = 0.0f;
    for (int px = lane; px < HoWo; px += 64) {
        const int oh = px / Wo, ow = px - oh * Wo;
        const float d = dp[px];
#pragma unroll
        for (int a = 0; a < DW_MAXK; ++a) {
            if (a >= kh) break;
            const int ih = oh * stride + a - pad;
#pragma unroll
            for (int b = 0; b < DW_MAXK; ++b) {
                if (b >= kw) break;
                const int iw = ow * stride + b - pad;
                const bool in = ih >= 0 && ih < H && iw >= 0 && iw < W;
                acc[a * DW_MAXK + b] = fmaf(d, in ? xp[ih * W + iw] : 0.0f, acc[a * DW_MAXK + b]);
            }
        }
    }
#pragma unroll
    for (int a = 0; a < DW_MAXK; ++a) {
        if (a >= kh) break;
#pragma unroll
        for (int b = 0; b < DW_MAXK; ++b) {
            if (b >= kw) break;
            float v = acc[a * DW_MAXK + b];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0) part[plane * taps + a * kw + b] = v;
        }
    }
}

// dW[c][tap] = (accumulate ? dW : 0) + scale * sum_r part[r][c][tap], images in order
__global__ __launch_bounds__(256) void dw_wgrad_fold_kernel(const float *__restrict__ part,
                                                            float *__restrict__ dW, int R, int per_image,
                                                            float scale, int accumulate)
{
    const int e = blockIdx.x * 256 + threadIdx.x;       // (channel, tap)
    if (e >= per_image) return;
    float s = 0.0f;
    for (int r = 0; r < R; ++r) s += part[(long long)r * per_image + e];
    dW[e] = accumulate ? dW[e] + scale * s : scale * s;
}

// Data gradient of the depthwise layer (un-encoded): the transpose of the
// forward map, dx[plane][i][j] = sum_{a,b} d[plane][(i+pad-a)/stride][(j+pad-b)/stride] w[a][b]
// over the taps for which both quotients are whole and inside the output.
__global__ __launch_bounds__(256) void dw_dgrad_kernel(const float *__restrict__ Wt, const float *__restrict__ d,
                                                       float *__restrict__ dx, int C, int H, int W, int kh,
                                                       int kw, int stride, int pad, int Ho, int Wo)
{
    const long long plane = blockIdx.x;
    const int c = (int)(plane % C);
    const int px = blockIdx.y * 256 + threadIdx.x;
    if (px >= H * W) return;
    const int i = px / W, j = px - i * W;
    const float *wc = Wt + (long long)c * kh * kw;
    const float *dp = d + plane * Ho * Wo;
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
            acc = fmaf(dp[h * Wo + w], wc[a * kw + b], acc);
        }
    }
    dx[plane * H * W + px] = acc;
}

} // namespace

bool dk_dw_supported(const dk_geom &g) { return g.kh <= DW_MAXK && g.kw <= DW_MAXK; }

size_t dk_dw_wgrad_part_bytes(const dk_geom &g, long long R)
{
    return ((size_t)R * g.Ci * g.kh * g.kw * sizeof(float) + 255) / 256 * 256;
}

dk_status dk_dw_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                        hipStream_t st)
{
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll, DK_ERR_SHAPE);
    const int HoWo = g.Ho * g.Wo;
    dk_prof_scope ps("dw_fwd", st);
    dw_fwd_kernel<<<dim3((unsigned)planes, (unsigned)((HoWo + 1023) / 1024)), dim3(256), 0, st>>>(
        W, xbar, ybar, g.Ci, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    return dk_launch_status();
}

dk_status dk_dw_wgrad_run(const dk_geom &g, const float *dtilde, const float *xbar, float *dW, long long R,
                          float scale, int accumulate, float *part, hipStream_t st)
{
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll && R <= 0x7fffffffll, DK_ERR_SHAPE);
    {
        dk_prof_scope ps("dw_wgrad_partial", st);
        dw_wgrad_partial_kernel<<<dim3((unsigned)planes), dim3(64), 0, st>>>(
            dtilde, xbar, part, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    const int per_image = g.Ci * g.kh * g.kw;
    dk_prof_scope ps("dw_wgrad_fold", st);
    dw_wgrad_fold_kernel<<<dim3((per_image + 255) / 256), dim3(256), 0, st>>>(part, dW, (int)R, per_image,
                                                                          scale, accumulate);
    return dk_launch_status();
}

dk_status dk_dw_dgrad_run(const dk_geom &g, const float *W, const float *delta, float *dx, long long R,
                          hipStream_t st)
{
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("dw_dgrad", st);
    dw_dgrad_kernel<<<dim3((unsigned)planes, (unsigned)((g.H * g.W + 255) / 256)), dim3(256), 0, st>>>(
        W, delta, dx, g.Ci, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    return dk_launch_status();
}
