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

// One thread per output element of one (image, channel) plane, consecutive
// lanes on consecutive elements, so stores and the bulk of the loads are
// coalesced; the plane is workgroup-uniform, so the filter taps come through
// scalar loads.  KH = KW = 0 selects the run-time filter size.
template <int KH, int KW>
__global__ void dw_fwd_kernel(const float *__restrict__ Wt, const float *__restrict__ x,
                              float *__restrict__ y, int C, int H, int W, int kh_rt, int kw_rt,
                              int stride, int pad, int Ho, int Wo)
{
    const int kh = KH ? KH : kh_rt, kw = KW ? KW : kw_rt;
    const long long plane = blockIdx.x;
    const int px = blockIdx.y * blockDim.x + threadIdx.x;
    const int HoWo = Ho * Wo;
    if (px >= HoWo) return;
    const int oh = px / Wo, ow = px - oh * Wo;
    const int c = (int)(plane % C);
    const float *wc = Wt + (long long)c * kh * kw;
    const float *xp = x + plane * H * W;
    const int ih0 = oh * stride - pad, iw0 = ow * stride - pad;
    float acc = 0.0f;
#pragma unroll
    for (int a = 0; a < (KH ? KH : DW_MAXK); ++a) {
        if (!KH && a >= kh) break;
        const int ih = ih0 + a;
#pragma unroll
        for (int b = 0; b < (KW ? KW : DW_MAXK); ++b) {
            if (!KW && b >= kw) break;
            const int iw = iw0 + b;
            const bool in = ih >= 0 && ih < H && iw >= 0 && iw < W;
            acc = fmaf(wc[a * kw + b], in ? xp[ih * W + iw] : 0.0f, acc);
        }
    }
    y[plane * HoWo + px] = acc;
}

// part[plane][chunk][tap] = sum over the chunk's pixels of
// dtilde[plane][px] * x[plane][px shifted by the tap]; one wave per (plane,
// chunk of up to 1024 pixels), lanes on consecutive pixels, fixed order.
template <int KH, int KW>
__global__ __launch_bounds__(64) void dw_wgrad_partial_kernel(const float *__restrict__ dt,
                                                              const float *__restrict__ x,
                                                              float *__restrict__ part, int H, int W, int kh_rt,
                                                              int kw_rt, int stride, int pad, int Ho, int Wo,
                                                              int chunks)
{
    const int kh = KH ? KH : kh_rt, kw = KW ? KW : kw_rt;
    constexpr int AH = KH ? KH : DW_MAXK, AW = KW ? KW : DW_MAXK;
    const long long plane = blockIdx.x;
    const int chunk = blockIdx.y;
    const int lane = threadIdx.x;
    const int HoWo = Ho * Wo, taps = kh * kw;
    const float *dp = dt + plane * HoWo;
    const float *xp = x + plane * H * W;
    float acc[AH * AW];
#pragma unroll
    for (int t = 0; t < AH * AW; ++t) acc[t] = 0.0f;
    const int p0 = chunk * 1024;
    const int p1 = p0 + 1024 < HoWo ? p0 + 1024 : HoWo;
    for (int px = p0 + lane; px < p1; px += 64) {
        const int oh = px / Wo, ow = px - oh * Wo;
        const float d = dp[px];
#pragma unroll
        for (int a = 0; a < AH; ++a) {
            if (!KH && a >= kh) break;
            const int ih = oh * stride + a - pad;
#pragma unroll
            for (int b = 0; b < AW; ++b) {
                if (!KW && b >= kw) break;
                const int iw = ow * stride + b - pad;
                const bool in = ih >= 0 && ih < H && iw >= 0 && iw < W;
                acc[a * AW + b] = fmaf(d, in ? xp[ih * W + iw] : 0.0f, acc[a * AW + b]);
            }
        }
    }
#pragma unroll
    for (int a = 0; a < AH; ++a) {
        if (!KH && a >= kh) break;
#pragma unroll
        for (int b = 0; b < AW; ++b) {
            if (!KW && b >= kw) break;
            float v = acc[a * AW + b];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0) part[(plane * chunks + chunk) * taps + a * kw + b] = v;
        }
    }
}

// dW[c][tap] = (accumulate ? dW : 0) + scale * sum_{r, chunk} part[r][c][chunk][tap]:
// one wave per (channel, tap); lane l adds entries l, l+64, ... of the
// (image, chunk) list in order, then the 64 sub-sums are combined by a fixed
// butterfly, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void dw_wgrad_fold_kernel(const float *__restrict__ part,
                                                            float *__restrict__ dW, int R, int C, int chunks,
                                                            int taps, float scale, int accumulate)
{
    const int e = blockIdx.x * 4 + (threadIdx.x >> 6);  // (channel, tap)
    const int lane = threadIdx.x & 63;
    if (e >= C * taps) return;
    const int c = e / taps, t = e - c * taps;
    const int n = R * chunks;
    float s = 0.0f;
    for (int i = lane; i < n; i += 64) {
        const int r = i / chunks, q = i - r * chunks;
        s += part[(((long long)r * C + c) * chunks + q) * taps + t];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) dW[e] = accumulate ? dW[e] + scale * s : scale * s;
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

static int dw_chunks(const dk_geom &g) { return (g.Ho * g.Wo + 1023) / 1024; }

size_t dk_dw_wgrad_part_bytes(const dk_geom &g, long long R)
{
    return ((size_t)R * g.Ci * dw_chunks(g) * g.kh * g.kw * sizeof(float) + 255) / 256 * 256;
}

dk_status dk_dw_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                        hipStream_t st)
{
    // small planes get one-wave workgroups
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll, DK_ERR_SHAPE);
    const int HoWo = g.Ho * g.Wo;
    const int bs = HoWo < 1024 ? 64 : 256;
    DK_REQUIRE((HoWo + bs - 1) / bs <= 65535, DK_ERR_SHAPE);
    dk_prof_scope ps("dw_fwd", st);
    if (g.kh == 3 && g.kw == 3)
        dw_fwd_kernel<3, 3><<<dim3((unsigned)planes, (HoWo + bs - 1) / bs), dim3(bs), 0, st>>>(
            W, xbar, ybar, g.Ci, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    else
        dw_fwd_kernel<0, 0><<<dim3((unsigned)planes, (HoWo + bs - 1) / bs), dim3(bs), 0, st>>>(
            W, xbar, ybar, g.Ci, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo);
    return dk_launch_status();
}

dk_status dk_dw_wgrad_run(const dk_geom &g, const float *dtilde, const float *xbar, float *dW, long long R,
                          float scale, int accumulate, float *part, hipStream_t st)
{
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll && R <= 0x7fffffffll, DK_ERR_SHAPE);
    const int chunks = dw_chunks(g);
    DK_REQUIRE(chunks <= 65535, DK_ERR_SHAPE);
    {
        dk_prof_scope ps("dw_wgrad_partial", st);
        if (g.kh == 3 && g.kw == 3)
            dw_wgrad_partial_kernel<3, 3><<<dim3((unsigned)planes, (unsigned)chunks), dim3(64), 0, st>>>(
                dtilde, xbar, part, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo, chunks);
        else
            dw_wgrad_partial_kernel<0, 0><<<dim3((unsigned)planes, (unsigned)chunks), dim3(64), 0, st>>>(
                dtilde, xbar, part, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo, chunks);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    const int taps = g.kh * g.kw;
    dk_prof_scope ps("dw_wgrad_fold", st);
    dw_wgrad_fold_kernel<<<dim3((g.Ci * taps + 3) / 4), dim3(256), 0, st>>>(part, dW, (int)R, g.Ci, chunks,
                                                                            taps, scale, accumulate);
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
