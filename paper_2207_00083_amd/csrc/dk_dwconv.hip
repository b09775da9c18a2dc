// Depthwise convolution on encoded rows (one filter per channel): the spatial
// half of a depthwise-separable layer.  Nine multiply-adds per output against
// one element read and one written: bandwidth-bound, so no matrix cores.  The
// 3x3 kernels give a thread a tile of 4 x 4 outputs of one (image, channel)
// plane: it walks the tile's input rows once, each as one 16-byte read plus
// the border columns, and keeps the 16 results in registers, so about 9 bytes
// per output pass through the vector L1 instead of 36 and the memory pipe, not
// the L1, sets the pace.  The taps of the plane's filter sit at a wave-uniform
// address (scalar loads).  Other filter sizes take one thread per output.
// The weight gradient reduces each plane to kh*kw partial sums with one wave
// per (plane, chunk) in a fixed order, then sums the planes of a channel over
// the images.
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

// Row ih of the input window of a 4-output-wide tile: image columns
// iw0 .. iw0 + NW - 1 (zero outside the image), NW = 3*S + KW.
//
// VEC (3-wide filters with pad 1, rows of whole 16-byte vectors): the columns
// the tile's outputs sit on come as one (stride 1) or two (stride 2) aligned
// 16-byte reads, and the border column(s) are the neighbouring lane's vector
// ends, fetched by a lane shuffle -- consecutive lanes own consecutive tiles of
// a tile row -- so that a border costs no second pass through the vector L1.
// Only where the neighbouring lane holds another tile row (or nothing) is the
// border read from memory.  Every lane of the wave must call this.
template <int NW, int S, bool VEC>
__device__ __forceinline__ void dw_load_row(float (&win)[NW], const float *__restrict__ xp, int ih, int H,
                                            int W, int iw0, bool active, bool has_left, bool has_right)
{
    const bool rok = active && ih >= 0 && ih < H;
    const float *row = xp + (long long)ih * W;
    if constexpr (VEC && S == 1) {
        static_assert(!VEC || S != 1 || NW == 6, "3-wide filter");
        const int c0 = iw0 + 1;                       // first output column
        const bool vok = rok && c0 + 3 < W;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vok) v = *reinterpret_cast<const float4 *>(row + c0);
        const float lv = __shfl_up(v.w, 1, 64), rv = __shfl_down(v.x, 1, 64);
        const int lok = __shfl_up((int)vok, 1, 64), rok2 = __shfl_down((int)vok, 1, 64);
        if (vok) {
            win[1] = v.x; win[2] = v.y; win[3] = v.z; win[4] = v.w;
        } else {
#pragma unroll
            for (int j = 1; j <= 4; ++j) win[j] = (rok && iw0 + j < W) ? row[iw0 + j] : 0.0f;
        }
        // left border: column c0 - 1 (never negative when has_left)
        if (has_left && lok) win[0] = lv;
        else win[0] = (rok && iw0 >= 0) ? row[iw0] : 0.0f;
        if (has_right && rok2) win[5] = rv;
        else win[5] = (rok && iw0 + 5 < W) ? row[iw0 + 5] : 0.0f;
    } else if constexpr (VEC && S == 2) {
        static_assert(!VEC || S != 2 || NW == 9, "3-wide filter");
        const int c0 = iw0 + 1;                       // 8 * tile column
        const bool vok = rok && c0 + 7 < W;
        float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
        if (vok) {
            v0 = *reinterpret_cast<const float4 *>(row + c0);
            v1 = *reinterpret_cast<const float4 *>(row + c0 + 4);
        }
        const float lv = __shfl_up(v1.w, 1, 64);
        const int lok = __shfl_up((int)vok, 1, 64);
        if (vok) {
            win[1] = v0.x; win[2] = v0.y; win[3] = v0.z; win[4] = v0.w;
            win[5] = v1.x; win[6] = v1.y; win[7] = v1.z; win[8] = v1.w;
        } else {
#pragma unroll
            for (int j = 1; j <= 8; ++j) win[j] = (rok && iw0 + j < W) ? row[iw0 + j] : 0.0f;
        }
        if (has_left && lok) win[0] = lv;
        else win[0] = (rok && iw0 >= 0) ? row[iw0] : 0.0f;
    } else {
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int iw = iw0 + j;
            win[j] = (rok && iw >= 0 && iw < W) ? row[iw] : 0.0f;
        }
    }
}

// Forward, KH x KW filter, stride S: a thread owns outputs [oh0, oh0+4) x [ow0, ow0+4)
// of one plane.  Threads are numbered over (plane, tile row, tile column), so
// that planes with few tiles still fill their waves.
template <int KH, int KW, int S, bool VEC>
__global__ __launch_bounds__(256) void dw_fwd_tile_kernel(const float *__restrict__ Wt,
                                                          const float *__restrict__ x,
                                                          float *__restrict__ y, int C, int H, int W,
                                                          int pad, int Ho, int Wo, int tiles_w, int tiles,
                                                          long long total)
{
    constexpr int NW = 3 * S + KW, NR = 3 * S + KH;
    const long long tg = (long long)blockIdx.x * 256 + threadIdx.x;
    const bool active = tg < total;
    const long long plane = active ? tg / tiles : 0;
    const int t = active ? (int)(tg - plane * tiles) : 0;
    const int th = t / tiles_w, tw = t - th * tiles_w;
    const int oh0 = th * 4, ow0 = tw * 4;
    const int lane = threadIdx.x & 63;
    const bool has_left = lane > 0 && tw > 0;
    const bool has_right = lane < 63 && tw + 1 < tiles_w && tg + 1 < total;
    const int c = (int)(plane % C);
    float w[KH * KW];
#pragma unroll
    for (int k = 0; k < KH * KW; ++k) w[k] = Wt[(long long)c * KH * KW + k];
    const float *xp = x + plane * H * W;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
    const int ih0 = oh0 * S - pad, iw0 = ow0 * S - pad;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float win[NW];
        dw_load_row<NW, S, VEC>(win, xp, ih0 + r, H, W, iw0, active, has_left, has_right);
#pragma unroll
        for (int orow = 0; orow < 4; ++orow) {
            const int a = r - orow * S;          // filter row that input row r is for output row orow
            if (a < 0 || a >= KH) continue;
#pragma unroll
            for (int oc = 0; oc < 4; ++oc)
#pragma unroll
                for (int b = 0; b < KW; ++b)
                    acc[orow][oc] = fmaf(w[a * KW + b], win[oc * S + b], acc[orow][oc]);
        }
    }
    if (!active) return;
    float *yp = y + plane * Ho * Wo;
#pragma unroll
    for (int orow = 0; orow < 4; ++orow) {
        const int oh = oh0 + orow;
        if (oh >= Ho) continue;
        float *d = yp + (long long)oh * Wo + ow0;
        if (VEC && ow0 + 3 < Wo) {
            *reinterpret_cast<float4 *>(d) = make_float4(acc[orow][0], acc[orow][1], acc[orow][2], acc[orow][3]);
        } else {
#pragma unroll
            for (int oc = 0; oc < 4; ++oc)
                if (ow0 + oc < Wo) d[oc] = acc[orow][oc];
        }
    }
}

// Weight gradient, first pass, on the same tiles.  Large planes: one wave per
// (plane, chunk of DW_TILES_PER_CHUNK tiles), a lane takes tiles lane, lane+64,
// ... of the chunk.  Planes of at most 32 tiles: a wave takes 64/slots planes,
// slots = the tile count rounded up to a power of two, one tile per lane.
// Either way a lane keeps kh*kw sums and the lanes of a plane are combined by
// a fixed butterfly into part[plane][chunk][tap].
constexpr int DW_TILES_PER_CHUNK = 256;

template <int KH, int KW, int S, bool VEC>
__global__ __launch_bounds__(64) void dw_wgrad_tile_kernel(const float *__restrict__ dt,
                                                           const float *__restrict__ x,
                                                           float *__restrict__ part, int H, int W, int pad,
                                                           int Ho, int Wo, int tiles_w, int tiles, int chunks,
                                                           int slots, long long planes)
{
    constexpr int NW = 3 * S + KW, NR = 3 * S + KH;
    const int lane = threadIdx.x;
    const int lt = lane & (slots - 1);                    // slots = 64: the lane itself
    const long long plane_raw = (long long)blockIdx.x * (64 / slots) + lane / slots;
    const bool pok = plane_raw < planes;
    const long long plane = pok ? plane_raw : 0;
    const int chunk = blockIdx.y;
    const float *dp = dt + plane * Ho * Wo;
    const float *xp = x + plane * H * W;
    float acc[KH * KW];
#pragma unroll
    for (int k = 0; k < KH * KW; ++k) acc[k] = 0.0f;
    const int t0 = chunk * DW_TILES_PER_CHUNK;
    const int t1 = t0 + DW_TILES_PER_CHUNK < tiles ? t0 + DW_TILES_PER_CHUNK : tiles;
    for (int tb = t0; tb < t1; tb += slots) {     // wave-uniform trip count
        const int t = tb + lt;
        const bool active = pok && t < t1;
        const int tt = active ? t : t0;
        const int th = tt / tiles_w, tw = tt - th * tiles_w;
        const int oh0 = th * 4, ow0 = tw * 4;
        const bool has_left = lane > 0 && tw > 0;
        const bool has_right = lane < 63 && tw + 1 < tiles_w && t + 1 < t1;
        float d[4][4];
#pragma unroll
        for (int orow = 0; orow < 4; ++orow) {
            const int oh = oh0 + orow;
            const float *src = dp + (long long)oh * Wo + ow0;
            if (VEC && active && oh < Ho && ow0 + 3 < Wo) {
                const float4 v = *reinterpret_cast<const float4 *>(src);
                d[orow][0] = v.x; d[orow][1] = v.y; d[orow][2] = v.z; d[orow][3] = v.w;
            } else {
#pragma unroll
                for (int oc = 0; oc < 4; ++oc)
                    d[orow][oc] = (active && oh < Ho && ow0 + oc < Wo) ? src[oc] : 0.0f;
            }
        }
        const int ih0 = oh0 * S - pad, iw0 = ow0 * S - pad;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float win[NW];
            dw_load_row<NW, S, VEC>(win, xp, ih0 + r, H, W, iw0, active, has_left, has_right);
#pragma unroll
            for (int orow = 0; orow < 4; ++orow) {
                const int a = r - orow * S;
                if (a < 0 || a >= KH) continue;
#pragma unroll
                for (int oc = 0; oc < 4; ++oc)
#pragma unroll
                    for (int b = 0; b < KW; ++b)
                        acc[a * KW + b] = fmaf(d[orow][oc], win[oc * S + b], acc[a * KW + b]);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < KH * KW; ++k) {
        float v = acc[k];
        for (int off = slots >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lt == 0 && pok) part[(plane * chunks + chunk) * (KH * KW) + k] = v;
    }
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

// 3x3 filters with stride 1 or 2 run on 4x4 output tiles
static bool dw_tiled(const dk_geom &g) { return g.kh == 3 && g.kw == 3 && (g.stride == 1 || g.stride == 2); }
static int dw_tiles_w(const dk_geom &g) { return (g.Wo + 3) / 4; }
static int dw_tiles(const dk_geom &g) { return ((g.Ho + 3) / 4) * dw_tiles_w(g); }

static int dw_chunks(const dk_geom &g)
{
    if (dw_tiled(g)) return (dw_tiles(g) + DW_TILES_PER_CHUNK - 1) / DW_TILES_PER_CHUNK;
    return (g.Ho * g.Wo + 1023) / 1024;
}

size_t dk_dw_wgrad_part_bytes(const dk_geom &g, long long R)
{
    return ((size_t)R * g.Ci * dw_chunks(g) * g.kh * g.kw * sizeof(float) + 255) / 256 * 256;
}

// 16-byte accesses: pad 1, rows of whole vectors on both sides, aligned bases
static bool dw_vec(const dk_geom &g, const void *a, const void *b)
{
    return g.pad == 1 && g.W % 4 == 0 && g.Wo % 4 == 0 && dk_aligned(a, 16) && dk_aligned(b, 16);
}

dk_status dk_dw_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                        hipStream_t st)
{
    const long long planes = R * g.Ci;
    DK_REQUIRE(planes <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps("dw_fwd", st);
    if (dw_tiled(g)) {
        const int tiles = dw_tiles(g), tw = dw_tiles_w(g);
        const long long total = planes * tiles;
        DK_REQUIRE((total + 255) / 256 <= 0x7fffffffll, DK_ERR_SHAPE);
        const dim3 grid((unsigned)((total + 255) / 256));
        const bool v = dw_vec(g, xbar, ybar);
#define DK_DW_FWD(S, V)                                                                          \
        dw_fwd_tile_kernel<3, 3, S, V><<<grid, dim3(256), 0, st>>>(W, xbar, ybar, g.Ci, g.H, g.W, g.pad, g.Ho, \
                                                                   g.Wo, tw, tiles, total)
        if (g.stride == 2) { if (v) DK_DW_FWD(2, true); else DK_DW_FWD(2, false); }
        else { if (v) DK_DW_FWD(1, true); else DK_DW_FWD(1, false); }
#undef DK_DW_FWD
        return dk_launch_status();
    }
    // small planes get one-wave workgroups
    const int HoWo = g.Ho * g.Wo;
    const int bs = HoWo < 1024 ? 64 : 256;
    DK_REQUIRE((HoWo + bs - 1) / bs <= 65535, DK_ERR_SHAPE);
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
        const dim3 grid((unsigned)planes, (unsigned)chunks);
        if (dw_tiled(g)) {
            const int tiles = dw_tiles(g), tw = dw_tiles_w(g);
            int slots = 64;
            if (tiles <= 32) { slots = 1; while (slots < tiles) slots <<= 1; }
            const dim3 tgrid((unsigned)((planes + 64 / slots - 1) / (64 / slots)), (unsigned)chunks);
#define DK_DW_WG(S, V)                                                                           \
            dw_wgrad_tile_kernel<3, 3, S, V><<<tgrid, dim3(64), 0, st>>>(dtilde, xbar, part, g.H, g.W, g.pad, g.Ho, \
                                                                         g.Wo, tw, tiles, chunks, slots, planes)
            const bool v = dw_vec(g, xbar, dtilde);
            if (g.stride == 2) { if (v) DK_DW_WG(2, true); else DK_DW_WG(2, false); }
            else { if (v) DK_DW_WG(1, true); else DK_DW_WG(1, false); }
#undef DK_DW_WG
        } else {
            dw_wgrad_partial_kernel<0, 0><<<grid, dim3(64), 0, st>>>(
                dtilde, xbar, part, g.H, g.W, g.kh, g.kw, g.stride, g.pad, g.Ho, g.Wo, chunks);
        }
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
