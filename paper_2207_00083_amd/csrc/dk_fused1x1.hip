// Fused forms of the masked layer for 1x1 convolutions (stride 1, no padding),
// where a virtual batch's K + 2 encodings are K + 2 independent products of the
// same filter matrix with [Ci][HW] images and the mixing steps around them move
// more bytes than the products themselves (K = 8, few channels, large images):
//
//  * forward + decode + integrity check: a workgroup owns a (filter tile x
//    pixel tile) of ONE virtual batch, runs the product for the batch's
//    encodings one after the other and folds each result tile straight into
//    the K decoded tiles and the two integrity sums it keeps in registers.
//    The encoded results never reach memory.
//  * weight gradient with the gradient mixing in its operand loader: the
//    contraction axis is walked as (virtual batch, 16-pixel chunk, encoding);
//    the K gradient tiles of a chunk are fetched once, and for each of the
//    K + 2 encodings the mixed tile is formed from them in registers on its way
//    to LDS.  The mixed gradients never reach memory.
//
// Both run on the same fp32 MFMA tile engine as the unfused kernels (operands
// k-major in LDS, register-staged double buffering, buffer loads with a scalar
// step offset and one precomputed lane offset per vector).
#include "dk_internal.h"
#include "dk_verify_slots.h"

namespace {

#include "dk_contract_tiles.h"

// ---------------------------------------------------------------------------
// forward + decode + verify
// ---------------------------------------------------------------------------

struct fused_fwd_params {
    const float *W, *xbar, *Ainv, *nvec;
    float *y;
    dk_verify_slot *slots;
    int *verdict;
    float *resid;
    int Co, Ci, HW, G;
    int tiles_m, tiles_n;          // filter tiles, pixel tiles of one image
    unsigned long long tag;
    float tol;
};

using FwdCfg = Cfg<64, 64, 16, 2, 2>;       // one 32x32 accumulator block per wave

template <int K, bool VEC>
__global__ __launch_bounds__(FwdCfg::NT) void fused1x1_fwd_kernel(fused_fwd_params p)
{
    using C = FwdCfg;
    constexpr int S = K + 2;
    __shared__ __attribute__((aligned(16))) float lds[C::LDS_FLOATS];
    constexpr int A_BUF = C::BK * C::LDA, B_BUF = C::BK * C::LDB;
    float *const As = lds;
    float *const Bs = lds + 2 * A_BUF;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % C::WM) * 32, wn0 = (wave / C::WM) * 32;
    const int li = lane & 31, lh = lane >> 5;

    // the filter tiles of one pixel tile are neighbours (they share the images'
    // pixel tile); a virtual batch's tiles are one run of the XCD-aware walk
    const int tiles = p.tiles_m * p.tiles_n;
    const int bid = dk_xcd_block();
    const int g = bid / tiles;
    const int t = bid - g * tiles;
    const int tile_n = t / p.tiles_m, tile_m = t - tile_n * p.tiles_m;
    const int row0 = tile_m * C::BM, col0 = tile_n * C::BN;

    using LA = LoadRowMajorK<C::BM, C::BK, C::NT, C::LDA, VEC>;      // W[Co][Ci]: rows = co, k = ci
    using LB = LoadKMajor<C::BN, C::BK, C::NT, C::LDB, VEC>;         // image [Ci][HW]: k = ci, rows = pixel
    const long long img = (long long)p.Ci * p.HW;
    const float *img0 = p.xbar + (long long)g * S * img;
    LA la; LB lb;
    la.init(MatParams{p.W, p.Ci, p.Co, p.Ci}, row0, tid);
    lb.init(MatParams{img0, p.HW, p.HW, p.Ci}, col0, tid);

    f32x16 acc, Tt, Sa, Y[K];
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[v] = 0.0f; Tt[v] = 0.0f; Sa[v] = 0.0f; }
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) Y[i][v] = 0.0f;

    const int KT = (p.Ci + C::BK - 1) / C::BK;
    const int T = S * KT;
    la.load(0); lb.load(0);
    la.store(As); lb.store(Bs);
    __syncthreads();
    int j = 0, kt = 0;
    for (int step = 0; step < T; ++step) {
        const int cur = step & 1;
        const bool more = step + 1 < T;
        int kt1 = kt + 1, j1 = j;
        if (kt1 == KT) { kt1 = 0; j1 = j + 1; }
        if (more) {
            if (kt1 == 0) lb.rebase(img0 + (long long)j1 * img);     // next encoding of the batch
            __builtin_amdgcn_s_setprio(3);
            la.load(kt1); lb.load(kt1);
            __builtin_amdgcn_s_setprio(0);
        }
        const float *a_s = As + cur * A_BUF + lh * C::LDA + wm0 + li;
        const float *b_s = Bs + cur * B_BUF + lh * C::LDB + wn0 + li;
#pragma unroll
        for (int kk = 0; kk < C::BK; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s[kk * C::LDA], b_s[kk * C::LDB], acc, 0, 0, 0);
        if (more) { la.store(As + (cur ^ 1) * A_BUF); lb.store(Bs + (cur ^ 1) * B_BUF); }
        __syncthreads();
        if (kt == KT - 1) {
            // encoding j of the batch is complete: fold its tile into the decoded
            // tiles (same order and operations as the decoding kernel: a product
            // for j = 0, fused multiply-adds after it) and into the integrity sums
            const float nj = p.nvec[(long long)g * S + j];
            float cj[K];
#pragma unroll
            for (int i = 0; i < K; ++i) cj[i] = p.Ainv[((long long)g * S + j) * S + i];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float a = acc[v];
#pragma unroll
                for (int i = 0; i < K; ++i) Y[i][v] = fmaf(cj[i], a, Y[i][v]);
                const float pr = nj * a;
                Tt[v] += pr;
                Sa[v] += fabsf(pr);
                acc[v] = 0.0f;
            }
        }
        kt = kt1; j = j1;
    }

    // lane holds pixel li, filters 8*(v/4) + 4*lh + v%4 of its wave's block
    const int col = col0 + wn0 + li;
    float tmax = 0.0f, smax = 0.0f;
    bool bad = false;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        bad |= !(Sa[v] <= 3.402823466e+38f) || !(fabsf(Tt[v]) <= 3.402823466e+38f);
        tmax = fmaxf(tmax, fabsf(Tt[v]));
        smax = fmaxf(smax, Sa[v]);
    }
    if (col < p.HW) {
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float *dst = p.y + ((long long)g * K + i) * p.Co * p.HW + col;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm0 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (row < p.Co) dst[(long long)row * p.HW] = Y[i][v];
            }
        }
    }
    // (rows and pixels outside the tensors hold zeros: their operands read as zero)
    dk_verify_publish_and_finish<C::NT>(tmax, smax, bad, p.slots, g, t, tiles, p.tag, p.tol, p.verdict,
                                        p.resid);
}

// The same for at most 64 input channels: the whole contraction is one step.  The filter
// tile goes to LDS once and serves all K + 2 encodings; an encoding is one 64 x 64 image tile,
// one barrier and 32 MFMAs per wave (the general kernel reloads the filter tile with every
// encoding and synchronises every 8 MFMAs, and its loader arithmetic weighs as much as its
// matrix work).  Same order of operations per output, so the same bits.
template <int K>
__global__ __launch_bounds__(FwdCfg::NT) void fused1x1_fwd64_kernel(fused_fwd_params p)
{
    constexpr int S = K + 2;
    constexpr int BM = 64, BN = 64, BKW = 64, NT = FwdCfg::NT, LDA = BM + 4, LDB = BN + 4;
    __shared__ __attribute__((aligned(16))) float lds[BKW * LDA + 2 * BKW * LDB];
    float *const As = lds;
    float *const Bs = lds + BKW * LDA;          // two buffers of BKW * LDB floats

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % 2) * 32, wn0 = (wave / 2) * 32;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    const int bid = dk_xcd_block();
    const int g = bid / tiles;
    const int t = bid - g * tiles;
    const int tile_n = t / p.tiles_m, tile_m = t - tile_n * p.tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    using LA = LoadRowMajorK<BM, BKW, NT, LDA, true>;       // W[Co][Ci]: rows = co, k = ci
    using LB = LoadKMajor<BN, BKW, NT, LDB, true>;          // image [Ci][HW]: k = ci, rows = pixel
    const long long img = (long long)p.Ci * p.HW;
    const float *img0 = p.xbar + (long long)g * S * img;
    LA la; LB lb;
    la.init(MatParams{p.W, p.Ci, p.Co, p.Ci}, row0, tid);
    lb.init(MatParams{img0, p.HW, p.HW, p.Ci}, col0, tid);

    f32x16 Tt, Sa, Y[K];
#pragma unroll
    for (int v = 0; v < 16; ++v) { Tt[v] = 0.0f; Sa[v] = 0.0f; }
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) Y[i][v] = 0.0f;

    la.load(0); lb.load(0);
    la.store(As); lb.store(Bs);
    __syncthreads();
    const float *a_s = As + lh * LDA + wm0 + li;
    for (int j = 0; j < S; ++j) {
        const int cur = j & 1;
        if (j + 1 < S) {
            lb.rebase(img0 + (long long)(j + 1) * img);            // next encoding of the batch
            lb.load(0);
        }
        // coefficients of this encoding (scalar loads, back before the MFMAs are through)
        const float nj = p.nvec[(long long)g * S + j];
        float cj[K];
#pragma unroll
        for (int i = 0; i < K; ++i) cj[i] = p.Ainv[((long long)g * S + j) * S + i];
        const float *b_s = Bs + cur * (BKW * LDB) + lh * LDB + wn0 + li;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < BKW; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s[kk * LDA], b_s[kk * LDB], acc, 0, 0, 0);
        if (j + 1 < S) lb.store(Bs + (cur ^ 1) * (BKW * LDB));
        // fold the encoding's tile into the decoded tiles (a product for j = 0, fused
        // multiply-adds after it: the decoding kernel's operations) and the integrity sums
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float a = acc[v];
#pragma unroll
            for (int i = 0; i < K; ++i) Y[i][v] = fmaf(cj[i], a, Y[i][v]);
            const float pr = nj * a;
            Tt[v] += pr;
            Sa[v] += fabsf(pr);
        }
        __syncthreads();
    }

    const int col = col0 + wn0 + li;
    float tmax = 0.0f, smax = 0.0f;
    bool bad = false;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        bad |= !(Sa[v] <= 3.402823466e+38f) || !(fabsf(Tt[v]) <= 3.402823466e+38f);
        tmax = fmaxf(tmax, fabsf(Tt[v]));
        smax = fmaxf(smax, Sa[v]);
    }
    if (col < p.HW) {
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float *dst = p.y + ((long long)g * K + i) * p.Co * p.HW + col;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm0 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (row < p.Co) dst[(long long)row * p.HW] = Y[i][v];
            }
        }
    }
    dk_verify_publish_and_finish<NT>(tmax, smax, bad, p.slots, g, t, tiles, p.tag, p.tol, p.verdict,
                                     p.resid);
}

// ---------------------------------------------------------------------------
// weight gradient with the gradient mixing in the operand loader
// ---------------------------------------------------------------------------

struct fused_wg_params {
    const float *delta, *xbar, *B, *gamma;
    float *out, *part;
    int Co, Ci, HW, G;
    int tiles_m, tiles_n;
    int cpi;                 // 16-pixel chunks per image
    int nch;                 // chunks in all virtual batches, G * cpi
    int per_split, splits;   // chunks per slice of the contraction, slices
    float alpha;
    int accumulate;
    long long out_elems;
};

template <class C, int K>
__global__ __launch_bounds__(C::NT) void fused1x1_wgrad_kernel(fused_wg_params p)
{
    constexpr int S = K + 2;
    static_assert(C::BK == 16, "a chunk is 16 pixels");
    constexpr int N4A = C::BM * 4 / C::NT, N4B = C::BN * 4 / C::NT;
    static_assert(N4A >= 1 && N4B >= 1, "tile/threads");
    __shared__ __attribute__((aligned(16))) float lds[C::LDS_FLOATS];
    constexpr int A_BUF = C::BK * C::LDA, B_BUF = C::BK * C::LDB;
    float *const As = lds;
    float *const Bs = lds + 2 * A_BUF;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % C::WM) * (C::BM / C::WM);
    const int wn0 = (wave / C::WM) * (C::BN / C::WN);
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    const int bid = dk_xcd_block();
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tile_m = t % p.tiles_m, tile_n = t / p.tiles_m;
    const int row0 = tile_m * C::BM, col0 = tile_n * C::BN;

    // both tensors as one buffer resource each; a lane keeps one byte offset per
    // 16-byte vector it fetches (rows beyond the tensor: out of range, read as 0)
    const __amdgpu_buffer_rsrc_t rsD = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.delta), 0, (int)((long long)p.G * K * p.Co * p.HW * 4), DK_RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rsX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.xbar), 0, (int)((long long)p.G * S * p.Ci * p.HW * 4), DK_RSRC_FLAGS);
    unsigned voffA[N4A], voffB[N4B];
#pragma unroll
    for (int e = 0; e < N4A; ++e) {
        const int idx = tid + e * C::NT, row = row0 + idx / 4, kc = idx % 4;
        voffA[e] = row < p.Co ? 4u * (unsigned)(row * p.HW + kc * 4) : DK_OOB;
    }
#pragma unroll
    for (int e = 0; e < N4B; ++e) {
        const int idx = tid + e * C::NT, row = col0 + idx / 4, kc = idx % 4;
        voffB[e] = row < p.Ci ? 4u * (unsigned)(row * p.HW + kc * 4) : DK_OOB;
    }

    float4 dreg[K][N4A];     // the chunk's K gradient tiles
    float4 breg[N4B];        // the encoding's tile of the current step

    // contraction step u = (chunk c, encoding j); chunk c = (virtual batch g, pixel chunk)
    // (the virtual batch g and the first pixel pix0 of a chunk are carried along by the loop:
    // a division per step, done on the vector ALU, costs as much as the mixing itself)
    auto fetch_delta = [&](int g, int pix0) {
#pragma unroll
        for (int i = 0; i < K; ++i) {
            const unsigned soff = 4u * ((unsigned)(g * K + i) * (unsigned)p.Co * (unsigned)p.HW + (unsigned)pix0);
#pragma unroll
            for (int e = 0; e < N4A; ++e) dreg[i][e] = dk_buffer_load4(rsD, voffA[e], soff);
        }
    };
    auto fetch_x = [&](int g, int pix0, int j) {
        const unsigned soff = 4u * ((unsigned)(g * S + j) * (unsigned)p.Ci * (unsigned)p.HW + (unsigned)pix0);
#pragma unroll
        for (int e = 0; e < N4B; ++e) breg[e] = dk_buffer_load4(rsX, voffB[e], soff);
    };
    // mixed gradient of encoding j from the chunk's K tiles (the mixing kernel's
    // own operations, in its order), written k-major like the other operand
    auto put = [&](int g, int j, float *as, float *bs) {
        const float gj = p.gamma[(long long)g * S + j];
        float cf[K];
#pragma unroll
        for (int i = 0; i < K; ++i) cf[i] = gj * p.B[((long long)g * S + j) * K + i];
#pragma unroll
        for (int e = 0; e < N4A; ++e) {
            float4 a = make_float4(cf[0] * dreg[0][e].x, cf[0] * dreg[0][e].y, cf[0] * dreg[0][e].z,
                                   cf[0] * dreg[0][e].w);
#pragma unroll
            for (int i = 1; i < K; ++i) {
                a.x = fmaf(cf[i], dreg[i][e].x, a.x);
                a.y = fmaf(cf[i], dreg[i][e].y, a.y);
                a.z = fmaf(cf[i], dreg[i][e].z, a.z);
                a.w = fmaf(cf[i], dreg[i][e].w, a.w);
            }
            const int idx = tid + e * C::NT, row = idx / 4, kc = idx % 4;
            float *d = as + (kc * 4) * C::LDA + row;
            d[0 * C::LDA] = a.x; d[1 * C::LDA] = a.y; d[2 * C::LDA] = a.z; d[3 * C::LDA] = a.w;
        }
#pragma unroll
        for (int e = 0; e < N4B; ++e) {
            const int idx = tid + e * C::NT, row = idx / 4, kc = idx % 4;
            float *d = bs + (kc * 4) * C::LDB + row;
            d[0 * C::LDB] = breg[e].x; d[1 * C::LDB] = breg[e].y; d[2 * C::LDB] = breg[e].z;
            d[3 * C::LDB] = breg[e].w;
        }
    };

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::TN; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const int c0 = split * p.per_split;
    int c1 = c0 + p.per_split;
    if (c1 > p.nch) c1 = p.nch;
    if (c0 < c1) {
        int g = c0 / p.cpi, pix0 = (c0 - g * p.cpi) * 16;         // of chunk c
        fetch_delta(g, pix0);
        fetch_x(g, pix0, 0);
        put(g, 0, As, Bs);
        __syncthreads();
        int c = c0, j = 0;
        for (int step = 0;; ++step) {
            const int cur = step & 1;
            int j1 = j + 1, cn = c, gn = g, pn = pix0;                 // ... of the next step's chunk
            if (j1 == S) {
                j1 = 0; cn = c + 1; pn = pix0 + 16;
                if (pn == p.cpi * 16) { pn = 0; gn = g + 1; }
            }
            const bool more = cn < c1;
            if (more) {
                // the chunk's last mixed tile was formed one step ago: its K tiles
                // can be overwritten by the next chunk's now
                __builtin_amdgcn_s_setprio(3);
                if (j1 == 0) fetch_delta(gn, pn);
                fetch_x(gn, pn, j1);
                __builtin_amdgcn_s_setprio(0);
            }
            const float *a_s = As + cur * A_BUF + lh * C::LDA + wm0 + li;
            const float *b_s = Bs + cur * B_BUF + lh * C::LDB + wn0 + li;
#pragma unroll
            for (int kk = 0; kk < C::BK; kk += 2) {
                float a[C::TM], b[C::TN];
#pragma unroll
                for (int mi = 0; mi < C::TM; ++mi) a[mi] = a_s[kk * C::LDA + mi * 32];
#pragma unroll
                for (int ni = 0; ni < C::TN; ++ni) b[ni] = b_s[kk * C::LDB + ni * 32];
#pragma unroll
                for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < C::TN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
            }
            if (more) put(gn, j1, As + (cur ^ 1) * A_BUF, Bs + (cur ^ 1) * B_BUF);
            __syncthreads();
            if (!more) break;
            c = cn; j = j1; g = gn; pix0 = pn;
        }
    }

    // dW[co][ci]: lane holds column (ci) li, rows (co) 8*(v/4) + 4*lh + v%4
    float *dst = p.splits > 1 ? p.part + (long long)split * p.out_elems : p.out;
    const bool direct = p.splits == 1;
#pragma unroll
    for (int ni = 0; ni < C::TN; ++ni) {
        const int col = col0 + wn0 + ni * 32 + li;
        if (col >= p.Ci) continue;
#pragma unroll
        for (int mi = 0; mi < C::TM; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm0 + mi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (row >= p.Co) continue;
                float *d = dst + (long long)row * p.Ci + col;
                float val = acc[mi][ni][v];
                if (direct) {
                    val *= p.alpha;
                    if (p.accumulate) val += *d;
                }
                *d = val;
            }
    }
}

using CfgSq = Cfg<128, 128, 16, 2, 2>;
using CfgWg64 = Cfg<64, 128, 16, 2, 2>;
using CfgTall = Cfg<128, 64, 16, 2, 2>;
using CfgSmall = Cfg<64, 64, 16, 2, 2>;

template <class Fn>
auto with_cfg(long long rows, long long cols, Fn fn)
{
    if (rows <= 64 && cols <= 64) return fn(CfgSmall{});
    if (rows <= 64) return fn(CfgWg64{});
    if (cols <= 64) return fn(CfgTall{});
    return fn(CfgSq{});
}

bool is_1x1_s1(const dk_geom &g)
{
    return g.conv && !g.dw && g.kh == 1 && g.kw == 1 && g.pad == 0 && g.stride == 1;
}

bool fused_k(int K) { return K == 2 || K == 4 || K == 8; }

struct wg_plan {
    int tiles_m, tiles_n, cpi, nch, per_split, splits;
    size_t part_bytes;
};

template <class C>
wg_plan plan_wgrad_cfg(const dk_geom &g, int G, int K)
{
    wg_plan pl;
    pl.tiles_m = (g.Co + C::BM - 1) / C::BM;
    pl.tiles_n = (g.Ci + C::BN - 1) / C::BN;
    pl.cpi = g.H * g.W / 16;
    pl.nch = G * pl.cpi;
    // a step of the plan is one chunk: K + 2 contraction steps of the tile
    const dk_split_plan sp = dk_plan_split((long long)pl.tiles_m * pl.tiles_n, pl.nch, (long long)g.Co * g.Ci,
                                           C::STEP_US * (K + 2));
    pl.splits = sp.splits;
    pl.per_split = sp.ktiles_per_split;
    pl.part_bytes = sp.splits > 1 ? (size_t)sp.splits * g.Co * g.Ci * sizeof(float) : 0;
    return pl;
}

wg_plan plan_wgrad(const dk_geom &g, int G, int K)
{
    return with_cfg(g.Co, g.Ci, [&](auto c) { return plan_wgrad_cfg<decltype(c)>(g, G, K); });
}

} // namespace

// ---- weight gradient ----

bool dk_fused1x1_wgrad_ok(const dk_geom &g, int G, int K, int M, const float *delta, const float *xbar)
{
    if (!is_1x1_s1(g) || M != 1 || !fused_k(K)) return false;
    const long long HW = (long long)g.H * g.W;
    if (HW % 16) return false;
    if (!dk_aligned(delta, 16) || !dk_aligned(xbar, 16)) return false;
    if ((long long)G * K * g.Co * HW * 4 > 0x7fffffffll) return false;
    if ((long long)G * (K + 2) * g.Ci * HW * 4 > 0x7fffffffll) return false;
    return true;
}

// Partial-sum bytes the fused weight gradient may need for R encoded rows,
// whatever K it is called with (the workspace query knows only R).
size_t dk_fused1x1_wgrad_part_bytes(const dk_geom &g, long long R)
{
    if (!is_1x1_s1(g) || ((long long)g.H * g.W) % 16) return 0;
    size_t b = 0;
    for (int K : {2, 4, 8})
        if (R % (K + 2) == 0 && R / (K + 2) < (1ll << 30)) {
            const wg_plan pl = plan_wgrad(g, (int)(R / (K + 2)), K);
            if (pl.part_bytes > b) b = pl.part_bytes;
        }
    return b;
}

dk_status dk_fused1x1_wgrad_run(const dk_geom &g, const float *delta, const float *B, const float *gamma,
                                const float *xbar, float *dW, int G, int K, float scale, int accumulate,
                                float *part, size_t part_bytes, hipStream_t st)
{
    const wg_plan pl = plan_wgrad(g, G, K);
    DK_REQUIRE(pl.part_bytes <= part_bytes, DK_ERR_WORKSPACE);
    fused_wg_params p;
    p.delta = delta; p.xbar = xbar; p.B = B; p.gamma = gamma;
    p.out = dW; p.part = part;
    p.Co = g.Co; p.Ci = g.Ci; p.HW = g.H * g.W; p.G = G;
    p.tiles_m = pl.tiles_m; p.tiles_n = pl.tiles_n; p.cpi = pl.cpi; p.nch = pl.nch;
    p.per_split = pl.per_split; p.splits = pl.splits;
    p.alpha = scale; p.accumulate = accumulate;
    p.out_elems = (long long)g.Co * g.Ci;
    const long long blocks = (long long)pl.tiles_m * pl.tiles_n * pl.splits;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    {
        dk_prof_scope ps("fused1x1_wgrad", st);
        with_cfg(g.Co, g.Ci, [&](auto c) {
            using C = decltype(c);
            const dim3 grid((unsigned)blocks), block(C::NT);
            if (K == 2) fused1x1_wgrad_kernel<C, 2><<<grid, block, 0, st>>>(p);
            else if (K == 4) fused1x1_wgrad_kernel<C, 4><<<grid, block, 0, st>>>(p);
            else fused1x1_wgrad_kernel<C, 8><<<grid, block, 0, st>>>(p);
            return 0;
        });
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    if (pl.splits > 1) return dk_fold_slices(part, dW, p.out_elems, pl.splits, scale, accumulate, st);
    return DK_OK;
}

// ---- forward + decode + verify ----

bool dk_fused1x1_fwd_ok(const dk_geom &g, int K)
{
    return is_1x1_s1(g) && fused_k(K);
}

// Integrity-check slots of the fused forward: one per (virtual batch, tile).
size_t dk_fused1x1_fwd_slot_bytes(const dk_geom &g, int G)
{
    const long long tiles = (long long)((g.Co + FwdCfg::BM - 1) / FwdCfg::BM) *
                            (((long long)g.H * g.W + FwdCfg::BN - 1) / FwdCfg::BN);
    return (size_t)G * tiles * sizeof(dk_verify_slot);
}

dk_status dk_fused1x1_fwd_run(const dk_geom &g, const float *W, const float *xbar, const float *Ainv,
                              const float *nvec, float tol, float *y, int *verdict, float *resid, int G,
                              int K, void *slots, hipStream_t st)
{
    fused_fwd_params p;
    p.W = W; p.xbar = xbar; p.Ainv = Ainv; p.nvec = nvec; p.y = y;
    p.slots = (dk_verify_slot *)slots; p.verdict = verdict; p.resid = resid;
    p.Co = g.Co; p.Ci = g.Ci; p.HW = g.H * g.W; p.G = G;
    p.tiles_m = (g.Co + FwdCfg::BM - 1) / FwdCfg::BM;
    p.tiles_n = (p.HW + FwdCfg::BN - 1) / FwdCfg::BN;
    const int tiles = p.tiles_m * p.tiles_n;
    const bool in_kernel = tiles <= DK_VERIFY_INLINE_MAX_CHUNKS;
    p.tag = in_kernel ? dk_next_verify_tag() : 0ull;
    p.tol = tol;
    const long long blocks = (long long)p.tiles_m * p.tiles_n * G;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const bool vec = g.Ci % 4 == 0 && p.HW % 4 == 0 && dk_aligned(W, 16) && dk_aligned(xbar, 16);
    const dim3 grid((unsigned)blocks), block(FwdCfg::NT);
    {
    dk_prof_scope ps("fused1x1_fwd_decode_verify", st);
#define DK_FF(KK)                                                                  \
    do {                                                                           \
        if (vec && g.Ci <= 64) fused1x1_fwd64_kernel<KK><<<grid, block, 0, st>>>(p); \
        else if (vec) fused1x1_fwd_kernel<KK, true><<<grid, block, 0, st>>>(p);    \
        else fused1x1_fwd_kernel<KK, false><<<grid, block, 0, st>>>(p);            \
    } while (0)
    if (K == 2) DK_FF(2); else if (K == 4) DK_FF(4); else DK_FF(8);
#undef DK_FF
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    return in_kernel ? DK_OK : dk_verify_finalize(p.slots, tiles, tol, verdict, resid, G, st);
}
