// Convolution forward on encoded images with the input staged as a zero-padded
// PATCH in LDS (stride-1/2 filters of compile-time size).
//
// The generic implicit-GEMM loader gathers every im2col element from global
// memory with its own bounds test (kh*kw-fold re-reads and a dozen VALU
// instructions per element).  Here a workgroup owns BM output channels x BN
// consecutive output pixels of one image (or several whole small images) and
// walks the input channels in chunks of CB: the chunk's input rows are copied
// once into LDS with the zero border materialised, and the MFMA B operand for
// filter tap (a, b) of channel c is read at
//     lane_base(pixel) + c*PLANE + a*PW + b
// i.e. a per-lane constant plus a wave-uniform offset: no bounds tests and
// almost no address arithmetic in the inner loop.  The filter bank is repacked
// once per call into the k-major, channel-pair order the MFMA steps consume,
// so its tile is a straight 16-byte copy into LDS.
#include "dk_internal.h"
#include "dk_patch.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Repack W[Co][Ci][KH][KW] -> wp[chunk][row][Co_pad], row = 2*step + h with
// step = (c' * KH + a) * KW + b and channel = chunk*CB + c' + h*CB/2; zero
// beyond Ci and Co.
__global__ __launch_bounds__(256) void pack_filters_kernel(const float *__restrict__ W,
                                                           float *__restrict__ wp, int Ci, int Co,
                                                           int KH, int KW, int CB, int Co_pad,
                                                           long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int co = (int)(i % Co_pad);
    long long t = i / Co_pad;
    const int rows = CB * KH * KW;
    const int row = (int)(t % rows);
    const int chunk = (int)(t / rows);
    const int h = row & 1, step = row >> 1;
    const int b = step % KW, a = (step / KW) % KH, cp = step / (KW * KH);
    const int ci = chunk * CB + cp + h * (CB / 2);
    float v = 0.0f;
    if (co < Co && ci < Ci) v = W[(((long long)co * Ci + ci) * KH + a) * KW + b];
    wp[i] = v;
}

template <int BM, int BN, int WM, int WN, int KH, int KW, int CB, int VEC, int MAXSLOT>
__global__ __launch_bounds__(64 * WM * WN) void conv_patch_fwd_kernel(dk_patch_params p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int NT = 64 * WM * WN;
    constexpr int KK = KH * KW;
    constexpr int LDA = BM + 4;
    constexpr int WROWS = CB * KK;                  // filter rows per chunk
    constexpr int W4 = WROWS * (BM / 4);            // 16-byte vectors in a filter tile
    constexpr int WSLOT = (W4 + NT - 1) / NT;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static_assert(CB % 2 == 0, "channel pairs");

    float *const patch = lds;
    float *const As = lds + p.patch_floats;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave % WM) * (BM / WM);
    const int wn0 = (wave / WM) * (BN / WN);

    const int tiles = p.tiles_m * p.tiles_n;
    // each XCD takes one contiguous run of tiles: neighbouring pixel tiles of an
    // image, which share their halo rows, then share an L2
    const int bid = dk_xcd_block();
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tile_n = t / p.tiles_m, tile_m = t - tile_n * p.tiles_m;
    const int co0 = tile_m * BM;

    // which images / pixels this tile covers
    int r0, p0, ho_a;
    if (!p.multi) {
        r0 = tile_n / p.tiles_per_img;
        p0 = (tile_n - r0 * p.tiles_per_img) * BN;
        ho_a = p0 / p.Wo;
    } else if (p.multi == 1) {
        r0 = tile_n * p.IPT;
        p0 = 0;
        ho_a = 0;
    } else {
        // BN consecutive pixels of the whole batch, starting anywhere in image r0: no column of
        // a tile is wasted whatever the image size; the patch holds every image they touch
        const long long g0 = (long long)tile_n * BN;
        r0 = (int)(g0 / p.HoWo);
        p0 = (int)(g0 - (long long)r0 * p.HoWo);
        ho_a = 0;
    }
    const int ih_a = ho_a * p.stride - p.pad;

    // per-lane output columns
    int fbase[TN], ooff[TN];
    bool okc[TN];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
        const int jn = wn0 + ni * 32 + li;
        int img_l, pix;
        bool ok;
        if (!p.multi) {
            img_l = 0; pix = p0 + jn; ok = pix < p.HoWo;
        } else if (p.multi == 1) {
            img_l = jn / p.HoWo; pix = jn - img_l * p.HoWo;
            ok = jn < p.BN_eff && r0 + img_l < p.R;
        } else {
            img_l = (p0 + jn) / p.HoWo; pix = p0 + jn - img_l * p.HoWo;
            ok = r0 + img_l < p.R;
        }
        if (!ok) { img_l = 0; pix = p.multi == 2 ? 0 : p0; }
        const int ho = pix / p.Wo, wo = pix - ho * p.Wo;
        fbase[ni] = img_l * CB * p.PLANE + (ho - ho_a) * p.stride * p.PW + p.LPAD - p.pad +
                    wo * p.stride + lh * (CB / 2) * p.PLANE;
        ooff[ni] = img_l * p.Co * p.HoWo + pix;
        okc[ni] = ok;
    }

    // patch copy slots of this lane (same positions for every channel chunk)
    int goff[MAXSLOT], loff[MAXSLOT], cch[MAXSLOT];
#pragma unroll
    for (int e = 0; e < MAXSLOT; ++e) {
        const int idx = tid + e * NT;
        const int xv = idx % p.XV;
        const int t1 = idx / p.XV;
        const int prow = t1 % p.PH;
        const int t2 = t1 / p.PH;
        const int c = t2 % CB;
        const int img_l = t2 / CB;
        const int ih = ih_a + prow;
        const bool act = idx < p.patch_slots && r0 + img_l < p.R && ih >= 0 && ih < p.H;
        goff[e] = act ? img_l * p.img_g + (c * p.H + ih) * p.W + xv * VEC : -1;
        loff[e] = img_l * CB * p.PLANE + c * p.PLANE + prow * p.PW + p.LPAD + xv * VEC;
        cch[e] = c;
    }

    for (int i = tid; i < p.patch_floats; i += NT) patch[i] = 0.0f;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const float *xbase = p.x + (long long)r0 * p.img_g;
    const int ch0 = split * p.per_split;
    int ch1 = ch0 + p.per_split;
    if (ch1 > p.n_chunks) ch1 = p.n_chunks;

    f32x4 pst[MAXSLOT];
    f32x4 wst[WSLOT];

    // Issue the global loads of one channel chunk into registers.
#define DK_PATCH_FETCH(CH)                                                                       \
    {                                                                                            \
        const int ci0_ = (CH) * CB;                                                              \
        const float *src_ = xbase + (long long)ci0_ * p.H * p.W;                                 \
        _Pragma("unroll") for (int e = 0; e < MAXSLOT; ++e) {                                    \
            const bool ok_ = goff[e] >= 0 && ci0_ + cch[e] < p.Ci;                               \
            const float *s_ = src_ + (ok_ ? goff[e] : 0);                                        \
            if constexpr (VEC == 4) {                                                            \
                f32x4 v_ = {0.f, 0.f, 0.f, 0.f};                                                 \
                if (ok_) v_ = *reinterpret_cast<const f32x4 *>(s_);                              \
                pst[e] = v_;                                                                     \
            } else {                                                                             \
                float v_ = 0.0f;                                                                 \
                if (ok_) v_ = *s_;                                                               \
                pst[e] = f32x4{v_, 0.f, 0.f, 0.f};                                               \
            }                                                                                    \
        }                                                                                        \
        const float *wsrc_ = p.wp + (long long)(CH) * WROWS * p.Co_pad + co0;                    \
        _Pragma("unroll") for (int e = 0; e < WSLOT; ++e) {                                      \
            int idx_ = tid + e * NT;                                                             \
            if (idx_ >= W4) idx_ = W4 - 1;                                                       \
            const int row_ = idx_ / (BM / 4), c4_ = idx_ % (BM / 4);                             \
            wst[e] = *reinterpret_cast<const f32x4 *>(wsrc_ + (long long)row_ * p.Co_pad + c4_ * 4); \
        }                                                                                        \
    }

    if (ch0 < ch1) DK_PATCH_FETCH(ch0)
    for (int ch = ch0; ch < ch1; ++ch) {
        __syncthreads();            // previous chunk fully consumed (and the zero fill done)
#pragma unroll
        for (int e = 0; e < MAXSLOT; ++e) {
            if (goff[e] < 0) continue;
            if constexpr (VEC == 4)
                *reinterpret_cast<f32x4 *>(patch + loff[e]) = pst[e];
            else
                patch[loff[e]] = pst[e].x;
        }
#pragma unroll
        for (int e = 0; e < WSLOT; ++e) {
            const int idx = tid + e * NT;
            const int row = idx / (BM / 4), c4 = idx % (BM / 4);
            if (idx < W4) *reinterpret_cast<f32x4 *>(As + row * LDA + c4 * 4) = wst[e];
        }
        __syncthreads();
        if (ch + 1 < ch1) DK_PATCH_FETCH(ch + 1)   // in flight during the MFMA loop

        const float *a_s = As + lh * LDA + wm0 + li;
#pragma unroll
        for (int cp = 0; cp < CB / 2; ++cp)
#pragma unroll
            for (int a = 0; a < KH; ++a) {
                const int soff = cp * p.PLANE + a * p.PW;      // wave-uniform
                const float *pb[TN];
#pragma unroll
                for (int ni = 0; ni < TN; ++ni) pb[ni] = patch + fbase[ni] + soff;
#pragma unroll
                for (int b = 0; b < KW; ++b) {
                    const int s = (cp * KH + a) * KW + b;
                    float av[TM], bv[TN];
#pragma unroll
                    for (int mi = 0; mi < TM; ++mi) av[mi] = a_s[2 * s * LDA + mi * 32];
#pragma unroll
                    for (int ni = 0; ni < TN; ++ni) bv[ni] = pb[ni][b];
#pragma unroll
                    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                        for (int ni = 0; ni < TN; ++ni)
                            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
                }
            }
    }

#undef DK_PATCH_FETCH

    float *dst = (p.splits > 1 ? p.part + (long long)split * p.out_elems : p.out) +
                 (long long)r0 * p.Co * p.HoWo;
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
        if (!okc[ni]) continue;
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = co0 + wm0 + mi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (row < p.Co) dst[(long long)row * p.HoWo + ooff[ni]] = acc[mi][ni][v];
            }
    }
}

// Repack W[Co][Ci][3][3] -> wq[chunk][Co_pad][72], position h*36 + (c'*3 + a)*3 + b
// holding channel chunk*8 + c' + 4h: per output channel, the 36 MFMA steps of
// each half-wave are contiguous, so four steps are one 16-byte LDS read.
__global__ __launch_bounds__(256) void pack_filters_quad_kernel(const float *__restrict__ W,
                                                                float *__restrict__ wq, int Ci,
                                                                int Co, int Co_pad, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int kk = (int)(i % 72);
    const long long t = i / 72;
    const int co = (int)(t % Co_pad);
    const int chunk = (int)(t / Co_pad);
    const int h = kk / 36, step = kk - h * 36;
    const int b = step % 3, a = (step / 3) % 3, cp = step / 9;
    const int ci = chunk * 8 + cp + 4 * h;
    float v = 0.0f;
    if (co < Co && ci < Ci) v = W[(((long long)co * Ci + ci) * 3 + a) * 3 + b];
    wq[i] = v;
}

// 3x3 stride-1 forward with 16-byte LDS reads (image and output widths
// multiples of 4).  A wave owns TM*32 output channels x 128 consecutive output
// pixels as four 32-column MFMA blocks, block t taking the pixels = t (mod 4):
// lane j then needs, for filter row a and the three filter columns, patch
// columns 4j .. 4j+5 -- an aligned 16-byte and an 8-byte read that feed 3 steps
// x 4 blocks.  The filter tile is stored [co][step] so that four steps of a lane
// are one 16-byte read too: about 0.2 LDS instructions per MFMA instead of one.
//
// Vector-ALU instructions of a wave that is copying queue behind the matrix
// instructions of the other waves on its SIMD, so the copy costs none per
// chunk: global reads are buffer loads (wave-uniform base in a scalar resource,
// the lane's byte offset precomputed; a slot outside the image or beyond the
// tile gets an offset past the resource's range and so reads as zero), LDS
// addresses are precomputed, and an unused slot stores into a dump area behind
// the tiles.  Only a last chunk with fewer than 8 channels tests its channels.
// Operands of the next filter row are read from LDS before the MFMAs of the
// current one are issued.
constexpr int DK_FWD_RSRC_FLAGS = 0x00020000;     // raw buffer resource, gfx9 family
constexpr unsigned DK_FWD_RANGE = 0x80000000u;    // resource range in bytes; offsets beyond read 0

template <int TM, int WM, int WN, int MAXSLOT>
__global__ __launch_bounds__(64 * WM * WN) void conv_quad_fwd_kernel(dk_patch_params p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int NT = 64 * WM * WN, CB = 8, BM = WM * TM * 32, BN = WN * 128;
    constexpr int WP = 76;                          // filter tile pitch: 72 steps + 4
    constexpr int W4 = BM * 18;                     // 16-byte vectors in a filter tile
    constexpr int WSLOT = (W4 + NT - 1) / NT;

    float *const patch = lds;
    float *const As = lds + p.patch_floats;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave % WM) * (TM * 32);
    const int wn0 = (wave / WM) * 128;
    float *const dump = As + BM * WP + lane * 4;    // 1 KB behind the filter tile

    const int tiles = p.tiles_m * p.tiles_n;
    // each XCD takes one contiguous run of tiles: neighbouring pixel tiles of an
    // image, which share their halo rows, then share an L2
    const int bid = dk_xcd_block();
    const int split = bid / tiles;
    const int t = bid - split * tiles;
    const int tile_n = t / p.tiles_m, tile_m = t - tile_n * p.tiles_m;
    const int co0 = tile_m * BM;

    int r0, p0, ho_a;
    if (!p.multi) {
        r0 = tile_n / p.tiles_per_img;
        p0 = (tile_n - r0 * p.tiles_per_img) * BN;
        ho_a = p0 / p.Wo;
    } else if (p.multi == 1) {
        r0 = tile_n * p.IPT;
        p0 = 0;
        ho_a = 0;
    } else {
        // BN consecutive pixels of the whole batch, starting anywhere in image r0: no column of
        // a tile is wasted whatever the image size; the patch holds every image they touch
        const long long g0 = (long long)tile_n * BN;
        r0 = (int)(g0 / p.HoWo);
        p0 = (int)(g0 - (long long)r0 * p.HoWo);
        ho_a = 0;
    }
    const int ih_a = ho_a - p.pad;

    // this lane's four pixels (one quad)
    int fbase, ooff;
    bool okc;
    {
        const int jn = wn0 + 4 * li;
        int img_l, pix;
        if (!p.multi) {
            img_l = 0; pix = p0 + jn; okc = pix < p.HoWo;
        } else {
            img_l = jn / p.HoWo; pix = jn - img_l * p.HoWo;
            okc = jn < p.BN_eff && r0 + img_l < p.R;
        }
        if (!okc) { img_l = 0; pix = p0; }
        const int ho = pix / p.Wo, wo = pix - ho * p.Wo;
        fbase = img_l * CB * p.PLANE + (ho - ho_a) * p.PW + wo + lh * (CB / 2) * p.PLANE;
        ooff = img_l * p.Co * p.HoWo + pix;
    }

    // copy slots of this lane, the same for every channel chunk
    unsigned goff[MAXSLOT];       // byte offset from the chunk's first channel, or out of range
    float *pdst[MAXSLOT];
    int cch[MAXSLOT];
#pragma unroll
    for (int e = 0; e < MAXSLOT; ++e) {
        const int idx = tid + e * NT;
        const int xv = idx % p.XV;
        const int t1 = idx / p.XV;
        const int prow = t1 % p.PH;
        const int t2 = t1 / p.PH;
        const int c = t2 % CB;
        const int img_l = t2 / CB;
        const int ih = ih_a + prow;
        const bool slot = idx < p.patch_slots;
        const bool act = slot && r0 + img_l < p.R && ih >= 0 && ih < p.H;
        goff[e] = act ? 4u * (unsigned)(img_l * p.img_g + (c * p.H + ih) * p.W + xv * 4) : DK_FWD_RANGE;
        // a slot outside the image still stores (zeros): the border stays clean
        pdst[e] = slot ? patch + img_l * CB * p.PLANE + c * p.PLANE + prow * p.PW + p.LPAD + xv * 4 : dump;
        cch[e] = c;
    }
    unsigned woff[WSLOT];
    float *wdst[WSLOT];
#pragma unroll
    for (int e = 0; e < WSLOT; ++e) {
        const int idx = tid + e * NT;
        const int row = idx / 18, c4 = idx - row * 18;
        woff[e] = idx < W4 ? 4u * (unsigned)(row * p.w_row + c4 * 4) : DK_FWD_RANGE;
        wdst[e] = idx < W4 ? As + row * WP + c4 * 4 : dump;
    }

    for (int i = tid; i < p.patch_floats; i += NT) patch[i] = 0.0f;

    f32x16 acc[TM][4];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const float *xbase = p.x + (long long)r0 * p.img_g;
    const int ch0 = split * p.per_split;
    int ch1 = ch0 + p.per_split;
    if (ch1 > p.n_chunks) ch1 = p.n_chunks;

    f32x4 pst[MAXSLOT];
    f32x4 wst[WSLOT];

#define DK_QUAD_FETCH(CH)                                                                        \
    {                                                                                            \
        const int ci0_ = (CH) * CB;                                                              \
        const __amdgpu_buffer_rsrc_t rx_ = __builtin_amdgcn_make_buffer_rsrc(                     \
            const_cast<float *>(xbase + (long long)ci0_ * p.H * p.W), 0, (int)DK_FWD_RANGE, DK_FWD_RSRC_FLAGS); \
        if (ci0_ + CB <= p.Ci) {                                                                 \
            _Pragma("unroll") for (int e = 0; e < MAXSLOT; ++e)                                  \
                pst[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx_, (int)goff[e], 0, 0)); \
        } else {                                                                                 \
            _Pragma("unroll") for (int e = 0; e < MAXSLOT; ++e) {                                \
                const unsigned o_ = ci0_ + cch[e] < p.Ci ? goff[e] : DK_FWD_RANGE;               \
                pst[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rx_, (int)o_, 0, 0)); \
            }                                                                                    \
        }                                                                                        \
        const __amdgpu_buffer_rsrc_t rw_ = __builtin_amdgcn_make_buffer_rsrc(                     \
            const_cast<float *>(p.wp + (long long)(CH) * p.w_chunk + (long long)co0 * p.w_row), 0, \
            (int)DK_FWD_RANGE, DK_FWD_RSRC_FLAGS);                                               \
        _Pragma("unroll") for (int e = 0; e < WSLOT; ++e)                                        \
            wst[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rw_, (int)woff[e], 0, 0)); \
    }

    if (ch0 < ch1) DK_QUAD_FETCH(ch0)
    for (int ch = ch0; ch < ch1; ++ch) {
        __syncthreads();            // previous chunk fully consumed (and the zero fill done)
#pragma unroll
        for (int e = 0; e < MAXSLOT; ++e) {
            float *d = pdst[e];                  // `pad` columns off 16-byte alignment
            d[0] = pst[e].x; d[1] = pst[e].y; d[2] = pst[e].z; d[3] = pst[e].w;
        }
#pragma unroll
        for (int e = 0; e < WSLOT; ++e) *reinterpret_cast<f32x4 *>(wdst[e]) = wst[e];
        __syncthreads();
        if (ch + 1 < ch1) DK_QUAD_FETCH(ch + 1)   // in flight during the MFMA loop

        const float *a_s = As + (wm0 + li) * WP + lh * 36;
        const float *pb = patch + fbase;
        // group g = (cp, a): three steps (b = 0..2) on one patch row; its six
        // columns are read one group ahead, the filter quads one quad ahead
        // (filter quad q = steps 4q .. 4q+3 lives in buffer q % 3: a group touches
        // at most two quads and the one after them is being read meanwhile)
        f32x4 wq[2];
        f32x2 wh[2];
        f32x4 aq[3][TM];
        wq[0] = *reinterpret_cast<const f32x4 *>(pb);
        wh[0] = *reinterpret_cast<const f32x2 *>(pb + 4);
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) aq[0][mi] = *reinterpret_cast<const f32x4 *>(a_s + mi * 32 * WP);
#pragma unroll
        for (int g = 0; g < 12; ++g) {
            if (g + 1 < 12) {
                const int cpn = (g + 1) / 3, an = (g + 1) % 3;
                const float *pr = pb + cpn * p.PLANE + an * p.PW;
                wq[(g + 1) & 1] = *reinterpret_cast<const f32x4 *>(pr);
                wh[(g + 1) & 1] = *reinterpret_cast<const f32x2 *>(pr + 4);
            }
            {
                const int qn = (3 * g + 2) / 4 + 1;                   // quad after this group's last
                const int qp = g ? (3 * (g - 1) + 2) / 4 + 1 : 0;     // what the group before fetched
                if (qn != qp && qn < 9) {
#pragma unroll
                    for (int mi = 0; mi < TM; ++mi)
                        aq[qn % 3][mi] = *reinterpret_cast<const f32x4 *>(a_s + mi * 32 * WP + 4 * qn);
                }
            }
            __builtin_amdgcn_sched_barrier(0);   // the reads go out before this group's MFMAs
            const f32x4 w0 = wq[g & 1];
            const f32x2 w1 = wh[g & 1];
            const float w[6] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y};
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                const int s = 3 * g + b;
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt)
                        acc[mi][tt] = __builtin_amdgcn_mfma_f32_32x32x2f32(aq[(s / 4) % 3][mi][s % 4], w[tt + b], acc[mi][tt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef DK_QUAD_FETCH

    if (!okc) return;
    float *dst = (p.splits > 1 ? p.part + (long long)split * p.out_elems : p.out) +
                 (long long)r0 * p.Co * p.HoWo + ooff;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = co0 + wm0 + mi * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
            if (row < p.Co)
                *reinterpret_cast<f32x4 *>(dst + (long long)row * p.HoWo) =
                    f32x4{acc[mi][0][v], acc[mi][1][v], acc[mi][2][v], acc[mi][3][v]};
        }
}

template <int TM, int WM, int WN>
struct QuadCfg {
    static constexpr int bm = WM * TM * 32, bn = WN * 128, cb = 8;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int MAXSLOT = 4;
    // a chunk of 8 channels: 36 k pairs on TM x 4 accumulator blocks, 64 cycles each, ~2.1 GHz
    static constexpr double STEP_US = TM * 4 * 36 * 64 / 2100.0;

    static dk_status launch(const dk_patch_params &p, size_t lds_bytes, hipStream_t st)
    {
        const long long blocks = (long long)p.tiles_m * p.tiles_n * p.splits;
        DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
        dk_prof_scope ps("conv_quad_fwd", st);
        conv_quad_fwd_kernel<TM, WM, WN, MAXSLOT><<<dim3((unsigned)blocks), dim3(NT), lds_bytes, st>>>(p);
        return dk_launch_status();
    }
};

using Q3Flat = QuadCfg<1, 2, 2>;     // 64 co x 256 px
using Q3Sq = QuadCfg<1, 4, 1>;       // 128 co x 128 px

template <int BM, int BN, int WM, int WN, int KH, int KW, int CB>
struct PatchCfg {
    static constexpr int bm = BM, bn = BN, cb = CB, kh = KH, kw = KW;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int MAXSLOT4 = 6, MAXSLOT1 = 14;
    static constexpr double STEP_US = (BM / WM / 32) * (BN / WN / 32) * (CB / 2 * KH * KW) * 64 / 2100.0;

    static dk_status launch(const dk_patch_params &p, int vec, size_t lds_bytes, hipStream_t st)
    {
        const long long blocks = (long long)p.tiles_m * p.tiles_n * p.splits;
        DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
        dk_prof_scope ps("conv_patch_fwd", st);
        if (vec == 4)
            conv_patch_fwd_kernel<BM, BN, WM, WN, KH, KW, CB, 4, MAXSLOT4>
                <<<dim3((unsigned)blocks), dim3(NT), lds_bytes, st>>>(p);
        else
            conv_patch_fwd_kernel<BM, BN, WM, WN, KH, KW, CB, 1, MAXSLOT1>
                <<<dim3((unsigned)blocks), dim3(NT), lds_bytes, st>>>(p);
        return dk_launch_status();
    }
};

using P3Flat = PatchCfg<64, 256, 1, 4, 3, 3, 8>;
using P3Sq = PatchCfg<128, 128, 2, 2, 3, 3, 8>;

inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

// Tile geometry for one configuration; returns false if the layer does not
// fit this kernel family (the caller then uses the generic implicit GEMM).
template <class C>
bool plan_cfg(const dk_geom &g, long long R, bool x_aligned16, dk_patch_plan *pl, bool sliding = false)
{
    dk_patch_params &p = pl->p;
    p = dk_patch_params();
    if (g.kh != C::kh || g.kw != C::kw || g.stride > 2) return false;
    const int HoWo = g.Ho * g.Wo;
    p.Ci = g.Ci; p.Co = g.Co; p.H = g.H; p.W = g.W; p.stride = g.stride; p.pad = g.pad;
    p.Ho = g.Ho; p.Wo = g.Wo; p.HoWo = HoWo; p.R = (int)R;
    p.img_g = (int)g.n;
    int n_img, rows_spanned;
    if (sliding) {
        // tiles of bn consecutive pixels of the batch; whole images in the patch
        p.multi = 2; p.BN_eff = C::bn;
        n_img = (C::bn - 1 + HoWo - 1) / HoWo + 1;      // images a tile can touch
        p.IPT = n_img;
        p.tiles_per_img = 0;
        const long long tn = (R * HoWo + C::bn - 1) / C::bn;
        if (tn >= (1ll << 30) || (long long)n_img * g.n >= (1ll << 30)) return false;
        p.tiles_n = (int)tn;
        rows_spanned = g.Ho;
    } else if (HoWo >= C::bn) {
        p.multi = 0; p.IPT = 1; p.BN_eff = C::bn;
        p.tiles_per_img = (HoWo + C::bn - 1) / C::bn;
        p.tiles_n = (int)(R * p.tiles_per_img);
        n_img = 1;
        rows_spanned = C::bn % g.Wo == 0 ? C::bn / g.Wo : (C::bn - 1) / g.Wo + 2;
        if (rows_spanned > g.Ho) rows_spanned = g.Ho;
    } else {
        p.multi = 1; p.IPT = C::bn / HoWo; p.BN_eff = p.IPT * HoWo;
        p.tiles_per_img = 0;
        p.tiles_n = (int)((R + p.IPT - 1) / p.IPT);
        n_img = p.IPT;
        rows_spanned = g.Ho;
        if ((long long)p.IPT * g.n >= (1ll << 30)) return false;
    }
    p.tiles_m = (g.Co + C::bm - 1) / C::bm;
    p.Co_pad = p.tiles_m * C::bm;
    p.LPAD = round_up(g.pad > 4 ? g.pad : 4, 4);
    p.PH = (rows_spanned - 1) * g.stride + C::kh;
    p.PW = round_up(p.LPAD + g.W + g.pad, 4);
    p.PLANE = p.PH * p.PW;
    p.patch_floats = round_up(n_img * C::cb * p.PLANE, 4);
    pl->vec = (g.W % 4 == 0 && x_aligned16) ? 4 : 1;
    p.XV = g.W / pl->vec;
    p.patch_slots = n_img * C::cb * p.PH * p.XV;
    const int maxslot = pl->vec == 4 ? C::MAXSLOT4 : C::MAXSLOT1;
    if ((p.patch_slots + C::NT - 1) / C::NT > maxslot) return false;
    pl->lds_bytes = (size_t)(p.patch_floats + C::cb * C::kh * C::kw * (C::bm + 4)) * sizeof(float);
    if (pl->lds_bytes > 64 * 1024) return false;
    p.n_chunks = (g.Ci + C::cb - 1) / C::cb;
    const dk_split_plan sp = dk_plan_split((long long)p.tiles_m * p.tiles_n, p.n_chunks, R * g.m, C::STEP_US);
    p.splits = sp.splits;
    p.per_split = sp.ktiles_per_split;
    p.out_elems = R * g.m;
    pl->wp_floats = (size_t)p.n_chunks * C::cb * C::kh * C::kw * p.Co_pad;
    pl->part_bytes = p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
    pl->cb = C::cb;
    return true;
}

// Same for the 16-byte-read kernels (3x3, stride 1, widths multiples of 4).
template <class C>
bool plan_quad(const dk_geom &g, long long R, dk_patch_plan *pl)
{
    dk_patch_params &p = pl->p;
    p = dk_patch_params();
    if (g.kh != 3 || g.kw != 3 || g.stride != 1 || g.W % 4 || g.Wo % 4 || g.pad > 4) return false;
    const int HoWo = g.Ho * g.Wo;
    p.Ci = g.Ci; p.Co = g.Co; p.H = g.H; p.W = g.W; p.stride = 1; p.pad = g.pad;
    p.Ho = g.Ho; p.Wo = g.Wo; p.HoWo = HoWo; p.R = (int)R;
    p.img_g = (int)g.n;
    int n_img, rows_spanned;
    if (HoWo >= C::bn) {
        p.multi = 0; p.IPT = 1; p.BN_eff = C::bn;
        p.tiles_per_img = (HoWo + C::bn - 1) / C::bn;
        p.tiles_n = (int)(R * p.tiles_per_img);
        n_img = 1;
        rows_spanned = C::bn % g.Wo == 0 ? C::bn / g.Wo : (C::bn - 1) / g.Wo + 2;
        if (rows_spanned > g.Ho) rows_spanned = g.Ho;
    } else {
        p.multi = 1; p.IPT = C::bn / HoWo; p.BN_eff = p.IPT * HoWo;
        p.tiles_per_img = 0;
        p.tiles_n = (int)((R + p.IPT - 1) / p.IPT);
        n_img = p.IPT;
        rows_spanned = g.Ho;
        if ((long long)p.IPT * g.n >= (1ll << 30)) return false;
    }
    // the copy addresses a tile through 32-bit byte offsets below 2^31
    if ((long long)(n_img - 1) * g.n + 8ll * g.H * g.W >= (1ll << 29)) return false;
    if (128ll * 9 * g.Ci >= (1ll << 29)) return false;
    p.tiles_m = (g.Co + C::bm - 1) / C::bm;
    p.Co_pad = p.tiles_m * C::bm;
    p.LPAD = g.pad;                      // output pixel wo sits over patch columns wo..wo+2
    p.PH = rows_spanned - 1 + 3;
    int pw = g.W + 2 * g.pad;
    if (pw < g.Wo + 4) pw = g.Wo + 4;    // the second 16-byte read of the last quad
    p.PW = round_up(pw, 4);
    p.PLANE = p.PH * p.PW;
    p.patch_floats = round_up(n_img * C::cb * p.PLANE, 4);
    pl->vec = 4;
    p.XV = g.W / 4;
    p.patch_slots = n_img * C::cb * p.PH * p.XV;
    if ((p.patch_slots + C::NT - 1) / C::NT > C::MAXSLOT) return false;
    pl->lds_bytes = (size_t)(p.patch_floats + C::bm * 76) * sizeof(float) + 1024;   // + dump area
    if (pl->lds_bytes > 64 * 1024) return false;
    p.n_chunks = (g.Ci + C::cb - 1) / C::cb;
    const dk_split_plan sp = dk_plan_split((long long)p.tiles_m * p.tiles_n, p.n_chunks, R * g.m, C::STEP_US);
    p.splits = sp.splits;
    p.per_split = sp.ktiles_per_split;
    p.out_elems = R * g.m;
    pl->wp_floats = (size_t)p.n_chunks * 72 * p.Co_pad;
    p.w_row = 72;
    p.w_chunk = 72ll * p.Co_pad;
    pl->part_bytes = p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
    pl->cb = C::cb;
    pl->quad = true;
    return true;
}

} // namespace

bool dk_patch_fwd_plan(const dk_geom &g, long long R, bool aligned16, dk_patch_plan *pl)
{
    if (!g.conv || R < 1) return false;
    pl->quad = false;
    if (g.kh == 3 && g.kw == 3) {
        pl->flat = g.Co <= 64;
        if (aligned16 && (pl->flat ? plan_quad<Q3Flat>(g, R, pl) : plan_quad<Q3Sq>(g, R, pl))) return true;
        pl->quad = false;
        // columns of the per-image tilings that carry pixels; below nine tenths, tiles that
        // slide over the batch are tried first (they need whole images in LDS)
        const int bn = pl->flat ? P3Flat::bn : P3Sq::bn;
        const int HoWo = g.Ho * g.Wo;
        const double used = HoWo >= bn ? (double)HoWo / ((HoWo + bn - 1) / bn * bn) : (double)(bn / HoWo * HoWo) / bn;
        if (used < 0.9 && (pl->flat ? plan_cfg<P3Flat>(g, R, aligned16, pl, true) : plan_cfg<P3Sq>(g, R, aligned16, pl, true)))
            return true;
        return pl->flat ? plan_cfg<P3Flat>(g, R, aligned16, pl) : plan_cfg<P3Sq>(g, R, aligned16, pl);
    }
    return false;
}

dk_status dk_patch_fwd_run(const dk_geom &g, dk_patch_plan &pl, const float *W, const float *xbar,
                           float *ybar, float *ws, hipStream_t st)
{
    dk_patch_params &p = pl.p;
    float *wp = ws;
    float *part = (float *)((char *)ws + dk_patch_wp_bytes(pl));
    const long long total = (long long)pl.wp_floats;
    // W[co][ci][3][3] already has the quad kernel's order inside a chunk of 8
    // input channels (position (c' + 4h)*9 + a*3 + b = h*36 + (c'*3 + a)*3 + b), so
    // with whole chunks, whole tiles and an aligned W the repack is skipped
    const bool direct = pl.quad && g.Ci % 8 == 0 && p.Co_pad == g.Co && dk_aligned(W, 16);
    if (direct) {
        p.w_row = 9ll * g.Ci;
        p.w_chunk = 72;
        wp = const_cast<float *>(W);
    } else {
        dk_prof_scope ps("pack_filters", st);
        if (pl.quad)
            pack_filters_quad_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
                W, wp, g.Ci, g.Co, p.Co_pad, total);
        else
            pack_filters_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(
                W, wp, g.Ci, g.Co, g.kh, g.kw, pl.cb, p.Co_pad, total);
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    p.x = xbar; p.wp = wp; p.out = ybar; p.part = part;
    dk_status s;
    if (pl.quad)
        s = pl.flat ? Q3Flat::launch(p, pl.lds_bytes, st) : Q3Sq::launch(p, pl.lds_bytes, st);
    else
        s = pl.flat ? P3Flat::launch(p, pl.vec, pl.lds_bytes, st) : P3Sq::launch(p, pl.vec, pl.lds_bytes, st);
    if (s != DK_OK) return s;
    if (p.splits > 1) return dk_fold_slices(part, ybar, p.out_elems, p.splits, 1.0f, 0, st);
    return DK_OK;
}
