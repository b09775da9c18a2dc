// Convolution weight gradient on encoded images with the input staged as a
// zero-padded patch in LDS.
//
//   dW[co][ci][a][b] = sum over encoded rows r and output pixels (ho, wo) of
//       dtilde[r][co][ho][wo] * xbar[r][ci][ho*s + a - pad][wo*s + b - pad]
//
// MFMA mapping: rows = co (A operand, from dtilde), columns = ci (B operand,
// from the patch), contraction = output pixels, taken two at a time (lanes
// 0-31 the even pixel of a pair, lanes 32-63 the odd one).  Every filter tap
// (a, b) is its own accumulator block fed by the SAME A value and by the patch
// read at a tap-shifted address, so one A fetch and KH*KW B fetches feed
// KH*KW MFMAs and the inner loop has no bounds tests and no per-element
// address arithmetic.  A workgroup owns 64 co x 64 ci x all taps and a
// contiguous range of pixel tiles (NI images x TR output rows each); partial
// sums of all workgroups are folded in a fixed order by a second kernel, which
// also applies scale / accumulate and writes dW's [co][ci][kh][kw] layout.
#include "dk_internal.h"
#include <type_traits>

#include "dk_patch.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int KH, int KW, int STRIDE, int VEC, int DSLOT, int PSLOT>
__global__ __launch_bounds__(256) void conv_patch_wgrad_kernel(dk_wgpatch_params p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int NT = 256, BM = 64, BCI = 64, KK = KH * KW;

    float *const Ad = lds;                       // [BM][LDQ]   dtilde tile
    float *const Pt = lds + p.ad_floats;         // [BCI][CPLANE] input patch

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave & 1) * 32, wn0 = (wave >> 1) * 32;

    const int tiles = p.tiles_co * p.tiles_ci;
    const int split = blockIdx.x / tiles;
    const int t = blockIdx.x - split * tiles;
    const int tci = t / p.tiles_co, tco = t - tci * p.tiles_co;
    const int co0 = tco * BM, ci0 = tci * BCI;

    // copy slots of this lane (tile-independent parts)
    int d_g[DSLOT], d_l[DSLOT], d_img[DSLOT], d_q[DSLOT];
#pragma unroll
    for (int e = 0; e < DSLOT; ++e) {
        const int idx = tid + e * NT;
        const int dv = idx % p.DV;
        const int t1 = idx / p.DV;
        const int img_l = t1 % p.NI;
        const int co_l = t1 / p.NI;
        const bool act = idx < p.d_slots && co0 + co_l < p.Co;
        d_g[e] = (img_l * p.Co + co_l) * p.HoWo + dv * VEC;
        d_l[e] = co_l * p.LDQ + img_l * p.TR * p.Wo + dv * VEC;
        d_img[e] = act ? img_l : -1;
        d_q[e] = dv * VEC;                       // pixel offset inside the row block
    }
    int p_g[PSLOT], p_l[PSLOT], p_img[PSLOT], p_row[PSLOT];
#pragma unroll
    for (int e = 0; e < PSLOT; ++e) {
        const int idx = tid + e * NT;
        const int xv = idx % p.XV;
        const int t1 = idx / p.XV;
        const int prow = t1 % p.PH;
        const int t2 = t1 / p.PH;
        const int img_l = t2 % p.NI;
        const int c_l = t2 / p.NI;
        const bool act = idx < p.p_slots && ci0 + c_l < p.Ci;
        p_g[e] = (img_l * p.Ci + c_l) * p.H * p.W + prow * p.W + xv * VEC;
        p_l[e] = c_l * p.CPLANE + img_l * p.PLANE + prow * p.PW + p.LPAD + xv * VEC;
        p_img[e] = act ? img_l : -1;
        p_row[e] = prow;
    }

    for (int i = tid; i < p.lds_floats; i += NT) lds[i] = 0.0f;

    f32x16 acc[KK];
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[k][v] = 0.0f;

    const int pt0 = split * p.per_split;
    int pt1 = pt0 + p.per_split;
    if (pt1 > p.n_ptiles) pt1 = p.n_ptiles;

    using stage_t = typename std::conditional<VEC == 4, f32x4, float>::type;
    stage_t dst_[DSLOT], pst_[PSLOT];

#define DK_WG_FETCH(PT)                                                                          \
    {                                                                                            \
        const int ig_ = (PT) / p.row_blocks;                                                     \
        const int rb_ = (PT) - ig_ * p.row_blocks;                                               \
        const int r0_ = ig_ * p.NI, row0_ = rb_ * p.TR;                                          \
        const int qlim_ = p.HoWo - row0_ * p.Wo; /* pixels left in the image from row0 */        \
        const float *dsrc_ = p.dt + ((long long)r0_ * p.Co + co0) * p.HoWo + (long long)row0_ * p.Wo; \
        _Pragma("unroll") for (int e = 0; e < DSLOT; ++e) {                                      \
            const bool ok_ = d_img[e] >= 0 && r0_ + d_img[e] < p.R && d_q[e] < qlim_;            \
            stage_t v_ = stage_t(0.0f);                                                          \
            if (ok_) v_ = *reinterpret_cast<const stage_t *>(dsrc_ + d_g[e]);                    \
            dst_[e] = v_;                                                                        \
        }                                                                                        \
        const int ih_a_ = row0_ * STRIDE - p.pad;                                                \
        const long long pbase_ = ((long long)r0_ * p.Ci + ci0) * p.H * p.W + (long long)ih_a_ * p.W; \
        _Pragma("unroll") for (int e = 0; e < PSLOT; ++e) {                                      \
            const int ih_ = ih_a_ + p_row[e];                                                    \
            const bool ok_ = p_img[e] >= 0 && r0_ + p_img[e] < p.R && ih_ >= 0 && ih_ < p.H;     \
            stage_t v_ = stage_t(0.0f);                                                          \
            if (ok_) v_ = *reinterpret_cast<const stage_t *>(p.x + pbase_ + p_g[e]);             \
            pst_[e] = v_;                                                                        \
        }                                                                                        \
    }

    if (pt0 < pt1) DK_WG_FETCH(pt0)
    for (int pt = pt0; pt < pt1; ++pt) {
        __syncthreads();                 // previous tile consumed (and the zero fill done)
#pragma unroll
        for (int e = 0; e < DSLOT; ++e) {
            if (d_img[e] < 0) continue;
            float *d = Ad + d_l[e];
            if constexpr (VEC == 4) { d[0] = dst_[e].x; d[1] = dst_[e].y; d[2] = dst_[e].z; d[3] = dst_[e].w; }
            else d[0] = dst_[e];
        }
#pragma unroll
        for (int e = 0; e < PSLOT; ++e) {
            if (p_img[e] < 0) continue;
            *reinterpret_cast<stage_t *>(Pt + p_l[e]) = pst_[e];
        }
        __syncthreads();
        if (pt + 1 < pt1) DK_WG_FETCH(pt + 1)   // in flight during the MFMA loop

        for (int img_l = 0; img_l < p.NI; ++img_l)
            for (int row = 0; row < p.TR; ++row) {
                const float *a_ptr = Ad + (wm0 + li) * p.LDQ + (img_l * p.TR + row) * p.Wo + lh;
                const float *b_ptr = Pt + (wn0 + li) * p.CPLANE + img_l * p.PLANE +
                                     row * STRIDE * p.PW + p.LPAD - p.pad + lh * STRIDE;
                const float *b_row[KH];
#pragma unroll
                for (int a = 0; a < KH; ++a) b_row[a] = b_ptr + a * p.PW;
                const int npair = p.Wo >> 1;
                // operands of pixel pair cp+1 are fetched while pair cp is in the
                // MFMA pipe (the last pair re-reads itself instead of running past the row)
                float av = a_ptr[0], bv[KK];
#pragma unroll
                for (int a = 0; a < KH; ++a)
#pragma unroll
                    for (int b = 0; b < KW; ++b) bv[a * KW + b] = b_row[a][b];
                for (int cp = 0; cp < npair; ++cp) {
                    const int cn = cp + 1 < npair ? cp + 1 : cp;
                    const float av_n = a_ptr[2 * cn];
                    float bv_n[KK];
#pragma unroll
                    for (int a = 0; a < KH; ++a)
#pragma unroll
                        for (int b = 0; b < KW; ++b) bv_n[a * KW + b] = b_row[a][2 * cn * STRIDE + b];
                    __builtin_amdgcn_sched_barrier(0);     // keep the LDS reads ahead of the MFMAs
#pragma unroll
                    for (int k = 0; k < KK; ++k)
                        acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[k], acc[k], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    av = av_n;
#pragma unroll
                    for (int k = 0; k < KK; ++k) bv[k] = bv_n[k];
                }
            }
    }
#undef DK_WG_FETCH

    // partial sums: part[split][tap][co][ci], lanes along ci
    float *dstp = p.part + (long long)split * p.part_elems;
    const int ci = ci0 + wn0 + li;
    if (ci < p.Ci) {
#pragma unroll
        for (int k = 0; k < KK; ++k)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int co = co0 + wm0 + 8 * (v / 4) + 4 * lh + (v % 4);
                if (co < p.Co) dstp[((long long)k * p.Co + co) * p.Ci + ci] = acc[k][v];
            }
    }
}

// dW[co][ci][tap] = (accumulate ? dW : 0) + scale * sum_s part[s][tap][co][ci].
// A workgroup folds 64 consecutive elements; its four 64-lane waves each sum
// every fourth slice (loads batched eight deep) and the four sub-sums are
// added in wave order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void wgrad_fold_kernel(const float *__restrict__ part,
                                                         float *__restrict__ dW, int Co, int Ci,
                                                         int KK, long long part_elems, int splits,
                                                         float scale, int accumulate)
{
    __shared__ float red[4][64];
    const int io = threadIdx.x & 63, sg = threadIdx.x >> 6;
    const long long i = (long long)blockIdx.x * 64 + io;
    float s = 0.0f;
    if (i < part_elems) {
        const float *src = part + i;
        int k = sg;
        for (; k + 28 < splits; k += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(long long)(k + 4 * u) * part_elems];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; k < splits; k += 4) s += src[(long long)k * part_elems];
    }
    red[sg][io] = s;
    __syncthreads();
    if (sg != 0 || i >= part_elems) return;
    s = ((red[0][io] + red[1][io]) + red[2][io]) + red[3][io];
    const int ci = (int)(i % Ci);
    const long long t = i / Ci;
    const int co = (int)(t % Co);
    const int tap = (int)(t / Co);
    float *d = dW + ((long long)co * Ci + ci) * KK + tap;
    s *= scale;
    if (accumulate) s += *d;
    *d = s;
}

inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

constexpr int DSLOT4 = 4, PSLOT4 = 8, DSLOT1 = 8, PSLOT1 = 24;
constexpr size_t LDS_LIMIT = 64 * 1024;

template <int KH, int KW>
dk_status launch_k(const dk_wgpatch_params &p, int vec, size_t lds_bytes, hipStream_t st)
{
    const long long blocks = (long long)p.tiles_co * p.tiles_ci * p.splits;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    const dim3 grid((unsigned)blocks), blk(256);
    if (p.stride == 1) {
        if (vec == 4) conv_patch_wgrad_kernel<KH, KW, 1, 4, DSLOT4, PSLOT4><<<grid, blk, lds_bytes, st>>>(p);
        else conv_patch_wgrad_kernel<KH, KW, 1, 1, DSLOT1, PSLOT1><<<grid, blk, lds_bytes, st>>>(p);
    } else {
        if (vec == 4) conv_patch_wgrad_kernel<KH, KW, 2, 4, DSLOT4, PSLOT4><<<grid, blk, lds_bytes, st>>>(p);
        else conv_patch_wgrad_kernel<KH, KW, 2, 1, DSLOT1, PSLOT1><<<grid, blk, lds_bytes, st>>>(p);
    }
    return dk_launch_status();
}

} // namespace

bool dk_patch_wgrad_plan(const dk_geom &g, long long R, bool aligned16, dk_wgpatch_plan *pl)
{
    if (!g.conv || R < 1) return false;
    if (!(g.kh == 3 && g.kw == 3)) return false;
    if (g.stride > 2 || (g.Wo & 1)) return false;
    dk_wgpatch_params &p = pl->p;
    p = dk_wgpatch_params();
    const int HoWo = g.Ho * g.Wo;
    p.Ci = g.Ci; p.Co = g.Co; p.H = g.H; p.W = g.W; p.stride = g.stride; p.pad = g.pad;
    p.Ho = g.Ho; p.Wo = g.Wo; p.HoWo = HoWo; p.R = (int)R;
    if ((long long)g.Co * HoWo >= (1ll << 26) || g.n >= (1ll << 26)) return false;
    const bool v4 = aligned16 && g.W % 4 == 0 && g.Wo % 4 == 0;
    pl->vec = v4 ? 4 : 1;
    const int dmax = (v4 ? DSLOT4 : DSLOT1) * 256, pmax = (v4 ? PSLOT4 : PSLOT1) * 256;
    p.LPAD = round_up(g.pad > 4 ? g.pad : 4, 4);
    p.PW = round_up(p.LPAD + g.W + g.pad, 4);

    // choose the pixel tile: as many output rows (then whole images) as the
    // copy slots and 64 KB of LDS allow
    int bestTR = 0, bestNI = 0;
    for (int pass = 0; pass < 2; ++pass) {
        // pass 0: row blocks of one image; pass 1: several whole images
        for (int cand = 1; cand <= 64; ++cand) {
            const int TR = pass == 0 ? cand : g.Ho;
            const int NI = pass == 0 ? 1 : cand;
            if (pass == 0 && TR > g.Ho) break;
            if (pass == 1 && (NI < 2 || NI > R)) { if (NI > R) break; else continue; }
            if (pass == 0 && v4 && (TR * g.Wo) % 4) continue;
            const int PH = (TR - 1) * g.stride + g.kh;
            const int PLANE = PH * p.PW;
            const int CPLANE = (NI * PLANE) | 1;
            const int QT = NI * TR * g.Wo;
            const int LDQ = QT | 1;
            const long long d_slots = 64ll * NI * (TR * g.Wo / pl->vec);
            const long long p_slots = 64ll * NI * PH * (g.W / pl->vec);
            const size_t bytes = ((size_t)round_up(64 * LDQ, 4) + 64 * (size_t)CPLANE) * 4;
            if (d_slots > dmax || p_slots > pmax || bytes > LDS_LIMIT) break;
            if ((long long)NI * g.Co * HoWo >= (1ll << 30) || (long long)NI * g.n >= (1ll << 30)) break;
            bestTR = TR; bestNI = NI;
        }
        if (bestTR < g.Ho) break;      // could not even fit one whole image: stay with row blocks
    }
    if (bestTR == 0) return false;
    p.TR = bestTR; p.NI = bestNI;
    p.PH = (p.TR - 1) * g.stride + g.kh;
    p.PLANE = p.PH * p.PW;
    p.CPLANE = (p.NI * p.PLANE) | 1;
    p.QT = p.NI * p.TR * g.Wo;
    p.LDQ = p.QT | 1;
    p.DV = p.TR * g.Wo / pl->vec;
    p.XV = g.W / pl->vec;
    p.d_slots = 64 * p.NI * p.DV;
    p.p_slots = 64 * p.NI * p.PH * p.XV;
    p.ad_floats = round_up(64 * p.LDQ, 4);
    p.lds_floats = p.ad_floats + 64 * p.CPLANE;
    pl->lds_bytes = (size_t)p.lds_floats * 4;
    p.row_blocks = (g.Ho + p.TR - 1) / p.TR;
    p.n_ptiles = (int)((R + p.NI - 1) / p.NI) * p.row_blocks;
    p.tiles_co = (g.Co + 63) / 64;
    p.tiles_ci = (g.Ci + 63) / 64;
    p.part_elems = (long long)g.kh * g.kw * g.Co * g.Ci;
    // about two workgroups per compute unit; never more partial sums than 256 MB
    long long s = 256 / ((long long)p.tiles_co * p.tiles_ci);   // one resident workgroup per compute unit
    if (s < 1) s = 1;
    if (s > p.n_ptiles) s = p.n_ptiles;
    while (s > 1 && s * p.part_elems * 4 > (256ll << 20)) --s;
    p.per_split = (int)((p.n_ptiles + s - 1) / s);
    p.splits = (p.n_ptiles + p.per_split - 1) / p.per_split;
    pl->part_bytes = (size_t)p.splits * p.part_elems * 4;
    return true;
}

dk_status dk_patch_wgrad_run(const dk_geom &g, dk_wgpatch_plan &pl, const float *dtilde,
                             const float *xbar, float *dW, float scale, int accumulate,
                             float *part, hipStream_t st)
{
    dk_wgpatch_params &p = pl.p;
    p.dt = dtilde; p.x = xbar; p.part = part;
    dk_status s = launch_k<3, 3>(p, pl.vec, pl.lds_bytes, st);
    if (s != DK_OK) return s;
    wgrad_fold_kernel<<<dim3((unsigned)((p.part_elems + 63) / 64)), dim3(256), 0, st>>>(
        part, dW, g.Co, g.Ci, g.kh * g.kw, p.part_elems, p.splits, scale, accumulate);
    return dk_launch_status();
}
