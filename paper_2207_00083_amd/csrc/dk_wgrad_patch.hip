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
typedef float f32x2 __attribute__((ext_vector_type(2)));

// last word of a raw (untyped, unstrided) buffer resource on gfx9-family parts
constexpr int DK_BUFFER_RSRC_FLAGS = 0x00020000;

// The copy waves (waves 4-7) of the weight-gradient kernels: tile pt of the
// workgroup's range goes to LDS buffer (pt - pt0) & 1 while the MFMA waves work
// on the other buffer; one barrier per tile hands the buffers over.  DVEC /
// PVEC: the dtilde tile / the patch take 16-byte LDS stores (else four 4-byte
// ones: odd pitch, or a position one column off alignment).
template <int DSLOT, int PSLOT, bool DVEC, bool PVEC>
__device__ __forceinline__ void wg_copy_waves(const dk_wgpatch_params &p, float *lds, int tid, int co0,
                                              int ci0, int pt0, int pt1)
{
    constexpr int NP = 256;
    // Vector-ALU instructions of this wave queue behind the matrix
    // instructions of the MFMA wave on the same SIMD (measured: about one
    // issue slot per MFMA), so a tile must cost as few of them as possible.
    // Everything a lane needs is computed once: byte offsets from a
    // wave-uniform base for the loads, LDS addresses in both buffers for the
    // stores (an unused slot loads offset 0 and stores into a dump area
    // behind the buffers, so nothing is predicated).  The tile position
    // advances in scalar registers, and a tile that lies wholly inside its
    // images and their rows is copied without any test.
    if constexpr (DVEC) __builtin_amdgcn_s_setprio(3);   // (measured: helps the 16-byte-read kernel, hurts the other)
    const int ptid = tid - 256;
    float *const dump = lds + 2 * p.buf_floats + (ptid & 63) * 4;
    unsigned d_g[DSLOT], p_g[PSLOT];          // byte offsets
    float *d_l[2][DSLOT], *p_l[2][PSLOT];
    int d_m[DSLOT], p_m[PSLOT];
#pragma unroll
    for (int e = 0; e < DSLOT; ++e) {
        const int idx = ptid + e * NP;
        const int dv = idx % p.DV;
        const int t1 = idx / p.DV;
        const int img_l = t1 % p.NI;
        const int co_l = t1 / p.NI;
        const bool act = idx < p.d_slots && co0 + co_l < p.Co;
        d_g[e] = act ? 4u * (unsigned)((img_l * p.Co + co_l) * p.HoWo + dv * 4) : 0u;
        const int l = co_l * p.LDQ + img_l * p.TR * p.Wo + dv * 4;
        d_l[0][e] = act ? lds + l : dump;
        d_l[1][e] = act ? lds + p.buf_floats + l : dump;
        d_m[e] = act ? (img_l | (dv * 4) << 8) : -1;
    }
#pragma unroll
    for (int e = 0; e < PSLOT; ++e) {
        const int idx = ptid + e * NP;
        const int xv = idx % p.XV;
        const int t1 = idx / p.XV;
        const int prow = t1 % p.PH;
        const int t2 = t1 / p.PH;
        const int img_l = t2 % p.NI;
        const int c_l = t2 / p.NI;
        const bool act = idx < p.p_slots && ci0 + c_l < p.Ci;
        p_g[e] = act ? 4u * (unsigned)((img_l * p.Ci + c_l) * p.H * p.W + prow * p.W + xv * 4) : 0u;
        const int l = p.ad_floats + c_l * p.CPLANE + img_l * p.PLANE + prow * p.PW + p.LPAD + xv * 4;
        p_l[0][e] = act ? lds + l : dump;
        p_l[1][e] = act ? lds + p.buf_floats + l : dump;
        p_m[e] = act ? (img_l | prow << 8) : -1;
    }
    int ig = pt0 / p.row_blocks, rb = pt0 - ig * p.row_blocks;
    // tile pt goes to buffer (pt - pt0) & 1: two tiles per trip, so that the
    // buffer is known at compile time
    auto copy_tile = [&](auto bufc) {
        constexpr int BUF = decltype(bufc)::value;
        const int r0 = ig * p.NI, row0 = rb * p.TR;
        const char *dsrc = reinterpret_cast<const char *>(
            p.dt + ((long long)r0 * p.Co + co0) * p.HoWo + (long long)row0 * p.Wo);
        const int ih_a = row0 - p.pad;
        const char *psrc = reinterpret_cast<const char *>(
            p.x + ((long long)r0 * p.Ci + ci0) * p.H * p.W + (long long)ih_a * p.W);
        f32x4 dst_[DSLOT], pst_[PSLOT];
        const bool clean = r0 + p.NI <= p.R && row0 + p.TR <= p.Ho && ih_a >= 0 && ih_a + p.PH <= p.H;
        if (clean) {
            // buffer loads: wave-uniform base in a scalar resource, the lane's
            // byte offset as it is -- no address arithmetic on the vector ALU
            const __amdgpu_buffer_rsrc_t rd =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(dsrc), 0, -1, DK_BUFFER_RSRC_FLAGS);
            const __amdgpu_buffer_rsrc_t rp =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(psrc), 0, -1, DK_BUFFER_RSRC_FLAGS);
#pragma unroll
            for (int e = 0; e < DSLOT; ++e)
                dst_[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rd, (int)d_g[e], 0, 0));
#pragma unroll
            for (int e = 0; e < PSLOT; ++e)
                pst_[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rp, (int)p_g[e], 0, 0));
        } else {
            // out of range for this tile: read the tile's first element, store zero
            const int qlim = p.HoWo - row0 * p.Wo;
            const int ilim = p.R - r0;
            const char *psrc0 = reinterpret_cast<const char *>(p.x + ((long long)r0 * p.Ci + ci0) * p.H * p.W);
            const int poffb = 4 * ih_a * p.W;
#pragma unroll
            for (int e = 0; e < DSLOT; ++e) {
                const bool ok = d_m[e] >= 0 && (d_m[e] & 255) < ilim && (d_m[e] >> 8) < qlim;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(dsrc + (ok ? d_g[e] : 0u));
                dst_[e] = ok ? v : f32x4(0.0f);
            }
#pragma unroll
            for (int e = 0; e < PSLOT; ++e) {
                const int ih = ih_a + (p_m[e] >> 8);
                const bool ok = p_m[e] >= 0 && (p_m[e] & 255) < ilim && ih >= 0 && ih < p.H;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(psrc0 + (ok ? (unsigned)((int)p_g[e] + poffb) : 0u));
                pst_[e] = ok ? v : f32x4(0.0f);
            }
        }
#pragma unroll
        for (int e = 0; e < DSLOT; ++e) {
            if constexpr (DVEC) {
                *reinterpret_cast<f32x4 *>(d_l[BUF][e]) = dst_[e];
            } else {
                float *d = d_l[BUF][e];           // odd pitch
                d[0] = dst_[e].x; d[1] = dst_[e].y; d[2] = dst_[e].z; d[3] = dst_[e].w;
            }
        }
#pragma unroll
        for (int e = 0; e < PSLOT; ++e) {
            if constexpr (PVEC) {
                *reinterpret_cast<f32x4 *>(p_l[BUF][e]) = pst_[e];
            } else {
                float *d = p_l[BUF][e];           // one column off 16-byte alignment
                d[0] = pst_[e].x; d[1] = pst_[e].y; d[2] = pst_[e].z; d[3] = pst_[e].w;
            }
        }
        if (++rb == p.row_blocks) { rb = 0; ++ig; }
        __syncthreads();     // this tile is in LDS; the one before has been consumed
    };
    for (int pt = pt0; pt < pt1; pt += 2) {
        copy_tile(std::integral_constant<int, 0>());
        if (pt + 1 < pt1) copy_tile(std::integral_constant<int, 1>());
    }
    if (pt0 < pt1) __syncthreads();   // matches the MFMA waves' last barrier
}

template <int KH, int KW, int DSLOT, int PSLOT>
__global__ __launch_bounds__(512) void conv_patch_wgrad_kernel(dk_wgpatch_params p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int BM = 64, BCI = 64, KK = KH * KW;
    constexpr int STRIDE = 1;              // stride-1 layers whose rows are whole 16-byte vectors

    // Two LDS buffers of [dtilde tile: BM x LDQ][input patch: BCI x CPLANE].
    // Waves 0-3 (one per SIMD) only run MFMAs on the current buffer; waves 4-7
    // only copy the next pixel tile from global memory into the other buffer.
    // One barrier per tile hands the buffers over.
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const bool producer = wave >= 4;

    const int tiles = p.tiles_co * p.tiles_ci;
    const int split = blockIdx.x / tiles;
    const int t = blockIdx.x - split * tiles;
    const int tci = t / p.tiles_co, tco = t - tci * p.tiles_co;
    const int co0 = tco * BM, ci0 = tci * BCI;

    const int pt0 = split * p.per_split;
    int pt1 = pt0 + p.per_split;
    if (pt1 > p.n_ptiles) pt1 = p.n_ptiles;

    for (int i = tid; i < 2 * p.buf_floats; i += 512) lds[i] = 0.0f;
    __syncthreads();

    if (producer) {
        wg_copy_waves<DSLOT, PSLOT, false, true>(p, lds, tid, co0, ci0, pt0, pt1);
        return;
    }

    // ---- MFMA waves ----
    const int lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave & 1) * 32, wn0 = (wave >> 1) * 32;

    f32x16 acc[KK];
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[k][v] = 0.0f;

    const int nrows = p.NI * p.TR;
    const int npair = p.Wo >> 1;
    const int total = nrows * npair;      // pixel pairs per tile
    if (pt0 < pt1) __syncthreads();       // tile pt0 is in LDS
    for (int pt = pt0; pt < pt1; ++pt) {
        const float *Ad = lds + ((pt - pt0) & 1) * p.buf_floats;
        const float *Pt = Ad + p.ad_floats;
        const float *a_base = Ad + (wm0 + li) * p.LDQ + lh;
        const float *b_base = Pt + (wn0 + li) * p.CPLANE + p.LPAD - p.pad + lh * STRIDE;

        // Load cursor: walks the tile's pixel pairs (row by row) one step ahead
        // of the MFMAs.  Past the last pair it stays on the last one.
        int ld_row = 0, ld_cp = 0;
        const float *a_ld = a_base, *b_ld[KH];
#pragma unroll
        for (int a = 0; a < KH; ++a) b_ld[a] = b_base + a * p.PW;
#define DK_WG_ADVANCE()                                                                          \
        if (ld_cp + 1 < npair) {                                                                 \
            ++ld_cp;                                                                             \
        } else if (ld_row + 1 < nrows) {                                                         \
            ld_cp = 0; ++ld_row;                                                                 \
            const int img_l_ = ld_row / p.TR, row_ = ld_row - img_l_ * p.TR;                     \
            a_ld = a_base + ld_row * p.Wo;                                                       \
            _Pragma("unroll") for (int a = 0; a < KH; ++a)                                       \
                b_ld[a] = b_base + img_l_ * p.PLANE + (row_ * STRIDE + a) * p.PW;                \
        }
        // Operands of the next pixel pair are read from LDS while the current
        // pair is in the MFMA pipe: the reads are spread between the MFMAs, and
        // two register sets alternate so nothing is copied.
#define DK_WG_STEP(AVN, BVN, AVC, BVC)                                                           \
        {                                                                                        \
            AVN = a_ld[2 * ld_cp];                                                               \
            _Pragma("unroll") for (int a = 0; a < KH; ++a)                                       \
                _Pragma("unroll") for (int b = 0; b < KW; ++b)                                   \
                    BVN[a * KW + b] = b_ld[a][2 * ld_cp * STRIDE + b];                           \
            _Pragma("unroll") for (int k = 0; k < KK; ++k)                                       \
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(AVC, BVC[k], acc[k], 0, 0, 0);     \
            _Pragma("unroll") for (int k = 0; k < KK; ++k) {                                     \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   /* one MFMA  */             \
                __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);   /* one VALU  */             \
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   /* one LDS read */          \
            }                                                                                    \
            __builtin_amdgcn_sched_barrier(0);                                                   \
            /* keep the consumed operand registers live to here: a register that an MFMA */     \
            /* in flight still reads must not be the target of the interleaved LDS reads */     \
            asm volatile("" ::"v"(AVC));                                                         \
            _Pragma("unroll") for (int k = 0; k < KK; ++k) asm volatile("" ::"v"(BVC[k]));       \
        }
        float av0, bv0[KK], av1, bv1[KK];
        av0 = a_ld[0];
#pragma unroll
        for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int b = 0; b < KW; ++b) bv0[a * KW + b] = b_ld[a][b];
        __builtin_amdgcn_sched_barrier(0);
        int f = 0;
        for (; f + 2 <= total; f += 2) {
            DK_WG_ADVANCE()
            DK_WG_STEP(av1, bv1, av0, bv0)
            DK_WG_ADVANCE()
            DK_WG_STEP(av0, bv0, av1, bv1)
        }
        if (f < total) {                     // odd number of pairs in the tile
#pragma unroll
            for (int k = 0; k < KK; ++k)
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0, bv0[k], acc[k], 0, 0, 0);
        }
#undef DK_WG_ADVANCE
#undef DK_WG_STEP
        __syncthreads();     // done with this buffer; the next tile is in the other one
    }

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

// Same contraction for stride 1 and output widths that are a multiple of 8
// (or of 4, with an even number of output rows), with 16-byte LDS reads.  Handing single floats from LDS to the matrix pipe
// costs one LDS instruction per operand and those, not the MFMAs, then set the
// pace.  Here the two half-waves take the left and the right half of an output
// row instead of even and odd pixels, so four consecutive pixels of a half are
// one aligned 16-byte read of dtilde, and the three filter columns of those four
// pixels lie in two aligned 16-byte reads of the patch row (the patch is stored
// with `pad` columns of left border, which puts output pixel wo over patch
// columns wo..wo+2).  Seven LDS instructions feed 36 MFMAs.  For widths that are
// not a multiple of 8 the half-waves take the even and the odd rows instead.
template <int DSLOT, int PSLOT>
__global__ __launch_bounds__(512) void conv_quad_wgrad_kernel(dk_wgpatch_params p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int BM = 64, BCI = 64, KH = 3, KW = 3, KK = 9;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const bool producer = wave >= 4;

    const int tiles = p.tiles_co * p.tiles_ci;
    const int split = blockIdx.x / tiles;
    const int t = blockIdx.x - split * tiles;
    const int tci = t / p.tiles_co, tco = t - tci * p.tiles_co;
    const int co0 = tco * BM, ci0 = tci * BCI;

    const int pt0 = split * p.per_split;
    int pt1 = pt0 + p.per_split;
    if (pt1 > p.n_ptiles) pt1 = p.n_ptiles;

    for (int i = tid; i < 2 * p.buf_floats; i += 512) lds[i] = 0.0f;
    __syncthreads();

    if (producer) {
        wg_copy_waves<DSLOT, PSLOT, true, false>(p, lds, tid, co0, ci0, pt0, pt1);
        return;
    }

    // ---- MFMA waves ----
    const int lane = tid & 63;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave & 1) * 32, wn0 = (wave >> 1) * 32;
    // The two half-waves split every output row in a left and a right half
    // (widths that are multiples of 8), or take the even and the odd rows of
    // the tile (other multiples of 4; tiles then have an even number of rows
    // per image): either way a half-wave walks whole 4-pixel steps.
    const bool rowsplit = (p.Wo & 7) != 0;
    const int rstep = rowsplit ? 2 : 1;
    const int a_half = rowsplit ? p.Wo : p.Wo >> 1;     // dtilde offset of the second half-wave
    const int b_half = rowsplit ? p.PW : p.Wo >> 1;     // patch offset of the second half-wave

    f32x16 acc[KK];
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[k][v] = 0.0f;

    const int nrows = p.NI * p.TR;
    const int nquad = (rowsplit ? p.Wo : p.Wo >> 1) >> 2;    // 4-pixel steps per row of a half-wave
    const int total = (nrows / rstep) * nquad;
    if (pt0 < pt1) __syncthreads();
    for (int pt = pt0; pt < pt1; ++pt) {
        const float *Ad = lds + ((pt - pt0) & 1) * p.buf_floats;
        const float *Pt = Ad + p.ad_floats;
        const float *a_base = Ad + (wm0 + li) * p.LDQ + lh * a_half;
        const float *b_base = Pt + (wn0 + li) * p.CPLANE + lh * b_half;

        // load cursor, one 4-pixel step ahead of the MFMAs; it stays on the
        // last step of the tile once it gets there
        int ld_row = 0, ld_q = 0, ld_img = 0, ld_r = 0;       // ld_row = ld_img * TR + ld_r
        const float *a_ld = a_base, *b_ld = b_base;
#define DK_WGQ_ADVANCE()                                                                         \
        if (ld_q + 1 < nquad) {                                                                  \
            ++ld_q;                                                                              \
        } else if (ld_row + rstep < nrows) {                                                     \
            ld_q = 0; ld_row += rstep; ld_r += rstep;                                            \
            if (ld_r == p.TR) { ld_r = 0; ++ld_img; }                                            \
            a_ld = a_base + ld_row * p.Wo;                                                       \
            b_ld = b_base + ld_img * p.PLANE + ld_r * p.PW;                                      \
        }
        // The six patch columns of a filter row come as a 16-byte and an 8-byte
        // read: a second 16-byte read would leave two registers dead, the
        // register allocator would overlap the tuples, and overlapping read
        // targets force a full wait between the reads.
#define DK_WGQ_LOAD(A, B, C)                                                                     \
        {                                                                                        \
            A = *reinterpret_cast<const f32x4 *>(a_ld + 4 * ld_q);                               \
            _Pragma("unroll") for (int a = 0; a < KH; ++a) {                                     \
                B[a] = *reinterpret_cast<const f32x4 *>(b_ld + a * p.PW + 4 * ld_q);             \
                C[a] = *reinterpret_cast<const f32x2 *>(b_ld + a * p.PW + 4 * ld_q + 4);         \
            }                                                                                    \
            __builtin_amdgcn_sched_barrier(0);   /* the reads go out before the MFMAs */         \
        }
#define DK_WGQ_MMA(A, B, C)                                                                      \
        {                                                                                        \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                        \
                _Pragma("unroll") for (int a = 0; a < KH; ++a)                                   \
                    _Pragma("unroll") for (int b = 0; b < KW; ++b) {                             \
                        const int c = i + b;                                                     \
                        const float bv = c < 4 ? B[a][c] : C[a][c - 4];                          \
                        acc[a * KW + b] = __builtin_amdgcn_mfma_f32_32x32x2f32(A[i], bv, acc[a * KW + b], 0, 0, 0); \
                    }                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                                   \
        }
        f32x4 A0, A1, B0[KH], B1[KH];
        f32x2 C0[KH], C1[KH];
        DK_WGQ_LOAD(A0, B0, C0)
        int f = 0;
        for (; f + 2 <= total; f += 2) {
            DK_WGQ_ADVANCE()
            DK_WGQ_LOAD(A1, B1, C1)
            DK_WGQ_MMA(A0, B0, C0)
            DK_WGQ_ADVANCE()
            DK_WGQ_LOAD(A0, B0, C0)
            DK_WGQ_MMA(A1, B1, C1)
        }
        if (f < total) DK_WGQ_MMA(A0, B0, C0)    // odd number of steps in the tile
#undef DK_WGQ_ADVANCE
#undef DK_WGQ_LOAD
#undef DK_WGQ_MMA
        __syncthreads();
    }

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

constexpr int DSLOT4 = 6, PSLOT4 = 10, DSLOTQ = 6, PSLOTQ = 11;
constexpr size_t LDS_LIMIT = 150 * 1024;     // of the 160 KB a compute unit has
constexpr size_t DUMP_BYTES = 1024;          // behind the buffers: where unused copy slots store

// `allowed` is the record of one kernel (the caller keeps one per kernel: the
// two kernels launched through here have the same function type, so a record
// inside this template would be shared between them).
template <class KernelT>
dk_status launch_one(KernelT kernel, std::atomic<unsigned long long> &allowed, const dk_wgpatch_params &p,
                     size_t lds_bytes, hipStream_t st, const char *label)
{
    const dk_status as = dk_allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)(LDS_LIMIT + DUMP_BYTES),
                                              allowed);
    if (as != DK_OK) return as;
    const long long blocks = (long long)p.tiles_co * p.tiles_ci * p.splits;
    DK_REQUIRE(blocks <= 0x7fffffffll, DK_ERR_SHAPE);
    dk_prof_scope ps(label, st);
    kernel<<<dim3((unsigned)blocks), dim3(512), lds_bytes, st>>>(p);
    return dk_launch_status();
}

} // namespace

bool dk_patch_wgrad_plan(const dk_geom &g, long long R, bool aligned16, dk_wgpatch_plan *pl)
{
    if (!g.conv || R < 1) return false;
    if (!(g.kh == 3 && g.kw == 3)) return false;
    // stride 1 and rows of whole 16-byte vectors only: with scalar copies or
    // stride 2 this kernel measured slower (51-74 TFLOP/s) than the gather
    // engine (78-80) on the same layers
    if (g.stride != 1 || (g.Wo & 1)) return false;
    // a workgroup's 64 input-channel columns would be mostly empty: the gather
    // engine packs (ci, tap) into its columns instead
    if (g.Ci <= 16) return false;
    dk_wgpatch_params &p = pl->p;
    p = dk_wgpatch_params();
    const int HoWo = g.Ho * g.Wo;
    p.Ci = g.Ci; p.Co = g.Co; p.H = g.H; p.W = g.W; p.stride = g.stride; p.pad = g.pad;
    p.Ho = g.Ho; p.Wo = g.Wo; p.HoWo = HoWo; p.R = (int)R;
    if ((long long)g.Co * HoWo >= (1ll << 26) || g.n >= (1ll << 26)) return false;
    const bool v4 = aligned16 && g.W % 4 == 0 && g.Wo % 4 == 0;
    if (!v4) return false;
    // 16-byte LDS reads need stride 1, vector copies and half-rows of whole quads
    // (widths that are multiples of 4 but not of 8 split the tile by rows: even row counts only)
    const bool quad = v4 && g.stride == 1 && g.pad <= 4 && (g.Wo % 8 == 0 || g.Ho % 2 == 0);
    const bool rowsplit = quad && g.Wo % 8 != 0;
    pl->vec = v4 ? 4 : 1;
    pl->quad = quad;
    const int dslot = quad ? DSLOTQ : DSLOT4;
    const int pslot = quad ? PSLOTQ : PSLOT4;
    const int dmax = dslot * 256, pmax = pslot * 256;
    if (quad) {
        p.LPAD = g.pad;
        int pw = g.W + 2 * g.pad;
        if (pw < g.Wo + 4) pw = g.Wo + 4;        // the second quad of the last step
        p.PW = round_up(pw, 4);
    } else {
        p.LPAD = round_up(g.pad > 4 ? g.pad : 4, 4);
        p.PW = round_up(p.LPAD + g.W + g.pad, 4);
    }
    // LDS pitches: odd for 4-byte reads, 4 mod 8 for 16-byte reads (both spread
    // the 32 rows a half-wave touches over all banks)
    auto pitch = [&](int n) { return quad ? (n % 8 == 0 ? n + 4 : n) : (n | 1); };

    // choose the pixel tile among those the copy slots and the LDS allow: the
    // one with the fewest matrix-pipe cycles on the busiest workgroup (large
    // tiles amortise the per-tile barrier, but a tile count that does not
    // divide over the workgroups, or a ragged last row block, leaves MFMA slots
    // empty)
    int bestTR = 0, bestNI = 0;
    double bestCost = 0.0;
    const long long wg_tiles = (long long)((g.Co + 63) / 64) * ((g.Ci + 63) / 64);
    bool fits_image = false;
    for (int pass = 0; pass < 2; ++pass) {
        // pass 0: row blocks of one image; pass 1: several whole images
        for (int cand = 1; cand <= 64; ++cand) {
            const int TR = pass == 0 ? cand : g.Ho;
            const int NI = pass == 0 ? 1 : cand;
            if (pass == 0 && TR > g.Ho) break;
            if (pass == 1 && (NI < 2 || NI > R || NI > 255)) { if (NI > R || NI > 255) break; else continue; }
            if (pass == 0 && v4 && (TR * g.Wo) % 4) continue;
            if (rowsplit && TR % 2) continue;
            const int PH = (TR - 1) * g.stride + g.kh;
            const int PLANE = PH * p.PW;
            const int CPLANE = pitch(NI * PLANE);
            const int QT = NI * TR * g.Wo;
            const int LDQ = pitch(QT);
            const long long d_slots = 64ll * NI * (TR * g.Wo / pl->vec);
            const long long p_slots = 64ll * NI * PH * (g.W / pl->vec);
            const size_t bytes = 2 * ((size_t)round_up(64 * LDQ, 4) + round_up(64 * CPLANE, 4)) * 4;
            if (d_slots > dmax || p_slots > pmax || bytes > LDS_LIMIT) break;
            if ((long long)NI * g.Co * HoWo >= (1ll << 30) || (long long)NI * g.n >= (1ll << 30)) break;
            if (pass == 0) fits_image = TR == g.Ho;
            const long long n_pt = ((R + NI - 1) / NI) * ((g.Ho + TR - 1) / TR);
            long long sp = 256 / wg_tiles;
            if (sp < 1) sp = 1;
            if (sp > n_pt) sp = n_pt;
            const long long per = (n_pt + sp - 1) / sp;
            // a step is 36 MFMAs on 8 pixels (16-byte reads) or 9 on 2; the single-float
            // reads pace the latter at about 730 cycles instead of 576
            const double steps = quad ? NI * TR * (g.Wo / 8.0) : NI * TR * (g.Wo / 2.0);
            const double cost = (double)per * (steps * (quad ? 2304.0 : 730.0) + 1000.0);
            if (bestTR == 0 || cost < bestCost) { bestTR = TR; bestNI = NI; bestCost = cost; }
        }
        if (!fits_image) break;        // could not even fit one whole image: stay with row blocks
    }
    if (bestTR == 0) return false;
    p.TR = bestTR; p.NI = bestNI;
    p.PH = (p.TR - 1) * g.stride + g.kh;
    p.PLANE = p.PH * p.PW;
    p.CPLANE = pitch(p.NI * p.PLANE);
    p.QT = p.NI * p.TR * g.Wo;
    p.LDQ = pitch(p.QT);
    p.DV = p.TR * g.Wo / pl->vec;
    p.XV = g.W / pl->vec;
    p.d_slots = 64 * p.NI * p.DV;
    p.p_slots = 64 * p.NI * p.PH * p.XV;
    p.ad_floats = round_up(64 * p.LDQ, 4);
    p.buf_floats = p.ad_floats + round_up(64 * p.CPLANE, 4);
    pl->lds_bytes = 2 * (size_t)p.buf_floats * 4 + DUMP_BYTES;
    p.row_blocks = (g.Ho + p.TR - 1) / p.TR;
    p.n_ptiles = (int)((R + p.NI - 1) / p.NI) * p.row_blocks;
    p.tiles_co = (g.Co + 63) / 64;
    p.tiles_ci = (g.Ci + 63) / 64;
    p.part_elems = (long long)g.kh * g.kw * g.Co * g.Ci;
    // one resident workgroup per compute unit; never more partial sums than 256 MB
    long long s = 256 / ((long long)p.tiles_co * p.tiles_ci);
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
    static std::atomic<unsigned long long> allowed_quad{0}, allowed_patch{0};
    dk_status s = pl.quad ? launch_one(conv_quad_wgrad_kernel<DSLOTQ, PSLOTQ>, allowed_quad, p, pl.lds_bytes, st,
                                       "conv_quad_wgrad")
                          : launch_one(conv_patch_wgrad_kernel<3, 3, DSLOT4, PSLOT4>, allowed_patch, p,
                                       pl.lds_bytes, st, "conv_patch_wgrad");
    if (s != DK_OK) return s;
    dk_prof_scope ps("wgrad_fold", st);
    wgrad_fold_kernel<<<dim3((unsigned)((p.part_elems + 63) / 64)), dim3(256), 0, st>>>(
        part, dW, g.Co, g.Ci, g.kh * g.kw, p.part_elems, p.splits, scale, accumulate);
    return dk_launch_status();
}
