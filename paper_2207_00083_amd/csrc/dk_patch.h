// Interface between the convolution entry points and the LDS-patch
// convolution kernels (internal).
#pragma once
#include "dk_internal.h"

struct dk_patch_params {
    const float *x;     // encoded images [R][Ci][H][W]
    const float *wp;    // repacked filters [chunk][CB*KH*KW][Co_pad]
    float *out;         // ybar [R][Co][Ho][Wo]
    float *part;        // split-K partial sums [splits][out_elems]
    int Ci, Co, H, W, stride, pad, Ho, Wo, HoWo, R;
    int img_g;          // Ci*H*W
    int multi;          // 0: a tile is BN pixels of one image; 1: IPT whole images; 2: BN pixels of the batch
    int IPT, BN_eff, tiles_per_img;
    int PH, PW, PLANE, LPAD;      // patch rows, row pitch, plane size, left pad (floats)
    int patch_floats;             // LDS floats of the patch region
    int patch_slots, XV;          // vectors to copy per chunk, vectors per image row
    int n_chunks, per_split, splits, Co_pad;
    int tiles_m, tiles_n;
    long long out_elems;
    long long w_row, w_chunk;     // filter tile addressing: floats between rows / chunks
};

struct dk_patch_plan {
    dk_patch_params p;
    int vec;            // 4: 16-byte copies, 1: scalar copies
    int cb;             // input channels per chunk
    bool flat;          // 64-row tile (Co <= 64) or 128-row tile
    bool quad;          // 16-byte LDS reads (3x3, stride 1, widths multiples of 4)
    size_t lds_bytes;
    size_t wp_floats;
    size_t part_bytes;
};

static inline size_t dk_patch_wp_bytes(const dk_patch_plan &pl)
{
    return (pl.wp_floats * sizeof(float) + 255) / 256 * 256;
}

// Fills the plan and returns true if the layer is covered by a patch kernel.
// aligned16: xbar and ybar are both 16-byte aligned.
bool dk_patch_fwd_plan(const dk_geom &g, long long R, bool aligned16, dk_patch_plan *pl);

// Repack the filters, run the kernel (and the split-K fold if any).  ws must
// hold dk_patch_wp_bytes(pl) + pl.part_bytes.
dk_status dk_patch_fwd_run(const dk_geom &g, dk_patch_plan &pl, const float *W, const float *xbar,
                           float *ybar, float *ws, hipStream_t st);

// ---- weight gradient with the input patch in LDS ----

struct dk_wgpatch_params {
    const float *dt;    // mixed gradients dtilde [R][Co][Ho][Wo]
    const float *x;     // encoded images [R][Ci][H][W]
    float *part;        // partial sums [splits][KH*KW][Co][Ci]
    int Ci, Co, H, W, stride, pad, Ho, Wo, HoWo, R;
    int NI, TR;         // a pixel tile is NI images x TR output rows
    int row_blocks, n_ptiles, per_split, splits;
    int PH, PW, PLANE, CPLANE, LPAD;   // patch rows, pitch, per-image plane, per-channel plane
    int LDQ, QT;        // dtilde tile pitch (odd) and pixels per tile
    int DV, XV, d_slots, p_slots;
    int ad_floats, buf_floats;   // dtilde tile floats; one LDS buffer (tile + patch) floats
    int tiles_co, tiles_ci;
    long long part_elems;
};

struct dk_wgpatch_plan {
    dk_wgpatch_params p;
    int vec;
    bool quad;          // 16-byte LDS reads (stride 1, output width a multiple of 8)
    size_t lds_bytes;
    size_t part_bytes;
};

bool dk_patch_wgrad_plan(const dk_geom &g, long long R, bool aligned16, dk_wgpatch_plan *pl);

// part must hold pl.part_bytes.
dk_status dk_patch_wgrad_run(const dk_geom &g, dk_wgpatch_plan &pl, const float *dtilde,
                             const float *xbar, float *dW, float scale, int accumulate,
                             float *part, hipStream_t st);
