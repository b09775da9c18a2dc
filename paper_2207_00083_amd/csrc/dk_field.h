// Internal helpers of the finite-field variant (not installed).
#pragma once
#include <initializer_list>
#include <math.h>
#include "dk_internal.h"
#include "darknight_field.h"

// Gradient mixing over the field (launcher; used by dkf_wgrad).  xscale (one
// normalisation factor per sample, device) may be null.  K inputs and M noise rows
// per group, S = K + M + 1.
dk_status dkf_delta_mix(const float *delta, const float *xscale, const uint32_t *B,
                        const uint32_t *gamma, uint32_t *dtilde, int G, int K, int M, long long m, int l,
                        hipStream_t st);

// Depthwise convolution over the field.
size_t dkf_dw_wgrad_part_bytes(const dk_geom &g, long long R);
dk_status dkf_dw_fwd_run(const dk_geom &g, const uint32_t *Wq, const uint32_t *xbar, uint32_t *ybar,
                         long long R, hipStream_t st);
dk_status dkf_dw_wgrad_run(const dk_geom &g, const uint32_t *dtilde, const uint32_t *xbar, float *dW,
                           uint32_t *dwq, long long R, int l, float scale, int accumulate, uint32_t *part,
                           hipStream_t st);

#ifdef __HIPCC__
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef i32x4 i32x4_u __attribute__((aligned(1)));     // for global loads at any byte address
typedef int i32x16 __attribute__((ext_vector_type(16)));

// v mod p for v < 2^56, by folding the bits above 2^25 twice with
// 2^25 = 39 (mod p) and one conditional subtraction.
static __device__ __forceinline__ uint32_t dkf_reduce(uint64_t v)
{
    const uint64_t t = (v >> 25) * 39u + (v & 0x1ffffffu);                   // < 2^37
    const uint32_t u = (uint32_t)(t >> 25) * 39u + ((uint32_t)t & 0x1ffffffu); // < 2^25 + 2^18
    return u >= DKF_P ? u - DKF_P : u;
}

// Field(Round(x * s)), s = 2^l: fp64 floor(x*s + 1/2) (the product is exact),
// clamped to int32, NaN -> 0, then the least non-negative residue.
static __device__ __forceinline__ uint32_t dkf_quant(float x, double s)
{
    double v = floor((double)x * s + 0.5);
    v = (v != v) ? 0.0 : v;
    v = fmin(fmax(v, -2147483648.0), 2147483647.0);
    int z = (int)v % (int)DKF_P;
    if (z < 0) z += (int)DKF_P;
    return (uint32_t)z;
}

// Centred lift, then Round(v * s) * s with s = 2^-l.
static __device__ __forceinline__ float dkf_dequant(uint32_t q, double s)
{
    int v = (int)q;
    if (q > DKF_P / 2) v -= (int)DKF_P;
    return (float)(floor((double)v * s + 0.5) * s);
}
#endif
