// Internal helpers shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "darknight.h"

#define DK_EXPORT extern "C" __attribute__((visibility("default")))

#define DK_REQUIRE(cond, err) \
    do {                      \
        if (!(cond)) return (err); \
    } while (0)

static inline bool dk_aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Kernels that use more than 64 KB of dynamic LDS have to be allowed to, once
// per kernel and device (HIP keeps the attribute per device).  `done` is the
// call site's own record, one bit per device ordinal; a race between two first
// calls sets the attribute twice, which is harmless.
static inline dk_status dk_allow_dynamic_lds(const void *kernel, int bytes, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DK_ERR_HIP;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return DK_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return DK_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
    return DK_OK;
}

static inline dk_status dk_launch_status()
{
    return hipGetLastError() == hipSuccess ? DK_OK : DK_ERR_HIP;
}

// Validated geometry of a layer, filled by dk_layer_geom().
struct dk_geom {
    bool conv;
    bool dw;              // depthwise convolution (conv is true too; Co == Ci, one filter per channel)
    long long n, m;       // per-sample input / output length
    int M, N;             // dense
    int Ci, Co, H, W, kh, kw, stride, pad, Ho, Wo;
    long long Kg;         // Ci*kh*kw
};

dk_status dk_layer_geom(const dk_layer *L, dk_geom *g);

// Workspace carving, identical in dk_workspace_bytes and in the entry points.
size_t dk_ws_fwd_bytes(const dk_geom &g, long long R);
size_t dk_ws_wgrad_bytes(const dk_geom &g, long long R);
size_t dk_ws_verify_bytes(int G);

// Split-K plan for a contraction: how many slices, steps per slice.  step_us =
// time one workgroup needs for one contraction step with a SIMD to itself.
struct dk_split_plan {
    int splits;
    int ktiles_per_split;
};
dk_split_plan dk_plan_split(long long out_tiles, long long ktiles, long long out_elems, double step_us);

// Second pass of a sliced contraction:
// out[i] = (accumulate ? out[i] : 0) + alpha * sum_s part[s][i], in a fixed order.
dk_status dk_fold_slices(const float *part, float *out, long long out_elems, int splits, float alpha,
                         int accumulate, hipStream_t st);

#define DK_VERIFY_MAX_BLOCKS 64
#define DK_MAX_SPLITS 256
#define DK_SPLIT_WS_CAP_BYTES (1ll << 30)

// Depthwise convolution kernels.
bool dk_dw_supported(const dk_geom &g);
size_t dk_dw_wgrad_part_bytes(const dk_geom &g, long long R);
dk_status dk_dw_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                        hipStream_t st);
dk_status dk_dw_wgrad_run(const dk_geom &g, const float *dtilde, const float *xbar, float *dW, long long R,
                          float scale, int accumulate, float *part, hipStream_t st);
dk_status dk_dw_dgrad_run(const dk_geom &g, const float *W, const float *delta, float *dx, long long R,
                          hipStream_t st);

// Gradient mixing kernel launcher (defined with the other bandwidth-bound
// kernels, used by dk_wgrad).
dk_status dk_delta_mix(const float *delta, const float *B, const float *gamma, float *dtilde,
                       int G, int K, int M, long long m, hipStream_t st);

// Direct (vector-ALU) kernels for 3x3 stride-1 pad-1 convolutions with at most
// four input channels.
bool dk_smallci_ok(const dk_geom &g, long long R, const float *x, const float *other);
size_t dk_smallci_wgrad_part_bytes(const dk_geom &g, long long R);
dk_status dk_smallci_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                             hipStream_t st);
dk_status dk_smallci_wgrad_run(const dk_geom &g, const float *dtilde, const float *xbar, float *dW, long long R,
                               float scale, int accumulate, float *part, size_t part_bytes, hipStream_t st);

// Fused kernels for 1x1 stride-1 convolutions.
bool dk_fused1x1_wgrad_ok(const dk_geom &g, int G, int K, int M, const float *delta, const float *xbar);
size_t dk_fused1x1_wgrad_part_bytes(const dk_geom &g, long long R);
dk_status dk_fused1x1_wgrad_run(const dk_geom &g, const float *delta, const float *B, const float *gamma,
                                const float *xbar, float *dW, int G, int K, float scale, int accumulate,
                                float *part, size_t part_bytes, hipStream_t st);
bool dk_fused1x1_fwd_ok(const dk_geom &g, int K);
size_t dk_fused1x1_fwd_slot_bytes(const dk_geom &g, int G);
dk_status dk_fused1x1_fwd_run(const dk_geom &g, const float *W, const float *xbar, const float *Ainv,
                              const float *nvec, float tol, float *y, int *verdict, float *resid, int G,
                              int K, void *slots, hipStream_t st);

// Tuning switches (dk_set_option).
int dk_option(int which);

// Optional per-kernel timing (dk_profile_enable): while enabled, a scope object
// brackets one kernel launch with two HIP events on the launch stream.
struct dk_prof_scope {
    dk_prof_scope(const char *kernel, hipStream_t st);
    ~dk_prof_scope();
    int slot;
    hipStream_t st;
};

#ifdef __HIPCC__
// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD
// b % 8) and each XCD has its own L2.  This maps the hardware index onto a
// logical one so that every XCD works through one contiguous run of logical
// indices: neighbouring tiles, which share operand panels, then share an L2.
// The mapping is a bijection on [0, gridDim.x) for any grid size.
static __device__ __forceinline__ int dk_xcd_block()
{
    const int nb = gridDim.x, b = blockIdx.x;
    const int q = nb >> 3, rem = nb & 7;
    const int xcd = b & 7, idx = b >> 3;
    return (xcd < rem ? xcd * (q + 1) : rem * (q + 1) + (xcd - rem) * q) + idx;
}
#endif
