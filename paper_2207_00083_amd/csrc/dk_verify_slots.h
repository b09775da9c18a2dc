// The integrity check's last step, shared by every kernel that ends with it.
#pragma once
#include <hip/hip_runtime.h>

// Host side: the tag of one integrity-check call, distinct from every tag this
// process drew before and never 0.
unsigned long long dk_next_verify_tag();

// Up to this many workgroups per virtual batch the verdict is taken inside the
// kernel that computes the maxima (DK_VERIFY_FINISH_IN_KERNEL below); with more,
// the look at every slot of the batch by every workgroup -- all on the same
// few cache lines, at device scope -- costs more than a second, tiny launch
// (measured, K = 8, 196 workgroups per batch: 0.097 ms against 0.076 + 0.006).
#define DK_VERIFY_INLINE_MAX_CHUNKS 32

// Second launch for the other case: one wave per virtual batch folds the slots
// the first kernel wrote (dk_verify_publish with finish = false).
dk_status dk_verify_finalize(const struct dk_verify_slot *slots, int chunks, float tol, int *verdict,
                             float *resid, int G, hipStream_t st);

#ifdef __HIPCC__
__device__ __forceinline__ float dk_wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ---- integrity check: per-workgroup maxima and the verdict, in one launch ----
//
// A group's feature axis is shared by `chunks` workgroups.  Each reduces its
// span to (max |t|, max s) and publishes the pair in its slot of the workspace;
// the workgroup that then finds every slot of its group published folds the
// pairs and writes the verdict.  max is order independent, so the result does
// not depend on which workgroup that is.
//
// A slot is two 64-bit words, (tag low half | bits of max |t|) and (tag high
// half | bits of max s), where the tag is a 64-bit number the host draws per
// call, never 0.  A word counts only if it carries this call's tag half, so
//   * nothing has to be cleared beforehand, whatever the workspace held;
//   * each word validates its own float: no ordering between different
//     addresses is needed, hence no release fence -- on this chip a fence at
//     device scope writes back every dirty line of the XCD's L2, which right
//     behind the decoded outputs cost ten times the kernel itself.
// The finishing workgroup resets the tags to 0, so a captured graph, whose
// replays all carry the tag of the capture, starts every replay from clean
// slots.  Publishing is an atomic exchange whose result is waited for: it
// has then been performed at the device's point of coherence, and the loads
// that follow are issued after it; of two workgroups of a group, at least the
// one whose exchange came second therefore sees the other's words, so at
// least one workgroup sees all of them.  If several do, they write the same
// verdict.
struct dk_verify_slot {
    unsigned long long t_word, s_word;
};
static_assert(sizeof(dk_verify_slot) == 16, "slot layout");

__device__ __forceinline__ unsigned long long dk_verify_word(float v, unsigned tag_half)
{
    return ((unsigned long long)tag_half << 32) | __float_as_uint(v);
}

// tag == 0: only store the pair (a second launch takes the verdict).
template <int NT>      // threads per workgroup (whole 64-lane waves); every thread calls
__device__ __forceinline__ void dk_verify_publish_and_finish(
    float tmax, float smax, bool bad, dk_verify_slot *__restrict__ slots, int g, int chunk, int chunks,
    unsigned long long tag, float tol, int *__restrict__ verdict, float *__restrict__ resid)
{
    if (bad) tmax = __builtin_inff();
    __shared__ float red[2][NT / 64];
    tmax = dk_wave_max(tmax);
    smax = dk_wave_max(smax);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) { red[0][wave] = tmax; red[1][wave] = smax; }
    __syncthreads();
    if (wave != 0) return;
    dk_verify_slot *grp = slots + (long long)g * chunks;
    const unsigned tag_lo = (unsigned)tag, tag_hi = (unsigned)(tag >> 32);
    if (lane == 0) {
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) {
            tmax = fmaxf(tmax, red[0][w]);
            smax = fmaxf(smax, red[1][w]);
        }
        if (tag == 0ull) {      // wave-uniform: the verdict is taken by dk_verify_finalize
            grp[chunk].t_word = dk_verify_word(tmax, 0u);
            grp[chunk].s_word = dk_verify_word(smax, 0u);
        }
    }
    if (tag == 0ull) return;
    if (lane == 0) {
        const unsigned long long o0 = __hip_atomic_exchange(&grp[chunk].t_word, dk_verify_word(tmax, tag_lo),
                                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long o1 = __hip_atomic_exchange(&grp[chunk].s_word, dk_verify_word(smax, tag_hi),
                                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("" ::"v"(o0), "v"(o1));          // the returning form: completion can be waited for
    }
    // both exchanges have returned before any of the loads below is issued
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    bool all_here = true;
    float t = 0.0f, sm = 0.0f;
    for (int c = lane; c < chunks; c += 64) {
        const unsigned long long w0 = __hip_atomic_load(&grp[c].t_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long w1 = __hip_atomic_load(&grp[c].s_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        all_here &= (unsigned)(w0 >> 32) == tag_lo && (unsigned)(w1 >> 32) == tag_hi;
        t = fmaxf(t, __uint_as_float((unsigned)w0));
        sm = fmaxf(sm, __uint_as_float((unsigned)w1));
    }
    if (!__all(all_here)) return;
    // fmaxf drops a NaN operand; the publishers turn every non-finite case into +inf beforehand
    t = dk_wave_max(t);
    sm = dk_wave_max(sm);
    for (int c = lane; c < chunks; c += 64) {
        __hip_atomic_store(&grp[c].t_word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&grp[c].s_word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane != 0) return;
    const bool nonfinite = !(t <= 3.402823466e+38f);
    const float rho = nonfinite ? __builtin_inff() : (sm > 0.0f ? t / sm : 0.0f);
    verdict[g] = (nonfinite || rho > tol) ? 1 : 0;
    if (resid) resid[g] = rho;
}

#endif
