// Host-side parts of the library: status strings, layer geometry, workspace
// sizing and the trusted-side coefficient derivation.  No device code here.
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <vector>

#include "dk_internal.h"

DK_EXPORT const char *dk_status_str(int s)
{
    switch (s) {
    case DK_OK: return "ok";
    case DK_ERR_NULL: return "required pointer is NULL";
    case DK_ERR_SHAPE: return "invalid size or K";
    case DK_ERR_UNSUPPORTED: return "unsupported layer geometry";
    case DK_ERR_ALIGN: return "device pointer not 4-byte aligned";
    case DK_ERR_WORKSPACE: return "workspace missing or too small";
    case DK_ERR_HIP: return "HIP launch failed";
    case DK_ERR_SINGULAR: return "singular encoding matrix or zero gamma";
    case DK_ERR_STATIC_LIMIT: return "more groups than the built-in scratch array serves";
    default: return "unknown status";
    }
}

DK_EXPORT int dk_version(void) { return 110; }

namespace {
std::atomic<int> g_options[DK_OPT_COUNT] = {{DK_FUSE_AUTO}, {DK_FUSE_AUTO}};
}

int dk_option(int which)
{
    return which >= 0 && which < DK_OPT_COUNT ? g_options[which].load(std::memory_order_relaxed) : 0;
}

DK_EXPORT dk_status dk_set_option(int which, int value)
{
    DK_REQUIRE(which >= 0 && which < DK_OPT_COUNT, DK_ERR_SHAPE);
    DK_REQUIRE(value == DK_FUSE_NEVER || value == DK_FUSE_ALWAYS || value == DK_FUSE_AUTO, DK_ERR_SHAPE);
    g_options[which].store(value, std::memory_order_relaxed);
    return DK_OK;
}

DK_EXPORT int dk_get_option(int which) { return which >= 0 && which < DK_OPT_COUNT ? dk_option(which) : -1; }

dk_status dk_layer_geom(const dk_layer *L, dk_geom *g)
{
    DK_REQUIRE(L && g, DK_ERR_NULL);
    memset(g, 0, sizeof(*g));
    if (L->kind == DK_LINEAR) {
        DK_REQUIRE(L->M >= 1 && L->N >= 1, DK_ERR_SHAPE);
        g->conv = false;
        g->M = L->M;
        g->N = L->N;
        g->n = L->N;
        g->m = L->M;
        return DK_OK;
    }
    DK_REQUIRE(L->kind == DK_CONV2D || L->kind == DK_DWCONV2D, DK_ERR_UNSUPPORTED);
    DK_REQUIRE(L->Ci >= 1 && L->Co >= 1 && L->H >= 1 && L->W >= 1, DK_ERR_SHAPE);
    DK_REQUIRE(L->kind == DK_CONV2D || L->Co == L->Ci, DK_ERR_SHAPE);
    DK_REQUIRE(L->kh >= 1 && L->kw >= 1 && L->stride >= 1 && L->pad >= 0, DK_ERR_SHAPE);
    DK_REQUIRE(L->kh <= 16 && L->kw <= 16 && L->stride <= 16 && L->pad <= 16, DK_ERR_UNSUPPORTED);
    DK_REQUIRE(L->H + 2 * L->pad >= L->kh && L->W + 2 * L->pad >= L->kw, DK_ERR_SHAPE);
    g->conv = true;
    g->Ci = L->Ci; g->Co = L->Co; g->H = L->H; g->W = L->W;
    g->kh = L->kh; g->kw = L->kw; g->stride = L->stride; g->pad = L->pad;
    g->Ho = (L->H + 2 * L->pad - L->kh) / L->stride + 1;
    g->Wo = (L->W + 2 * L->pad - L->kw) / L->stride + 1;
    g->n = (long long)L->Ci * L->H * L->W;
    g->m = (long long)L->Co * g->Ho * g->Wo;
    g->Kg = (long long)L->Ci * L->kh * L->kw;
    if (L->kind == DK_DWCONV2D) {
        g->dw = true;
        g->Kg = (long long)L->kh * L->kw;
        DK_REQUIRE(dk_dw_supported(*g), DK_ERR_UNSUPPORTED);
    }
    // the kernels index one sample's image and the filter bank with 32-bit ints
    DK_REQUIRE(g->n < (1ll << 30) && g->m < (1ll << 30) && g->Kg * L->Co < (1ll << 30), DK_ERR_SHAPE);
    return DK_OK;
}

DK_EXPORT long long dk_layer_in_len(const dk_layer *L)
{
    dk_geom g;
    return dk_layer_geom(L, &g) == DK_OK ? g.n : 0;
}

DK_EXPORT long long dk_layer_out_len(const dk_layer *L)
{
    dk_geom g;
    return dk_layer_geom(L, &g) == DK_OK ? g.m : 0;
}

DK_EXPORT size_t dk_workspace_bytes(const dk_layer *L, int op, int G, int K)
{
    if (G < 1 || K < 1 || K > DK_MAX_K) return 0;
    if (op == DK_OP_VERIFY) return dk_ws_verify_bytes(G);
    dk_geom g;
    if (dk_layer_geom(L, &g) != DK_OK) return 0;
    const long long R = (long long)G * (K + 2);
    if (op == DK_OP_FWD) return dk_ws_fwd_bytes(g, R);
    if (op == DK_OP_WGRAD) return dk_ws_wgrad_bytes(g, R);
    return 0;
}

DK_EXPORT size_t dk_workspace_bytes_m(const dk_layer *L, int op, int G, int K, int M)
{
    if (G < 1 || K < 1 || M < 1 || K + M - 1 > DK_MAX_K) return 0;
    if (op == DK_OP_VERIFY) return dk_ws_verify_bytes(G);
    dk_geom g;
    if (dk_layer_geom(L, &g) != DK_OK) return 0;
    const long long R = (long long)G * (K + M + 1);
    if (op == DK_OP_FWD) return dk_ws_fwd_bytes(g, R);
    if (op == DK_OP_WGRAD) return dk_ws_wgrad_bytes(g, R);
    return 0;
}

DK_EXPORT size_t dk_fwd_workspace_bytes(const dk_layer *L, long long R)
{
    dk_geom g;
    if (R < 1 || R >= (1ll << 31) || dk_layer_geom(L, &g) != DK_OK) return 0;
    return dk_ws_fwd_bytes(g, R);
}

dk_split_plan dk_plan_split(long long out_tiles, long long ktiles, long long out_elems, double step_us)
{
    // One workgroup per (output tile, K slice), handed out evenly over the 256
    // compute units.  A unit's matrix pipe is shared by the workgroups resident
    // on it, so the kernel lasts about
    //     (workgroups on the busiest unit) x (steps per slice x step_us + fixed cost per workgroup),
    // a single workgroup per unit cannot hide its own load latency
    // (measured: 10-25 % slower; two hide most of it), and the slices are written and read once
    // more by the fold.  Take the slice count that minimises the sum.
    dk_split_plan p = {1, (int)ktiles};
    if (ktiles < 1) { p.ktiles_per_split = 0; return p; }
    if (ktiles == 1) return p;
    const double fixed_us = 3.0;                    // prologue latency + epilogue of a workgroup
    const double fold_us_per_byte = 1.5 / 5.0e6;    // one write + about half a read at 5 TB/s
    long long smax = ktiles < DK_MAX_SPLITS ? ktiles : DK_MAX_SPLITS;
    double best = 0.0;
    for (long long s = 1; s <= smax; ++s) {
        if (s > 1 && s * out_elems * 4 > DK_SPLIT_WS_CAP_BYTES) break;
        const long long per = (ktiles + s - 1) / s;
        const long long sl = (ktiles + per - 1) / per;       // slices actually used
        if (sl != s) continue;
        const long long per_cu = (out_tiles * s + 255) / 256;
        double t = (double)per_cu * ((double)per * step_us + fixed_us);
        if (per_cu < 2) t *= 1.25; else if (per_cu < 3) t *= 1.05;
        if (s > 1) t += (double)s * (double)out_elems * 4.0 * fold_us_per_byte;
        if (s == 1 || t < best) { best = t; p.splits = (int)s; p.ktiles_per_split = (int)per; }
    }
    return p;
}

// Gauss-Jordan inversion in fp64 with partial pivoting; a is destroyed.
static bool invert(std::vector<double> &a, std::vector<double> &inv, int n)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) inv[i * n + j] = (i == j);
    for (int c = 0; c < n; ++c) {
        int piv = c;
        for (int r = c + 1; r < n; ++r)
            if (std::fabs(a[r * n + c]) > std::fabs(a[piv * n + c])) piv = r;
        const double d = a[piv * n + c];
        if (!(std::fabs(d) > 0.0) || !std::isfinite(d)) return false;
        if (piv != c)
            for (int j = 0; j < n; ++j) {
                std::swap(a[c * n + j], a[piv * n + j]);
                std::swap(inv[c * n + j], inv[piv * n + j]);
            }
        for (int j = 0; j < n; ++j) { a[c * n + j] /= d; inv[c * n + j] /= d; }
        for (int r = 0; r < n; ++r) {
            if (r == c) continue;
            const double f = a[r * n + c];
            if (f == 0.0) continue;
            for (int j = 0; j < n; ++j) {
                a[r * n + j] -= f * a[c * n + j];
                inv[r * n + j] -= f * inv[c * n + j];
            }
        }
    }
    for (int q = 0; q < n * n; ++q)
        if (!std::isfinite(inv[q])) return false;
    return true;
}

// Coefficients for K private inputs and S encodings per group.
static dk_status coeffs_impl(const float *A, const float *gamma, int G, int K, int S,
                             float *Ainv, float *nvec, float *B)
{
    DK_REQUIRE(A, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && S >= K + 2 && S <= DK_MAX_K + 2, DK_ERR_SHAPE);
    DK_REQUIRE(!B || gamma, DK_ERR_NULL);
    std::vector<double> a(S * S), inv(S * S);
    // first pass: validate everything so that nothing is written on error
    for (int pass = 0; pass < 2; ++pass)
        for (int g = 0; g < G; ++g) {
            if (pass == 0 && B)
                for (int j = 0; j < S; ++j) {
                    const float gj = gamma[(size_t)g * S + j];
                    DK_REQUIRE(gj != 0.0f && std::isfinite(gj), DK_ERR_SINGULAR);
                }
            for (int q = 0; q < S * S; ++q) a[q] = (double)A[(size_t)g * S * S + q];
            DK_REQUIRE(invert(a, inv, S), DK_ERR_SINGULAR);
            if (pass == 0) continue;
            if (Ainv)
                for (int q = 0; q < S * S; ++q) Ainv[(size_t)g * S * S + q] = (float)inv[q];
            if (nvec)
                for (int j = 0; j < S; ++j) nvec[(size_t)g * S + j] = (float)inv[j * S + (S - 1)];
            if (B)
                for (int j = 0; j < S; ++j)
                    for (int i = 0; i < K; ++i)
                        B[((size_t)g * S + j) * K + i] =
                            (float)(inv[j * S + i] / (double)gamma[(size_t)g * S + j]);
        }
    return DK_OK;
}

DK_EXPORT dk_status dk_coeffs(const float *A, const float *gamma, int G, int K,
                              float *Ainv, float *nvec, float *B)
{
    DK_REQUIRE(K >= 1 && K <= DK_MAX_K, DK_ERR_SHAPE);
    return coeffs_impl(A, gamma, G, K, K + 2, Ainv, nvec, B);
}

DK_EXPORT dk_status dk_coeffs_m(const float *A, const float *gamma, int G, int K, int M,
                                float *Ainv, float *nvec, float *B)
{
    DK_REQUIRE(K >= 1 && M >= 1 && K + M - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    return coeffs_impl(A, gamma, G, K, K + M + 1, Ainv, nvec, B);
}

// ---------------------------------------------------------------------------
// Per-kernel timing for benchmarks.
// ---------------------------------------------------------------------------
namespace {
constexpr int PROF_MAX = 8192;
struct prof_state {
    bool on = false;
    int used = 0;
    std::vector<hipEvent_t> ev;          // 2 per record, created on first use
    std::vector<const char *> name;
} g_prof;
} // namespace

dk_prof_scope::dk_prof_scope(const char *kernel, hipStream_t st_) : slot(-1), st(st_)
{
    if (!g_prof.on || g_prof.used >= PROF_MAX) return;
    slot = g_prof.used++;
    if ((int)g_prof.ev.size() < 2 * (slot + 1)) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { slot = -1; --g_prof.used; return; }
        g_prof.ev.push_back(a);
        g_prof.ev.push_back(b);
        g_prof.name.push_back(kernel);
    }
    g_prof.name[slot] = kernel;
    (void)hipEventRecord(g_prof.ev[2 * slot], st);
}

dk_prof_scope::~dk_prof_scope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof.ev[2 * slot + 1], st);
}

DK_EXPORT dk_status dk_profile_enable(int on)
{
    if (on) g_prof.used = 0;
    g_prof.on = on != 0;
    return DK_OK;
}

DK_EXPORT int dk_profile_read(int index, char *name, int name_cap, double *avg_ms, int *launches)
{
    // aggregate by kernel label, in order of first appearance
    std::vector<const char *> labels;
    std::vector<double> sum;
    std::vector<int> cnt;
    for (int i = 0; i < g_prof.used; ++i) {
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess) continue;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess) continue;
        size_t k = 0;
        while (k < labels.size() && strcmp(labels[k], g_prof.name[i]) != 0) ++k;
        if (k == labels.size()) { labels.push_back(g_prof.name[i]); sum.push_back(0.0); cnt.push_back(0); }
        sum[k] += ms;
        cnt[k] += 1;
    }
    if (index >= 0 && index < (int)labels.size()) {
        if (name && name_cap > 0) { strncpy(name, labels[index], name_cap - 1); name[name_cap - 1] = 0; }
        if (avg_ms) *avg_ms = sum[index] / cnt[index];
        if (launches) *launches = cnt[index];
    }
    return (int)labels.size();
}
