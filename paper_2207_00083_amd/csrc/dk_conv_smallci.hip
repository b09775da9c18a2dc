// 3x3 convolutions with at most four input channels (the first layer of an
// image network): 27 or 36 multiply-adds per output element against 4 bytes
// written, so neither the forward nor the weight gradient is a job for the
// matrix cores -- the forward is bound by writing the results, the weight
// gradient by reading the mixed gradients, and the arithmetic fits the vector
// ALUs several times over.  Both kernels give a thread four consecutive pixels
// of a row: it keeps the 3 x 6 input patch of each channel in registers, so
// results leave and gradients arrive as 16-byte vectors.
#include "dk_internal.h"
#include "dk_patch.h"

namespace {

constexpr int NT = 256;

typedef float f4 __attribute__((ext_vector_type(4)));

struct smallci_params {
    const float *x;        // xbar[R][CI][H][W]
    const float *w;        // W[Co][CI][3][3]        (forward)
    const float *d;        // dtilde[R][Co][H][W]    (weight gradient)
    float *y;              // ybar[R][Co][H][W]      (forward)
    float *part;           // [slices][Co][CI*9]     (weight gradient)
    int Co, H, W, R;
    long long nq;          // pixel quads: R*H*W/4
    int qpt;               // quads per thread (weight gradient)
};

// The 3 x 6 patch around pixels (h, w0..w0+3) of every channel, zero outside.
template <int CI>
__device__ __forceinline__ void load_patch(float (&p)[CI][3][6], const float *__restrict__ img, int H, int W,
                                           int h, int w0)
{
#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const int hh = h + a - 1;
            const bool row_ok = (unsigned)hh < (unsigned)H;
            const float *row = img + ((long long)c * H + (row_ok ? hh : 0)) * W + w0;
            f4 m = {0.f, 0.f, 0.f, 0.f};
            float l = 0.0f, r = 0.0f;
            if (row_ok) {
                m = *reinterpret_cast<const f4 *>(row);
                if (w0 > 0) l = row[-1];
                if (w0 + 4 < W) r = row[4];
            }
            p[c][a][0] = l; p[c][a][1] = m.x; p[c][a][2] = m.y; p[c][a][3] = m.z; p[c][a][4] = m.w; p[c][a][5] = r;
        }
}

// Forward: blockIdx.y picks COB output channels (their filters sit at a
// wave-uniform address: scalar loads), a thread writes one 16-byte vector per
// channel.
template <int CI, int COB>
__global__ __launch_bounds__(NT) void smallci_fwd_kernel(smallci_params p)
{
    const long long q0 = (long long)blockIdx.x * NT + threadIdx.x;
    const bool live = q0 < p.nq;
    const long long q = live ? q0 : 0;               // idle lanes shadow quad 0 and store nothing
    const int WQ = p.W / 4;
    const int wq = (int)(q % WQ);
    const long long t = q / WQ;
    const int h = (int)(t % p.H);
    const long long r = t / p.H;
    const int w0 = wq * 4;
    float patch[CI][3][6];
    load_patch<CI>(patch, p.x + r * CI * p.H * p.W, p.H, p.W, h, w0);
    const int co0 = blockIdx.y * COB;
    float *dst = p.y + ((r * p.Co + co0) * p.H + h) * p.W + w0;
    const long long chs = (long long)p.H * p.W;
    // the chunk's filters through LDS (every lane reads the same word: a broadcast)
    __shared__ float wsh[COB * CI * 9];
    __syncthreads();
    for (int e = threadIdx.x; e < COB * CI * 9; e += NT)
        wsh[e] = co0 * CI * 9 + e < p.Co * CI * 9 ? p.w[(long long)co0 * CI * 9 + e] : 0.0f;
    __syncthreads();
#pragma unroll 2
    for (int k = 0; k < COB; ++k) {
        const int co = co0 + k;
        if (co >= p.Co) break;                      // wave-uniform
        const float *wf = wsh + k * CI * 9;
        float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < CI; ++c)
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    const float wv = wf[(c * 3 + a) * 3 + b];
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = fmaf(wv, patch[c][a][j + b], o[j]);
                }
        const f4 v = {o[0], o[1], o[2], o[3]};
        if (live) __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(dst + k * chs));
    }
}

// Weight gradient: blockIdx.y picks COB output channels, blockIdx.x a slice of
// the pixel quads; a thread walks its quads (stride = workgroups x threads, so
// a wave reads consecutive vectors of the gradients), keeps COB x CI x 9 sums
// and the workgroup adds them up in a fixed order through LDS.
template <int CI, int COB>
__global__ __launch_bounds__(NT) void smallci_wgrad_kernel(smallci_params p)
{
    constexpr int NA = COB * CI * 9;
    float acc[COB][CI][3][3];
#pragma unroll
    for (int k = 0; k < COB; ++k)
#pragma unroll
        for (int c = 0; c < CI; ++c)
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) acc[k][c][a][b] = 0.0f;

    const int WQ = p.W / 4;
    const int co0 = blockIdx.y * COB;
    const long long chs = (long long)p.H * p.W;
    const long long stride = (long long)gridDim.x * NT;
    long long q = (long long)blockIdx.x * NT + threadIdx.x;
    for (int it = 0; it < p.qpt; ++it, q += stride) {
        if (q >= p.nq) break;
        const int wq = (int)(q % WQ);
        const long long t = q / WQ;
        const int h = (int)(t % p.H);
        const long long r = t / p.H;
        const int w0 = wq * 4;
        float patch[CI][3][6];
        load_patch<CI>(patch, p.x + r * CI * chs, p.H, p.W, h, w0);
        const float *src = p.d + ((r * p.Co + co0) * p.H + h) * p.W + w0;
#pragma unroll
        for (int k = 0; k < COB; ++k) {
            f4 dv = {0.f, 0.f, 0.f, 0.f};
            if (co0 + k < p.Co) dv = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(src + k * chs));
            const float d[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
            for (int c = 0; c < CI; ++c)
#pragma unroll
                for (int a = 0; a < 3; ++a)
#pragma unroll
                    for (int b = 0; b < 3; ++b)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[k][c][a][b] = fmaf(d[j], patch[c][a][j + b], acc[k][c][a][b]);
        }
    }

    // Sum over the workgroup in a fixed order.  A butterfly over the lanes would
    // cost six cross-lane moves per sum; instead a wave lays 32 sums at a time
    // out in LDS as [sum][lane], two lanes add up the halves of one row (each
    // starting at its own offset, so the 64 lanes spread over the banks), one
    // cross-lane move joins the halves; the four waves' results meet in `red`.
    __shared__ float red[NT / 64][NA];
    __shared__ float tile[NT / 64][32][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *av = &acc[0][0][0][0];
#pragma unroll
    for (int v0 = 0; v0 < NA; v0 += 32) {
#pragma unroll
        for (int v = 0; v < 32; ++v)
            if (v0 + v < NA) tile[wave][v][lane] = av[v0 + v];
        // (a wave's own writes are visible to its later reads: LDS operations of a wave stay in order)
        const int row = lane >> 1, half = lane & 1;
        float sum = 0.0f;
        if (v0 + row < NA) {
#pragma unroll
            for (int i = 0; i < 32; ++i) sum += tile[wave][row][half * 32 + ((i + row) & 31)];
        }
        sum += __shfl_xor(sum, 1, 64);
        if (half == 0 && v0 + row < NA) red[wave][v0 + row] = sum;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < NA; e += NT) {
        const int k = e / (CI * 9);
        if (co0 + k >= p.Co) continue;
        float s = red[0][e];
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) s += red[w][e];
        p.part[((long long)blockIdx.x * p.Co + co0) * (CI * 9) + e] = s;
    }
}

constexpr int FWD_COB = 16, WG_COB = 4;

} // namespace

bool dk_smallci_ok(const dk_geom &g, long long R, const float *x, const float *other)
{
    if (!g.conv || g.dw) return false;
    if (g.kh != 3 || g.kw != 3 || g.stride != 1 || g.pad != 1) return false;
    if (g.Ci < 1 || g.Ci > 4 || g.W % 4 || g.W < 4) return false;
    if (!dk_aligned(x, 16) || !dk_aligned(other, 16)) return false;
    if (R * g.H * (g.W / 4) > (1ll << 40)) return false;
    return true;
}

// Slices of the pixel quads in the weight gradient: enough workgroups for the
// chip (with Co / 2 channel pairs each), at least four quads per thread.
static int smallci_slices(const dk_geom &g, long long R)
{
    const long long nq = R * g.H * (g.W / 4);
    const long long chunks = (g.Co + WG_COB - 1) / WG_COB;
    long long s = (1024 + chunks - 1) / chunks;
    const long long most = (nq + NT * 4 - 1) / (NT * 4);
    if (s > most) s = most;
    if (s < 1) s = 1;
    if (s > DK_MAX_SPLITS) s = DK_MAX_SPLITS;
    return (int)s;
}

size_t dk_smallci_wgrad_part_bytes(const dk_geom &g, long long R)
{
    if (!g.conv || g.dw || g.kh != 3 || g.kw != 3 || g.stride != 1 || g.pad != 1 || g.Ci > 4 || g.W % 4) return 0;
    return (size_t)smallci_slices(g, R) * g.Co * g.Ci * 9 * sizeof(float);
}

dk_status dk_smallci_fwd_run(const dk_geom &g, const float *W, const float *xbar, float *ybar, long long R,
                             hipStream_t st)
{
    smallci_params p = {};
    p.x = xbar; p.w = W; p.y = ybar;
    p.Co = g.Co; p.H = g.H; p.W = g.W; p.R = (int)R;
    p.nq = R * g.H * (g.W / 4);
    const long long bx = (p.nq + NT - 1) / NT;
    DK_REQUIRE(bx <= 0x7fffffffll, DK_ERR_SHAPE);
    const dim3 grid((unsigned)bx, (unsigned)((g.Co + FWD_COB - 1) / FWD_COB));
    DK_REQUIRE(grid.y <= 65535u, DK_ERR_SHAPE);
    dk_prof_scope ps("conv_smallci_fwd", st);
    switch (g.Ci) {
    case 1: smallci_fwd_kernel<1, FWD_COB><<<grid, dim3(NT), 0, st>>>(p); break;
    case 2: smallci_fwd_kernel<2, FWD_COB><<<grid, dim3(NT), 0, st>>>(p); break;
    case 3: smallci_fwd_kernel<3, FWD_COB><<<grid, dim3(NT), 0, st>>>(p); break;
    default: smallci_fwd_kernel<4, FWD_COB><<<grid, dim3(NT), 0, st>>>(p); break;
    }
    return dk_launch_status();
}

dk_status dk_smallci_wgrad_run(const dk_geom &g, const float *dtilde, const float *xbar, float *dW, long long R,
                               float scale, int accumulate, float *part, size_t part_bytes, hipStream_t st)
{
    const int slices = smallci_slices(g, R);
    DK_REQUIRE(part && part_bytes >= (size_t)slices * g.Co * g.Ci * 9 * sizeof(float), DK_ERR_WORKSPACE);
    smallci_params p = {};
    p.x = xbar; p.d = dtilde; p.part = part;
    p.Co = g.Co; p.H = g.H; p.W = g.W; p.R = (int)R;
    p.nq = R * g.H * (g.W / 4);
    const long long per_pass = (long long)slices * NT;
    p.qpt = (int)((p.nq + per_pass - 1) / per_pass);
    const dim3 grid((unsigned)slices, (unsigned)((g.Co + WG_COB - 1) / WG_COB));
    DK_REQUIRE(grid.y <= 65535u, DK_ERR_SHAPE);
    {
        dk_prof_scope ps("conv_smallci_wgrad", st);
        switch (g.Ci) {
        case 1: smallci_wgrad_kernel<1, WG_COB><<<grid, dim3(NT), 0, st>>>(p); break;
        case 2: smallci_wgrad_kernel<2, WG_COB><<<grid, dim3(NT), 0, st>>>(p); break;
        case 3: smallci_wgrad_kernel<3, WG_COB><<<grid, dim3(NT), 0, st>>>(p); break;
        default: smallci_wgrad_kernel<4, WG_COB><<<grid, dim3(NT), 0, st>>>(p); break;
        }
    }
    DK_REQUIRE(hipGetLastError() == hipSuccess, DK_ERR_HIP);
    // part[slice][co][ci*9] has dW's own layout per slice
    return dk_fold_slices(part, dW, (long long)g.Co * g.Ci * 9, slices, scale, accumulate, st);
}
