// Pieces of the fp32 MFMA contraction engine that more than one translation
// unit uses: tile configuration, the buffer-load fast path and the two plain
// matrix loaders.  Included inside each unit's unnamed namespace.
#pragma once

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Loader fast path.  Vector-ALU instructions of a wave that is fetching queue
// behind the matrix instructions of the other waves on its SIMD, so the common
// case -- a whole contraction step of an operand whose rows are whole 16-byte
// vectors -- is fetched with buffer loads: the matrix is a scalar resource, the
// step advances a scalar offset, and each lane keeps one precomputed byte
// offset per vector (an offset past the resource's range for rows outside the
// matrix, which then read as zero).  No address arithmetic, no predicates.
constexpr int DK_RSRC_FLAGS = 0x00020000;         // raw buffer resource, gfx9 family
constexpr unsigned DK_OOB = 0x80000000u;          // beyond any resource range used here
constexpr long long DK_RSRC_MAX = 0x7fffffffll;   // largest operand (bytes) the fast path takes

// A resource over `bytes` bytes at p.  Both are wave-uniform by construction, but a size
// that went through an integer division was computed on the vector ALU, and a resource in
// vector registers makes the compiler wrap every load in a loop over the wave's distinct
// descriptors: pin the words to scalar registers.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t dk_uniform_rsrc(const float *p, int bytes)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<float *>(((unsigned long long)hi << 32) | lo), 0,
                                             __builtin_amdgcn_readfirstlane(bytes), DK_RSRC_FLAGS);
}

__device__ __forceinline__ float4 dk_buffer_load4(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff)
{
    const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, (int)soff, 0));
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = 64 * WM * WN;          // threads per workgroup
    static constexpr int TM = BM / WM / 32;          // 32x32 blocks per wave, rows
    static constexpr int TN = BN / WN / 32;          // 32x32 blocks per wave, cols
    static constexpr int LDA = BM + 4;               // LDS row pitch (floats)
    static constexpr int LDB = BN + 4;
    static constexpr int LDS_FLOATS = 2 * BK * (LDA + LDB);
    // one contraction step of a wave: TM*TN MFMAs of 64 cycles per k pair, at about 2.1 GHz
    static constexpr double STEP_US = TM * TN * (BK / 2) * 64 / 2100.0;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 4 == 0, "tile shape");
};

// ---------------------------------------------------------------------------
// Operand loaders.  Each fetches a BK x ROWS operand tile of contraction step
// kt into registers (load) and later writes it k-major into LDS (store).
// Elements outside the matrix read as zero.
// ---------------------------------------------------------------------------

struct MatParams {
    const float *p;
    long long ld;   // leading dimension (floats)
    int rows;       // extent along the tile's row axis
    int kdim;       // extent along the contraction axis
};

// Source stored [kdim][ld] with the tile's row axis contiguous.
template <int ROWS, int BK, int NT, int LD, bool VEC>
struct LoadKMajor {
    using Params = MatParams;
    static constexpr int PER_K = ROWS / 4;
    static constexpr int N4 = BK * PER_K / NT;
    static_assert(BK * PER_K % NT == 0, "tile/threads");
    float4 st[N4];
    const float *p; long long ld; int rows, kdim, row0, tid;
    __amdgpu_buffer_rsrc_t rs; unsigned voff[N4]; bool fast;

    __device__ __forceinline__ void init(const Params &a, int row0_, int tid_)
    {
        p = a.p; ld = a.ld; rows = a.rows; kdim = a.kdim; row0 = row0_; tid = tid_;
        const long long bytes = (long long)a.kdim * a.ld * 4;
        fast = VEC && bytes <= DK_RSRC_MAX;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int kr = idx / PER_K, row = row0 + (idx % PER_K) * 4;
            voff[e] = row + 3 < rows ? 4u * (unsigned)(kr * (int)ld + row) : DK_OOB;
        }
    }

    // the same tile of another matrix of the same shape (e.g. the next image)
    __device__ __forceinline__ void rebase(const float *np)
    {
        p = np;
        rs = dk_uniform_rsrc(np, (int)((long long)kdim * ld * 4));
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= kdim) {
            const unsigned soff = 4u * (unsigned)(kt * BK) * (unsigned)ld;
#pragma unroll
            for (int e = 0; e < N4; ++e) st[e] = dk_buffer_load4(rs, voff[e], soff);
            return;
        }
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int kr = idx / PER_K, c4 = idx % PER_K;
            const int k = kt * BK + kr, row = row0 + c4 * 4;
            const float *s = p + (long long)k * ld + row;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < kdim) {
                if (VEC && row + 3 < rows) {
                    v = *reinterpret_cast<const float4 *>(s);
                } else {
                    if (row + 0 < rows) v.x = s[0];
                    if (row + 1 < rows) v.y = s[1];
                    if (row + 2 < rows) v.z = s[2];
                    if (row + 3 < rows) v.w = s[3];
                }
            }
            st[e] = v;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int kr = idx / PER_K, c4 = idx % PER_K;
            *reinterpret_cast<float4 *>(buf + kr * LD + c4 * 4) = st[e];
        }
    }
};

// Source stored [rows][ld] with the contraction axis contiguous.
template <int ROWS, int BK, int NT, int LD, bool VEC>
struct LoadRowMajorK {
    using Params = MatParams;
    static constexpr int PER_ROW = BK / 4;
    static constexpr int N4 = ROWS * PER_ROW / NT;
    static_assert(ROWS * PER_ROW % NT == 0, "tile/threads");
    float4 st[N4];
    const float *p; long long ld; int rows, kdim, row0, tid;
    __amdgpu_buffer_rsrc_t rs; unsigned voff[N4]; bool fast;

    __device__ __forceinline__ void init(const Params &a, int row0_, int tid_)
    {
        p = a.p; ld = a.ld; rows = a.rows; kdim = a.kdim; row0 = row0_; tid = tid_;
        const long long bytes = (long long)a.rows * a.ld * 4;
        fast = VEC && bytes <= DK_RSRC_MAX;
        rs = dk_uniform_rsrc(a.p, (int)bytes);
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int r = row0 + idx / PER_ROW, kc = idx % PER_ROW;
            voff[e] = r < rows ? 4u * (unsigned)(r * (int)ld + kc * 4) : DK_OOB;
        }
    }

    __device__ __forceinline__ void load(int kt)
    {
        if (fast && (kt + 1) * BK <= kdim) {
            const unsigned soff = 4u * (unsigned)(kt * BK);
#pragma unroll
            for (int e = 0; e < N4; ++e) st[e] = dk_buffer_load4(rs, voff[e], soff);
            return;
        }
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int row = idx / PER_ROW, kc = idx % PER_ROW;
            const int k = kt * BK + kc * 4, r = row0 + row;
            const float *s = p + (long long)r * ld + k;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rows) {
                if (VEC && k + 3 < kdim) {
                    v = *reinterpret_cast<const float4 *>(s);
                } else {
                    if (k + 0 < kdim) v.x = s[0];
                    if (k + 1 < kdim) v.y = s[1];
                    if (k + 2 < kdim) v.z = s[2];
                    if (k + 3 < kdim) v.w = s[3];
                }
            }
            st[e] = v;
        }
    }

    __device__ __forceinline__ void store(float *buf) const
    {
#pragma unroll
        for (int e = 0; e < N4; ++e) {
            const int idx = tid + e * NT;
            const int row = idx / PER_ROW, kc = idx % PER_ROW;
            float *d = buf + (kc * 4) * LD + row;
            d[0 * LD] = st[e].x;
            d[1 * LD] = st[e].y;
            d[2 * LD] = st[e].z;
            d[3 * LD] = st[e].w;
        }
    }
};

