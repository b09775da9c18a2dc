// Finite-field variant, host side: coefficient derivation modulo p.
#include <vector>

#include "dk_field.h"

namespace {

constexpr uint64_t P = DKF_P;

// a^-1 mod p by the extended Euclidean algorithm (a in [1, p)).
uint32_t inv_mod(uint32_t a)
{
    int64_t r0 = (int64_t)P, r1 = a, t0 = 0, t1 = 1;
    while (r1 != 0) {
        const int64_t q = r0 / r1;
        const int64_t r2 = r0 - q * r1; r0 = r1; r1 = r2;
        const int64_t t2 = t0 - q * t1; t0 = t1; t1 = t2;
    }
    return (uint32_t)(t0 < 0 ? t0 + (int64_t)P : t0);
}

// Gauss-Jordan elimination of [M | I] over the field; false if M is singular.
bool invert(std::vector<uint32_t> &M, std::vector<uint32_t> &inv, int n)
{
    inv.assign((size_t)n * n, 0);
    for (int i = 0; i < n; ++i) inv[(size_t)i * n + i] = 1;
    for (int c = 0; c < n; ++c) {
        int piv = -1;
        for (int r = c; r < n && piv < 0; ++r)
            if (M[(size_t)r * n + c]) piv = r;
        if (piv < 0) return false;
        if (piv != c)
            for (int j = 0; j < n; ++j) {
                std::swap(M[(size_t)c * n + j], M[(size_t)piv * n + j]);
                std::swap(inv[(size_t)c * n + j], inv[(size_t)piv * n + j]);
            }
        const uint64_t f = inv_mod(M[(size_t)c * n + c]);
        for (int j = 0; j < n; ++j) {
            M[(size_t)c * n + j] = (uint32_t)(M[(size_t)c * n + j] * f % P);
            inv[(size_t)c * n + j] = (uint32_t)(inv[(size_t)c * n + j] * f % P);
        }
        for (int r = 0; r < n; ++r) {
            const uint64_t m = M[(size_t)r * n + c];
            if (r == c || m == 0) continue;
            for (int j = 0; j < n; ++j) {
                M[(size_t)r * n + j] = (uint32_t)((M[(size_t)r * n + j] + (P - m) * M[(size_t)c * n + j]) % P);
                inv[(size_t)r * n + j] = (uint32_t)((inv[(size_t)r * n + j] + (P - m) * inv[(size_t)c * n + j]) % P);
            }
        }
    }
    return true;
}

} // namespace

DK_EXPORT dk_status dkf_coeffs(const uint32_t *A, const uint32_t *gamma, int G, int K,
                               uint32_t *Ainv, uint32_t *nvec, uint32_t *B)
{
    return dkf_coeffs_m(A, gamma, G, K, 1, Ainv, nvec, B);
}

DK_EXPORT dk_status dkf_coeffs_m(const uint32_t *A, const uint32_t *gamma, int G, int K, int Mn,
                                 uint32_t *Ainv, uint32_t *nvec, uint32_t *B)
{
    DK_REQUIRE(A && gamma, DK_ERR_NULL);
    DK_REQUIRE(G >= 1 && K >= 1 && Mn >= 1 && K + Mn - 1 <= DK_MAX_K, DK_ERR_SHAPE);
    const int S = K + Mn + 1;
    for (long long i = 0; i < (long long)G * S * S; ++i) DK_REQUIRE(A[i] < P, DK_ERR_SHAPE);
    for (long long i = 0; i < (long long)G * S; ++i) DK_REQUIRE(gamma[i] < P, DK_ERR_SHAPE);
    // Validate everything before writing anything.
    std::vector<uint32_t> all((size_t)G * S * S), M((size_t)S * S), inv;
    for (int g = 0; g < G; ++g) {
        for (int i = 0; i < S * S; ++i) M[i] = A[(size_t)g * S * S + i];
        if (!invert(M, inv, S)) return DK_ERR_SINGULAR;
        for (int j = 0; j < S; ++j)
            if (gamma[(size_t)g * S + j] == 0) return DK_ERR_SINGULAR;
        for (int i = 0; i < S * S; ++i) all[(size_t)g * S * S + i] = inv[i];
    }
    for (int g = 0; g < G; ++g) {
        const uint32_t *inv_g = &all[(size_t)g * S * S];
        for (int j = 0; j < S; ++j) {
            const uint64_t gi = inv_mod(gamma[(size_t)g * S + j]);
            if (Ainv)
                for (int i = 0; i < S; ++i) Ainv[((size_t)g * S + j) * S + i] = inv_g[j * S + i];
            if (nvec) nvec[(size_t)g * S + j] = inv_g[j * S + S - 1];
            if (B)
                for (int i = 0; i < K; ++i)
                    B[((size_t)g * S + j) * K + i] = (uint32_t)(inv_g[j * S + i] * gi % P);
        }
    }
    return DK_OK;
}
