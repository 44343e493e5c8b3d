// Shared device-side helpers for the ASI kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asi {

// bf16 storage is handled as raw 16-bit patterns: widening to fp32 is a shift.
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

template <typename T>
__device__ __forceinline__ float ldf(const T* __restrict__ p, long long idx) { return to_f32(p[idx]); }

// Guarded loads: the index is clamped to element 0 (always valid) and the value is selected
// afterwards, so that the load itself needs no branch.  The compiler may still wrap load and
// widening in a conditional block of its own (it does for bf16 when the guard is a single
// comparison), and the load is then waited for inside that block; loops whose speed depends on
// many loads in flight keep what they load as raw bits and mask it later (asi_ttm.hip, k_pair).
template <typename T>
__device__ __forceinline__ float ldg_f32(const T* __restrict__ p, long long idx, bool ok) {
    const T v = p[ok ? idx : 0];
    return ok ? to_f32(v) : 0.f;
}
__device__ __forceinline__ double ldg_f64(const double* __restrict__ p, long long idx, bool ok) {
    const double v = p[ok ? idx : 0];
    return ok ? v : 0.0;
}

// A tensor seen from one mode: X[o, i, j], o < outer, i < n (the mode), j < inner.
// Column c of the mode unfolding (Sec. 3.2) is the pair (o, j) = (c / inner, c % inner).
struct ModeView {
    long long outer;
    int n;
    long long inner;
};

// ---------------------------------------------------------------------------
// The standard-normal matrix V of Alg. 1's first iteration (t = 0), never stored: entry V[c, 4g + k] of
// mode m is a pure function of (seed, m, c, g).  Philox4x32-10 (Salmon et al., SC 2011) keyed by the seed
// is called on the counter (c mod 2^32, c div 2^32, g, m); each of its four words gives a uniform
// u = (top 23 bits + 0.5) / 2^23, strictly inside (0, 1), and each pair of uniforms one Box-Muller pair
// sqrt(-2 ln u1) * (cos 2 pi u2, sin 2 pi u2), evaluated in fp64 and rounded once to fp32: any correct
// fp64 evaluation of the same formula then gives the same fp32 value (up to the rare tie within an fp64
// rounding error), so V does not depend on a library's fp32 log / sin / cos.  The draw happens once per
// training run, so its cost is of no account.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                              uint32_t out[4]) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0, hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
__device__ __forceinline__ double uniform23(uint32_t x) { return ((double)(x >> 9) + 0.5) * 0x1p-23; }
__device__ __forceinline__ void gauss4(uint32_t seed_lo, uint32_t seed_hi, int mode, long long c, uint32_t g, float z[4]) {
    uint32_t w[4];
    philox4x32_10((uint32_t)((unsigned long long)c & 0xffffffffu), (uint32_t)((unsigned long long)c >> 32), g, (uint32_t)mode,
                  seed_lo, seed_hi, w);
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        const double rad = sqrt(-2.0 * log(uniform23(w[2 * pr])));
        double sn, cs;
        sincospi(2.0 * uniform23(w[2 * pr + 1]), &sn, &cs);
        z[2 * pr] = (float)(rad * cs);
        z[2 * pr + 1] = (float)(rad * sn);
    }
}

}  // namespace asi
