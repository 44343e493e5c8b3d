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

}  // namespace asi
