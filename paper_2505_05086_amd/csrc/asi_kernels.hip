// Generic kernels of the ASI hot path for gfx950 (wave64).
//
// Contractions over a tensor seen from a mode, X[o,i,j] (outer, n, inner):
//   pair: P[i,q]    = sum_{o,j} X[o,i,j] Y[o,q,j]      (A_m V of Alg. 1)
// plus partial-sum reduction, the step-4 correlation of Eq. 14 and its grouped step 5.
#include "asi_device.h"
#include "asi_kernels.h"

#include <cstdarg>
#include <cstdio>

namespace asi {

static thread_local char g_last_label[160] = "";
void set_last_label(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_label, sizeof(g_last_label), fmt, ap);
    va_end(ap);
}
const char* last_label() { return g_last_label; }

// ---------------------------------------------------------------------------
// pair: P[i,q] = sum_c X[i,c] Y[q,c] on fp64 MFMA.  A workgroup owns 64 rows i x 32 outputs q
// over one split of the unfolding columns; chunks of 32 columns are prefetched into registers
// while the previous chunk is multiplied.  Wave w multiplies rows 16w..16w+15:
//   A operand (16 i x 4 c) = Xs[4ks + lane/16][16w + lane%16],  B operand (4 c x 16 q) = Ys[4ks + lane/16][16nb + lane%16]
// fp32 values are widened to fp64, so every product is exact and the sums are carried in fp64.
// ---------------------------------------------------------------------------
constexpr int PR_TI = 64, PR_TQ = 32, PR_TK = 32;
typedef double v4d __attribute__((ext_vector_type(4)));

template <typename T, bool LASTMODE>
__global__ __launch_bounds__(256) void k_pair(const T* __restrict__ X, long long outer, int n, long long inner,
                                              const float* __restrict__ Y, int r, double* __restrict__ part,
                                              long long cols_per_split) {
    __shared__ float Xs[PR_TK][PR_TI + 4];
    __shared__ float Ys[PR_TK][PR_TQ + 4];
    const long long ncols = outer * inner;
    const int i0 = blockIdx.x * PR_TI, q0 = blockIdx.y * PR_TQ, s = blockIdx.z;
    const long long cbeg = (long long)s * cols_per_split;
    const long long cend = (cbeg + cols_per_split < ncols) ? cbeg + cols_per_split : ncols;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;

    float xr[8], yr[4];
    auto fetch = [&](long long c0) {
        if (!LASTMODE) {
            const int cl = tid & 31;
            const long long c = c0 + cl;
            const bool valid = c < cend;
            long long xbase = 0, ybase = 0;
            if (valid) {
                const long long o = c / inner, j = c - o * inner;
                xbase = o * (long long)n * inner + j;
                ybase = o * (long long)r * inner + j;
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int i = i0 + (tid >> 5) + 8 * t;
                xr[t] = ldg_f32(X, xbase + (long long)i * inner, valid && i < n);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int q = q0 + (tid >> 5) + 8 * t;
                yr[t] = ldg_f32(Y, ybase + (long long)q * inner, valid && q < r);
            }
        } else {  // inner == 1
            const int i = i0 + (tid & 63);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const long long c = c0 + (tid >> 6) + 4 * t;
                xr[t] = ldg_f32(X, c * (long long)n + i, c < cend && i < n);
            }
            const int q = q0 + (tid & 31);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const long long c = c0 + (tid >> 5) + 8 * t;
                yr[t] = ldg_f32(Y, c * (long long)r + q, c < cend && q < r);
            }
        }
    };
    auto stash = [&]() {
        if (!LASTMODE) {
            const int cl = tid & 31;
#pragma unroll
            for (int t = 0; t < 8; ++t) Xs[cl][(tid >> 5) + 8 * t] = xr[t];
#pragma unroll
            for (int t = 0; t < 4; ++t) Ys[cl][(tid >> 5) + 8 * t] = yr[t];
        } else {
#pragma unroll
            for (int t = 0; t < 8; ++t) Xs[(tid >> 6) + 4 * t][tid & 63] = xr[t];
#pragma unroll
            for (int t = 0; t < 4; ++t) Ys[(tid >> 5) + 8 * t][tid & 31] = yr[t];
        }
    };

    v4d acc[2] = {{0.0, 0.0, 0.0, 0.0}, {0.0, 0.0, 0.0, 0.0}};
    if (cbeg < cend) fetch(cbeg);
    for (long long c0 = cbeg; c0 < cend; c0 += PR_TK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (c0 + PR_TK < cend) fetch(c0 + PR_TK);
#pragma unroll
        for (int ks = 0; ks < PR_TK / 4; ++ks) {
            const double a = (double)Xs[4 * ks + lg][16 * wave + ll];
            acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)Ys[4 * ks + lg][ll], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)Ys[4 * ks + lg][16 + ll], acc[1], 0, 0, 0);
        }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + 16 * wave + lg + 4 * v, q = q0 + 16 * nb + ll;    // fp64 MFMA result layout
            if (i < n && q < r) part[((long long)s * n + i) * r + q] = acc[nb][v];
        }
}

static long long pair_cols_per_split(long long ncols, int nsplit) {
    long long cps = (ncols + nsplit - 1) / nsplit;
    cps = (cps + PR_TK - 1) / PR_TK * PR_TK;
    return cps;
}

int pair_splits(long long outer, int n, long long inner, int r) {
    const long long ncols = outer * inner;
    const long long tiles = (long long)((n + PR_TI - 1) / PR_TI) * ((r + PR_TQ - 1) / PR_TQ);
    long long want = 512 / (tiles > 0 ? tiles : 1);           // aim at ~512 workgroups
    const long long maxs = (ncols + 511) / 512;               // at least 512 columns per split
    if (want > maxs) want = maxs;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    // no empty split: shrink until the last split starts inside the column range
    int ns = (int)want;
    while (ns > 1 && pair_cols_per_split(ncols, ns) * (ns - 1) >= ncols) --ns;
    return ns;
}

hipError_t launch_pair(DType xt, const void* X, long long outer, int n, long long inner, const float* Y, int r,
                       double* part, int nsplit, hipStream_t st) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0 || nsplit <= 0) return hipErrorInvalidValue;
    const long long cps = pair_cols_per_split(ncols, nsplit);
    dim3 grid((unsigned)((n + PR_TI - 1) / PR_TI), (unsigned)((r + PR_TQ - 1) / PR_TQ), (unsigned)nsplit);
    const bool last = (inner == 1);
    set_last_label("k_pair<%s, %s>", xt == F32 ? "float" : "asi::bf16_t", last ? "true" : "false");
    if (xt == F32) {
        if (last) hipLaunchKernelGGL((k_pair<float, true>), grid, 256, 0, st, (const float*)X, outer, n, inner, Y, r, part, cps);
        else      hipLaunchKernelGGL((k_pair<float, false>), grid, 256, 0, st, (const float*)X, outer, n, inner, Y, r, part, cps);
    } else {
        if (last) hipLaunchKernelGGL((k_pair<bf16_t, true>), grid, 256, 0, st, (const bf16_t*)X, outer, n, inner, Y, r, part, cps);
        else      hipLaunchKernelGGL((k_pair<bf16_t, false>), grid, 256, 0, st, (const bf16_t*)X, outer, n, inner, Y, r, part, cps);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// sum of split partials
// ---------------------------------------------------------------------------
template <typename PT>
__global__ __launch_bounds__(256) void k_sum_partials(const PT* __restrict__ part, int nsplit, long long count,
                                                      float* __restrict__ out, int beta) {
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    double s = 0.0;
    for (int sp = 0; sp < nsplit; ++sp) s += (double)part[(long long)sp * count + e];
    out[e] = beta ? out[e] + (float)s : (float)s;
}

hipError_t launch_sum_partials(const float* part, int nsplit, long long count, float* out, int beta, hipStream_t st) {
    if (count <= 0) return hipErrorInvalidValue;
    const long long gx = (count + 255) / 256;
    set_last_label("k_sum_partials<float>");
    hipLaunchKernelGGL(k_sum_partials<float>, dim3((unsigned)gx), 256, 0, st, part, nsplit, count, out, beta);
    return hipGetLastError();
}
hipError_t launch_sum_partials_f64(const double* part, int nsplit, long long count, float* out, int beta,
                                   hipStream_t st) {
    if (count <= 0) return hipErrorInvalidValue;
    const long long gx = (count + 255) / 256;
    set_last_label("k_sum_partials<double>");
    hipLaunchKernelGGL(k_sum_partials<double>, dim3((unsigned)gx), 256, 0, st, part, nsplit, count, out, beta);
    return hipGetLastError();
}

__global__ void k_set_i32(int32_t* p, int32_t v) { *p = v; }
hipError_t launch_set_i32(int32_t* p, int32_t v, hipStream_t st) {
    hipLaunchKernelGGL(k_set_i32, 1, 1, 0, st, p, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Step 5 of Eq. 14 for grouped convolutions
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_expand_grouped(const float* __restrict__ T, const float* __restrict__ U2,
                                                        float* __restrict__ dW, int cout, int r2, int taps, int cg,
                                                        int og, int beta) {
    const long long total = (long long)cout * cg * taps;
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int t = (int)(e % taps);
    const int c = (int)((e / taps) % cg);
    const int o = (int)(e / ((long long)taps * cg));
    const float* tp = T + (long long)o * r2 * taps + t;
    const float* up = U2 + ((long long)(o / og) * cg + c) * r2;
    float acc = 0.f;
    for (int j = 0; j < r2; ++j) acc = fmaf(tp[(long long)j * taps], up[j], acc);
    dW[e] = beta ? dW[e] + acc : acc;
}

hipError_t launch_expand_grouped(const float* T, const float* U2, float* dW, int cout, int r2, int taps, int cg,
                                 int og, int beta, hipStream_t st) {
    const long long total = (long long)cout * cg * taps;
    if (total <= 0) return hipErrorInvalidValue;
    set_last_label("k_expand_grouped");
    hipLaunchKernelGGL(k_expand_grouped, dim3((unsigned)((total + 255) / 256)), 256, 0, st, T, U2, dW, cout, r2,
                       taps, cg, og, beta);
    return hipGetLastError();
}

}  // namespace asi
