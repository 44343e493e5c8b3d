// Generic kernels of the ASI hot path for gfx950 (wave64).
//
// Every contraction of the path is one of two shapes over a tensor seen from a
// mode, X[o,i,j] (outer, n, inner):
//   ttm : Y[o,q,j]  = sum_i X[o,i,j] M(i,q)            (m-mode product, Eq. 4)
//   pair: P[i,q]    = sum_{o,j} X[o,i,j] Y[o,q,j]      (A_m V of Alg. 1)
// plus the Gram/Cholesky orthonormalisation and the step-4 correlation of Eq. 14.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

// ---------------------------------------------------------------------------
// ttm: block = 128 unfolding columns x 32 outputs q, K (= mode index i) in chunks of 16
// ---------------------------------------------------------------------------
constexpr int TTM_TC = 128, TTM_TQ = 32, TTM_TK = 16;

template <typename T, bool LASTMODE>
__global__ __launch_bounds__(256) void k_ttm(const T* __restrict__ X, long long outer, int n, long long inner,
                                             const float* __restrict__ Mp, long long ms_i, long long ms_q, int r,
                                             float* __restrict__ Y, int beta) {
    __shared__ float Xs[TTM_TK][TTM_TC + 1];
    __shared__ float Ms[TTM_TK][TTM_TQ + 1];
    const long long ncols = outer * inner;
    const long long c0 = (long long)blockIdx.x * TTM_TC;
    const int q0 = blockIdx.y * TTM_TQ;
    const int tid = threadIdx.x;
    const int tcg = tid & 31, tqg = tid >> 5;
    float acc[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[u][k] = 0.f;

    long long ld_base = -1;  // offset of element (o, 0, j) for this thread's loader column
    if (!LASTMODE) {
        const long long c = c0 + (tid & 127);
        if (c < ncols) {
            const long long o = c / inner, j = c - o * inner;
            ld_base = o * (long long)n * inner + j;
        }
    }
    for (int k0 = 0; k0 < n; k0 += TTM_TK) {
        if (!LASTMODE) {
            const int cl = tid & 127;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int il = (tid >> 7) + 2 * t, i = k0 + il;
                Xs[il][cl] = (ld_base >= 0 && i < n) ? ldf(X, ld_base + (long long)i * inner) : 0.f;
            }
        } else {  // inner == 1: fibres are contiguous, X[c*n + i]
            const int il = tid & 15, i = k0 + il;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int cl = (tid >> 4) + 16 * t;
                const long long c = c0 + cl;
                Xs[il][cl] = (c < ncols && i < n) ? ldf(X, c * (long long)n + i) : 0.f;
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int e = tid + 256 * t, il = e >> 5, ql = e & 31;
            const int i = k0 + il, q = q0 + ql;
            Ms[il][ql] = (i < n && q < r) ? Mp[(long long)i * ms_i + (long long)q * ms_q] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TTM_TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) a[k] = Xs[kk][tcg + 32 * k];
#pragma unroll
            for (int u = 0; u < 4; ++u) b[u] = Ms[kk][tqg * 4 + u];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[u][k] = fmaf(b[u], a[k], acc[u][k]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long long c = c0 + tcg + 32 * k;
        if (c >= ncols) continue;
        const long long o = c / inner, j = c - o * inner;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = q0 + tqg * 4 + u;
            if (q < r) {
                const long long idx = (o * r + q) * inner + j;
                Y[idx] = beta ? Y[idx] + acc[u][k] : acc[u][k];
            }
        }
    }
}

hipError_t launch_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp,
                      long long ms_i, long long ms_q, int r, float* Y, int beta, hipStream_t st) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0) return hipErrorInvalidValue;
    const long long gx = (ncols + TTM_TC - 1) / TTM_TC;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)gx, (unsigned)((r + TTM_TQ - 1) / TTM_TQ));
    const bool last = (inner == 1);
    if (xt == F32) {
        if (last) hipLaunchKernelGGL((k_ttm<float, true>), grid, 256, 0, st, (const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
        else      hipLaunchKernelGGL((k_ttm<float, false>), grid, 256, 0, st, (const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
    } else {
        if (last) hipLaunchKernelGGL((k_ttm<bf16_t, true>), grid, 256, 0, st, (const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
        else      hipLaunchKernelGGL((k_ttm<bf16_t, false>), grid, 256, 0, st, (const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// pair: block = 64 rows i x 32 outputs q over one split of the unfolding columns
// ---------------------------------------------------------------------------
constexpr int PR_TI = 64, PR_TQ = 32, PR_TK = 32;

template <typename T, bool LASTMODE>
__global__ __launch_bounds__(256) void k_pair(const T* __restrict__ X, long long outer, int n, long long inner,
                                              const float* __restrict__ Y, int r, double* __restrict__ part,
                                              long long cols_per_split) {
    __shared__ float Xs[PR_TK][PR_TI + 1];
    __shared__ float Ys[PR_TK][PR_TQ + 1];
    const long long ncols = outer * inner;
    const int i0 = blockIdx.x * PR_TI, q0 = blockIdx.y * PR_TQ, s = blockIdx.z;
    const long long cbeg = (long long)s * cols_per_split;
    const long long cend = (cbeg + cols_per_split < ncols) ? cbeg + cols_per_split : ncols;
    const int tid = threadIdx.x;
    const int ti = tid & 15, tq = tid >> 4;
    // fp64 accumulation: P must keep components ~(sigma_r/sigma_1)^2 below its largest ones,
    // which fp32 sums cannot hold when the columns of U_prev are not aligned with singular vectors
    double acc[4][2];
#pragma unroll
    for (int x = 0; x < 4; ++x) { acc[x][0] = 0.0; acc[x][1] = 0.0; }

    for (long long c0 = cbeg; c0 < cend; c0 += PR_TK) {
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
                const int il = (tid >> 5) + 8 * t, i = i0 + il;
                Xs[cl][il] = (valid && i < n) ? ldf(X, xbase + (long long)i * inner) : 0.f;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int ql = (tid >> 5) + 8 * t, q = q0 + ql;
                Ys[cl][ql] = (valid && q < r) ? Y[ybase + (long long)q * inner] : 0.f;
            }
        } else {  // inner == 1
            const int il = tid & 63, i = i0 + il;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int cl = (tid >> 6) + 4 * t;
                const long long c = c0 + cl;
                Xs[cl][il] = (c < cend && i < n) ? ldf(X, c * (long long)n + i) : 0.f;
            }
            const int ql = tid & 31, q = q0 + ql;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int cl = (tid >> 5) + 8 * t;
                const long long c = c0 + cl;
                Ys[cl][ql] = (c < cend && q < r) ? Y[c * (long long)r + q] : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < PR_TK; ++kk) {
            double a[4], b[2];
#pragma unroll
            for (int x = 0; x < 4; ++x) a[x] = (double)Xs[kk][ti + 16 * x];
            b[0] = (double)Ys[kk][tq];
            b[1] = (double)Ys[kk][tq + 16];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                acc[x][0] = fma(a[x], b[0], acc[x][0]);
                acc[x][1] = fma(a[x], b[1], acc[x][1]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int i = i0 + ti + 16 * x, q = q0 + tq + 16 * y;
            if (i < n && q < r) part[((long long)s * n + i) * r + q] = acc[x][y];
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
    long long want = 1024 / (tiles > 0 ? tiles : 1);
    if (want < 1) want = 1;
    long long maxs = (ncols + 4 * PR_TK - 1) / (4 * PR_TK);   // at least 128 columns per split
    if (want > maxs) want = maxs;
    if (want > 1024) want = 1024;
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
    hipLaunchKernelGGL(k_sum_partials<float>, dim3((unsigned)gx), 256, 0, st, part, nsplit, count, out, beta);
    return hipGetLastError();
}
hipError_t launch_sum_partials_f64(const double* part, int nsplit, long long count, float* out, int beta,
                                   hipStream_t st) {
    if (count <= 0) return hipErrorInvalidValue;
    const long long gx = (count + 255) / 256;
    hipLaunchKernelGGL(k_sum_partials<double>, dim3((unsigned)gx), 256, 0, st, part, nsplit, count, out, beta);
    return hipGetLastError();
}

__global__ void k_set_i32(int32_t* p, int32_t v) { *p = v; }
hipError_t launch_set_i32(int32_t* p, int32_t v, hipStream_t st) {
    hipLaunchKernelGGL(k_set_i32, 1, 1, 0, st, p, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Step 4 of Eq. 14: one thread per T[o,j,kh,kw] and split of the r1 axis
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_corr(const float* __restrict__ G1, const float* __restrict__ Z,
                                              float* __restrict__ Tpart, CorrGeom g, int i_per_split) {
    const int taps = g.kh * g.kw;
    const long long total = (long long)g.cout * g.r2 * taps;
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int t = (int)(e % taps);
    const int j = (int)((e / taps) % g.r2);
    const int o = (int)(e / ((long long)taps * g.r2));
    const int kh = t / g.kw, kw = t - kh * g.kw;
    const int ibeg = blockIdx.y * i_per_split;
    const int iend = (ibeg + i_per_split < g.r1) ? ibeg + i_per_split : g.r1;
    const int hoff = kh * g.dh - g.ph, woff = kw * g.dw - g.pw;
    float acc = 0.f;
    for (int i = ibeg; i < iend; ++i) {
        const float* g1p = G1 + ((long long)i * g.cout + o) * g.Ho * g.Wo;
        const float* zp = Z + ((long long)i * g.r2 + j) * g.H * g.W;
        for (int y = 0; y < g.Ho; ++y) {
            const int hh = y * g.sh + hoff;
            if (hh < 0 || hh >= g.H) continue;
            for (int x = 0; x < g.Wo; ++x) {
                const int ww = x * g.sw + woff;
                if (ww >= 0 && ww < g.W) acc = fmaf(g1p[y * g.Wo + x], zp[hh * g.W + ww], acc);
            }
        }
    }
    Tpart[(long long)blockIdx.y * total + e] = acc;
}

int corr_splits(const CorrGeom& g) {
    const long long total = (long long)g.cout * g.r2 * g.kh * g.kw;
    const long long blocks = (total + 255) / 256;
    long long want = (2048 + blocks - 1) / blocks;
    if (want > g.r1) want = g.r1;
    if (want < 1) want = 1;
    int ips = (int)((g.r1 + want - 1) / want);
    return (g.r1 + ips - 1) / ips;
}

hipError_t launch_corr(const float* G1, const float* Z, float* Tpart, const CorrGeom& g, int nsplit, hipStream_t st) {
    const long long total = (long long)g.cout * g.r2 * g.kh * g.kw;
    if (total <= 0 || nsplit <= 0) return hipErrorInvalidValue;
    const int ips = (g.r1 + nsplit - 1) / nsplit;
    dim3 grid((unsigned)((total + 255) / 256), (unsigned)nsplit);
    hipLaunchKernelGGL(k_corr, grid, 256, 0, st, G1, Z, Tpart, g, ips);
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
    hipLaunchKernelGGL(k_expand_grouped, dim3((unsigned)((total + 255) / 256)), 256, 0, st, T, U2, dW, cout, r2,
                       taps, cg, og, beta);
    return hipGetLastError();
}

}  // namespace asi
