// m-mode product (Eq. 4) on fp32 MFMA:  Y[o,q,j] = sum_i X[o,i,j] M(i,q).
//
// Seen as a GEMM the unfolding's columns c = (o,j) are the long dimension, the mode index i
// is K and q is N.  A workgroup owns 64 columns and up to 64 outputs q; K is walked in
// chunks of 32 that are prefetched into registers while the previous chunk is multiplied
// (LDS double use, one barrier pair per chunk).  Wave w multiplies columns 16w..16w+15:
//   A operand (16 columns x 4 i)   = Xs[4ks + lane/16][16w + lane%16]
//   B operand (4 i x 16 q)         = Ms[4ks + lane/16][16nb + lane%16]
// The result tile is transposed through LDS so that stores run along the contiguous index.
// With KRON the matrix is the Kronecker product of two factors, M(i,q) = M1(i/n2, q/r2) *
// M2(i%n2, q%r2), which contracts two adjacent modes (H and W) in one pass.
//
// k_ttm_ksplit serves long fibres with few unfolding columns (the channel mode of a late conv
// layer): a workgroup owns only 16 columns, its four waves split the mode index between them,
// every operand goes from global memory straight into the MFMA registers (all loads of a round
// are in flight together) and the four partial tiles are added through LDS.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TM_TC = 64, TM_KC = 32, TM_TQ = 64, TM_LD = TM_TC + 4;

struct KronSpec {
    const float* M2;       // second factor; element (i2, q2) at M2[i2 * ms_i + q2 * ms_q]
    long long ms_i, ms_q;
    int n2, r2;            // i = i1 * n2 + i2,  q = q1 * r2 + q2
};

template <typename T, bool LASTMODE, int NBR, bool KRON>
__global__ __launch_bounds__(256) void k_ttm_mfma(const T* __restrict__ X, long long outer, int n, long long inner,
                                                  const float* __restrict__ Mp, long long ms_i, long long ms_q, int r,
                                                  float* __restrict__ Y, int beta, KronSpec kr) {
    __shared__ float smem[2 * TM_KC * TM_LD];       // Xs | Ms during the K loop, Ys (64 x TM_LD) afterwards
    float (*Xs)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem);
    float (*Ms)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem + TM_KC * TM_LD);
    float (*Ys)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem);
    const long long ncols = outer * inner;
    const long long c0 = (long long)blockIdx.x * TM_TC;
    const int q0 = blockIdx.y * TM_TQ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;

    // loader coordinates
    long long ld_base = -1;
    int l_c, l_i;
    if (!LASTMODE) {
        l_c = tid & 63; l_i = tid >> 6;              // rows l_i + 4t
        const long long c = c0 + l_c;
        if (c < ncols) {
            const long long o = c / inner, j = c - o * inner;
            ld_base = o * (long long)n * inner + j;
        }
    } else {
        l_i = tid & 31; l_c = tid >> 5;              // columns l_c + 8t
    }
    const int m_q = tid & 63, m_i = tid >> 6;        // Ms loader: rows m_i + 4t

    float xr[8], mr[8];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (!LASTMODE) {
                const int i = k0 + l_i + 4 * t;
                xr[t] = ldg_f32(X, ld_base + (long long)i * inner, ld_base >= 0 && i < n);
            } else {
                const long long c = c0 + l_c + 8 * t;
                const int i = k0 + l_i;
                xr[t] = ldg_f32(X, c * (long long)n + i, c < ncols && i < n);
            }
            const int i = k0 + m_i + 4 * t, q = q0 + m_q;
            if (!KRON) {
                mr[t] = ldg_f32(Mp, (long long)i * ms_i + (long long)q * ms_q, i < n && q < r);
            } else {
                const int i1 = i / kr.n2, i2 = i - i1 * kr.n2, q1 = q / kr.r2, q2 = q - q1 * kr.r2;
                const bool ok = i < n && q < r;
                mr[t] = ldg_f32(Mp, (long long)i1 * ms_i + (long long)q1 * ms_q, ok) *
                        ldg_f32(kr.M2, (long long)i2 * kr.ms_i + (long long)q2 * kr.ms_q, ok);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (!LASTMODE) Xs[l_i + 4 * t][l_c] = xr[t];
            else Xs[l_i][l_c + 8 * t] = xr[t];
            Ms[m_i + 4 * t][m_q] = mr[t];
        }
    };

    v4f acc[NBR];
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb) acc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};

    fetch(0);
    for (int k0 = 0; k0 < n; k0 += TM_KC) {
        __syncthreads();                 // previous chunk fully consumed
        stash();
        __syncthreads();
        if (k0 + TM_KC < n) fetch(k0 + TM_KC);
#pragma unroll
        for (int ks = 0; ks < TM_KC / 4; ++ks) {
            if (k0 + 4 * ks < n) {
                const float a = Xs[4 * ks + lg][16 * wave + ll];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, Ms[4 * ks + lg][16 * nb + ll], acc[nb], 0, 0, 0);
            }
        }
    }
    __syncthreads();
    // result layout: lane holds column 16w + 4*lg + v, output 16nb + ll
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) Ys[16 * nb + ll][16 * wave + 4 * lg + v] = acc[nb][v];
    __syncthreads();
    const int rq = (r - q0 < TM_TQ) ? r - q0 : TM_TQ;
    if (!LASTMODE) {
        const int cl = tid & 63;
        const long long c = c0 + cl;
        if (c < ncols) {
            const long long o = c / inner, j = c - o * inner;
            for (int ql = tid >> 6; ql < rq; ql += 4) {
                const long long idx = (o * r + q0 + ql) * inner + j;
                Y[idx] = beta ? Y[idx] + Ys[ql][cl] : Ys[ql][cl];
            }
        }
    } else {
        for (int e = tid; e < TM_TC * rq; e += 256) {
            const int cl = e / rq, ql = e - cl * rq;
            const long long c = c0 + cl;
            if (c < ncols) {
                const long long idx = c * r + q0 + ql;
                Y[idx] = beta ? Y[idx] + Ys[ql][cl] : Ys[ql][cl];
            }
        }
    }
}

// ---- long fibres, few columns ------------------------------------------------------------------
// Round = 16*KS mode indices: wave w, step s multiplies rows k0 + 16s + 4w .. +3.
//   A operand (16 columns x 4 i) and B operand (4 i x 16 q) are loaded by the lanes that use them.
template <typename T, int NBR, int KS>
__global__ __launch_bounds__(256) void k_ttm_ksplit(const T* __restrict__ X, long long outer, int n, long long inner,
                                                    const float* __restrict__ Mp, long long ms_i, long long ms_q, int r,
                                                    float* __restrict__ Y, int beta) {
    __shared__ float red[4][NBR * 16][17];
    const long long ncols = outer * inner;
    const long long c0 = (long long)blockIdx.x * 16;
    const int q0 = blockIdx.y * (NBR * 16);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const long long c = c0 + ll;
    const bool cok = c < ncols;
    long long xbase = 0;
    if (cok) {
        const long long o = c / inner, j = c - o * inner;
        xbase = o * (long long)n * inner + j;
    }
    v4f acc[NBR];
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb) acc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < n; k0 += 16 * KS) {
        float xr[KS], mr[NBR][KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int i = k0 + 16 * s + 4 * wave + lg;
            xr[s] = ldg_f32(X, xbase + (long long)i * inner, cok && i < n);
#pragma unroll
            for (int nb = 0; nb < NBR; ++nb) {
                const int q = q0 + 16 * nb + ll;
                mr[nb][s] = ldg_f32(Mp, (long long)i * ms_i + (long long)q * ms_q, i < n && q < r);
            }
        }
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int nb = 0; nb < NBR; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[s], mr[nb][s], acc[nb], 0, 0, 0);
    }
    // lane holds column 4*lg + v, output 16nb + ll
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][16 * nb + ll][4 * lg + v] = acc[nb][v];
    __syncthreads();
    const int cl = tid & 15;
    const long long cc = c0 + cl;
    if (cc < ncols) {
        const long long o = cc / inner, j = cc - o * inner;
        for (int ql = tid >> 4; ql < NBR * 16; ql += 16) {
            const int q = q0 + ql;
            if (q < r) {
                const float v = (red[0][ql][cl] + red[1][ql][cl]) + (red[2][ql][cl] + red[3][ql][cl]);
                const long long idx = (o * r + q) * inner + j;
                Y[idx] = beta ? Y[idx] + v : v;
            }
        }
    }
}

template <typename T, int NBR>
static hipError_t launch_ksplit_n(const T* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                                  long long ms_q, int r, float* Y, int beta, dim3 grid, hipStream_t st) {
    const int ks = n <= 64 ? 4 : (n <= 128 ? 8 : 16);
    set_last_label("k_ttm_ksplit<%s, %d, %d>", sizeof(T) == 4 ? "float" : "asi::bf16_t", NBR, ks);
    if (ks == 4) hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 4>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
    else if (ks == 8) hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 8>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
    else hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 16>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_ksplit_t(const T* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                                  long long ms_q, int r, float* Y, int beta, hipStream_t st) {
    const long long ncols = outer * inner;
    const long long gx = (ncols + 15) / 16;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    const int nbr = r >= 64 ? 4 : (r + 15) / 16;
    dim3 grid((unsigned)gx, (unsigned)((r + nbr * 16 - 1) / (nbr * 16)));
    switch (nbr) {
        case 1: return launch_ksplit_n<T, 1>(X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, grid, st);
        case 2: return launch_ksplit_n<T, 2>(X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, grid, st);
        case 3: return launch_ksplit_n<T, 3>(X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, grid, st);
        default: return launch_ksplit_n<T, 4>(X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, grid, st);
    }
}

// The tiled kernel walks the mode index in n/32 dependent steps with ncols/64 workgroups; when that
// leaves most of the chip idle the split kernel is the faster one.
static bool prefer_ksplit(long long ncols, int n, long long inner) {
    return inner > 1 && n > 64 && (ncols + TM_TC - 1) / TM_TC < 512;
}

template <typename T, bool LAST, bool KRON>
static hipError_t launch_ttm_t(const T* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                               long long ms_q, int r, float* Y, int beta, const KronSpec& kr, hipStream_t st) {
    const long long ncols = outer * inner;
    const long long gx = (ncols + TM_TC - 1) / TM_TC;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)gx, (unsigned)((r + TM_TQ - 1) / TM_TQ));
    const int rr = r < TM_TQ ? r : TM_TQ;
    const int nbr = (rr + 15) / 16;
    set_last_label("k_ttm_mfma<%s, %s, %d, %s>", sizeof(T) == 4 ? "float" : "asi::bf16_t", LAST ? "true" : "false",
                   nbr > 4 ? 4 : nbr, KRON ? "true" : "false");
    switch (nbr) {
        case 1: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 1, KRON>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, kr); break;
        case 2: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 2, KRON>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, kr); break;
        case 3: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 3, KRON>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, kr); break;
        default: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 4, KRON>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, kr); break;
    }
    return hipGetLastError();
}

hipError_t launch_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp,
                      long long ms_i, long long ms_q, int r, float* Y, int beta, hipStream_t st) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0) return hipErrorInvalidValue;
    const bool last = (inner == 1);
    const KronSpec none = {nullptr, 0, 0, 1, 1};
    if (prefer_ksplit(ncols, n, inner)) {
        return xt == F32 ? launch_ksplit_t<float>((const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st)
                         : launch_ksplit_t<bf16_t>((const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st);
    }
    if (xt == F32) {
        return last ? launch_ttm_t<float, true, false>((const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, none, st)
                    : launch_ttm_t<float, false, false>((const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, none, st);
    }
    return last ? launch_ttm_t<bf16_t, true, false>((const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, none, st)
                : launch_ttm_t<bf16_t, false, false>((const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, none, st);
}

// Two adjacent trailing modes at once: X is (cols, n1*n2) row-major, Y is (cols, r1*r2),
//   Y[c, q1*r2 + q2] = sum_{i1,i2} X[c, i1*n2 + i2] * M1(i1,q1) * M2(i2,q2),  Mk(i,q) = Mk[i*msk_i + q*msk_q].
hipError_t launch_ttm_kron(DType xt, const void* X, long long cols, int n1, int n2, const float* M1, long long ms1_i,
                           long long ms1_q, int r1, const float* M2, long long ms2_i, long long ms2_q, int r2, float* Y,
                           int beta, hipStream_t st) {
    if (cols <= 0 || n1 <= 0 || n2 <= 0 || r1 <= 0 || r2 <= 0 || !M1 || !M2) return hipErrorInvalidValue;
    const KronSpec kr = {M2, ms2_i, ms2_q, n2, r2};
    const int n = n1 * n2, r = r1 * r2;
    if (xt == F32) return launch_ttm_t<float, true, true>((const float*)X, cols, n, 1, M1, ms1_i, ms1_q, r, Y, beta, kr, st);
    return launch_ttm_t<bf16_t, true, true>((const bf16_t*)X, cols, n, 1, M1, ms1_i, ms1_q, r, Y, beta, kr, st);
}

}  // namespace asi
