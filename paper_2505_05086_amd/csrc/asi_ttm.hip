// m-mode product (Eq. 4) on fp32 MFMA:  Y[o,q,j] = sum_i X[o,i,j] M(i,q).
//
// Seen as a GEMM the unfolding's columns c = (o,j) are the long dimension, the mode index i
// is K and q is N.  A workgroup owns 64 columns and up to 64 outputs q; K is walked in
// chunks of 32 that are prefetched into registers while the previous chunk is multiplied
// (LDS double use, one barrier pair per chunk).  Wave w multiplies columns 16w..16w+15:
//   A operand (16 columns x 4 i)   = Xs[4ks + lane/16][16w + lane%16]
//   B operand (4 i x 16 q)         = Ms[4ks + lane/16][16nb + lane%16]
// The result tile is transposed through LDS so that stores run along the contiguous index.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TM_TC = 64, TM_KC = 32, TM_TQ = 64, TM_LD = TM_TC + 4;

template <typename T, bool LASTMODE, int NBR>
__global__ __launch_bounds__(256) void k_ttm_mfma(const T* __restrict__ X, long long outer, int n, long long inner,
                                                  const float* __restrict__ Mp, long long ms_i, long long ms_q, int r,
                                                  float* __restrict__ Y, int beta) {
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
            mr[t] = ldg_f32(Mp, (long long)i * ms_i + (long long)q * ms_q, i < n && q < r);
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

template <typename T, bool LAST>
static hipError_t launch_ttm_t(const T* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                               long long ms_q, int r, float* Y, int beta, hipStream_t st) {
    const long long ncols = outer * inner;
    const long long gx = (ncols + TM_TC - 1) / TM_TC;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)gx, (unsigned)((r + TM_TQ - 1) / TM_TQ));
    const int rr = r < TM_TQ ? r : TM_TQ;
    const int nbr = (rr + 15) / 16;
    set_last_label("k_ttm_mfma<%s, %s, %d>", sizeof(T) == 4 ? "float" : "asi::bf16_t", LAST ? "true" : "false", nbr > 4 ? 4 : nbr);
    switch (nbr) {
        case 1: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 1>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta); break;
        case 2: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 2>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta); break;
        case 3: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 3>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta); break;
        default: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 4>), grid, 256, 0, st, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta); break;
    }
    return hipGetLastError();
}

hipError_t launch_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp,
                      long long ms_i, long long ms_q, int r, float* Y, int beta, hipStream_t st) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0) return hipErrorInvalidValue;
    const bool last = (inner == 1);
    if (xt == F32) {
        return last ? launch_ttm_t<float, true>((const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st)
                    : launch_ttm_t<float, false>((const float*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st);
    }
    return last ? launch_ttm_t<bf16_t, true>((const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st)
                : launch_ttm_t<bf16_t, false>((const bf16_t*)X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, st);
}

}  // namespace asi
