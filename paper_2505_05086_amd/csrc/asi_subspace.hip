// Fused subspace-iteration step for modes with a short fibre (n <= 64): B, H, W of a
// conv activation, the batch mode of a token tensor.
//
// For such a mode the two products of Alg. 1, V = A_m^T U_prev and P = A_m V, are done
// on the same LDS tile of complete mode-m fibres, so V never exists in memory and the
// activation is read once:   P = sum over fibres x of  x (x^T U_prev).
//   step A (fp32 MFMA 16x16x4):  V[c,q]  = sum_i X[i,c] U[i,q]      16 fibres at a time
//   step B (fp64 MFMA 16x16x4):  P[i,q] += sum_c X[i,c] V[c,q]      accumulators stay in registers
// The accumulator layout of step A (lane l, register v holds fibre 4*(l/16)+v, column l%16)
// is exactly the B-operand layout step B needs if step B walks the 16 fibres in the order
// k-step v -> fibres {v, 4+v, 8+v, 12+v}; the A operand is fetched from LDS in that order.
// P is summed in fp64: the columns of U_prev need not be aligned with singular vectors, so
// P holds components (sigma_r/sigma_1)^2 below its largest ones that fp32 sums would lose.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int SS_TC = 128;                 // fibres (unfolding columns) per tile
constexpr int SS_PAD = 4;
constexpr int SS_LDS_FLOATS = 64 * (SS_TC + SS_PAD);   // 33 KB

struct SmallJob {
    const void* X;
    const float* U;      // (n, r) previous factor
    double* part;        // (nwg, n, r) partial sums of P
    long long outer, inner;
    int n, r;
    int whole_o;         // 1: a tile is `To` complete outer slices (contiguous memory)
    int To;
    long long tiles_per_o;   // whole_o == 0: ceil(inner / SS_TC)
    long long ntiles;
};

template <typename T, int NBM, int NBR>
__global__ __launch_bounds__(256) void k_subspace_small(SmallJob jb) {
    __shared__ float smem[SS_LDS_FLOATS];
    __shared__ int colofs[SS_TC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 4, ll = lane & 15;
    const int n = jb.n, r = jb.r;
    const long long inner = jb.inner;
    const T* __restrict__ X = static_cast<const T*>(jb.X);

    // previous factor in B-operand layout: k-step ks, column block nb -> U[4ks + lg][16nb + ll]
    float ureg[NBM * 4][NBR];
#pragma unroll
    for (int ks = 0; ks < NBM * 4; ++ks)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) {
            const int i = 4 * ks + lg, q = 16 * nb + ll;
            ureg[ks][nb] = (i < n && q < r) ? jb.U[(long long)i * r + q] : 0.f;
        }

    int sI;
    if (jb.whole_o) {
        sI = (int)inner;
        for (int c = tid; c < SS_TC; c += 256) colofs[c] = (int)((c / inner) * n * inner + (c % inner));
    } else {
        sI = SS_TC + SS_PAD;
        for (int c = tid; c < SS_TC; c += 256) colofs[c] = c;
    }

    v4d pacc[NBM][NBR];
#pragma unroll
    for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) pacc[mb][nb] = (v4d){0.0, 0.0, 0.0, 0.0};

    for (long long tile = blockIdx.x; tile < jb.ntiles; tile += gridDim.x) {
        __syncthreads();   // everyone is done with the previous tile (and colofs is written)
        int valid_cols;
        if (jb.whole_o) {
            const long long o0 = tile * jb.To;
            const int no = (int)((jb.outer - o0 < jb.To) ? jb.outer - o0 : jb.To);
            const int count = no * n * (int)inner;
            const long long base = o0 * n * inner;
            for (int e0 = 0; e0 < count; e0 += 256 * 8) {      // 8 loads in flight per thread
                float t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256 + tid;
                    t[u] = (e < count) ? ldf(X, base + e) : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256 + tid;
                    if (e < count) smem[e] = t[u];
                }
            }
            valid_cols = no * (int)inner;
        } else {
            const long long o = tile / jb.tiles_per_o;
            const long long j0 = (tile - o * jb.tiles_per_o) * SS_TC;
            valid_cols = (int)((inner - j0 < SS_TC) ? inner - j0 : SS_TC);
            const long long base = o * n * inner + j0;
            const int c = tid & (SS_TC - 1);
            const bool okc = c < valid_cols;
            for (int i0 = tid / SS_TC; i0 < n; i0 += 16) {      // 2 rows per pass, 8 passes in flight
                float t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + 2 * u;
                    t[u] = (okc && i < n) ? ldf(X, base + (long long)i * inner + c) : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + 2 * u;
                    if (i < n) smem[i * sI + c] = t[u];
                }
            }
        }
        __syncthreads();
        for (int cb = wave; cb * 16 < valid_cols; cb += 4) {
            // step A: V for 16 fibres
            v4f vacc[NBR];
#pragma unroll
            for (int nb = 0; nb < NBR; ++nb) vacc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};
            const int cA = cb * 16 + ll;
            const bool okA = cA < valid_cols;
            const int ofsA = colofs[cA];
#pragma unroll
            for (int ks = 0; ks < NBM * 4; ++ks) {
                if (4 * ks < n) {
                    const int i = 4 * ks + lg;
                    const float a = (okA && i < n) ? smem[ofsA + i * sI] : 0.f;
#pragma unroll
                    for (int nb = 0; nb < NBR; ++nb)
                        vacc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, ureg[ks][nb], vacc[nb], 0, 0, 0);
                }
            }
            // step B: P += X V over the same 16 fibres
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int cB = cb * 16 + 4 * lg + v;
                const bool okB = cB < valid_cols;
                const int ofsB = colofs[cB];
                double bv[NBR];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) bv[nb] = (double)vacc[nb][v];
#pragma unroll
                for (int mb = 0; mb < NBM; ++mb) {
                    if (16 * mb < n) {
                        const int i = 16 * mb + ll;
                        const double a = (okB && i < n) ? (double)smem[ofsB + i * sI] : 0.0;
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb)
                            pacc[mb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bv[nb], pacc[mb][nb], 0, 0, 0);
                    }
                }
            }
        }
    }
    // sum the four waves' accumulators through LDS, wave after wave (fixed order)
    __syncthreads();
    double* red = reinterpret_cast<double*>(smem);   // (NBM*16) x (NBR*16) doubles <= 32 KB
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int i = 16 * mb + lg + 4 * v, q = 16 * nb + ll;   // fp64 MFMA result layout
                        double* p = red + i * (NBR * 16) + q;
                        *p = (w == 0) ? pacc[mb][nb][v] : *p + pacc[mb][nb][v];
                    }
        }
        __syncthreads();
    }
    double* out = jb.part + (long long)blockIdx.x * n * r;
    for (int e = tid; e < n * r; e += 256) {
        const int i = e / r, q = e - i * r;
        out[e] = red[i * (NBR * 16) + q];
    }
}

// ---- host side ---------------------------------------------------------------------
bool subspace_small_supported(int n, int r) { return n <= 64 && r <= 64 && r <= n; }

int subspace_small_nwg(long long outer, int n, long long inner) {
    SmallJob jb;
    jb.outer = outer; jb.inner = inner; jb.n = n;
    long long ntiles;
    if (inner < SS_TC && (long long)n * inner <= SS_LDS_FLOATS) {
        long long To = SS_TC / inner;
        const long long cap = SS_LDS_FLOATS / ((long long)n * inner);
        if (To > cap) To = cap;
        ntiles = (outer + To - 1) / To;
    } else {
        ntiles = outer * ((inner + SS_TC - 1) / SS_TC);
    }
    return (int)(ntiles < 256 ? ntiles : 256);
}

template <typename T>
static hipError_t launch_small_t(const SmallJob& jb, int nwg, hipStream_t st) {
    const int nbm = (jb.n + 15) / 16, nbr = (jb.r + 15) / 16;
#define ASI_SS_CASE(M, R)                                                                       \
    if (nbm == M && nbr == R) {                                                                 \
        hipLaunchKernelGGL((k_subspace_small<T, M, R>), dim3(nwg), 256, 0, st, jb);             \
        return hipGetLastError();                                                               \
    }
    ASI_SS_CASE(1, 1) ASI_SS_CASE(2, 1) ASI_SS_CASE(2, 2) ASI_SS_CASE(3, 1) ASI_SS_CASE(3, 2) ASI_SS_CASE(3, 3)
    ASI_SS_CASE(4, 1) ASI_SS_CASE(4, 2) ASI_SS_CASE(4, 3) ASI_SS_CASE(4, 4)
#undef ASI_SS_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_subspace_small(DType xt, const void* X, long long outer, int n, long long inner, const float* U,
                                 int r, double* part, int nwg, hipStream_t st) {
    if (!subspace_small_supported(n, r) || nwg <= 0) return hipErrorInvalidValue;
    SmallJob jb;
    jb.X = X; jb.U = U; jb.part = part; jb.outer = outer; jb.inner = inner; jb.n = n; jb.r = r;
    if (inner < SS_TC && (long long)n * inner <= SS_LDS_FLOATS) {
        jb.whole_o = 1;
        long long To = SS_TC / inner;
        const long long cap = SS_LDS_FLOATS / ((long long)n * inner);
        if (To > cap) To = cap;
        jb.To = (int)To;
        jb.tiles_per_o = 0;
        jb.ntiles = (outer + To - 1) / To;
    } else {
        jb.whole_o = 0;
        jb.To = 1;
        jb.tiles_per_o = (inner + SS_TC - 1) / SS_TC;
        jb.ntiles = outer * jb.tiles_per_o;
    }
    if (nwg > jb.ntiles) return hipErrorInvalidValue;
    return xt == F32 ? launch_small_t<float>(jb, nwg, st) : launch_small_t<bf16_t>(jb, nwg, st);
}

}  // namespace asi
