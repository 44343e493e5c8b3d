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
//
// A tile is either a run of complete outer slices (contiguous memory; the H and W modes,
// which then share one tile as two "views" of the same planes) or, for a long inner
// extent, n rows of 128 consecutive elements.  All loads of a tile are issued before the
// first is stored (one memory latency per tile); two or more workgroups per CU overlap one
// tile's loads with another's MFMAs.
#include "asi_device.h"
#include "asi_kernels.h"
#include <algorithm>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int SS_TC = 128;                 // fibres (unfolding columns) per tile and view
constexpr int SS_PAD = 4;
constexpr int SS_LDS_FLOATS = 64 * (SS_TC + SS_PAD);   // 33 KB
constexpr int SS_PRE = (SS_LDS_FLOATS + 255) / 256;    // prefetch registers per thread

struct SmallView {
    const float* U;      // (n, r) previous factor
    double* part;        // (nwg, n, r) partial sums of P
    int n, r;
    int sI;              // LDS stride between consecutive mode indices
    int div, mulA, mulB; // LDS offset of fibre c at mode index 0: (c / div) * mulA + (c % div) * mulB
    int cols_per_o;      // fibres one outer slice contributes (whole_o tiles)
};
struct SmallJob {
    const void* X;
    long long outer;     // outer slices (whole_o) / rows of tiles
    long long o_elems;   // elements per outer slice
    long long inner;     // whole_o == 0: row length; tile = n rows x 128 columns
    int whole_o, To;
    long long tiles_per_o;
    long long ntiles;
    int nviews;
    SmallView v[2];
};

template <typename T, int NBM, int NBR, int NV, bool WHOLE_O>
__global__ __launch_bounds__(256, 2) void k_subspace_small(SmallJob jb) {
    __shared__ float smem[SS_LDS_FLOATS];
    __shared__ int colofs[NV][SS_TC];
    __shared__ float Us[NV][NBM * 16][NBR * 16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 4, ll = lane & 15;
    const T* __restrict__ X = static_cast<const T*>(jb.X);

    for (int e = tid; e < NV * NBM * 16 * NBR * 16; e += 256) {
        const int vi = e / (NBM * 16 * NBR * 16), rem = e - vi * (NBM * 16 * NBR * 16);
        const int i = rem / (NBR * 16), q = rem - i * (NBR * 16);
        const SmallView& sv = jb.v[vi];
        Us[vi][i][q] = ldg_f32(sv.U, (long long)i * sv.r + q, i < sv.n && q < sv.r);
    }
    for (int e = tid; e < NV * SS_TC; e += 256) {
        const int vi = e / SS_TC, c = e - vi * SS_TC;
        const SmallView& sv = jb.v[vi];
        colofs[vi][c] = (c / sv.div) * sv.mulA + (c % sv.div) * sv.mulB;
    }

    v4d pacc[NV][NBM][NBR];
#pragma unroll
    for (int vi = 0; vi < NV; ++vi)
#pragma unroll
        for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBR; ++nb) pacc[vi][mb][nb] = (v4d){0.0, 0.0, 0.0, 0.0};

    const int n0 = jb.v[0].n;
    const int rowI = SS_TC + SS_PAD;
    for (long long tile = blockIdx.x; tile < jb.ntiles; tile += gridDim.x) {
        __syncthreads();   // everyone is done with the previous tile (and Us / colofs are written)
        int no_or_vc;
        // the whole tile is requested before any of it is stored: one memory latency per tile
        if (WHOLE_O) {
            const long long o0 = tile * jb.To;
            const int no = (int)((jb.outer - o0 < jb.To) ? jb.outer - o0 : jb.To);
            const int count = no * (int)jb.o_elems;
            const T* src = X + o0 * jb.o_elems;
            T pre[SS_PRE];
#pragma unroll
            for (int u = 0; u < SS_PRE; ++u) {
                const int e = u * 256 + tid;
                pre[u] = src[e < count ? e : 0];          // clamped, not branched: all loads stay in flight
            }
#pragma unroll
            for (int u = 0; u < SS_PRE; ++u) {
                const int e = u * 256 + tid;
                if (e < count) smem[e] = to_f32(pre[u]);
            }
            no_or_vc = no;
        } else {
            const long long o = tile / jb.tiles_per_o;
            const long long j0 = (tile - o * jb.tiles_per_o) * SS_TC;
            const int vc = (int)((jb.inner - j0 < SS_TC) ? jb.inner - j0 : SS_TC);
            const int c = tid & (SS_TC - 1);
            const T* src = X + o * n0 * jb.inner + j0 + c;
            T pre[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int i = (tid >> 7) + 2 * u;
                pre[u] = src[(c < vc && i < n0) ? (long long)i * jb.inner : 0];
            }
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int i = (tid >> 7) + 2 * u;
                if (i < n0) smem[i * rowI + c] = (c < vc) ? to_f32(pre[u]) : 0.f;
            }
            no_or_vc = vc;
        }
        __syncthreads();
#pragma unroll
        for (int vi = 0; vi < NV; ++vi) {
            const SmallView& sv = jb.v[vi];
            const int n = sv.n, sI = sv.sI;
            const int valid_cols = WHOLE_O ? no_or_vc * sv.cols_per_o : no_or_vc;
            for (int cb = wave; cb * 16 < valid_cols; cb += 4) {
                // step A: V for 16 fibres
                v4f vacc[NBR];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) vacc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};
                const int cA = cb * 16 + ll;
                const bool okA = cA < valid_cols;
                const int ofsA = colofs[vi][cA];
#pragma unroll
                for (int ks = 0; ks < NBM * 4; ++ks) {
                    if (4 * ks < n) {
                        const int i = 4 * ks + lg;
                        const float a = ldg_f32(smem, ofsA + i * sI, okA && i < n);
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb)
                            vacc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, Us[vi][i][16 * nb + ll], vacc[nb], 0, 0, 0);
                    }
                }
                // step B: P += X V over the same 16 fibres
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int cB = cb * 16 + 4 * lg + v;
                    const bool okB = cB < valid_cols;
                    const int ofsB = colofs[vi][cB];
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
                                pacc[vi][mb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bv[nb], pacc[vi][mb][nb], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }
    // sum the four waves' accumulators through LDS, wave after wave (fixed order)
    double* red = reinterpret_cast<double*>(smem);   // (NBM*16) x (NBR*16) doubles <= 32 KB
#pragma unroll
    for (int vi = 0; vi < NV; ++vi) {
        __syncthreads();
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
                            *p = (w == 0) ? pacc[vi][mb][nb][v] : *p + pacc[vi][mb][nb][v];
                        }
            }
            __syncthreads();
        }
        const int n = jb.v[vi].n, r = jb.v[vi].r;
        double* out = jb.v[vi].part + (long long)blockIdx.x * n * r;
        for (int e = tid; e < n * r; e += 256) {
            const int i = e / r, q = e - i * r;
            out[e] = red[i * (NBR * 16) + q];
        }
    }
}

// ---- host side ---------------------------------------------------------------------
bool subspace_small_supported(int n, int r) { return n <= 64 && r <= 64 && r <= n; }

static const int SS_MAX_WG = 512;

// tile geometry of one mode seen as (outer, n, inner)
static void single_geometry(long long outer, int n, long long inner, SmallJob* jb) {
    jb->outer = outer; jb->inner = inner; jb->o_elems = (long long)n * inner;
    if (inner < SS_TC && (long long)n * inner <= SS_LDS_FLOATS) {
        long long To = SS_TC / inner;
        const long long cap = SS_LDS_FLOATS / ((long long)n * inner);
        if (To > cap) To = cap;
        jb->whole_o = 1; jb->To = (int)To; jb->tiles_per_o = 0;
        jb->ntiles = (outer + To - 1) / To;
    } else {
        jb->whole_o = 0; jb->To = 1;
        jb->tiles_per_o = (inner + SS_TC - 1) / SS_TC;
        jb->ntiles = outer * jb->tiles_per_o;
    }
}

int subspace_small_nwg(long long outer, int n, long long inner) {
    SmallJob jb;
    single_geometry(outer, n, inner, &jb);
    return (int)(jb.ntiles < SS_MAX_WG ? jb.ntiles : SS_MAX_WG);
}

// The last two modes of a tensor (planes, rows, cols) can share tiles of whole planes.
bool subspace_pair_supported(int rows, int cols, int r_rows, int r_cols) {
    if (!subspace_small_supported(rows, r_rows) || !subspace_small_supported(cols, r_cols)) return false;
    if ((rows + 15) / 16 != (cols + 15) / 16) return false;           // one register shape for both views
    const int nbr = std::max((r_rows + 15) / 16, (r_cols + 15) / 16);
    if (nbr > 2) return false;
    return (long long)rows * cols <= SS_LDS_FLOATS && rows <= SS_TC && cols <= SS_TC;
}
static int pair_To(int rows, int cols) {
    long long To = std::min(SS_TC / rows, SS_TC / cols);
    const long long cap = SS_LDS_FLOATS / ((long long)rows * cols);
    if (To > cap) To = cap;
    return (int)To;
}
int subspace_pair_nwg(long long planes, int rows, int cols) {
    const int To = pair_To(rows, cols);
    const long long ntiles = (planes + To - 1) / To;
    return (int)(ntiles < SS_MAX_WG ? ntiles : SS_MAX_WG);
}

template <typename T, int NV>
static hipError_t launch_small_t(const SmallJob& jb, int nbm, int nbr, int nwg, hipStream_t st) {
#define ASI_SS_CASE(M, R)                                                                       \
    if (nbm == M && nbr == R) {                                                                 \
        set_last_label("k_subspace_small<%s, %d, %d, %d, %s>", sizeof(T) == 4 ? "float" : "asi::bf16_t", M, R, NV,   \
                       jb.whole_o ? "true" : "false");                                                          \
        if (jb.whole_o) hipLaunchKernelGGL((k_subspace_small<T, M, R, NV, true>), dim3(nwg), 256, 0, st, jb);   \
        else if constexpr (NV == 1) hipLaunchKernelGGL((k_subspace_small<T, M, R, NV, false>), dim3(nwg), 256, 0, st, jb); \
        return hipGetLastError();                                                               \
    }
    ASI_SS_CASE(1, 1) ASI_SS_CASE(2, 1) ASI_SS_CASE(2, 2) ASI_SS_CASE(3, 1) ASI_SS_CASE(3, 2)
    ASI_SS_CASE(4, 1) ASI_SS_CASE(4, 2)
    if constexpr (NV == 1) {
        ASI_SS_CASE(3, 3) ASI_SS_CASE(4, 3) ASI_SS_CASE(4, 4)
    }
#undef ASI_SS_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_subspace_small(DType xt, const void* X, long long outer, int n, long long inner, const float* U,
                                 int r, double* part, int nwg, hipStream_t st) {
    if (!subspace_small_supported(n, r) || nwg <= 0) return hipErrorInvalidValue;
    SmallJob jb;
    jb.X = X;
    single_geometry(outer, n, inner, &jb);
    jb.nviews = 1;
    SmallView& v = jb.v[0];
    v.U = U; v.part = part; v.n = n; v.r = r;
    if (jb.whole_o) {
        v.sI = (int)inner; v.div = (int)inner; v.mulA = n * (int)inner; v.mulB = 1; v.cols_per_o = (int)inner;
    } else {
        v.sI = SS_TC + SS_PAD; v.div = SS_TC; v.mulA = 0; v.mulB = 1; v.cols_per_o = 0;
    }
    jb.v[1] = jb.v[0];
    if (nwg > jb.ntiles) return hipErrorInvalidValue;
    const int nbm = (n + 15) / 16, nbr = (r + 15) / 16;
    return xt == F32 ? launch_small_t<float, 1>(jb, nbm, nbr, nwg, st) : launch_small_t<bf16_t, 1>(jb, nbm, nbr, nwg, st);
}

// Modes "rows" and "cols" of X seen as (planes, rows, cols), both from one read of X.
hipError_t launch_subspace_pair(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows,
                                int r_rows, double* part_rows, const float* U_cols, int r_cols, double* part_cols,
                                int nwg, hipStream_t st) {
    if (!subspace_pair_supported(rows, cols, r_rows, r_cols) || nwg <= 0) return hipErrorInvalidValue;
    SmallJob jb;
    jb.X = X; jb.outer = planes; jb.inner = cols; jb.o_elems = (long long)rows * cols;
    jb.whole_o = 1; jb.To = pair_To(rows, cols); jb.tiles_per_o = 0;
    jb.ntiles = (planes + jb.To - 1) / jb.To;
    jb.nviews = 2;
    SmallView& a = jb.v[0];      // fibres run along rows: element (i, c = (plane, col)) at plane*rows*cols + i*cols + col
    a.U = U_rows; a.part = part_rows; a.n = rows; a.r = r_rows;
    a.sI = cols; a.div = cols; a.mulA = rows * cols; a.mulB = 1; a.cols_per_o = cols;
    SmallView& b = jb.v[1];      // fibres run along cols: element (i, c = (plane, row)) at plane*rows*cols + row*cols + i
    b.U = U_cols; b.part = part_cols; b.n = cols; b.r = r_cols;
    b.sI = 1; b.div = rows; b.mulA = rows * cols; b.mulB = cols; b.cols_per_o = rows;
    if (nwg > jb.ntiles) return hipErrorInvalidValue;
    const int nbm = (rows + 15) / 16, nbr = std::max((r_rows + 15) / 16, (r_cols + 15) / 16);
    return xt == F32 ? launch_small_t<float, 2>(jb, nbm, nbr, nwg, st) : launch_small_t<bf16_t, 2>(jb, nbm, nbr, nwg, st);
}

}  // namespace asi
