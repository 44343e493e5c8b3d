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
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int SS_TC = 128;                 // fibres (unfolding columns) per tile and view
constexpr int SS_PAD = 4;
constexpr int SS_LDS_FLOATS = 64 * (SS_TC + SS_PAD);   // 33 KB
constexpr int SS_PRE = (SS_LDS_FLOATS + 255) / 256;    // prefetch registers per thread
static const int SS_MAX_WG = 1024;

struct SmallView {
    const float* U;      // (n, r) previous factor
    double* part;        // (nwg, n, r) partial sums of P
    int n, r;
    int sI;              // LDS stride between consecutive mode indices
    int div, mulA, mulB; // LDS offset of fibre c at mode index 0: (c / div) * mulA + (c % div) * mulB
    float inv_div;       // 1 / div: c stays below 2^14, so the rounded float quotient is exact
    int cols_per_o;      // fibres one outer slice contributes (whole_o tiles)
};
struct SmallJob {
    const void* X;
    long long outer;     // outer slices (whole_o) / rows of tiles
    long long o_elems;   // elements per outer slice
    long long inner;     // whole_o == 0: row length; tile = To groups of (n rows x 128 columns), stacked in LDS
    int whole_o, To;     // To: outer slices per tile (whole_o), else column groups per tile
    long long tiles_per_o;
    long long ntiles;
    int nviews;
    int nwg;             // workgroups of this job; each walks tiles nwg apart
    int32_t* zero;       // nullable: `nzero` int32 to clear (arrival counters of the orth launches that follow)
    int nzero;
    SmallView v[2];
};


template <typename T, int NBM, int NBR, int NV, bool WHOLE_O, bool STACK = false>   // STACK: several column groups per tile
__global__ __launch_bounds__(256, 2) void k_subspace_small(Batch<SmallJob> bt) {
    int lb;
    const SmallJob& jb = bt.job[locate(bt, &lb)];
    __shared__ float smem[SS_LDS_FLOATS];
    __shared__ float Us[NV][NBM * 16][NBR * 16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 4, ll = lane & 15;
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;

    // the factors: all loads first (addresses valid for every lane), then the stores; written as a loop of
    // load and store, every element paid its own round trip to memory
    {
        constexpr int PV = NBM * 16 * NBR * 16, NU = PV / 256;
        static_assert(NU * 256 == PV, "whole passes");
        float ut[NV][NU];
        bool uok[NV][NU];
#pragma unroll
        for (int vi = 0; vi < NV; ++vi) {
            const float* Uv = jb.v[vi].U;
            const int nv = jb.v[vi].n, rv = jb.v[vi].r;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int rem = tid + 256 * u, i = rem / (NBR * 16), q = rem - i * (NBR * 16);
                uok[vi][u] = i < nv && q < rv;
                ut[vi][u] = Uv[uok[vi][u] ? (long long)i * rv + q : 0LL];
            }
        }
#pragma unroll
        for (int vi = 0; vi < NV; ++vi)
#pragma unroll
            for (int u = 0; u < NU; ++u) (&Us[vi][0][0])[tid + 256 * u] = uok[vi][u] ? ut[vi][u] : 0.f;
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
    // Tiles of a long inner extent (!WHOLE_O): a short mode leaves most of the 64 LDS rows empty, so a tile
    // takes To groups of 128 columns and stacks them: LDS row g * n + i holds mode index i of columns
    // 128 g .. 128 g + 127.  The loads of a tile are issued (clamped, not branched, so that all stay in
    // flight) while the previous tile is multiplied and stored to LDS when that is done.
    T pre[WHOLE_O ? 1 : 32];
    const float inv_n0 = 1.0f / (float)n0;
    auto tile_origin = [&](long long tile, const T** src, int* vc) {
        const int tcols = SS_TC * jb.To;
        const long long o = tile / jb.tiles_per_o;
        const long long j0 = (tile - o * jb.tiles_per_o) * tcols;
        *vc = (int)((jb.inner - j0 < tcols) ? jb.inner - j0 : tcols);
        *src = X + o * n0 * jb.inner + j0;
    };
    auto issue = [&](long long tile) {
        const T* src;
        int vc;
        tile_origin(tile, &src, &vc);
        const int c = tid & (SS_TC - 1);
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const int row = (tid >> 7) + 2 * u;
            if constexpr (!STACK) {      // one group: LDS row = mode index
                pre[u] = src[(c < vc && row < n0) ? (long long)row * jb.inner + c : 0];
            } else {
                const int g = (int)(((float)row + 0.5f) * inv_n0), i = row - g * n0, col = g * SS_TC + c;
                pre[u] = src[(g < jb.To && col < vc) ? (long long)i * jb.inner + col : 0];
            }
        }
    };
    auto commit = [&](long long tile) -> int {
        const T* src;
        int vc;
        tile_origin(tile, &src, &vc);
        const int c = tid & (SS_TC - 1);
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const int row = (tid >> 7) + 2 * u;
            if constexpr (!STACK) {
                if (row < n0) smem[row * rowI + c] = (c < vc) ? to_f32(pre[u]) : 0.f;
            } else {
                const int g = (int)(((float)row + 0.5f) * inv_n0), col = g * SS_TC + c;
                if (g < jb.To) smem[row * rowI + c] = (col < vc) ? to_f32(pre[u]) : 0.f;
            }
        }
        return vc;
    };
    if constexpr (!WHOLE_O) {
        if (lb < jb.ntiles) issue(lb);
    }
    for (long long tile = lb; tile < jb.ntiles; tile += jb.nwg) {
        __syncthreads();   // everyone is done with the previous tile (and Us is written)
        int no_or_vc;
        if constexpr (WHOLE_O) {
            // the whole tile is requested before any of it is stored: one memory latency per tile
            const long long o0 = tile * jb.To;
            const int no = (int)((jb.outer - o0 < jb.To) ? jb.outer - o0 : jb.To);
            const int count = no * (int)jb.o_elems;
            const T* src = X + o0 * jb.o_elems;
            T prw[SS_PRE];
#pragma unroll
            for (int u = 0; u < SS_PRE; ++u) {
                const int e = u * 256 + tid;
                prw[u] = src[e < count ? e : 0];          // clamped, not branched: all loads stay in flight
            }
#pragma unroll
            for (int u = 0; u < SS_PRE; ++u) {
                const int e = u * 256 + tid;
                if (e < count) smem[e] = to_f32(prw[u]);
            }
            no_or_vc = no;
        } else {
            no_or_vc = commit(tile);
        }
        __syncthreads();
        if constexpr (!WHOLE_O) {
            if (tile + jb.nwg < jb.ntiles) issue(tile + jb.nwg);
        }
#pragma unroll
        for (int vi = 0; vi < NV; ++vi) {
            const SmallView& sv = jb.v[vi];
            const int n = sv.n, sI = sv.sI;
            const int valid_cols = WHOLE_O ? no_or_vc * sv.cols_per_o : no_or_vc;
            // The loop body is free of branches and every group of LDS reads is issued before the
            // products that consume it, so that a fibre block pays LDS latency twice, not once per product.
            // B operands of step A do not depend on the fibre block (rows i >= n of Us are zero)
            float ub[NBM * 4][NBR];
#pragma unroll
            for (int ks = 0; ks < NBM * 4; ++ks)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) ub[ks][nb] = Us[vi][4 * ks + lg][16 * nb + ll];
            for (int cb = wave; cb * 16 < valid_cols; cb += 4) {
                // step A: V for 16 fibres
                const int cA = cb * 16 + ll;
                const bool okA = cA < valid_cols;
                const int qA = (int)(((float)cA + 0.5f) * sv.inv_div);
                const int ofsA = qA * sv.mulA + (cA - qA * sv.div) * sv.mulB;
                float av[NBM * 4];
#pragma unroll
                for (int ks = 0; ks < NBM * 4; ++ks) {
                    const int i = 4 * ks + lg;
                    const bool ok = okA && i < n;
                    const float x = smem[ok ? ofsA + i * sI : 0];
                    av[ks] = ok ? x : 0.f;
                }
                v4f vacc[NBR];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) vacc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NBM * 4; ++ks)
#pragma unroll
                    for (int nb = 0; nb < NBR; ++nb)
                        vacc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ks], ub[ks][nb], vacc[nb], 0, 0, 0);
                // step B: P += X V over the same 16 fibres
                double a2[4][NBM];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int cB = cb * 16 + 4 * lg + v;
                    const bool okB = cB < valid_cols;
                    const int qB = (int)(((float)cB + 0.5f) * sv.inv_div);
                    const int ofsB = qB * sv.mulA + (cB - qB * sv.div) * sv.mulB;
#pragma unroll
                    for (int mb = 0; mb < NBM; ++mb) {
                        const int i = 16 * mb + ll;
                        const bool ok = okB && i < n;
                        const float x = smem[ok ? ofsB + i * sI : 0];
                        a2[v][mb] = ok ? (double)x : 0.0;
                    }
                }
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb)
                            pacc[vi][mb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a2[v][mb], (double)vacc[nb][v],
                                                                                    pacc[vi][mb][nb], 0, 0, 0);
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
        double* out = jb.v[vi].part + (long long)lb * n * r;
        for (int e = tid; e < n * r; e += 256) {
            const int i = e / r, q = e - i * r;
            out[e] = red[i * (NBR * 16) + q];
        }
    }
}

// ---- host side ---------------------------------------------------------------------
bool subspace_small_supported(int n, int r) { return n <= 64 && r <= 64 && r <= n; }

// Outer slices per tile when a tile is a run of whole slices: as many as the LDS buffer holds, but
// no fewer than ~SS_MAX_WG tiles in all: the MFMA chains of a tile are latency bound, and only
// several resident workgroups per CU hide that.
static long long whole_To(long long outer, long long o_elems) {
    long long To = SS_LDS_FLOATS / o_elems;
    const long long spread = (outer + SS_MAX_WG - 1) / SS_MAX_WG;
    if (To > spread) To = spread;
    return To < 1 ? 1 : To;
}

// tile geometry of one mode seen as (outer, n, inner)
static void single_geometry(long long outer, int n, long long inner, SmallJob* jb) {
    jb->outer = outer; jb->inner = inner; jb->o_elems = (long long)n * inner;
    if (inner < SS_TC && (long long)n * inner <= SS_LDS_FLOATS) {
        long long To = whole_To(outer, (long long)n * inner);
        jb->whole_o = 1; jb->To = (int)To; jb->tiles_per_o = 0;
        jb->ntiles = (outer + To - 1) / To;
    } else {
        // groups of 128 columns per tile: as many as the 64 LDS rows hold, while ~SS_MAX_WG tiles remain
        int G = 64 / n;
        while (G > 1 && outer * ((inner + (long long)SS_TC * G - 1) / ((long long)SS_TC * G)) < SS_MAX_WG) --G;
        if (G < 1) G = 1;
        jb->whole_o = 0; jb->To = G;
        jb->tiles_per_o = (inner + (long long)SS_TC * G - 1) / ((long long)SS_TC * G);
        jb->ntiles = outer * jb->tiles_per_o;
    }
}

int subspace_small_nwg(long long outer, int n, long long inner) {
    SmallJob jb;
    single_geometry(outer, n, inner, &jb);
    // tiles of a long inner extent are prefetched behind the previous tile's products: two resident
    // workgroups per CU, each walking several tiles, instead of further rounds of workgroups
    const int cap = jb.whole_o ? SS_MAX_WG : SS_MAX_WG / 2;
    return (int)(jb.ntiles < cap ? jb.ntiles : cap);
}

// The last two modes of a tensor (planes, rows, cols) can share tiles of whole planes.
bool subspace_pair_supported(int rows, int cols, int r_rows, int r_cols) {
    if (!subspace_small_supported(rows, r_rows) || !subspace_small_supported(cols, r_cols)) return false;
    if ((rows + 15) / 16 != (cols + 15) / 16) return false;           // one register shape for both views
    const int nbr = std::max((r_rows + 15) / 16, (r_cols + 15) / 16);
    if (nbr > 2) return false;
    return (long long)rows * cols <= SS_LDS_FLOATS;
}
static int pair_To(long long planes, int rows, int cols) { return (int)whole_To(planes, (long long)rows * cols); }
int subspace_pair_nwg(long long planes, int rows, int cols) {
    const int To = pair_To(planes, rows, cols);
    const long long ntiles = (planes + To - 1) / To;
    return (int)(ntiles < SS_MAX_WG ? ntiles : SS_MAX_WG);
}

// key: [0] bf16, [1] two views, [2] whole_o, [3] stacked column groups (n <= 32), [4..6] NBM, [8..10] NBR
static bool small_key_ok(int nbm, int nbr, int nv) {
    if (nbm < 1 || nbm > 4 || nbr < 1 || nbr > nbm) return false;
    return nv == 1 || nbr <= 2;
}
static bool finish_small(DType xt, SmallJob& jb, int nbm, int nbr, int nwg, Item* out) {
    if (!small_key_ok(nbm, nbr, jb.nviews) || nwg <= 0 || nwg > jb.ntiles) return false;
    if (jb.nviews == 2 && !jb.whole_o) return false;
    jb.nwg = nwg;
    *out = Item();
    out->kind = IT_SMALL;
    const bool stack = !jb.whole_o && jb.To > 1;
    out->key = (xt == BF16 ? 1u : 0u) | (jb.nviews == 2 ? 2u : 0u) | (jb.whole_o ? 4u : 0u) | (stack ? 8u : 0u) |
               ((unsigned)nbm << 4) | ((unsigned)nbr << 8);
    out->nblocks = nwg;
    std::snprintf(out->label, sizeof(out->label), "k_subspace_small<%s, %d, %d, %d, %s, %s>", xt == F32 ? "float" : "asi::bf16_t",
                  nbm, nbr, jb.nviews, jb.whole_o ? "true" : "false", stack ? "true" : "false");
    static_assert(sizeof(SmallJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

bool make_subspace_small(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r,
                         double* part, int nwg, int32_t* zero, int nzero, Item* out) {
    if (!subspace_small_supported(n, r) || !X || !U || !part || nzero < 0 || nzero > 256) return false;
    SmallJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.zero = zero; jb.nzero = zero ? nzero : 0;
    single_geometry(outer, n, inner, &jb);
    jb.nviews = 1;
    SmallView& v = jb.v[0];
    v.U = U; v.part = part; v.n = n; v.r = r;
    if (jb.whole_o) {
        v.sI = (int)inner; v.div = (int)inner; v.mulA = n * (int)inner; v.mulB = 1; v.cols_per_o = (int)inner;
    } else {
        v.sI = SS_TC + SS_PAD; v.div = SS_TC; v.mulA = n * (SS_TC + SS_PAD); v.mulB = 1; v.cols_per_o = 0;   // group g starts n rows further down
    }
    v.inv_div = 1.0f / (float)v.div;
    jb.v[1] = jb.v[0];
    return finish_small(xt, jb, (n + 15) / 16, (r + 15) / 16, nwg, out);
}

// Modes "rows" and "cols" of X seen as (planes, rows, cols), both from one read of X.
bool make_subspace_pair(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                        double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, Item* out) {
    if (!subspace_pair_supported(rows, cols, r_rows, r_cols) || !X || !U_rows || !U_cols || !part_rows || !part_cols)
        return false;
    SmallJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.outer = planes; jb.inner = cols; jb.o_elems = (long long)rows * cols;
    jb.whole_o = 1; jb.To = pair_To(planes, rows, cols); jb.tiles_per_o = 0;
    jb.ntiles = (planes + jb.To - 1) / jb.To;
    jb.nviews = 2;
    SmallView& a = jb.v[0];      // fibres run along rows: element (i, c = (plane, col)) at plane*rows*cols + i*cols + col
    a.U = U_rows; a.part = part_rows; a.n = rows; a.r = r_rows;
    a.sI = cols; a.div = cols; a.mulA = rows * cols; a.mulB = 1; a.cols_per_o = cols;
    a.inv_div = 1.0f / (float)cols;
    SmallView& b = jb.v[1];      // fibres run along cols: element (i, c = (plane, row)) at plane*rows*cols + row*cols + i
    b.U = U_cols; b.part = part_cols; b.n = cols; b.r = r_cols;
    b.sI = 1; b.div = rows; b.mulA = rows * cols; b.mulB = cols; b.cols_per_o = rows;
    b.inv_div = 1.0f / (float)rows;
    return finish_small(xt, jb, (rows + 15) / 16, std::max((r_rows + 15) / 16, (r_cols + 15) / 16), nwg, out);
}

// ---- the last two modes when both are tiny (rows, cols <= 8, ranks <= 8) ------------------------------
// For a 7x7 plane and rank 5 the 16x16 MFMA blocks above are 14 % full, so here the vector ALU does
// the work with no padding beyond 8: thread (plane, view) keeps the plane's contribution
//   P += X (X^T U)   (view 0, fibres along rows)     or     P += X^T (X U)   (view 1, fibres along cols)
// for its planes in fp64 registers (V = fibre^T U in fp32, the products of P exact in fp64).  Sums over
// the planes of a workgroup are taken in a fixed order: lanes of a wave by xor shuffles, then waves.
constexpr int TY_PL = 128;           // planes per tile: 256 threads = 128 planes x 2 views

// value of the lane a data-parallel move selects (every lane of a row active)
template <int CTRL>
__device__ __forceinline__ double dpp_move(double x) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}
typedef float v4f_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4f_t tiny_widen(const v4f_t& p) { return p; }
__device__ __forceinline__ v4f_t tiny_widen(const uint2& p) {
    v4f_t o;
    o[0] = __uint_as_float(p.x << 16); o[1] = __uint_as_float(p.x & 0xffff0000u);
    o[2] = __uint_as_float(p.y << 16); o[3] = __uint_as_float(p.y & 0xffff0000u);
    return o;
}
struct TinyJob {
    const void* X;
    long long planes, ntiles;
    const float* U[2];    // (rows, r[0]) and (cols, r[1])
    double* part[2];      // (nwg, rows, r[0]) and (nwg, cols, r[1])
    int rows, cols, r[2];
    int nwg;
};

template <typename T, bool VEC> struct TinyPiece { typedef T type; };
template <> struct TinyPiece<float, true> { typedef v4f_t type; };
template <> struct TinyPiece<bf16_t, true> { typedef uint2 type; };
template <typename T, bool VEC, typename PC>
__device__ __forceinline__ void tiny_store(float* dst, const PC& v) {
    if constexpr (VEC) *reinterpret_cast<v4f_t*>(dst) = tiny_widen(v);
    else *dst = to_f32(v);
}

template <typename T, int RP, bool VEC>
__global__ __launch_bounds__(256) void k_subspace_tiny(Batch<TinyJob> bt) {
    __shared__ __align__(16) float tile[TY_PL * 64];
    __shared__ float Us[2][8][RP];
    __shared__ double red[4][2][8 * RP];
    int lb;
    const TinyJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const int tid = threadIdx.x, view = tid & 1, pl = tid >> 1, wave = tid >> 6, lane = tid & 63;
    const int rows = jb.rows, cols = jb.cols, pe = rows * cols;
    const int n_v = view ? cols : rows;          // length of this view's fibres (the mode size)
    const int m_v = view ? rows : cols;          // fibres per plane
    const int sI = view ? 1 : cols, sC = view ? cols : 1;    // element (i, c) of the plane at i*sI + c*sC
    // A tile (TY_PL consecutive planes, one contiguous run of X) travels in pieces of W elements.  VEC (X is
    // aligned, so every tile of 128 planes is): W = 4, one 16-byte load (8 bytes for bf16) and one 16-byte LDS
    // store; the up to three elements after the last whole piece of a ragged last tile go one by one.
    // The first tile is requested before the factors are staged, and a workgroup with a further tile requests it
    // before it multiplies: a tile's round trip to memory costs as much as its arithmetic.
    typedef typename TinyPiece<T, VEC>::type Piece;
    constexpr int W = VEC ? 4 : 1;
    constexpr int NPC = TY_PL * 64 / W / 256;                // pieces per thread
    Piece pre[NPC];
    T pre_tail;
    auto fetch = [&](long long t) __attribute__((always_inline)) {
        const long long p0 = t * TY_PL;
        const int np = (int)((jb.planes - p0 < TY_PL) ? jb.planes - p0 : TY_PL);
        const int count = np * pe;
        const T* src = X + p0 * pe;
#pragma unroll
        for (int k = 0; k < NPC; ++k) {
            const int e = W * (k * 256 + tid);
            pre[k] = *reinterpret_cast<const Piece*>(src + (e + W - 1 < count ? e : 0));      // clamped, not branched: all loads stay in flight
        }
        const int et = (count & ~(W - 1)) + (tid & 3);
        pre_tail = src[et < count ? et : 0];
    };
    if (lb < jb.ntiles) fetch(lb);
    {
        float ut = 0.f;                                      // 2 * 8 * RP <= 128 elements: one per thread
        const int e = tid, vi = e / (8 * RP), rem = e - vi * (8 * RP), i = rem / RP, q = rem - i * RP;
        const bool in = e < 2 * 8 * RP;
        const int nn = vi ? cols : rows, rr = in ? jb.r[vi] : 1;
        const bool ok = in && i < nn && q < rr;
        ut = jb.U[in ? vi : 0][ok ? (long long)i * rr + q : 0];
        if (in) Us[vi][i][q] = ok ? ut : 0.f;
    }
    __syncthreads();
    float u[8][RP];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < RP; ++q) u[i][q] = Us[view][i][q];
    double P[8][RP];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < RP; ++q) P[i][q] = 0.0;

    for (long long t = lb; t < jb.ntiles; t += jb.nwg) {
        const long long p0 = t * TY_PL;
        const int np = (int)((jb.planes - p0 < TY_PL) ? jb.planes - p0 : TY_PL);
        const int count = np * pe;
        __syncthreads();                          // previous tile consumed
#pragma unroll
        for (int k = 0; k < NPC; ++k) {
            const int e = W * (k * 256 + tid);
            if (e + W - 1 < count) tiny_store<T, VEC>(tile + e, pre[k]);
        }
        {
            const int et = (count & ~(W - 1)) + (tid & 3);
            if (tid < 4 && et < count) tile[et] = to_f32(pre_tail);
        }
        if (t + jb.nwg < jb.ntiles) fetch(t + jb.nwg);       // on its way during this tile's arithmetic
        __syncthreads();
        if (pl < np) {
            const float* xp = tile + pl * pe;
#pragma unroll 1
            for (int c = 0; c < m_v; ++c) {                  // one fibre at a time keeps the register count down
                float x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = ldg_f32(xp, i * sI + c * sC, i < n_v);
                float v[RP];
#pragma unroll
                for (int q = 0; q < RP; ++q) v[q] = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int q = 0; q < RP; ++q) v[q] = fmaf(x[i], u[i][q], v[q]);
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int q = 0; q < RP; ++q) P[i][q] = fma((double)x[i], (double)v[q], P[i][q]);
            }
        }
    }
    // Sum over the lanes of the same view (same lane parity).  Inside a row of 16 lanes by data-parallel
    // moves: partner lane^2, then rotations by 4 and 8; across the four rows by two xor shuffles.  One
    // step for all accumulators at a time, so that their moves are in flight together.
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < RP; ++q) P[i][q] += dpp_move<0x4E>(P[i][q]);        // quad_perm [2,3,0,1]
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < RP; ++q) P[i][q] += dpp_move<0x124>(P[i][q]);       // row_ror:4
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < RP; ++q) P[i][q] += dpp_move<0x128>(P[i][q]);       // row_ror:8
#pragma unroll
    for (int m = 16; m <= 32; m <<= 1)
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < RP; ++q) P[i][q] += __shfl_xor(P[i][q], m);
    if (lane < 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < RP; ++q) red[wave][lane][i * RP + q] = P[i][q];
    }
    __syncthreads();
    for (int e = tid; e < 2 * 8 * RP; e += 256) {
        const int vi = e / (8 * RP), rem = e - vi * (8 * RP), i = rem / RP, q = rem - i * RP;
        const int nn = vi ? cols : rows, rr = jb.r[vi];
        if (i < nn && q < rr) {
            const double s = (red[0][vi][rem] + red[1][vi][rem]) + (red[2][vi][rem] + red[3][vi][rem]);
            jb.part[vi][((long long)lb * nn + i) * rr + q] = s;
        }
    }
}

bool subspace_tiny_supported(int rows, int cols, int r_rows, int r_cols) {
    return rows <= 8 && cols <= 8 && r_rows <= 8 && r_cols <= 8 && r_rows <= rows && r_cols <= cols;
}
// Two workgroups are resident per CU (a thread holds its P in ~100 fp64 registers), and a workgroup's fixed costs
// (factor staging, the first tile's round trip, the sum over its lanes and waves) are several times a tile's
// arithmetic: no more workgroups than are resident, every one walking the same number of tiles, the next
// tile on its way while the current one is multiplied.
constexpr int TY_MAX_WG = 512;
int subspace_tiny_nwg(long long planes) {
    const long long ntiles = (planes + TY_PL - 1) / TY_PL;
    const long long per = (ntiles + TY_MAX_WG - 1) / TY_MAX_WG;
    return (int)((ntiles + per - 1) / per);
}
bool make_subspace_tiny(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                        double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, Item* out) {
    if (!subspace_tiny_supported(rows, cols, r_rows, r_cols) || !X || !U_rows || !U_cols || !part_rows || !part_cols)
        return false;
    TinyJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.planes = planes; jb.ntiles = (planes + TY_PL - 1) / TY_PL;
    jb.U[0] = U_rows; jb.U[1] = U_cols; jb.part[0] = part_rows; jb.part[1] = part_cols;
    jb.rows = rows; jb.cols = cols; jb.r[0] = r_rows; jb.r[1] = r_cols; jb.nwg = nwg;
    if (nwg <= 0 || nwg > jb.ntiles) return false;
    const int rmax = std::max(r_rows, r_cols);
    const int rp = rmax <= 4 ? 4 : (rmax <= 6 ? 6 : 8);
    *out = Item();
    out->kind = IT_TINY;
    const bool vec = reinterpret_cast<uintptr_t>(X) % (xt == F32 ? 16 : 8) == 0;
    out->key = (xt == BF16 ? 1u : 0u) | (vec ? 2u : 0u) | ((unsigned)rp << 4);
    out->nblocks = nwg;
    std::snprintf(out->label, sizeof(out->label), "k_subspace_tiny<%s, %d, %s>", xt == F32 ? "float" : "asi::bf16_t", rp,
                  vec ? "true" : "false");
    static_assert(sizeof(TinyJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}
hipError_t launch_tiny_items(const Item* const* items, int n, hipStream_t st) {
    Batch<TinyJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int rp = (int)(key >> 4);
    const bool bf = key & 1u, vec = key & 2u;
#define ASI_TINY_CASE(R)                                                                                  \
    if (rp == R) {                                                                                        \
        if (bf) {                                                                                         \
            if (vec) hipLaunchKernelGGL((k_subspace_tiny<bf16_t, R, true>), grid, 256, 0, st, b);         \
            else hipLaunchKernelGGL((k_subspace_tiny<bf16_t, R, false>), grid, 256, 0, st, b);            \
        } else {                                                                                          \
            if (vec) hipLaunchKernelGGL((k_subspace_tiny<float, R, true>), grid, 256, 0, st, b);          \
            else hipLaunchKernelGGL((k_subspace_tiny<float, R, false>), grid, 256, 0, st, b);             \
        }                                                                                                 \
        return hipGetLastError();                                                                         \
    }
    ASI_TINY_CASE(4) ASI_TINY_CASE(6) ASI_TINY_CASE(8)
#undef ASI_TINY_CASE
    return hipErrorInvalidValue;
}

template <typename T, int NV>
static bool launch_small_t(const Batch<SmallJob>& b, dim3 grid, int nbm, int nbr, bool whole_o, bool stack, hipStream_t st) {
    if constexpr (NV == 1) {
        if (stack) {
            if (whole_o || nbm > 2) return false;
            if (nbm == 1 && nbr == 1) hipLaunchKernelGGL((k_subspace_small<T, 1, 1, 1, false, true>), grid, 256, 0, st, b);
            else if (nbm == 2 && nbr == 1) hipLaunchKernelGGL((k_subspace_small<T, 2, 1, 1, false, true>), grid, 256, 0, st, b);
            else if (nbm == 2 && nbr == 2) hipLaunchKernelGGL((k_subspace_small<T, 2, 2, 1, false, true>), grid, 256, 0, st, b);
            else return false;
            return true;
        }
    } else if (stack) {
        return false;
    }
#define ASI_SS_CASE(M, R)                                                                                \
    if (nbm == M && nbr == R) {                                                                          \
        if (whole_o) hipLaunchKernelGGL((k_subspace_small<T, M, R, NV, true>), grid, 256, 0, st, b);     \
        else if constexpr (NV == 1) hipLaunchKernelGGL((k_subspace_small<T, M, R, NV, false>), grid, 256, 0, st, b); \
        return true;                                                                                     \
    }
    ASI_SS_CASE(1, 1) ASI_SS_CASE(2, 1) ASI_SS_CASE(2, 2) ASI_SS_CASE(3, 1) ASI_SS_CASE(3, 2)
    ASI_SS_CASE(4, 1) ASI_SS_CASE(4, 2)
    if constexpr (NV == 1) {
        ASI_SS_CASE(3, 3) ASI_SS_CASE(4, 3) ASI_SS_CASE(4, 4)
    }
#undef ASI_SS_CASE
    return false;
}

hipError_t launch_small_items(const Item* const* items, int n, hipStream_t st) {
    Batch<SmallJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const bool bf16 = key & 1u, two = key & 2u, whole_o = key & 4u, stack = key & 8u;
    const int nbm = (int)((key >> 4) & 7u), nbr = (int)((key >> 8) & 7u);
    bool ok;
    if (!bf16) ok = two ? launch_small_t<float, 2>(b, grid, nbm, nbr, whole_o, stack, st) : launch_small_t<float, 1>(b, grid, nbm, nbr, whole_o, stack, st);
    else ok = two ? launch_small_t<bf16_t, 2>(b, grid, nbm, nbr, whole_o, stack, st) : launch_small_t<bf16_t, 1>(b, grid, nbm, nbr, whole_o, stack, st);
    return ok ? hipGetLastError() : hipErrorInvalidValue;
}

}  // namespace asi
