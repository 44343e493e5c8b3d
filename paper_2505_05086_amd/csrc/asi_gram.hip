// Subspace-iteration step of a short mode with a long inner extent (the batch mode of an activation:
// n <= 64 indices, millions of unfolding columns) through the mode's Gram matrix.
//
// Alg. 1 asks for P = A_m V with V = A_m^T U_prev, i.e. P = (A_m A_m^T) U_prev.  For a short mode the
// n x n matrix G = A_m A_m^T is tiny, so the step is one pass over the activation that accumulates G
// and a product G U_prev at the end; V (columns x r) is never formed, not even in registers:
//     G[i][i'] = sum_c X[i][c] X[i'][c]      fp64 MFMA 16x16x4, both operands from ONE LDS read
//     P        = G U_prev                    n * n * r multiply-adds per workgroup, fp64
// Products of fp32 (or bf16) values are exact in fp64 and the sums are carried in fp64, so P is at least
// as accurate as the two-product form (which rounds V to fp32 in between).
//
// A lane reads 16 bytes of one LDS row: columns c0 + 4 (lane / 16) .. + 3 of row lane % 16.  Element s of
// those four is the lane's operand of K step s, for the row block as A operand and as B operand alike
// (A[i][k] and B[k][j] of the instruction both come from lane (k, i) resp. (k, j)), so which column a K
// slot stands for does not matter.  Per 16 columns and row block a wave issues one LDS read and four
// conversions for 4 * (blocks on or above the diagonal) MFMAs: the matrix pipe is the only busy unit.
//
// A mode of at most 8 indices would leave half of the 16 x 16 result unused.  Its tile holds S = 2 (4 for
// n <= 4) ranges of columns stacked in the 16 rows (row s n + i = index i of range s); the diagonal
// n x n sub-blocks of the result are the Gram matrices of the ranges (the rest mixes ranges and is
// dropped), so each instruction covers S times the columns.
#include "asi_device.h"
#include "asi_kernels.h"

#include <cstdio>
#include <cstring>

namespace asi {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int SG_NT = 256;
constexpr int SG_MAX_WG = 512;             // two resident workgroups per CU, each walking several tiles
template <int NBM>
constexpr int sg_tc() { return NBM == 1 ? 512 : (NBM == 2 ? 256 : 128); }      // columns per tile: ~33 KB of LDS

struct GramJob {
    const void* X;       // (outer, n, inner)
    const float* U;      // (n, r) previous factor
    double* part;        // (nwg, n, r) partial sums of P
    long long outer, inner;
    long long tiles_per_o, ntiles;
    int n, r, nwg;
    int S;               // n <= 8: S = 2 (n <= 4: 4) column ranges of a tile are stacked in the 16 LDS rows
    int32_t* zero;       // nullable: `nzero` int32 to clear
    int nzero;
};

template <typename T> struct Vec4;
template <> struct Vec4<float> { typedef v4f type; };
template <> struct Vec4<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ v4f widen4(v4f x) { return x; }
__device__ __forceinline__ v4f widen4(uint2 x) {
    v4f o;
    o[0] = __uint_as_float(x.x << 16); o[1] = __uint_as_float(x.x & 0xffff0000u);
    o[2] = __uint_as_float(x.y << 16); o[3] = __uint_as_float(x.y & 0xffff0000u);
    return o;
}

// VEC: rows of X start 16-byte (fp32) / 8-byte (bf16) aligned and inner is a multiple of 4, so a thread
// moves four consecutive columns at a time; otherwise single elements.
template <typename T, int NBM, bool VEC>
__global__ __launch_bounds__(SG_NT, 2) void k_subspace_gram(Batch<GramJob> bt) {
    constexpr int TC = sg_tc<NBM>(), PITCH = TC + 4, ROWS = 16 * NBM;
    constexpr int NPAIR = NBM * (NBM + 1) / 2;
    __shared__ __align__(16) float Xs[ROWS * PITCH];
    static_assert(sizeof(float) * ROWS * PITCH >= sizeof(double) * ROWS * ROWS, "the Gram matrix fits the tile buffer");
    int lb;
    const GramJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int n = jb.n, r = jb.r;
    const int S = NBM == 1 ? jb.S : 1;
    const float inv_n = 1.0f / (float)n;
    const long long inner = jb.inner;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    for (int e = tid; e < ROWS * PITCH; e += SG_NT) Xs[e] = 0.f;      // rows >= n stay zero for good
    // U_prev for the product at the end: fetched now (all loads of the workgroup together, addresses valid for
    // every lane), so that the last step reads it from LDS instead of one word at a time from memory
    __shared__ float Us[ROWS * 64];
    {
        constexpr int NU = ROWS * 64 / SG_NT;
        float ut[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int e = tid + SG_NT * u;
            ut[u] = jb.U[e < n * r ? e : 0];
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) Us[tid + SG_NT * u] = ut[u];
    }

    // a thread's share of a tile: NL pieces (VEC: of four columns) in rows (piece / pieces per row)
    constexpr int W = VEC ? 4 : 1, PPR = TC / W, NL = ROWS * PPR / SG_NT;
    static_assert(ROWS * PPR % SG_NT == 0, "whole pieces per thread");
    typename Vec4<T>::type pv[VEC ? NL : 1];
    T ps[VEC ? 1 : NL];
    auto origin = [&](long long tile, long long* base, int* vc) {
        const long long o = tile / jb.tiles_per_o, j0 = (tile - o * jb.tiles_per_o) * (TC * S);
        *vc = (int)(inner - j0 < TC * S ? inner - j0 : TC * S);
        *base = o * n * inner + j0;
    };
    // LDS row -> (column range, mode index); the rounded float quotient is exact for these small integers
    auto split_row = [&](int row, int* sidx, int* i) {
        if (NBM == 1) { *sidx = (int)(((float)row + 0.5f) * inv_n); *i = row - *sidx * n; }
        else { *sidx = row < n ? 0 : 1; *i = row; }
    };
    // Loads go to clamped addresses (always inside X) rather than behind branches, so that all of a
    // tile's loads are in flight together, and are issued while the previous tile is multiplied.
    auto issue = [&](long long tile) {
        long long base;
        int vc;
        origin(tile, &base, &vc);
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int e = u * SG_NT + tid, row = e / PPR, c = (e - row * PPR) * W;
            int sidx, i;
            split_row(row, &sidx, &i);
            const bool ok = sidx < S && sidx * TC + c < vc;
            const long long idx = ok ? base + (long long)i * inner + sidx * TC + c : 0;
            if constexpr (VEC) pv[u] = *reinterpret_cast<const typename Vec4<T>::type*>(X + idx);
            else ps[u] = X[idx];
        }
    };
    auto commit = [&](long long tile) -> int {
        long long base;
        int vc;
        origin(tile, &base, &vc);
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int e = u * SG_NT + tid, row = e / PPR, c = (e - row * PPR) * W;
            int sidx, i;
            split_row(row, &sidx, &i);
            if (sidx < S) {
                const bool in = sidx * TC + c < vc;
                if constexpr (VEC) {
                    const v4f z = {0.f, 0.f, 0.f, 0.f};
                    *reinterpret_cast<v4f*>(&Xs[row * PITCH + c]) = in ? widen4(pv[u]) : z;
                } else {
                    Xs[row * PITCH + c] = in ? to_f32(ps[u]) : 0.f;
                }
            }
        }
        return vc;
    };

    v4d acc[NPAIR];
#pragma unroll
    for (int p = 0; p < NPAIR; ++p) acc[p] = (v4d){0.0, 0.0, 0.0, 0.0};
    if (lb < jb.ntiles) issue(lb);
    for (long long tile = lb; tile < jb.ntiles; tile += jb.nwg) {
        __syncthreads();                                   // the previous tile is no longer read
        const int vc = commit(tile);
        __syncthreads();
        if (tile + jb.nwg < jb.ntiles) issue(tile + jb.nwg);
        const int nch = ((vc < TC ? vc : TC) + 15) >> 4;   // columns past vc are zero in LDS
        for (int ch = wave; ch < nch; ch += 4) {
            double d[NBM][4];
#pragma unroll
            for (int mb = 0; mb < NBM; ++mb) {
                const v4f x = *reinterpret_cast<const v4f*>(&Xs[(16 * mb + ll) * PITCH + 16 * ch + 4 * lg]);
#pragma unroll
                for (int s = 0; s < 4; ++s) d[mb][s] = (double)x[s];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                int p = 0;
#pragma unroll
                for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
                    for (int nb = mb; nb < NBM; ++nb, ++p)
                        acc[p] = __builtin_amdgcn_mfma_f64_16x16x4f64(d[mb][s], d[nb][s], acc[p], 0, 0, 0);
            }
        }
    }
    // G = sum of the four waves' accumulators, wave after wave (fixed order); blocks on or above the diagonal
    double* G = reinterpret_cast<double*>(Xs);             // [ROWS][ROWS]
    for (int w = 0; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
            int p = 0;
#pragma unroll
            for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
                for (int nb = mb; nb < NBM; ++nb, ++p)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        double* g = G + (16 * mb + lg + 4 * v) * ROWS + 16 * nb + ll;      // fp64 MFMA result layout
                        *g = (w == 0) ? acc[p][v] : *g + acc[p][v];
                    }
        }
    }
    __syncthreads();
    // P = G U_prev for this workgroup's columns; a block below the diagonal is its mirror image's transpose
    double* out = jb.part + (long long)lb * n * r;
    for (int e = tid; e < n * r; e += SG_NT) {
        const int i = e / r, q = e - i * r;
        double sum = 0.0;
        for (int k = 0; k < n; ++k) {
            double g;
            if (NBM == 1) {
                g = G[i * ROWS + k];
                for (int sidx = 1; sidx < S; ++sidx) g += G[(sidx * n + i) * ROWS + sidx * n + k];
            } else {
                g = ((i >> 4) <= (k >> 4)) ? G[i * ROWS + k] : G[k * ROWS + i];
            }
            sum = fma(g, (double)Us[k * r + q], sum);
        }
        out[e] = sum;
    }
}

// ---- host side ---------------------------------------------------------------------
bool subspace_gram_supported(long long outer, int n, long long inner, int r) {
    if (n < 1 || n > 64 || r < 1 || r > 64 || outer < 1) return false;
    // The Gram matrix costs n (n + 16) / 2 multiply-adds per column in fp64 against 2 n r for the two
    // products (one of them fp32): with four row blocks and a rank of at most 16 the products are cheaper.
    if (n > 48 && r <= 16) return false;
    return inner >= 128;                  // a long inner extent: tiles of consecutive columns
}
static int gram_nbm(int n) { return (n + 15) / 16; }
static int gram_stack(int n) { return n <= 4 ? 4 : (n <= 8 ? 2 : 1); }
// columns per tile
static int gram_tc(int n) { const int b = gram_nbm(n); return b == 1 ? 512 * gram_stack(n) : (b == 2 ? 256 : 128); }
int subspace_gram_nwg(long long outer, int n, long long inner) {
    const long long tiles = outer * ((inner + gram_tc(n) - 1) / gram_tc(n));
    return (int)(tiles < SG_MAX_WG ? tiles : SG_MAX_WG);
}

// key: [0] bf16, [1] vector loads, [4..6] NBM
bool make_subspace_gram(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r, double* part,
                        int nwg, int32_t* zero, int nzero, Item* out) {
    if (!subspace_gram_supported(outer, n, inner, r) || !X || !U || !part || nzero < 0 || nzero > 256) return false;
    if (nwg != subspace_gram_nwg(outer, n, inner)) return false;
    GramJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.U = U; jb.part = part; jb.outer = outer; jb.inner = inner; jb.n = n; jb.r = r; jb.nwg = nwg;
    jb.tiles_per_o = (inner + gram_tc(n) - 1) / gram_tc(n);
    jb.ntiles = outer * jb.tiles_per_o;
    jb.S = gram_stack(n);
    jb.zero = zero; jb.nzero = zero ? nzero : 0;
    const size_t esz = xt == F32 ? 4 : 2;
    const bool vec = inner % 4 == 0 && reinterpret_cast<uintptr_t>(X) % (4 * esz) == 0;
    const int nbm = gram_nbm(n);
    *out = Item();
    out->kind = IT_GRAM_MODE;
    out->key = (xt == BF16 ? 1u : 0u) | (vec ? 2u : 0u) | ((unsigned)nbm << 4);
    out->nblocks = nwg;
    std::snprintf(out->label, sizeof(out->label), "k_subspace_gram<%s, %d, %s>", xt == F32 ? "float" : "asi::bf16_t", nbm,
                  vec ? "true" : "false");
    static_assert(sizeof(GramJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

template <typename T, bool VEC>
static void launch_gram_nbm(int nbm, dim3 grid, hipStream_t st, const Batch<GramJob>& b) {
    switch (nbm) {
        case 1: hipLaunchKernelGGL((k_subspace_gram<T, 1, VEC>), grid, SG_NT, 0, st, b); break;
        case 2: hipLaunchKernelGGL((k_subspace_gram<T, 2, VEC>), grid, SG_NT, 0, st, b); break;
        case 3: hipLaunchKernelGGL((k_subspace_gram<T, 3, VEC>), grid, SG_NT, 0, st, b); break;
        default: hipLaunchKernelGGL((k_subspace_gram<T, 4, VEC>), grid, SG_NT, 0, st, b); break;
    }
}

hipError_t launch_gram_items(const Item* const* items, int n, hipStream_t st) {
    Batch<GramJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int nbm = (int)((key >> 4) & 7u);
    if (nbm < 1 || nbm > 4) return hipErrorInvalidValue;
    if (key & 1u) {
        if (key & 2u) launch_gram_nbm<bf16_t, true>(nbm, grid, st, b);
        else          launch_gram_nbm<bf16_t, false>(nbm, grid, st, b);
    } else {
        if (key & 2u) launch_gram_nbm<float, true>(nbm, grid, st, b);
        else          launch_gram_nbm<float, false>(nbm, grid, st, b);
    }
    return hipGetLastError();
}

}  // namespace asi
