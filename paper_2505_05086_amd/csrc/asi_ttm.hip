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
//
// k_ttm_thin serves modes of at most 16 entries over very many columns on the vector ALU (further down).
//
// All kernels take the argument blocks of several layers side by side (Batch<TtmJob>).
#include "asi_device.h"
#include "asi_kernels.h"

#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TM_TC = 64, TM_TQ = 64;
// Row pitch of the LDS tiles in floats.  An operand read takes rows 4ks + lane / 16 at columns lane % 16 of
// a wave's block; a pitch of 16 banks more than a multiple of 64 puts the four rows on disjoint banks (a
// pitch of 68 puts them 4 banks apart: up to four lanes per bank).  Along the last mode the tile is stored
// transposed (lanes along the row index), where that pitch would send 16 lanes to one bank; an odd
// multiple of the bank width (17) spreads the rows of the store and keeps the reads nearly disjoint.
// Measured bank-conflict cycles per active LDS cycle: 0.08-0.24 (was 0.50) and 0.38-0.40 (was 0.54-0.60).
template <bool LASTMODE> constexpr int tm_ld() { return LASTMODE ? TM_TC + 17 : TM_TC + 16; }
constexpr int TM_LD_MAX = TM_TC + 17;
constexpr int TM_KCMAX = 64;

// KM: 0 = plain matrix, 1 = Kronecker product, 2 = Kronecker product with K chunks of 64 (long merged
// modes with few columns; otherwise chunks of 32, which overlap across workgroups), 3 = plain matrix with
// K chunks of 64 (a long last mode with at most one workgroup per CU: a chunk is a dependent round trip
// to memory, and nothing else on the CU hides it)
constexpr int TM_SMEM = 2 * TM_KCMAX * TM_LD_MAX;   // floats: Xs | Ms during the K loop, Ys (64 x TM_LD) afterwards

// one tile (workgroup lb of job jb); smem holds TM_SMEM floats
template <typename T, bool LASTMODE, int NBR, int KM>
__device__ __forceinline__ void ttm_tile(const TtmJob& jb, int lb, float* smem) {
    constexpr bool KRON = KM == 1 || KM == 2;
    constexpr int TM_KC = KM >= 2 ? 64 : 32;
    constexpr int TM_LR = TM_KC / 4;      // loads per thread and operand for one chunk
    constexpr int TM_LD = tm_ld<LASTMODE>();
    float (*Xs)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem);
    float (*Ms)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem + TM_KCMAX * TM_LD);
    float (*Ys)[TM_LD] = reinterpret_cast<float (*)[TM_LD]>(smem);
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const float* __restrict__ Mp = jb.Mp;
    float* __restrict__ Y = jb.Y;
    const long long outer = jb.outer, inner = jb.inner, ms_i = jb.ms_i, ms_q = jb.ms_q;
    const int n = jb.n, r = jb.r, beta = jb.beta;
    const KronSpec kr = jb.kr;
    const int bx = lb / jb.gy, by = lb - bx * jb.gy;      // output tiles of the same columns are neighbours (one L2)
    const long long ncols = outer * inner;
    const int tcols = jb.tile_cols;                  // columns of a tile in use (<= TM_TC)
    const long long c0 = (long long)bx * tcols;
    const int q0 = by * TM_TQ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;

    // loader coordinates
    long long ld_base = -1;
    int l_c, l_i;
    if (!LASTMODE) {
        l_c = tid & 63; l_i = tid >> 6;              // rows l_i + 4t
        const long long c = c0 + l_c;
        if (c < ncols && l_c < tcols) {
            const long long o = c / inner, j = c - o * inner;
            ld_base = o * (long long)n * inner + j;
        }
    } else {
        l_i = tid & (TM_KC - 1); l_c = tid / TM_KC;   // columns l_c + (256 / TM_KC) t
    }
    const int m_q = tid & 63, m_i = tid >> 6;        // Ms loader: rows m_i + 4t
    // a matrix stored with the mode index contiguous (the transposed factor of step 5 of Eq. 14) is
    // loaded with the lanes along that index instead: row tid % KC, outputs tid / KC + (256 / KC) t
    const bool m_tr = !KRON && ms_i == 1 && ms_q != 1;
    const int t_i = tid & (TM_KC - 1), t_q = tid / TM_KC;

    // Kronecker indices by a rounded float quotient: exact for arguments below 2^14 (checked on the host)
    const float inv_n2 = 1.0f / (float)kr.n2, inv_r2 = 1.0f / (float)kr.r2;

    v4f acc[NBR];
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb) acc[nb] = (v4f){0.f, 0.f, 0.f, 0.f};

    // The K loop, compiled once per matrix layout (MTR) so that the layout is no test inside it.
    auto kloop = [&](auto mtr_c) {
        constexpr bool MTR = decltype(mtr_c)::value;
        // Every load goes to an address that is always valid: a lane outside the tile reads the tile's
        // first column / first output instead, a row past n reads row n - 1.  What the loads return
        // stays untouched in registers until stash() masks and widens it, after the previous chunk's
        // MFMAs: the chunk's loads are one straight run of instructions, all in flight together, and
        // nothing waits for one of them before the multiply.
        T xr[TM_LR];
        float mr[TM_LR], m2[KRON ? TM_LR : 1];
        const bool x_in = LASTMODE ? true : ld_base >= 0;
        long long x_org;                              // element index of (this lane's column, row 0 / l_i)
        if (!LASTMODE) {
            const long long o = c0 / inner, j = c0 - o * inner;
            x_org = x_in ? ld_base : o * (long long)n * inner + j;
        } else {
            x_org = c0 * (long long)n;
        }
        const bool qm_in = q0 + m_q < r;                             // plain and Kronecker layouts
        const int qm = qm_in ? q0 + m_q : q0;
        const int qm1 = (int)(((float)qm + 0.5f) * inv_r2), qm2 = qm - qm1 * kr.r2;
        // PART: the chunk may reach past n (rows are clamped, empty row groups skipped: a uniform test);
        // otherwise it lies wholly below n and no test on the mode index remains
        auto fetch = [&](int k0, auto part_c) {
            constexpr bool PART = decltype(part_c)::value;
            auto row = [&](int i) { return (PART && i >= n) ? n - 1 : i; };
#pragma unroll
            for (int t = 0; t < TM_LR; ++t) {
                const bool live = !PART || k0 + 4 * t < n;
                if (!LASTMODE) {
                    if (live) xr[t] = X[x_org + (long long)row(k0 + l_i + 4 * t) * inner];
                    else xr[t] = T{};
                } else {
                    const int cl = l_c + (256 / TM_KC) * t;
                    const bool in = c0 + cl < ncols && cl < tcols;
                    xr[t] = X[x_org + row(k0 + l_i) + (in ? (long long)cl * n : 0LL)];
                }
                if (MTR) {
                    const int qt = q0 + t_q + (256 / TM_KC) * t;
                    mr[t] = Mp[(long long)row(k0 + t_i) + (long long)(qt < r ? qt : q0) * ms_q];
                } else if (!live) {
                    mr[t] = 0.f;
                    if (KRON) m2[t] = 0.f;
                } else if (!KRON) {
                    mr[t] = Mp[(long long)row(k0 + m_i + 4 * t) * ms_i + (long long)qm * ms_q];
                } else {
                    const int i = row(k0 + m_i + 4 * t);
                    const int i1 = (int)(((float)i + 0.5f) * inv_n2), i2 = i - i1 * kr.n2;
                    mr[t] = Mp[(long long)i1 * ms_i + (long long)qm1 * ms_q];
                    m2[t] = kr.M2[(long long)i2 * kr.ms_i + (long long)qm2 * kr.ms_q];
                }
            }
        };
        auto stash = [&](int k0) {
#pragma unroll
            for (int t = 0; t < TM_LR; ++t) {
                if (!LASTMODE) {
                    Xs[l_i + 4 * t][l_c] = (x_in && k0 + l_i + 4 * t < n) ? to_f32(xr[t]) : 0.f;
                } else {
                    const int cl = l_c + (256 / TM_KC) * t;
                    Xs[l_i][cl] = (c0 + cl < ncols && cl < tcols && k0 + l_i < n) ? to_f32(xr[t]) : 0.f;
                }
                if (MTR) {
                    const int ql = t_q + (256 / TM_KC) * t;
                    Ms[t_i][ql] = (q0 + ql < r && k0 + t_i < n) ? mr[t] : 0.f;
                } else {
                    const float v = KRON ? mr[t] * m2[t] : mr[t];
                    Ms[m_i + 4 * t][m_q] = (qm_in && k0 + m_i + 4 * t < n) ? v : 0.f;
                }
            }
        };
        // operands of two K steps at a time, read one group ahead of the MFMAs that use them
        constexpr int GS = 2, NG = TM_KC / 4 / GS;
        auto operands = [&](int g, float (&a)[GS], float (&b)[GS][NBR]) {
#pragma unroll
            for (int s = 0; s < GS; ++s) {
                a[s] = Xs[4 * (GS * g + s) + lg][16 * wave + ll];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) b[s][nb] = Ms[4 * (GS * g + s) + lg][16 * nb + ll];
            }
        };
        auto multiply = [&](const float (&a)[GS], const float (&b)[GS][NBR]) {
#pragma unroll
            for (int s = 0; s < GS; ++s)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[s][nb], acc[nb], 0, 0, 0);
        };

        const std::true_type partial{};
        const std::false_type whole{};
        if (TM_KC <= n) fetch(0, whole); else fetch(0, partial);
        for (int k0 = 0; k0 < n; k0 += TM_KC) {
            __syncthreads();                 // previous chunk fully consumed
            stash(k0);
            __syncthreads();
            const int nx = k0 + TM_KC;
            if (nx + TM_KC <= n) fetch(nx, whole);
            else if (nx < n) fetch(nx, partial);
            if (nx <= n) {
                float a0[GS], b0[GS][NBR], a1[GS], b1[GS][NBR];
                // (scheduling fences: without them the compiler moves every read back next to its MFMA
                // and waits for it there)
                operands(0, a0, b0);
#pragma unroll
                for (int g = 0; g < NG; g += 2) {
                    operands(g + 1, a1, b1);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(a0, b0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (g + 2 < NG) operands(g + 2, a0, b0);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(a1, b1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
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
        }
    };
    if (m_tr) kloop(std::true_type{}); else kloop(std::false_type{});
    __syncthreads();
    // result layout: lane holds column 16w + 4*lg + v, output 16nb + ll
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) Ys[16 * nb + ll][16 * wave + 4 * lg + v] = acc[nb][v];
    __syncthreads();
    const int rq = (r - q0 < TM_TQ) ? r - q0 : TM_TQ;
    if (!LASTMODE && inner < TM_TC) {
        // short inner extent: a tile holds whole outer indices, and for one outer index the (q, j)
        // pairs of this workgroup are one contiguous run of Y
        const int k_o = tcols / (int)inner;
        const long long o0 = (long long)bx * k_o;
        const int nvo = (int)((outer - o0 < k_o) ? outer - o0 : k_o);
        const int run = rq * (int)inner, total = nvo * run;          // total <= 4096: float quotients are exact
        const float inv_run = 1.0f / (float)run, inv_in = 1.0f / (float)inner;
        for (int e = tid; e < total; e += 256) {
            const int ol = (int)(((float)e + 0.5f) * inv_run), rem = e - ol * run;
            const int ql = (int)(((float)rem + 0.5f) * inv_in), j = rem - ql * (int)inner;
            const long long idx = ((o0 + ol) * r + q0) * inner + rem;
            const float v = Ys[ql][ol * (int)inner + j];
            Y[idx] = beta ? Y[idx] + v : v;
        }
    } else if (!LASTMODE) {
        const int cl = tid & 63;
        const long long c = c0 + cl;
        if (c < ncols && cl < tcols) {
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
            if (c < ncols && cl < tcols) {
                const long long idx = c * r + q0 + ql;
                Y[idx] = beta ? Y[idx] + Ys[ql][cl] : Ys[ql][cl];
            }
        }
    }
}

template <typename T, bool LASTMODE, int NBR, int KM>
__global__ __launch_bounds__(256) void k_ttm_mfma(Batch<TtmJob> bt) {
    __shared__ float smem[TM_SMEM];
    int lb;
    const TtmJob& jb = bt.job[locate_xcd(bt, &lb)];
    ttm_tile<T, LASTMODE, NBR, KM>(jb, lb, smem);
}

// Two independent products in one launch: a plain product along a leading mode (G1 = grad_out x_1 U1^T
// of Eq. 14) and, in extra workgroups, a small merged product of fp32 data (Z = S x_3 U3 x_4 U4).
struct TtmDuoJob {
    TtmJob a;        // dtype T, not the last mode, plain matrix, NBR column blocks
    TtmJob z;        // fp32, trailing modes merged by a Kronecker product, K chunks of 32
    int a_blocks;
};
template <typename T, int NBR>
__global__ __launch_bounds__(256) void k_ttm_duo(Batch<TtmDuoJob> bt) {
    __shared__ float smem[TM_SMEM];
    int lb;
    const TtmDuoJob& jb = bt.job[locate(bt, &lb)];
    if (lb < jb.a_blocks) ttm_tile<T, false, NBR, 0>(jb.a, xcd_order(lb, jb.a_blocks), smem);
    else ttm_tile<float, true, 4, 1>(jb.z, lb - jb.a_blocks, smem);
}

// ---- long fibres, few columns ------------------------------------------------------------------
// A workgroup owns 16*CB columns.  Round = 16*KS mode indices: wave w, step s multiplies rows
// k0 + 16s + 4w .. +3.  A operands (16 columns x 4 i, one per column block) and B operands
// (4 i x 16 q) are loaded by the lanes that use them; CB column blocks share each B operand.
template <typename T, int NBR, int KS, int CB>
__global__ __launch_bounds__(256) void k_ttm_ksplit(Batch<TtmJob> bt) {
    __shared__ float red[4][NBR * 16][16 * CB + 1];
    int lb;
    const TtmJob& jb = bt.job[locate_xcd(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const float* __restrict__ Mp = jb.Mp;
    float* __restrict__ Y = jb.Y;
    const long long outer = jb.outer, inner = jb.inner, ms_i = jb.ms_i, ms_q = jb.ms_q;
    const int n = jb.n, r = jb.r, beta = jb.beta;
    const int bx = lb / jb.gy, by = lb - bx * jb.gy;      // output tiles of the same columns are neighbours (one L2)
    const long long ncols = outer * inner;
    const long long c0 = (long long)bx * (16 * CB);
    const int q0 = by * (NBR * 16);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    long long xbase[CB];
    bool cok[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const long long c = c0 + 16 * cb + ll;
        cok[cb] = c < ncols;
        const long long cc = cok[cb] ? c : 0;
        const long long o = cc / inner, j = cc - o * inner;
        xbase[cb] = o * (long long)n * inner + j;
    }
    v4f acc[CB][NBR];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) acc[cb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < n; k0 += 16 * KS) {
        float xr[CB][KS], mr[NBR][KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int i = k0 + 16 * s + 4 * wave + lg;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) xr[cb][s] = ldg_f32(X, xbase[cb] + (long long)i * inner, cok[cb] && i < n);
#pragma unroll
            for (int nb = 0; nb < NBR; ++nb) {
                const int q = q0 + 16 * nb + ll;
                mr[nb][s] = ldg_f32(Mp, (long long)i * ms_i + (long long)q * ms_q, i < n && q < r);
            }
        }
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
                    acc[cb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[cb][s], mr[nb][s], acc[cb][nb], 0, 0, 0);
    }
    // lane holds column 16cb + 4*lg + v, output 16nb + ll
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][16 * nb + ll][16 * cb + 4 * lg + v] = acc[cb][nb][v];
    __syncthreads();
    constexpr int W = 16 * CB;
    const int cl = tid % W;
    const long long cc = c0 + cl;
    if (cc < ncols) {
        const long long o = cc / inner, j = cc - o * inner;
        for (int ql = tid / W; ql < NBR * 16; ql += 256 / W) {
            const int q = q0 + ql;
            if (q < r) {
                const float v = (red[0][ql][cl] + red[1][ql][cl]) + (red[2][ql][cl] + red[3][ql][cl]);
                const long long idx = (o * r + q) * inner + j;
                Y[idx] = beta ? Y[idx] + v : v;
            }
        }
    }
}

// ---- very short modes on the vector ALU ---------------------------------------------------------
// A mode of at most 16 entries with at most 16 outputs (the batch mode of a high-resolution layer:
// 8 x 8 over a million columns) gives the MFMA tiles of k_ttm_mfma nothing to do — a 64-column tile is
// 2 KB of data, and the launch is bound by the number of workgroups.  Here a thread owns TH_CPT
// columns: it loads their n values (lanes along the contiguous index), multiplies by the matrix held
// in LDS (read as whole rows, the same address in every lane) and stores r values per column.
constexpr int TH_CPT = 2, TH_COLS = 256 * TH_CPT;
template <typename T, int NMAX>
__global__ __launch_bounds__(256) void k_ttm_thin(Batch<TtmJob> bt) {
    __shared__ __align__(16) float Ms[16][16];
    int lb;
    const TtmJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    float* __restrict__ Y = jb.Y;
    const long long outer = jb.outer, inner = jb.inner, ncols = outer * inner;
    const int n = jb.n, r = jb.r, beta = jb.beta, tid = threadIdx.x;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    {
        const int i = tid >> 4, q = tid & 15;
        Ms[i][q] = ldg_f32(jb.Mp, (long long)i * jb.ms_i + (long long)q * jb.ms_q, i < n && q < r);
    }
    // (o, j) of the workgroup's first column by one division (uniform), of a thread's columns by additions
    const long long cw = (long long)lb * TH_COLS;
    const long long ow = cw / inner, jw = cw - ow * inner;
    long long xb[TH_CPT], yb[TH_CPT];
    bool ok[TH_CPT];
    T xv[TH_CPT][NMAX];
#pragma unroll
    for (int t = 0; t < TH_CPT; ++t) {
        long long o = ow, j = jw + t * 256 + tid;
        while (j >= inner) { j -= inner; ++o; }
        ok[t] = cw + t * 256 + tid < ncols;
        xb[t] = ok[t] ? o * (long long)n * inner + j : 0;          // past the end: column 0, dropped at the store
        yb[t] = ok[t] ? o * (long long)r * inner + j : 0;
#pragma unroll
        for (int i = 0; i < NMAX; ++i) xv[t][i] = X[xb[t] + (long long)(i < n ? i : n - 1) * inner];
    }
    __syncthreads();
    float acc[TH_CPT][16];
#pragma unroll
    for (int t = 0; t < TH_CPT; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;
#pragma unroll
    for (int i = 0; i < NMAX; ++i) {
        float m[16];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const v4f row = *reinterpret_cast<const v4f*>(&Ms[i][4 * q4]);      // rows i >= n are zero
            m[4 * q4] = row[0]; m[4 * q4 + 1] = row[1]; m[4 * q4 + 2] = row[2]; m[4 * q4 + 3] = row[3];
        }
#pragma unroll
        for (int t = 0; t < TH_CPT; ++t) {
            const float x = i < n ? to_f32(xv[t][i]) : 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[t][q] = fmaf(x, m[q], acc[t][q]);
        }
    }
#pragma unroll
    for (int t = 0; t < TH_CPT; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (ok[t] && q < r) {
                const long long idx = yb[t] + (long long)q * inner;
                Y[idx] = beta ? Y[idx] + acc[t][q] : acc[t][q];
            }
}

// ---- a short last mode expanded to many outputs, on the vector ALU ------------------------------
// Y[c, q] (+)= sum_k X[c, k] M(k, q) with at most 32 terms and 256 or more outputs per column: the last
// step of the linear weight gradient (dW = T U_3^T: rank 20, thousands of features).  The output is the
// only large tensor, so the kernel is built around its stores: a workgroup owns 32 columns x 256 outputs,
// lane l holds the four consecutive outputs 4 l .. 4 l + 3 of eight columns, and every store instruction of
// a wave writes 1 KB of one output row.  M's tile sits in LDS as Ms[k][q] (one 16-byte read per term), X's
// tile as Xs[c][k] (every lane of a wave reads the same word).
constexpr int EX_C = 32, EX_Q = 256, EX_K = 32;
__global__ __launch_bounds__(256) void k_ttm_expand(Batch<TtmJob> bt) {
    __shared__ __align__(16) float Ms[EX_K][EX_Q + 4];
    __shared__ float Xs[EX_C][EX_K + 1];
    int lb;
    const TtmJob& jb = bt.job[locate(bt, &lb)];
    const float* __restrict__ X = static_cast<const float*>(jb.X);
    const float* __restrict__ Mp = jb.Mp;
    float* __restrict__ Y = jb.Y;
    const long long ncols = jb.outer, ms_i = jb.ms_i, ms_q = jb.ms_q;
    const int n = jb.n, r = jb.r, beta = jb.beta;
    const int bx = lb / jb.gy, by = lb - bx * jb.gy;
    const long long c0 = (long long)bx * EX_C;
    const int q0 = by * EX_Q;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    // tiles: consecutive threads along the index that is contiguous in memory; every load of the workgroup is
    // issued before the first is stored (clamped addresses, masks at the store: nothing waits in between)
    const bool k_fast = ms_i == 1;
    const float inv_n = 1.0f / (float)n;             // e < 2^13: the rounded float quotients are exact
    float mt[EX_K], xt[EX_C * EX_K / 256];
#pragma unroll
    for (int u = 0; u < EX_K; ++u) {
        const int e = tid + 256 * u;
        const int eq = (int)(((float)e + 0.5f) * inv_n);
        const int k = k_fast ? e - eq * n : u, q = k_fast ? eq : tid;       // (e / 256 = u, e % 256 = tid)
        const bool ok = e < EX_Q * n && q0 + q < r;
        mt[u] = Mp[ok ? (long long)k * ms_i + (long long)(q0 + q) * ms_q : 0LL];
    }
#pragma unroll
    for (int u = 0; u < EX_C * EX_K / 256; ++u) {
        const int e = tid + 256 * u;
        const int c = (int)(((float)e + 0.5f) * inv_n), k = e - c * n;
        const bool ok = e < EX_C * n && c0 + c < ncols;
        xt[u] = X[ok ? (c0 + c) * n + k : 0LL];
    }
#pragma unroll
    for (int u = 0; u < EX_K; ++u) {
        const int e = tid + 256 * u;
        const int eq = (int)(((float)e + 0.5f) * inv_n);
        const int k = k_fast ? e - eq * n : u, q = k_fast ? eq : tid;
        if (e < EX_Q * n) Ms[k][q] = (q0 + q < r) ? mt[u] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < EX_C * EX_K / 256; ++u) {
        const int e = tid + 256 * u;
        const int c = (int)(((float)e + 0.5f) * inv_n), k = e - c * n;
        if (e < EX_C * n) Xs[c][k] = (c0 + c < ncols) ? xt[u] : 0.f;
    }
    __syncthreads();
    v4f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < n; ++k) {
        const v4f m = *reinterpret_cast<const v4f*>(&Ms[k][4 * lane]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float x = Xs[8 * wave + j][k];
            acc[j][0] = fmaf(x, m[0], acc[j][0]); acc[j][1] = fmaf(x, m[1], acc[j][1]);
            acc[j][2] = fmaf(x, m[2], acc[j][2]); acc[j][3] = fmaf(x, m[3], acc[j][3]);
        }
    }
    const int q = q0 + 4 * lane;
    if (q < r) {                                      // r is a multiple of four (host check): a piece is whole
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const long long c = c0 + 8 * wave + j;
            if (c < ncols) {
                v4f* yp = reinterpret_cast<v4f*>(Y + c * r + q);
                v4f out = acc[j];
                if (beta) out += *yp;
                *yp = out;
            }
        }
    }
}
static bool ttm_expand_supported(DType xt, long long inner, int n, int r, const float* Y) {
    return xt == F32 && inner == 1 && n <= EX_K && r >= EX_Q && r % 4 == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
}

// ---- host side -----------------------------------------------------------------------------------
// key bits: [0] bf16 input, [1] LASTMODE, [2] KRON, [3] split kernel, [4..6] NBR-1, [8..12] KS,
// [13] split kernel with several column blocks per workgroup (4 up to NBR = 3, else 2),
// [14] K chunks of 64 (tiled kernel along the last mode), [15] the vector-ALU kernel for very short modes.
// Bits 4..12 only bound sizes.
static unsigned ttm_key(bool bf16, bool last, bool kron, bool ksplit, int nbr, int ks, bool wide, bool kc64) {
    return (bf16 ? 1u : 0u) | (last ? 2u : 0u) | (kron ? 4u : 0u) | (ksplit ? 8u : 0u) | ((unsigned)(nbr - 1) << 4) |
           ((unsigned)ks << 8) | (wide ? 0x2000u : 0u) | (kc64 ? 0x4000u : 0u);
}
static int ksplit_cb(int nbr, bool wide) { return !wide ? 1 : (nbr <= 3 ? 4 : 2); }

// The tiled kernel walks the mode index in n/32 dependent steps with ncols/64 workgroups; when that
// leaves most of the chip idle the split kernel is the faster one.
static bool prefer_ksplit(long long ncols, int n, long long inner) {
    return inner > 1 && n > 64 && (ncols + TM_TC - 1) / TM_TC < 512;
}

static bool fill_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                     long long ms_q, int r, float* Y, int beta, const KronSpec& kr, Item* out) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0 || !X || !Mp || !Y) return false;
    const bool last = (inner == 1), kron = kr.M2 != nullptr;
    TtmJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.outer = outer; jb.inner = inner; jb.Mp = Mp; jb.ms_i = ms_i; jb.ms_q = ms_q; jb.Y = Y;
    jb.kr = kr; jb.n = n; jb.r = r; jb.beta = beta;
    const char* tn = xt == F32 ? "float" : "asi::bf16_t";
    *out = Item();
    if (!kron && ttm_expand_supported(xt, inner, n, r, Y)) {
        const long long gx = (ncols + EX_C - 1) / EX_C;
        jb.gx = (int)gx; jb.gy = (r + EX_Q - 1) / EX_Q;
        if (gx * jb.gy > 0x3fffffffLL) return false;
        out->kind = IT_TTM_EXPAND; out->key = 0;
        std::snprintf(out->label, sizeof(out->label), "k_ttm_expand");
    } else if (!kron && !last && n <= 16 && r <= 16 && ncols >= (1LL << 18)) {
        const long long gx = (ncols + TH_COLS - 1) / TH_COLS;
        if (gx > 0x3fffffffLL) return false;
        jb.gx = (int)gx; jb.gy = 1;
        out->kind = IT_TTM; out->key = ttm_key(xt == BF16, false, false, false, 1, 0, false, false) | 0x8000u;
        std::snprintf(out->label, sizeof(out->label), "k_ttm_thin<%s, %d>", tn, n <= 8 ? 8 : 16);
    } else if (!kron && prefer_ksplit(ncols, n, inner)) {
        const int nbr = r >= 64 ? 4 : (r + 15) / 16;
        // several column blocks per workgroup share the matrix operand; worth it once that still
        // leaves a workgroup for every other CU
        const bool wide = ncols / (16 * ksplit_cb(nbr, true)) >= 128;
        const int ks = n <= 64 ? 4 : (wide ? 8 : (n <= 128 ? 8 : 16));
        const int wcols = 16 * ksplit_cb(nbr, wide);
        const long long gx = (ncols + wcols - 1) / wcols;
        jb.gx = (int)gx; jb.gy = (r + nbr * 16 - 1) / (nbr * 16);
        if (gx * jb.gy > 0x3fffffffLL) return false;
        out->kind = IT_KSPLIT; out->key = ttm_key(xt == BF16, false, false, true, nbr, ks, wide, false);
        std::snprintf(out->label, sizeof(out->label), "k_ttm_ksplit<%s, %d, %d, %d>", tn, nbr, ks, ksplit_cb(nbr, wide));
    } else {
        // short inner extents: tiles of whole outer indices (stores then run contiguously)
        jb.tile_cols = (!last && inner < TM_TC) ? (int)(TM_TC / inner * inner) : TM_TC;
        const long long gx = (!last && inner < TM_TC) ? (outer + TM_TC / inner - 1) / (TM_TC / inner)
                                                      : (ncols + TM_TC - 1) / TM_TC;
        const int rr = r < TM_TQ ? r : TM_TQ;
        const int nbr = (rr + 15) / 16;
        jb.gx = (int)gx; jb.gy = (r + TM_TQ - 1) / TM_TQ;
        if (gx * jb.gy > 0x3fffffffLL) return false;
        const bool kc64 = kron ? n > 64 : (last && n >= 256 && gx * jb.gy <= 256);   // (at most one workgroup per CU)
        out->kind = IT_TTM; out->key = ttm_key(xt == BF16, last, kron, false, nbr, 0, false, kc64);
        std::snprintf(out->label, sizeof(out->label), "k_ttm_mfma<%s, %s, %d, %d>", tn, last ? "true" : "false", nbr,
                      kron ? (kc64 ? 2 : 1) : (kc64 ? 3 : 0));
    }
    out->nblocks = jb.gx * jb.gy;
    static_assert(sizeof(TtmJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

bool make_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
              long long ms_q, int r, float* Y, int beta, Item* out, bool stream_ok) {
    const KronSpec none = {nullptr, 0, 0, 1, 1};
    const long long ncols = outer * inner;
    const bool thin = n <= 16 && r <= 16 && ncols >= (1LL << 18);
    // the streaming kernel pays once the tensor is large enough to keep the chip busy with its loads
    // (the split kernel's 16-column workgroups spread few columns further: it keeps the products below 256 spans)
    if (stream_ok && inner > 1 && !thin && ncols * n >= kStreamMinElems && (ncols >= 256 * 64 || !prefer_ksplit(ncols, n, inner)) &&
        ttm_stream_supported(xt, X, outer, n, inner, Mp, ms_i, ms_q, r, Y))
        return make_ttm_stream(xt, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, out);
    return fill_ttm(xt, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, none, out);
}

bool make_ttm_kron(DType xt, const void* X, long long cols, int n1, int n2, const float* M1, long long ms1_i,
                   long long ms1_q, int r1, const float* M2, long long ms2_i, long long ms2_q, int r2, float* Y,
                   int beta, Item* out) {
    if (cols <= 0 || n1 <= 0 || n2 <= 0 || r1 <= 0 || r2 <= 0 || !M1 || !M2) return false;
    const KronSpec kr = {M2, ms2_i, ms2_q, n2, r2};
    return fill_ttm(xt, X, cols, n1 * n2, 1, M1, ms1_i, ms1_q, r1 * r2, Y, beta, kr, out);
}

template <typename T, bool LAST, int KM>
static void launch_tiled(int nbr, const Batch<TtmJob>& b, dim3 grid, hipStream_t st) {
    switch (nbr) {
        case 1: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 1, KM>), grid, 256, 0, st, b); break;
        case 2: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 2, KM>), grid, 256, 0, st, b); break;
        case 3: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 3, KM>), grid, 256, 0, st, b); break;
        default: hipLaunchKernelGGL((k_ttm_mfma<T, LAST, 4, KM>), grid, 256, 0, st, b); break;
    }
}
template <typename T, int NBR>
static void launch_split(int ks, bool wide, const Batch<TtmJob>& b, dim3 grid, hipStream_t st) {
    constexpr int CB = NBR <= 3 ? 4 : 2;
    if (wide) {
        if (ks == 4) hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 4, CB>), grid, 256, 0, st, b);
        else hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 8, CB>), grid, 256, 0, st, b);
    } else {
        if (ks == 4) hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 4, 1>), grid, 256, 0, st, b);
        else if (ks == 8) hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 8, 1>), grid, 256, 0, st, b);
        else hipLaunchKernelGGL((k_ttm_ksplit<T, NBR, 16, 1>), grid, 256, 0, st, b);
    }
}

// a: a tiled plain product that is not along the last mode; z: a Kronecker product with short K.
// Fails (and leaves *out alone) if the two do not have these forms; the caller then launches them apart.
bool make_ttm_duo(const Item& a, const Item& z, Item* out) {
    if (a.kind != IT_TTM || z.kind != IT_TTM) return false;
    if ((a.key & 0xe00eu) != 0u) return false;                 // not last mode, plain, tiled, chunks of 32
    if ((z.key & 0x600fu) != (2u | 4u)) return false;          // fp32, last mode, Kronecker, tiled, chunks of 32
    TtmDuoJob jb;
    std::memcpy(&jb.a, a.arg, sizeof(TtmJob));
    std::memcpy(&jb.z, z.arg, sizeof(TtmJob));
    jb.a_blocks = a.nblocks;
    if ((long long)a.nblocks + z.nblocks > 0x3fffffffLL) return false;
    const int nbr = (int)((a.key >> 4) & 7u) + 1;
    Item it;
    it.kind = IT_TTM_DUO;
    it.key = (a.key & 1u) | ((unsigned)(nbr - 1) << 4);
    it.nblocks = a.nblocks + z.nblocks;
    std::snprintf(it.label, sizeof(it.label), "k_ttm_duo<%s, %d>", (a.key & 1u) ? "asi::bf16_t" : "float", nbr);
    std::snprintf(it.role, sizeof(it.role), "%s+%s", a.role, z.role);
    it.bytes = a.bytes + z.bytes; it.flops = a.flops + z.flops;
    static_assert(sizeof(TtmDuoJob) <= kItemArgMax, "argument block");
    std::memcpy(it.arg, &jb, sizeof(jb));
    *out = it;
    return true;
}

hipError_t launch_ttm_duo_items(const Item* const* items, int n, hipStream_t st, char* label_out) {
    Batch<TtmDuoJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const bool bf16 = items[0]->key & 1u;
    int nbr = 1;
    for (int j = 0; j < n; ++j) {
        const int nj = (int)((items[j]->key >> 4) & 7u) + 1;
        nbr = nj > nbr ? nj : nbr;
    }
    if (label_out) std::snprintf(label_out, 96, "k_ttm_duo<%s, %d>", bf16 ? "asi::bf16_t" : "float", nbr);
#define ASI_DUO(TT)                                                                              \
    switch (nbr) {                                                                               \
        case 1: hipLaunchKernelGGL((k_ttm_duo<TT, 1>), grid, 256, 0, st, b); break;              \
        case 2: hipLaunchKernelGGL((k_ttm_duo<TT, 2>), grid, 256, 0, st, b); break;              \
        case 3: hipLaunchKernelGGL((k_ttm_duo<TT, 3>), grid, 256, 0, st, b); break;              \
        default: hipLaunchKernelGGL((k_ttm_duo<TT, 4>), grid, 256, 0, st, b); break;             \
    }
    if (!bf16) { ASI_DUO(float) } else { ASI_DUO(bf16_t) }
#undef ASI_DUO
    return hipGetLastError();
}

hipError_t launch_ttm_expand_items(const Item* const* items, int n, hipStream_t st) {
    Batch<TtmJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_ttm_expand, grid, 256, 0, st, b);
    return hipGetLastError();
}

hipError_t launch_ttm_items(const Item* const* items, int n, hipStream_t st, char* label_out) {
    Batch<TtmJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const bool bf16 = key & 1u, last = key & 2u, kron = key & 4u, ksplit = key & 8u;
    const bool wide = key & 0x2000u, kc64 = key & 0x4000u;
    if (key & 0x8000u) {             // very short mode: one instantiation per bound on n
        int nmax = 8;
        for (int j = 0; j < n; ++j) {
            TtmJob tj;
            std::memcpy(&tj, items[j]->arg, sizeof(tj));
            if (tj.n > 8) nmax = 16;
        }
        if (label_out) std::snprintf(label_out, 96, "k_ttm_thin<%s, %d>", bf16 ? "asi::bf16_t" : "float", nmax);
        if (!bf16) { if (nmax == 8) hipLaunchKernelGGL((k_ttm_thin<float, 8>), grid, 256, 0, st, b); else hipLaunchKernelGGL((k_ttm_thin<float, 16>), grid, 256, 0, st, b); }
        else { if (nmax == 8) hipLaunchKernelGGL((k_ttm_thin<bf16_t, 8>), grid, 256, 0, st, b); else hipLaunchKernelGGL((k_ttm_thin<bf16_t, 16>), grid, 256, 0, st, b); }
        return hipGetLastError();
    }
    // the instantiation with the most column blocks / steps serves every item
    int nbr = 1, ks = 0;
    for (int j = 0; j < n; ++j) {
        const int nj = (int)((items[j]->key >> 4) & 7u) + 1, kj = (int)((items[j]->key >> 8) & 31u);
        nbr = nj > nbr ? nj : nbr;
        ks = kj > ks ? kj : ks;
    }
    if (label_out) {
        const char* tn = bf16 ? "asi::bf16_t" : "float";
        if (ksplit) std::snprintf(label_out, 96, "k_ttm_ksplit<%s, %d, %d, %d>", tn, nbr, ks, ksplit_cb(nbr, wide));
        else std::snprintf(label_out, 96, "k_ttm_mfma<%s, %s, %d, %d>", tn, last ? "true" : "false", nbr, kron ? (kc64 ? 2 : 1) : (kc64 ? 3 : 0));
    }
    if (ksplit) {
        if (!bf16) {
            switch (nbr) {
                case 1: launch_split<float, 1>(ks, wide, b, grid, st); break;
                case 2: launch_split<float, 2>(ks, wide, b, grid, st); break;
                case 3: launch_split<float, 3>(ks, wide, b, grid, st); break;
                default: launch_split<float, 4>(ks, wide, b, grid, st); break;
            }
        } else {
            switch (nbr) {
                case 1: launch_split<bf16_t, 1>(ks, wide, b, grid, st); break;
                case 2: launch_split<bf16_t, 2>(ks, wide, b, grid, st); break;
                case 3: launch_split<bf16_t, 3>(ks, wide, b, grid, st); break;
                default: launch_split<bf16_t, 4>(ks, wide, b, grid, st); break;
            }
        }
    } else if (kron) {           // always LASTMODE
        if (!bf16) { if (kc64) launch_tiled<float, true, 2>(nbr, b, grid, st); else launch_tiled<float, true, 1>(nbr, b, grid, st); }
        else { if (kc64) launch_tiled<bf16_t, true, 2>(nbr, b, grid, st); else launch_tiled<bf16_t, true, 1>(nbr, b, grid, st); }
    } else if (!bf16) {
        if (last && kc64) launch_tiled<float, true, 3>(nbr, b, grid, st);
        else if (last) launch_tiled<float, true, 0>(nbr, b, grid, st);
        else launch_tiled<float, false, 0>(nbr, b, grid, st);
    } else {
        if (last && kc64) launch_tiled<bf16_t, true, 3>(nbr, b, grid, st);
        else if (last) launch_tiled<bf16_t, true, 0>(nbr, b, grid, st);
        else launch_tiled<bf16_t, false, 0>(nbr, b, grid, st);
    }
    return hipGetLastError();
}

}  // namespace asi
