// Generic kernels of the ASI hot path for gfx950 (wave64).
//
// Contractions over a tensor seen from a mode, X[o,i,j] (outer, n, inner):
//   pair: P[i,q]    = sum_{o,j} X[o,i,j] Y[o,q,j]      (A_m V of Alg. 1)
// plus partial-sum reduction and the grouped step 5 of Eq. 14.  Every kernel serves the
// argument blocks of several layers side by side.
#include "asi_device.h"
#include "asi_kernels.h"

#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

// ---------------------------------------------------------------------------
// pair: P[i,q] = sum_c X[i,c] Y[q,c] on fp64 MFMA.  A workgroup owns 64 rows i x 32 outputs q
// over one split of the unfolding columns; chunks of 64 columns are prefetched into registers
// while the previous chunk is multiplied.  Wave w multiplies rows 16w..16w+15:
//   A operand (16 i x 4 c) = Xs[4ks + lane/16][16w + lane%16],  B operand (4 c x 16 q) = Ys[4ks + lane/16][16nb + lane%16]
// fp32 values are widened to fp64, so every product is exact and the sums are carried in fp64.
// ---------------------------------------------------------------------------
constexpr int PR_TI = 64, PR_TQ = 32, PR_TK = 64;
// Waves per workgroup: 4 own 16 rows of the tile each; the second four take every other K step of
// a chunk on accumulators of their own, added through LDS at the end.  One wave per SIMD pays its
// operand reads and conversions on top of its products; two waves per SIMD overlap them.
constexpr int PR_NW = 8, PR_NT = 64 * PR_NW, PR_KG = PR_NW / 4;
typedef double v4d __attribute__((ext_vector_type(4)));

template <typename T, bool LASTMODE>
__global__ __launch_bounds__(PR_NT) void k_pair(Batch<PairJob> bt) {
    // Along the last mode the tiles are held widened (a Y element is an operand of four waves, so widening
    // once at the store saves most of the conversions); otherwise the stores run down the columns of the
    // tiles, where 8-byte elements would collide in the LDS banks.
    using S = std::conditional_t<LASTMODE, double, float>;
    __shared__ S Xs[PR_TK][PR_TI + 1];
    __shared__ S Ys[PR_TK][PR_TQ + 1];
    int lb;
    const PairJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const float* __restrict__ Y = jb.Y;
    double* __restrict__ part = jb.part;
    const long long outer = jb.outer, inner = jb.inner, cols_per_split = jb.cols_per_split;
    const int n = jb.n, r = jb.r;
    if (lb >= jb.gx * jb.gy * jb.gz) {             // extra workgroups: another mode's partial-sum tree
        if (threadIdx.x < 256) presum_block(jb.pre.job, jb.pre.njobs, lb - jb.gx * jb.gy * jb.gz);
        return;
    }
    // Neighbouring blocks (one XCD after the renumbering) are the output tiles of the same rows of X,
    // then the row tiles of the same split: the large operand is fetched from memory once.
    lb = xcd_order(lb, jb.gx * jb.gy * jb.gz);
    const int bz = lb / (jb.gx * jb.gy), rem = lb - bz * (jb.gx * jb.gy), bx = rem / jb.gy, by = rem - bx * jb.gy;
    const long long ncols = outer * inner;
    const int i0 = bx * PR_TI, q0 = by * PR_TQ, s = bz;
    const long long cbeg = (long long)s * cols_per_split;
    const long long cend = (cbeg + cols_per_split < ncols) ? cbeg + cols_per_split : ncols;
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, kgrp = tid >> 8, lg = lane >> 4, ll = lane & 15;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;   // arrival counters of later launches

    constexpr int NX = PR_TI * PR_TK / PR_NT, NY = PR_TQ * PR_TK / PR_NT, RS = PR_NT / PR_TK;   // loads per thread, row step
    // A chunk's loads go to addresses that are always valid (a lane outside the tile, the split or the
    // tensor reads a clamped position instead) and what they return stays untouched in registers until
    // stash() masks and widens it after the previous chunk's MFMAs: the loads are one straight run of
    // instructions, all in flight together, and nothing waits for one of them before the multiply.
    T xr[NX];
    float yr[NY];
    const int cl = tid & (PR_TK - 1), rl = tid / PR_TK;
    // not the last mode: column c = (o, j) of this lane in the chunk to fetch next, carried from chunk
    // to chunk by additions (PR_TK = so * inner + sj with sj < inner, so at most one carry into o)
    // (a lane whose column lies beyond the tensor keeps base 0: with a row offset it still reads inside X)
    long long lc = cbeg + cl, lj = 0, xbase = 0, ybase = 0;
    const int so = LASTMODE || inner > PR_TK ? 0 : PR_TK / (int)inner;
    const long long sj = LASTMODE ? 0 : PR_TK - so * inner;
    const long long xplane = (long long)n * inner, yplane = (long long)r * inner;
    if (!LASTMODE && lc < ncols) {
        // quotient by a double division (exact below 2^52) with one correction step
        long long o = (long long)((double)lc / (double)inner);
        lj = lc - o * inner;
        if (lj < 0) { --o; lj += inner; } else if (lj >= inner) { ++o; lj -= inner; }
        xbase = o * xplane + lj;
        ybase = o * yplane + lj;
    }
    // last mode: offsets of this lane's elements from the chunk's first element (PR_TK * n < 2^32: host check);
    // a column past the split's end reads column 0 instead, a row or output past the end the tile's first
    unsigned xoff[LASTMODE ? NX : 1], yoff[LASTMODE ? NY : 1];
    const unsigned xoff0 = (i0 + (tid & 63) < n) ? (tid & 63) : 0, yoff0 = (q0 + (tid & 31) < r) ? (tid & 31) : 0;
    if (LASTMODE) {
#pragma unroll
        for (int t = 0; t < NX; ++t) xoff[t] = (unsigned)((tid >> 6) + PR_NW * t) * (unsigned)n + xoff0;
#pragma unroll
        for (int t = 0; t < NY; ++t) yoff[t] = (unsigned)((tid >> 5) + 2 * PR_NW * t) * (unsigned)r + yoff0;
    }
    auto fetch = [&](long long c0) {
        if (!LASTMODE) {
#pragma unroll
            for (int t = 0; t < NX; ++t) {
                const int i = i0 + rl + RS * t;
                xr[t] = X[xbase + (long long)(i < n ? i : i0) * inner];
            }
#pragma unroll
            for (int t = 0; t < NY; ++t) {
                const int q = q0 + rl + RS * t;
                yr[t] = Y[ybase + (long long)(q < r ? q : q0) * inner];
            }
            lc += PR_TK; lj += sj; xbase += so * xplane + sj; ybase += so * yplane + sj;
            if (lj >= inner) { lj -= inner; xbase += xplane - inner; ybase += yplane - inner; }
            if (lc >= ncols) { xbase = 0; ybase = 0; }
        } else {  // inner == 1: one 64-bit base per chunk (uniform) and 32-bit lane offsets, fixed for the whole split
            const T* __restrict__ xb = X + (c0 * (long long)n + i0);
            const float* __restrict__ yb = Y + (c0 * (long long)r + q0);
            const int lim = (int)(cend - c0 < PR_TK ? cend - c0 : PR_TK);     // columns of the chunk inside the split
#pragma unroll
            for (int t = 0; t < NX; ++t) xr[t] = xb[(tid >> 6) + PR_NW * t < lim ? xoff[t] : xoff0];
#pragma unroll
            for (int t = 0; t < NY; ++t) yr[t] = yb[(tid >> 5) + 2 * PR_NW * t < lim ? yoff[t] : yoff0];
        }
    };
    auto stash = [&](long long c0) {
        if (!LASTMODE) {
            const bool valid = c0 + cl < cend;
#pragma unroll
            for (int t = 0; t < NX; ++t) Xs[cl][rl + RS * t] = (valid && i0 + rl + RS * t < n) ? to_f32(xr[t]) : 0.f;
#pragma unroll
            for (int t = 0; t < NY; ++t) Ys[cl][rl + RS * t] = (valid && q0 + rl + RS * t < r) ? yr[t] : 0.f;
        } else {
            const bool iv = i0 + (tid & 63) < n, qv = q0 + (tid & 31) < r;
#pragma unroll
            for (int t = 0; t < NX; ++t)
                Xs[(tid >> 6) + PR_NW * t][tid & 63] = (iv && c0 + (tid >> 6) + PR_NW * t < cend) ? (S)to_f32(xr[t]) : (S)0;
#pragma unroll
            for (int t = 0; t < NY; ++t)
                Ys[(tid >> 5) + 2 * PR_NW * t][tid & 31] = (qv && c0 + (tid >> 5) + 2 * PR_NW * t < cend) ? (S)yr[t] : (S)0;
        }
    };

    v4d acc[2] = {{0.0, 0.0, 0.0, 0.0}, {0.0, 0.0, 0.0, 0.0}};
    if (cbeg < cend) fetch(cbeg);
    for (long long c0 = cbeg; c0 < cend; c0 += PR_TK) {
        __syncthreads();
        stash(c0);
        __syncthreads();
        if (c0 + PR_TK < cend) fetch(c0 + PR_TK);
#pragma unroll
        for (int ks = kgrp; ks < PR_TK / 4; ks += PR_KG) {
            const double a = (double)Xs[4 * ks + lg][16 * wave + ll];
            acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)Ys[4 * ks + lg][ll], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)Ys[4 * ks + lg][16 + ll], acc[1], 0, 0, 0);
        }
    }
    // the K groups add their accumulators through LDS (the tiles are no longer read), then group 0 stores
    double* red = reinterpret_cast<double*>(&Xs[0][0]);           // 64 x 32 doubles = 16 KB <= sizeof(Xs)
    static_assert(sizeof(float) * PR_TK * (PR_TI + 1) >= sizeof(double) * PR_TI * PR_TQ, "reduction buffer fits the X tile");
#pragma unroll
    for (int kg = PR_KG - 1; kg >= 1; --kg) {
        __syncthreads();
        if (kgrp == kg) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double* p = red + (16 * wave + lg + 4 * v) * PR_TQ + 16 * nb + ll;
                    *p = (kg == PR_KG - 1) ? acc[nb][v] : *p + acc[nb][v];
                }
        }
    }
    __syncthreads();
    if (kgrp == 0) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 16 * wave + lg + 4 * v, q = q0 + 16 * nb + ll;    // fp64 MFMA result layout
                const double sum = PR_KG > 1 ? acc[nb][v] + red[(16 * wave + lg + 4 * v) * PR_TQ + 16 * nb + ll] : acc[nb][v];
                if (i < n && q < r) part[((long long)s * n + i) * r + q] = sum;
            }
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
    long long maxs = (ncols + 255) / 256;                     // at least 256 columns per split
    if (maxs > 64) maxs = 64;
    if (maxs < 1) maxs = 1;
    // The chip holds two workgroups per CU at full rate (512 slots; a single workgroup per CU leaves the
    // MFMA pipe idle while it loads and stores tiles).  Workgroups beyond that run in further rounds, so
    // the time goes as rounds x (columns of a split + a fixed cost per workgroup, worth ~128 columns);
    // the number of splits minimises it.  Few tiles: as many splits as allowed (one round anyway); many
    // tiles (a 3072 x 192 result is 288): a count that fills whole rounds, not one workgroup per CU.
    int best = 1;
    long long best_cost = -1;
    for (int ns = 1; ns <= (int)maxs; ++ns) {
        const long long cps = pair_cols_per_split(ncols, ns);
        if (ns > 1 && cps * (ns - 1) >= ncols) continue;     // the last split would be empty
        const long long rounds = (tiles * ns + 511) / 512;
        // beyond 32 splits the partial sums need a tree level: one more launch on the chain (~600 columns' worth)
        const long long cost = rounds * (cps + 128) + (ns > 32 ? 600 : 0);
        if (best_cost < 0 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    return best;
}

int presum_blocks(const PresumArgs& a) {
    if (a.njobs <= 0 || a.njobs > 4) return -1;
    long long blocks = 0;
    for (int j = 0; j < a.njobs; ++j) {
        const PresumJob& jb = a.job[j];
        if (!jb.in || !jb.out || jb.cnt <= 0 || jb.nsplit <= 0) return -1;
        if (jb.nchunks != (int)((jb.cnt + 255) / 256) || jb.ngroups != (jb.nsplit + 31) / 32) return -1;
        blocks += (long long)jb.nchunks * jb.ngroups;
    }
    return blocks > 0x3fffffffLL ? -1 : (int)blocks;
}

bool make_pair(DType xt, const void* X, long long outer, int n, long long inner, const float* Y, int r, double* part,
               int nsplit, int32_t* zero, int nzero, const PresumArgs* pre, Item* out) {
    const long long ncols = outer * inner;
    if (ncols <= 0 || n <= 0 || r <= 0 || nsplit <= 0 || !X || !Y || !part || nzero < 0 || nzero > 256) return false;
    if (inner == 1 && (n >= (1 << 24) || r >= (1 << 24))) return false;      // 32-bit offsets inside a chunk of the last mode
    PairJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.outer = outer; jb.inner = inner; jb.cols_per_split = pair_cols_per_split(ncols, nsplit);
    jb.Y = Y; jb.part = part; jb.n = n; jb.r = r;
    jb.gx = (n + PR_TI - 1) / PR_TI; jb.gy = (r + PR_TQ - 1) / PR_TQ; jb.gz = nsplit;
    jb.zero = zero; jb.nzero = zero ? nzero : 0;
    if (pre) {
        jb.pre_blocks = presum_blocks(*pre);
        if (jb.pre_blocks < 0) return false;
        jb.pre = *pre;
    }
    const bool last = (inner == 1);
    *out = Item();
    out->kind = IT_PAIR; out->key = (xt == BF16 ? 1u : 0u) | (last ? 2u : 0u);
    out->nblocks = jb.gx * jb.gy * jb.gz + jb.pre_blocks;
    std::snprintf(out->label, sizeof(out->label), "k_pair<%s, %s>", xt == F32 ? "float" : "asi::bf16_t", last ? "true" : "false");
    static_assert(sizeof(PairJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

hipError_t launch_pair_items(const Item* const* items, int n, hipStream_t st) {
    Batch<PairJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    if (!(key & 1u)) {
        if (key & 2u) hipLaunchKernelGGL((k_pair<float, true>), grid, PR_NT, 0, st, b);
        else          hipLaunchKernelGGL((k_pair<float, false>), grid, PR_NT, 0, st, b);
    } else {
        if (key & 2u) hipLaunchKernelGGL((k_pair<bf16_t, true>), grid, PR_NT, 0, st, b);
        else          hipLaunchKernelGGL((k_pair<bf16_t, false>), grid, PR_NT, 0, st, b);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// sum of split partials
// ---------------------------------------------------------------------------
template <typename PT>
__global__ __launch_bounds__(256) void k_sum_partials(Batch<SumJob> bt) {
    int lb;
    const SumJob& jb = bt.job[locate(bt, &lb)];
    const PT* __restrict__ part = static_cast<const PT*>(jb.part);
    const long long count = jb.count;
    const long long e = (long long)lb * 256 + threadIdx.x;
    if (e >= count) return;
    double s = 0.0;
    constexpr int SU = 16;                                   // loads in flight per round (a round is one memory latency)
    for (int sp0 = 0; sp0 < jb.nsplit; sp0 += SU) {
        PT t[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) t[u] = part[(sp0 + u < jb.nsplit) ? (long long)(sp0 + u) * count + e : e];
#pragma unroll
        for (int u = 0; u < SU; ++u) s += (sp0 + u < jb.nsplit) ? (double)t[u] : 0.0;
    }
    jb.out[e] = jb.beta ? jb.out[e] + (float)s : (float)s;
}

static bool fill_sum(const void* part, bool f64, int nsplit, long long count, float* out, int beta, Item* it) {
    if (count <= 0 || nsplit <= 0 || !part || !out || (count + 255) / 256 > 0x3fffffffLL) return false;
    SumJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.part = part; jb.out = out; jb.count = count; jb.nsplit = nsplit; jb.beta = beta;
    *it = Item();
    it->kind = f64 ? IT_SUM_F64 : IT_SUM_F32;
    it->nblocks = (int)((count + 255) / 256);
    std::snprintf(it->label, sizeof(it->label), "k_sum_partials<%s>", f64 ? "double" : "float");
    std::memcpy(it->arg, &jb, sizeof(jb));
    return true;
}
bool make_sum_partials(const float* part, int nsplit, long long count, float* out, int beta, Item* it) {
    return fill_sum(part, false, nsplit, count, out, beta, it);
}
bool make_sum_partials_f64(const double* part, int nsplit, long long count, float* out, int beta, Item* it) {
    return fill_sum(part, true, nsplit, count, out, beta, it);
}
hipError_t launch_sum_items(const Item* const* items, int n, hipStream_t st) {
    Batch<SumJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    if (items[0]->kind == IT_SUM_F64) hipLaunchKernelGGL(k_sum_partials<double>, grid, 256, 0, st, b);
    else hipLaunchKernelGGL(k_sum_partials<float>, grid, 256, 0, st, b);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Step 5 of Eq. 14 for grouped convolutions
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_expand_grouped(Batch<ExpandJob> bt) {
    int lb;
    const ExpandJob& jb = bt.job[locate(bt, &lb)];
    const int r2 = jb.r2, taps = jb.taps, cg = jb.cg, og = jb.og;
    const long long total = (long long)jb.cout * cg * taps;
    const long long e = (long long)lb * 256 + threadIdx.x;
    if (e >= total) return;
    const int t = (int)(e % taps);
    const int c = (int)((e / taps) % cg);
    const int o = (int)(e / ((long long)taps * cg));
    const float* tp = jb.T + (long long)o * r2 * taps + t;
    const float* up = jb.U2 + ((long long)(o / og) * cg + c) * r2;
    float acc = 0.f;
    for (int j = 0; j < r2; ++j) acc = fmaf(tp[(long long)j * taps], up[j], acc);
    jb.dW[e] = jb.beta ? jb.dW[e] + acc : acc;
}

bool make_expand_grouped(const float* T, const float* U2, float* dW, int cout, int r2, int taps, int cg, int og,
                         int beta, Item* out) {
    const long long total = (long long)cout * cg * taps;
    if (total <= 0 || !T || !U2 || !dW || (total + 255) / 256 > 0x3fffffffLL) return false;
    ExpandJob jb = {T, U2, dW, cout, r2, taps, cg, og, beta};
    *out = Item();
    out->kind = IT_EXPAND;
    out->nblocks = (int)((total + 255) / 256);
    std::snprintf(out->label, sizeof(out->label), "k_expand_grouped");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}
hipError_t launch_expand_items(const Item* const* items, int n, hipStream_t st) {
    Batch<ExpandJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_expand_grouped, grid, 256, 0, st, b);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// one launch for the items of several layers
// ---------------------------------------------------------------------------
// key bits of the mode-product kernels that only bound sizes (see asi_ttm.hip): NBR, KS
static unsigned launch_class(const Item& it) {
    if (it.kind == IT_TTM || it.kind == IT_KSPLIT) return it.key & 0xe00fu;
    if (it.kind == IT_TTM_DUO) return it.key & 0xfu;
    return it.key;
}
bool same_launch(const Item& a, const Item& b) {
    return a.kind == b.kind && a.aux == b.aux && launch_class(a) == launch_class(b);
}

hipError_t launch_items(const Item* const* items, int n, hipStream_t st, char* label_out) {
    if (n <= 0 || n > kMaxBatch) return hipErrorInvalidValue;
    for (int j = 1; j < n; ++j)
        if (!same_launch(*items[0], *items[j])) return hipErrorInvalidValue;
    if (label_out) std::snprintf(label_out, 96, "%s", items[0]->label);
    switch (items[0]->kind) {
        case IT_TTM: case IT_KSPLIT: return launch_ttm_items(items, n, st, label_out);
        case IT_TTM_DUO: return launch_ttm_duo_items(items, n, st, label_out);
        case IT_PAIR: return launch_pair_items(items, n, st);
        case IT_SUM_F32: case IT_SUM_F64: return launch_sum_items(items, n, st);
        case IT_EXPAND: return launch_expand_items(items, n, st);
        case IT_SMALL: return launch_small_items(items, n, st);
        case IT_TINY: return launch_tiny_items(items, n, st);
        case IT_LONG: return launch_long_items(items, n, st);
        case IT_PLANES: return launch_planes_items(items, n, st);
        case IT_SPLIT_BF16: case IT_GEMM_BF16: return launch_bf16_items(items, n, st);
        case IT_PRESUM: case IT_GRAM0: case IT_APPLY: case IT_ORTHW_GRAM: case IT_ORTHW_CHOL: case IT_ORTHW_APPLY:
        case IT_ORTH_BIG: case IT_INIT: return launch_orth_items(items, n, st, label_out);
        case IT_CORR_MFMA: case IT_CORR: return launch_corr_items(items, n, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace asi
