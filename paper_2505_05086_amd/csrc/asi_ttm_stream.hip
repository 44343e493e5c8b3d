// m-mode product (Eq. 4) for large tensors whose contiguous index runs in multiples of four:
//   Y[o,q,j] = sum_i X[o,i,j] M(i,q),   r <= 64 outputs, not the last mode.
//
// The product reads X once and has little arithmetic per byte, so the kernel is built around the loads.
// A wave owns a span of 64 unfolding columns.  Lane (lg, ll) = (lane / 16, lane % 16) loads, for K step
// rows i = k + lg, the FOUR consecutive columns 4 ll .. 4 ll + 3 of the span with one 16-byte load (8 bytes
// for bf16): the 16 lanes of a row read 256 contiguous bytes.  Register v of that load is exactly the A
// operand (16 columns x 4 rows) of a 16x16x4 MFMA for the interleaved column block {4 l + v}: no LDS
// staging of X, no transposition, and a load instruction feeds 4 NBR MFMAs.  The result registers
// then hold, for output q = 16 nb + ll, the 16 consecutive columns 16 lg .. 16 lg + 15, which go to Y as
// 16-byte stores in runs of 256 bytes.
//
// The matrix (n x r, at most 96 KB padded) is staged once per workgroup in LDS, permuted so that one
// 16-byte read gives a lane its B operands of four K steps (a round of 16 rows).
//
// KW waves share a span and split the rounds between them (their partial tiles are added through LDS,
// in the space of the matrix); 4 / KW spans make a workgroup.  KW = 1 suits short modes over very many
// columns, KW = 4 long modes or few columns.
//
// k_ttm_stream_short: modes of 17..32 entries over very many columns (the batch mode of grad_out, G1 of
// Eq. 14).  A wave's whole fibre block is two rounds, and a lane's matrix operands are 8 words per block of
// 16 outputs, which it reads straight from memory (every wave of the launch reads the same few KB): no LDS,
// no barrier, a third of the registers, so four times as many waves stay resident per CU.  Such a launch
// has nothing but its loads to wait for, and the resident waves are what keeps them in flight.
#include "asi_device.h"
#include "asi_kernels.h"

#include <atomic>
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int TS_RP = 68;                 // pitch of a partial tile's row (64 columns) in floats
constexpr size_t TS_LDS_MAX = 96 * 1024;     // of the CU's 160 KB: a 512-long mode with 32 outputs takes 66 KB

extern __shared__ __align__(16) float ts_dyn[];

template <typename T> struct StreamPiece { typedef v4f type; };
template <> struct StreamPiece<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ v4f stream_widen(const v4f& p) { return p; }
__device__ __forceinline__ v4f stream_widen(const uint2& p) {
    v4f o;
    o[0] = __uint_as_float(p.x << 16); o[1] = __uint_as_float(p.x & 0xffff0000u);
    o[2] = __uint_as_float(p.y << 16); o[3] = __uint_as_float(p.y & 0xffff0000u);
    return o;
}

template <typename T, int NBR, int KW>
__global__ __launch_bounds__(256, 2) void k_ttm_stream(Batch<TtmJob> bt) {
    typedef typename StreamPiece<T>::type P;
    constexpr int SPANS = 4 / KW, QP = 16 * NBR;
    constexpr int RB = NBR <= 3 ? 4 : 2;                // rounds (of 16 rows) whose loads are in flight together
    int lb;
    const TtmJob& jb = bt.job[locate_xcd(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const float* __restrict__ Mp = jb.Mp;
    float* __restrict__ Y = jb.Y;
    const unsigned inner = (unsigned)jb.inner, ncols = (unsigned)(jb.outer * jb.inner);   // below 2^31 (host check)
    const int n = jb.n, r = jb.r, beta = jb.beta;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int span = wave / KW, kp = wave % KW;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;

    const int NR = (n + 15) >> 4;                       // rounds of the whole mode
    const int NRW = (NR + KW - 1) / KW;                 // rounds of a wave
    const int S0 = kp * NRW, S1 = (S0 + NRW < NR) ? S0 + NRW : NR;
    const int MP = 16 * NR + 4;                         // pitch of a matrix row in LDS (4 times an odd number)
    float* Ms = ts_dyn;                                 // [QP][MP]: output q, permuted mode index
    float* red = ts_dyn;                                // [4][QP][TS_RP] after the K loop

    // this lane's piece of the span, and where its fibre starts
    const unsigned cs = ((unsigned)lb * SPANS + span) * 64u;
    const unsigned c = cs + 4u * ll;
    const bool c_in = c < ncols;
    const unsigned cc = c_in ? c : 0u;                  // past the end: the first piece (valid), dropped at the store
    const unsigned o = cc / inner, j = cc - o * inner;
    const T* __restrict__ xp = X + ((size_t)o * n * inner + j);

    // The matrix goes to LDS as Ms[q][16 S + 4 lg + s] = M(16 S + 4 s + lg, q), zero for i >= n or q >= r, in
    // pieces of four outputs (the host checks that rows of M are contiguous, aligned and a multiple of four
    // long).  The first MU pieces of a thread are requested before X (loads return in order: the matrix must
    // not wait behind the tensor) and stored once X is on its way; a larger matrix takes further passes.
    const long long ms_i = jb.ms_i;
    constexpr int QP4 = QP / 4, MU = 8;
    const int npc = 16 * NR * QP4;                      // pieces of the padded matrix
    v4f mreg[MU];
    auto m_load = [&](int e0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            const int e = e0 + tid + 256 * u, i = e / QP4, q = 4 * (e - i * QP4);
            mreg[u] = *reinterpret_cast<const v4f*>(Mp + ((i < n && q < r) ? i * ms_i + q : 0LL));
        }
    };
    auto m_store = [&](int e0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            const int e = e0 + tid + 256 * u, i = e / QP4, q = 4 * (e - i * QP4);
            if (e < npc) {
                const bool ok = i < n && q < r;
                const int pos = (i & ~15) | ((i & 3) << 2) | ((i >> 2) & 3);
#pragma unroll
                for (int t = 0; t < 4; ++t) Ms[(q + t) * MP + pos] = ok ? mreg[u][t] : 0.f;
            }
        }
    };
    m_load(0);

    P x[RB][4];
    auto fetch = [&](int Sb) __attribute__((always_inline)) {
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            if (Sb + rr < S1) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int i = 16 * (Sb + rr) + 4 * s + lg;
                    // a row past n is read as row n - 1 and meets a zero row of the matrix
                    x[rr][s] = *reinterpret_cast<const P*>(xp + (unsigned)(i < n ? i : n - 1) * inner);
                }
            }
        }
    };
    if (S0 < S1) fetch(S0);

    m_store(0);
    for (int e0 = 256 * MU; e0 < npc; e0 += 256 * MU) {
        m_load(e0);
        m_store(e0);
    }
    __syncthreads();

    v4f acc[4][NBR];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) acc[v][nb] = (v4f){0.f, 0.f, 0.f, 0.f};

    for (int Sb = S0; Sb < S1; Sb += RB) {
        if (Sb != S0) fetch(Sb);
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            if (Sb + rr < S1) {
                v4f b[NBR];
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
                    b[nb] = *reinterpret_cast<const v4f*>(Ms + (16 * nb + ll) * MP + 16 * (Sb + rr) + 4 * lg);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const v4f a = stream_widen(x[rr][s]);
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb)
                            acc[v][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v], b[nb][s], acc[v][nb], 0, 0, 0);
                }
            }
        }
    }

    // acc[v][nb][e]: column cs + 16 lg + 4 e + v, output 16 nb + ll: a lane owns 64 contiguous bytes of one output
    // row, and a store from there would write 16-byte pieces 64 bytes apart in 16 rows.  The tiles go through
    // LDS (for KW > 1 the partial tiles meet there anyway) and a store instruction writes whole runs of a row.
    {
        __syncthreads();                                // every wave has read its last matrix operand
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const v4f out = {acc[0][nb][e], acc[1][nb][e], acc[2][nb][e], acc[3][nb][e]};
                *reinterpret_cast<v4f*>(red + ((wave * QP + 16 * nb + ll) * TS_RP + 16 * lg + 4 * e)) = out;
            }
        __syncthreads();
        // thread: piece pc of span sp, outputs q0, q0 + 16 / SPANS, ...
        const int pc = tid & 15, sp = (tid >> 4) % SPANS, q0 = tid / (16 * SPANS);
        const unsigned ce = ((unsigned)lb * SPANS + sp) * 64u + 4u * pc;
        if (ce < ncols) {
            const unsigned oe = ce / inner, je = ce - oe * inner;
            for (int q = q0; q < r; q += 16 / SPANS) {
                v4f out = *reinterpret_cast<const v4f*>(red + ((sp * KW * QP + q) * TS_RP + 4 * pc));
#pragma unroll
                for (int k = 1; k < KW; ++k)
                    out += *reinterpret_cast<const v4f*>(red + (((sp * KW + k) * QP + q) * TS_RP + 4 * pc));
                v4f* yp = reinterpret_cast<v4f*>(Y + (((size_t)oe * r + q) * inner + je));
                if (beta) out += *yp;
                *yp = out;
            }
        }
    }
}

template <typename T, int NBR>
__global__ __launch_bounds__(256, NBR <= 2 ? 4 : 2) void k_ttm_stream_short(Batch<TtmJob> bt) {
    typedef typename StreamPiece<T>::type P;
    __shared__ __align__(16) float ss_tile[4 * 16 * NBR * TS_RP];       // a result tile per wave
    int lb;
    const TtmJob& jb = bt.job[locate_xcd(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const float* __restrict__ Mp = jb.Mp;
    float* __restrict__ Y = jb.Y;
    const unsigned inner = (unsigned)jb.inner, ncols = (unsigned)(jb.outer * jb.inner);   // below 2^31 (host check)
    const int n = jb.n, r = jb.r, beta = jb.beta, msi = (int)jb.ms_i;                      // 32 ms_i below 2^31 (host check)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;

    const unsigned cs = ((unsigned)lb * 4u + wave) * 64u;
    const unsigned c = cs + 4u * ll;
    const unsigned cc = c < ncols ? c : 0u;             // past the end: the first piece (valid), dropped at the store
    const unsigned o = cc / inner, j = cc - o * inner;
    const T* __restrict__ xp = X + ((size_t)o * n * inner + j);

    // B operands: step s of round S multiplies row i = 16 S + 4 s + lg of the mode; this lane's output is 16 nb + ll.
    // Requested before X (loads return in order), from addresses valid for every lane, masked afterwards.
    float bm[2][NBR][4];
#pragma unroll
    for (int S = 0; S < 2; ++S)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int i = 16 * S + 4 * s + lg, q = 16 * nb + ll;
                bm[S][nb][s] = Mp[(i < n && q < r) ? i * msi + q : 0];
            }
    P x[2][4];
#pragma unroll
    for (int S = 0; S < 2; ++S)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int i = 16 * S + 4 * s + lg;
            // a row past n is read as row n - 1 and meets a zero of the matrix
            x[S][s] = *reinterpret_cast<const P*>(xp + (unsigned)(i < n ? i : n - 1) * inner);
        }
#pragma unroll
    for (int S = 0; S < 2; ++S)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int i = 16 * S + 4 * s + lg, q = 16 * nb + ll;
                bm[S][nb][s] = (i < n && q < r) ? bm[S][nb][s] : 0.f;
            }

    v4f acc[4][NBR];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) acc[v][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int S = 0; S < 2; ++S)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const v4f a = stream_widen(x[S][s]);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
                    acc[v][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v], bm[S][nb][s], acc[v][nb], 0, 0, 0);
        }

    // acc[v][nb][e]: column cs + 16 lg + 4 e + v, output 16 nb + ll: a lane owns 64 contiguous bytes of one output
    // row.  Stored from there, an instruction would write 16-byte pieces 64 bytes apart in 16 rows; the tile goes
    // through the wave's own LDS block instead (LDS serves a wave's accesses in order: no barrier), and every
    // store instruction then writes four whole rows of the span, 256 contiguous bytes each, like the loads.
    float* tile = ss_tile + wave * (16 * NBR * TS_RP);
#pragma unroll
    for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const v4f out = {acc[0][nb][e], acc[1][nb][e], acc[2][nb][e], acc[3][nb][e]};
            *reinterpret_cast<v4f*>(tile + (16 * nb + ll) * TS_RP + 16 * lg + 4 * e) = out;
        }
    const unsigned ce = cs + 4u * ll;                   // this lane's piece of every row
    if (ce < ncols) {
        const unsigned oe = ce / inner, je = ce - oe * inner;
        float* yb = Y + ((size_t)oe * r * inner + je);
#pragma unroll
        for (int k = 0; k < 4 * NBR; ++k) {
            const int q = 4 * k + lg;
            if (q < r) {
                v4f out = *reinterpret_cast<const v4f*>(tile + q * TS_RP + 4 * ll);
                v4f* yp = reinterpret_cast<v4f*>(yb + (size_t)q * inner);
                if (beta) out += *yp;
                *yp = out;
            }
        }
    }
}

// ---- host side -----------------------------------------------------------------------------------
static size_t stream_lds(int n, int nbr, int kw) {
    const size_t ms = sizeof(float) * (size_t)(16 * nbr) * (size_t)(16 * ((n + 15) / 16) + 4);
    const size_t rd = sizeof(float) * 4u * (size_t)(16 * nbr) * TS_RP;       // the four waves' result tiles
    (void)kw;
    return ms > rd ? ms : rd;
}

// waves per span: the fewest that still give every CU two workgroups, and every wave a round
static int stream_kw(long long ncols, int n) {
    const long long spans = (ncols + 63) / 64;
    int kw = 1;
    while (kw < 4 && (spans * kw / 4 < 512 || n > 64 * kw) && n >= 32 * kw) kw *= 2;
    return kw;
}

bool ttm_stream_supported(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp,
                          long long ms_i, long long ms_q, int r, const float* Y) {
    if (ms_q != 1 || ms_i % 4 != 0 || r % 4 != 0 || reinterpret_cast<uintptr_t>(Mp) % 16 != 0) return false;
    if (inner < 4 || inner % 4 != 0 || r > 64 || n < 16) return false;
    if (outer * inner >= (1LL << 31) - 256 || (long long)n * inner >= (1LL << 31)) return false;
    if (reinterpret_cast<uintptr_t>(X) % (xt == F32 ? 16 : 8) != 0 || reinterpret_cast<uintptr_t>(Y) % 16 != 0) return false;
    const int nbr = (r + 15) / 16;
    return stream_lds(n, nbr, 4) <= TS_LDS_MAX;
}

// key: [0] bf16, [4..6] NBR - 1, [8..10] KW, [12] k_ttm_stream_short
bool make_ttm_stream(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                     long long ms_q, int r, float* Y, int beta, Item* out) {
    if (!X || !Mp || !Y || !ttm_stream_supported(xt, X, outer, n, inner, Mp, ms_i, ms_q, r, Y)) return false;
    TtmJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.outer = outer; jb.inner = inner; jb.Mp = Mp; jb.ms_i = ms_i; jb.ms_q = ms_q; jb.Y = Y;
    jb.n = n; jb.r = r; jb.beta = beta;
    const long long ncols = outer * inner;
    const int nbr = (r + 15) / 16, kw = stream_kw(ncols, n);
    const long long wcols = 64LL * (4 / kw);
    jb.gx = (int)((ncols + wcols - 1) / wcols); jb.gy = 1;
    *out = Item();
    out->kind = IT_TTM_STREAM;
    const bool shrt = kw == 1 && n > 16 && n <= 32 && ms_i < (1LL << 25);
    out->key = (xt == BF16 ? 1u : 0u) | ((unsigned)(nbr - 1) << 4) | ((unsigned)kw << 8) | (shrt ? 1u << 12 : 0u);
    out->nblocks = jb.gx;
    if (shrt) std::snprintf(out->label, sizeof(out->label), "k_ttm_stream_short<%s, %d>", xt == F32 ? "float" : "asi::bf16_t", nbr);
    else std::snprintf(out->label, sizeof(out->label), "k_ttm_stream<%s, %d, %d>", xt == F32 ? "float" : "asi::bf16_t", nbr, kw);
    static_assert(sizeof(TtmJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

template <typename T, int NBR, int KW>
static hipError_t launch_stream_one(const Batch<TtmJob>& b, dim3 grid, size_t lds, hipStream_t st) {
    if (lds > 65536) {                // more than a static array may take: allowed once per kernel
        static std::atomic<bool> allowed{false};
        if (!allowed.load()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_ttm_stream<T, NBR, KW>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)TS_LDS_MAX);
            if (e != hipSuccess) return e;
            allowed.store(true);
        }
    }
    hipLaunchKernelGGL((k_ttm_stream<T, NBR, KW>), grid, 256, lds, st, b);
    return hipGetLastError();
}
template <typename T, int NBR>
static hipError_t launch_stream_kw(int kw, const Batch<TtmJob>& b, dim3 grid, size_t lds, hipStream_t st) {
    if (kw == 1) return launch_stream_one<T, NBR, 1>(b, grid, lds, st);
    if (kw == 2) return launch_stream_one<T, NBR, 2>(b, grid, lds, st);
    return launch_stream_one<T, NBR, 4>(b, grid, lds, st);
}
template <typename T>
static hipError_t launch_stream_short_t(int nbr, const Batch<TtmJob>& b, dim3 grid, hipStream_t st) {
    switch (nbr) {
        case 1: hipLaunchKernelGGL((k_ttm_stream_short<T, 1>), grid, 256, 0, st, b); break;
        case 2: hipLaunchKernelGGL((k_ttm_stream_short<T, 2>), grid, 256, 0, st, b); break;
        case 3: hipLaunchKernelGGL((k_ttm_stream_short<T, 3>), grid, 256, 0, st, b); break;
        default: hipLaunchKernelGGL((k_ttm_stream_short<T, 4>), grid, 256, 0, st, b); break;
    }
    return hipGetLastError();
}
template <typename T>
static hipError_t launch_stream_t(int nbr, int kw, const Batch<TtmJob>& b, dim3 grid, size_t lds, hipStream_t st) {
    switch (nbr) {
        case 1: return launch_stream_kw<T, 1>(kw, b, grid, lds, st);
        case 2: return launch_stream_kw<T, 2>(kw, b, grid, lds, st);
        case 3: return launch_stream_kw<T, 3>(kw, b, grid, lds, st);
        default: return launch_stream_kw<T, 4>(kw, b, grid, lds, st);
    }
}

hipError_t launch_ttm_stream_items(const Item* const* items, int n, hipStream_t st) {
    Batch<TtmJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int nbr = (int)((key >> 4) & 7u) + 1, kw = (int)((key >> 8) & 7u);
    if ((key >> 12) & 1u) {                             // the short form holds exactly two rounds of a mode
        for (int j = 0; j < n; ++j) {
            TtmJob tj;
            std::memcpy(&tj, items[j]->arg, sizeof(tj));
            if (tj.n <= 16 || tj.n > 32 || tj.ms_i >= (1LL << 25)) return hipErrorInvalidValue;
        }
        if (key & 1u) return launch_stream_short_t<bf16_t>(nbr, b, grid, st);
        return launch_stream_short_t<float>(nbr, b, grid, st);
    }
    size_t lds = 0;
    for (int j = 0; j < n; ++j) {                       // items of one launch share the instantiation; the largest matrix sizes the LDS
        TtmJob tj;
        std::memcpy(&tj, items[j]->arg, sizeof(tj));
        const size_t l = stream_lds(tj.n, nbr, kw);
        lds = l > lds ? l : lds;
    }
    if (lds > TS_LDS_MAX) return hipErrorInvalidValue;
    if (key & 1u) return launch_stream_t<bf16_t>(nbr, kw, b, grid, lds, st);
    return launch_stream_t<float>(nbr, kw, b, grid, lds, st);
}

}  // namespace asi
