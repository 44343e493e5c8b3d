// m-mode product along the LAST mode of a bf16 tensor on the bf16 MFMA (Eq. 4 with inner extent 1):
//     Y[c, q] = sum_i X[c, i] M[i, q],     X: (ncols, n) bf16 row-major,  M: (n, r) fp32,  Y: (ncols, r) fp32.
// Serves V = A_m^T U_prev for the hidden mode of a transformer activation (Alg. 1) and the first
// product of the core projection along that mode.
//
// The activation is exactly bf16; the fp32 factor is split once (k_split_bf16) into two bf16 terms,
// M = Mh + Ml with |M - Mh - Ml| <= 2^-17 |M|, and both terms are multiplied on
// v_mfma_f32_16x16x32_bf16 with fp32 accumulation: 2 x 16 cycles per 16 x 16 x 32 block against 8 x 32
// cycles on the fp32 MFMA.  The split factor is stored in the order the lanes read it,
//     Mb[term][k chunk of 32][q][4 lane groups][8 consecutive i],
// so that a chunk is copied to LDS as it is and a B operand (the 8 values of lane (q = l % 16, group l / 16))
// is one 16-byte LDS read.  A and B operands take their K indices from memory in the same way (lane
// group g, element e -> i = 32 chunk + 8 g + e), so the result does not depend on how the hardware numbers K.
//
// A workgroup (8 waves as WM x WN) owns 16 CBW WM columns and all r <= 48 WN outputs; K runs in chunks
// of 64 through two LDS buffers (one barrier per chunk), the next two chunks travelling in registers.
#include "asi_device.h"
#include "asi_kernels.h"

#include <atomic>
#include <cstdio>
#include <cstring>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int BG_NT = 512;

struct SplitJob {
    const float* M;          // (n, r), element (i, q) at M[i * ms_i + q * ms_q]
    long long ms_i, ms_q;
    unsigned short* Mb;      // [2][kchunks][rpad][4][8]
    int n, r, rpad, kchunks;
};
struct GemmBfJob {
    const void* X;           // (ncols, n) bf16
    const unsigned short* Mb;
    float* Y;                // (ncols, r), or (ksplit, ncols, r) partial products when ksplit > 1
    long long ncols;
    int n, r, rpad, kchunks;
    int ksplit, ntiles;      // workgroup lb: column tile lb % ntiles, K range lb / ntiles
    int32_t* zero;
    int nzero;
};

__device__ __forceinline__ unsigned short bf16_rne(float x) {
    unsigned u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

__global__ __launch_bounds__(256) void k_split_bf16(Batch<SplitJob> bt) {
    int lb;
    const SplitJob& jb = bt.job[locate(bt, &lb)];
    const long long total = (long long)jb.kchunks * jb.rpad * 32;
    const long long e = (long long)lb * 256 + threadIdx.x;
    if (e >= total) return;
    // e = ((kc * rpad + q) * 4 + g) * 8 + el
    const int el = (int)(e & 7), g = (int)((e >> 3) & 3);
    const long long t = e >> 5;
    const int q = (int)(t % jb.rpad), kc = (int)(t / jb.rpad);
    const int i = 32 * kc + 8 * g + el;
    const bool ok = i < jb.n && q < jb.r;
    const float x = ok ? jb.M[(long long)i * jb.ms_i + (long long)q * jb.ms_q] : 0.f;
    const unsigned short hi = bf16_rne(x);
    const float rest = x - __uint_as_float((unsigned)hi << 16);
    jb.Mb[e] = hi;
    jb.Mb[total + e] = bf16_rne(rest);
}

extern __shared__ __align__(16) unsigned char bg_dyn[];

constexpr int BG_KST = 2;                              // MFMA K steps (of 32) per chunk and barrier
constexpr int BG_APITCH_B = BG_KST * 64 + 16;          // bytes per A row in LDS: 16 more than a multiple of 128

template <int NBN, int WN, int CBW>
struct GemmShape {
    static constexpr int WM = 8 / WN;
    static constexpr int TCOLS = 16 * CBW * WM;
    static constexpr int RP = 16 * NBN * WN;                       // outputs the workgroup covers (>= rpad)
    static constexpr int A_BYTES = TCOLS * BG_APITCH_B;            // one buffer of the A tile
    static constexpr int B_BYTES = 2 * BG_KST * RP * 64;           // both terms of a chunk: RP outputs x 32 KST i x 2 bytes
    static constexpr int BUF = A_BYTES + B_BYTES;
    static constexpr size_t lds_bytes = 2 * (size_t)BUF;
};

// NBN: 16-blocks of outputs per wave, WN: waves along the outputs, CBW: 16-blocks of columns per wave.
// Chunk kc + 2 is requested while chunk kc is multiplied (two register sets), chunk kc + 1 sits in the
// other LDS buffer: a request has two chunks of products to arrive behind.
template <int NBN, int WN, int CBW>
__global__ __launch_bounds__(BG_NT) void k_gemm_bf16(Batch<GemmBfJob> bt) {
    using SH = GemmShape<NBN, WN, CBW>;
    constexpr int TCOLS = SH::TCOLS, RP = SH::RP, A_BYTES = SH::A_BYTES, BUF = SH::BUF;
    constexpr int NAL = TCOLS * BG_KST * 4 / BG_NT;               // 16-byte loads of A per thread and chunk
    constexpr int NBL = (SH::B_BYTES / 16 + BG_NT - 1) / BG_NT;   // 16-byte loads of B per thread and chunk
    static_assert(TCOLS * BG_KST * 4 % BG_NT == 0 && NAL >= 1, "whole 16-byte loads of A per thread");
    int lb;
    const GemmBfJob& jb = bt.job[locate(bt, &lb)];
    const unsigned short* __restrict__ X = static_cast<const unsigned short*>(jb.X);
    const unsigned short* __restrict__ Mb = jb.Mb;
    const int n = jb.n, r = jb.r, rpad = jb.rpad, kchunks = jb.kchunks;
    const int nck = (kchunks + BG_KST - 1) / BG_KST;              // chunks of this kernel
    const long long ncols = jb.ncols;
    const int tid = threadIdx.x, lane = tid & 63, lg = lane >> 4, ll = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wv / WN, wn = wv - wm * WN;
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    // Few columns (a (tokens x hidden) activation of some thousand tokens) make few column tiles: the
    // contraction is then split over `ksplit` workgroups per tile, each writing its partial product.
    const int kpart = lb / jb.ntiles, ctile = lb - kpart * jb.ntiles;
    const int ck_per = (nck + jb.ksplit - 1) / jb.ksplit;
    const int ck_beg = kpart * ck_per, ck_end = (ck_beg + ck_per < nck) ? ck_beg + ck_per : nck;
    float* __restrict__ Yout = jb.Y + (long long)kpart * ncols * r;
    const long long c0 = (long long)ctile * TCOLS;
    const long long term_stride = (long long)kchunks * rpad * 32;            // bf16 elements per term
    constexpr int PPR = BG_KST * 4;                                          // 16-byte pieces per A row and chunk

    v4u a_r[2][NAL], b_r[2][NBL];
    // A piece u of this thread: row (u * BG_NT + tid) / PPR of the tile, piece (..) % PPR of the row
    auto fetch = [&](int ck, v4u (&ar)[NAL], v4u (&br)[NBL]) {
#pragma unroll
        for (int u = 0; u < NAL; ++u) {
            const int p = u * BG_NT + tid, row = p / PPR, pc = p - row * PPR;
            // a piece beyond n is not read (rows are multiples of 8 long: host check), it is zero
            const bool in = (c0 + row < ncols) & (32 * BG_KST * ck + 8 * pc < n);
            const v4u v = *reinterpret_cast<const v4u*>(X + (in ? (c0 + row) * (long long)n + 32 * BG_KST * ck + 8 * pc : 0));
            ar[u] = in ? v : (v4u){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < NBL; ++u) {
            // piece p of the chunk: term, K step, then (q, lane group) as stored
            const int p = u * BG_NT + tid;
            const int per = rpad * 4;                 // pieces of one K step and term
            const int term = p / (BG_KST * per), rest = p - term * (BG_KST * per);
            const int ks = rest / per, pr = rest - ks * per;
            const int kc = BG_KST * ck + ks;
            const bool ok = (p < 2 * BG_KST * per) & (kc < kchunks);
            const v4u v = *reinterpret_cast<const v4u*>(Mb + (ok ? term * term_stride + ((long long)kc * per + pr) * 8 : 0));
            br[u] = ok ? v : (v4u){0u, 0u, 0u, 0u};
        }
    };
    auto stash = [&](int buf, const v4u (&ar)[NAL], const v4u (&br)[NBL]) {
        unsigned char* base = bg_dyn + buf * BUF;
#pragma unroll
        for (int u = 0; u < NAL; ++u) {
            const int p = u * BG_NT + tid, row = p / PPR, pc = p - row * PPR;
            *reinterpret_cast<v4u*>(base + row * BG_APITCH_B + pc * 16) = ar[u];
        }
#pragma unroll
        for (int u = 0; u < NBL; ++u) {
            const int p = u * BG_NT + tid;
            const int per = rpad * 4;
            const int term = p / (BG_KST * per), rest = p - term * (BG_KST * per);
            const int ks = rest / per, pr = rest - ks * per;
            if (p < 2 * BG_KST * per) *reinterpret_cast<v4u*>(base + A_BYTES + ((term * BG_KST + ks) * RP * 4 + pr) * 16) = br[u];
        }
    };

    v4f acc[CBW][NBN];
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int nb = 0; nb < NBN; ++nb) acc[cb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
    // outputs of this wave that exist at all (uniform): blocks beyond rpad are skipped
    const int nb_live = (rpad - 16 * NBN * wn + 15) / 16;

    if (ck_beg < ck_end) fetch(ck_beg, a_r[0], b_r[0]);
    if (ck_beg + 1 < ck_end) fetch(ck_beg + 1, a_r[1], b_r[1]);
    for (int ck = ck_beg; ck < ck_end; ck += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {                 // two chunks per trip: register set and LDS buffer h
            if (ck + h < ck_end) {
                stash(h, a_r[h], b_r[h]);
                __syncthreads();   // chunk ck + h is in LDS; every wave has finished the chunk before it (its buffer is free again)
                if (ck + h + 2 < ck_end) fetch(ck + h + 2, a_r[h], b_r[h]);
                const unsigned char* base = bg_dyn + h * BUF;
                const unsigned char* ap = base + (16 * CBW * wm + ll) * BG_APITCH_B + lg * 16;
                const unsigned char* bp = base + A_BYTES + ((16 * NBN * wn + ll) * 4 + lg) * 16;
#pragma unroll
                for (int ks = 0; ks < BG_KST; ++ks) {
                    v8bf a[CBW];
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb) a[cb] = *reinterpret_cast<const v8bf*>(ap + cb * 16 * BG_APITCH_B + ks * 64);
#pragma unroll
                    for (int nb = 0; nb < NBN; ++nb) {
                        if (nb < nb_live) {
                            const v8bf bh = *reinterpret_cast<const v8bf*>(bp + (ks * RP + nb * 16) * 64);
                            const v8bf bl = *reinterpret_cast<const v8bf*>(bp + ((BG_KST + ks) * RP + nb * 16) * 64);
#pragma unroll
                            for (int cb = 0; cb < CBW; ++cb) {
                                acc[cb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[cb], bl, acc[cb][nb], 0, 0, 0);
                                acc[cb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[cb], bh, acc[cb][nb], 0, 0, 0);
                            }
                        }
                    }
                }
            }
        }
    }
    // result layout: lane holds column 16 cb + 4 lg + v, output 16 nb + ll
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int nb = 0; nb < NBN; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long long c = c0 + 16 * (CBW * wm + cb) + 4 * lg + v;
                const int q = 16 * (NBN * wn + nb) + ll;
                if (c < ncols && q < r) Yout[c * r + q] = acc[cb][nb][v];
            }
}

// ---- host side ---------------------------------------------------------------------------------
static int bf_rpad(int r) { return (r + 15) / 16 * 16; }
static int bf_kchunks(int n) { return (n + 31) / 32; }

bool gemm_bf16_supported(long long ncols, int n, int r) {
    // 16-byte loads along a row: rows of a multiple of 8 elements; up to 192 outputs; enough work to pay for the split
    return n >= 64 && n % 8 == 0 && r >= 1 && r <= 192 && ncols >= 1024;
}
size_t split_bf16_elems(int n, int r) { return (size_t)2 * bf_kchunks(n) * bf_rpad(r) * 32; }

bool make_split_bf16(const float* M, long long ms_i, long long ms_q, int n, int r, unsigned short* Mb, Item* out) {
    if (!M || !Mb || n <= 0 || r <= 0) return false;
    SplitJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.M = M; jb.ms_i = ms_i; jb.ms_q = ms_q; jb.Mb = Mb; jb.n = n; jb.r = r; jb.rpad = bf_rpad(r); jb.kchunks = bf_kchunks(n);
    const long long total = (long long)jb.kchunks * jb.rpad * 32;
    *out = Item();
    out->kind = IT_SPLIT_BF16;
    out->nblocks = (int)((total + 255) / 256);
    std::snprintf(out->label, sizeof(out->label), "k_split_bf16");
    static_assert(sizeof(SplitJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

// shape of the instantiation: outputs per wave (16-blocks), waves along the outputs, column blocks per wave
static void gemm_shape(int r, int* nbn, int* wn, int* cbw) {
    const int nb = (r + 15) / 16;
    if (nb <= 2) { *nbn = nb; *wn = 1; *cbw = 1; }            // 8 waves x 16 columns
    else if (nb <= 3) { *nbn = 3; *wn = 1; *cbw = 1; }
    else if (nb <= 6) { *nbn = 3; *wn = 2; *cbw = 1; }        // 4 x 2 waves, 64 columns
    else { *nbn = 3; *wn = 4; *cbw = 4; }                     // 2 x 4 waves, 128 columns
}

static int gemm_tcols(int r) {
    int nbn, wn, cbw;
    gemm_shape(r, &nbn, &wn, &cbw);
    return 16 * cbw * (8 / wn);
}
// Workgroups per column tile: enough to give every CU one when the columns alone make fewer tiles, while
// each keeps at least four chunks of the contraction (a chunk is 64 elements long).
int gemm_bf16_ksplit(long long ncols, int n, int r) {
    const int tc = gemm_tcols(r);
    const long long tiles = (ncols + tc - 1) / tc;
    const int nck = (bf_kchunks(n) + BG_KST - 1) / BG_KST;
    if (tiles >= 128) return 1;
    long long ks = 256 / tiles;
    if (ks > nck / 4) ks = nck / 4;
    if (ks > 16) ks = 16;
    return ks < 2 ? 1 : (int)ks;
}

// key: [4..5] NBN, [8..10] WN, [12..13] CBW.  ksplit > 1: Y takes ksplit partial products of (ncols, r), to be summed.
bool make_gemm_bf16(const void* X, long long ncols, int n, const unsigned short* Mb, int r, float* Y, int ksplit,
                    int32_t* zero, int nzero, Item* out) {
    if (!gemm_bf16_supported(ncols, n, r) || !X || !Mb || !Y || nzero < 0 || nzero > 256) return false;
    if (ksplit < 1 || (ksplit != 1 && ksplit != gemm_bf16_ksplit(ncols, n, r))) return false;
    GemmBfJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.Mb = Mb; jb.Y = Y; jb.ncols = ncols; jb.n = n; jb.r = r; jb.rpad = bf_rpad(r); jb.kchunks = bf_kchunks(n);
    jb.zero = zero; jb.nzero = zero ? nzero : 0;
    int nbn, wn, cbw;
    gemm_shape(r, &nbn, &wn, &cbw);
    const int tcols = 16 * cbw * (8 / wn);
    const long long tiles = (ncols + tcols - 1) / tcols;
    const long long blocks = tiles * ksplit;
    if (blocks > 0x3fffffffLL) return false;
    jb.ksplit = ksplit; jb.ntiles = (int)tiles;
    *out = Item();
    out->kind = IT_GEMM_BF16;
    out->key = ((unsigned)nbn << 4) | ((unsigned)wn << 8) | ((unsigned)cbw << 12);
    out->nblocks = (int)blocks;
    std::snprintf(out->label, sizeof(out->label), "k_gemm_bf16<%d, %d, %d>", nbn, wn, cbw);
    static_assert(sizeof(GemmBfJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

template <int NBN, int WN, int CBW>
static hipError_t launch_gemm_one(const Batch<GemmBfJob>& b, dim3 grid, hipStream_t st) {
    constexpr size_t lds = GemmShape<NBN, WN, CBW>::lds_bytes;
    static_assert(lds <= 160 * 1024, "LDS of a CU");
    if (lds > 65536) {                // more than a static array may take: allowed once per kernel
        static std::atomic<bool> allowed{false};
        if (!allowed.load()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_bf16<NBN, WN, CBW>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            allowed.store(true);
        }
    }
    hipLaunchKernelGGL((k_gemm_bf16<NBN, WN, CBW>), grid, BG_NT, lds, st, b);
    return hipGetLastError();
}

hipError_t launch_bf16_items(const Item* const* items, int n, hipStream_t st) {
    dim3 grid;
    if (items[0]->kind == IT_SPLIT_BF16) {
        Batch<SplitJob> b;
        if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k_split_bf16, grid, 256, 0, st, b);
        return hipGetLastError();
    }
    Batch<GemmBfJob> b;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int nbn = (int)((key >> 4) & 3u), wn = (int)((key >> 8) & 7u), cbw = (int)((key >> 12) & 7u);
    if (wn == 1 && cbw == 1 && nbn == 1) return launch_gemm_one<1, 1, 1>(b, grid, st);
    if (wn == 1 && cbw == 1 && nbn == 2) return launch_gemm_one<2, 1, 1>(b, grid, st);
    if (wn == 1 && cbw == 1 && nbn == 3) return launch_gemm_one<3, 1, 1>(b, grid, st);
    if (wn == 2 && cbw == 1 && nbn == 3) return launch_gemm_one<3, 2, 1>(b, grid, st);
    if (wn == 4 && cbw == 4 && nbn == 3) return launch_gemm_one<3, 4, 4>(b, grid, st);
    return hipErrorInvalidValue;
}

}  // namespace asi
