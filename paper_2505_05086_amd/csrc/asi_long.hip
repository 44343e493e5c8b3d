// Fused subspace-iteration step for modes with long fibres (64 < n <= 512, r <= 64): the
// channel mode of a conv activation, the token mode of a transformer activation.
//
// Both products of Alg. 1 for the mode, V = A_m^T U_prev and P = A_m V, are taken from ONE LDS
// tile of complete mode-m fibres: P = sum over fibres x of x (x^T U_prev).  V never exists in
// memory and the activation is read once for the mode.
//
// A tile holds TC = 16 NCB unfolding columns (fibres), all n <= 128 NRB entries of each, as
// Xs[i][c] in fp32.  Eight waves:
//   step A (fp32 MFMA 16x16x4)  V[c,q] = sum_i X[i,c] U[i,q]:  the mode index is split four ways and
//          the columns two ways among the waves; a wave keeps its rows of U in registers for the whole
//          kernel (B operands), reads its A operands from LDS at fixed offsets and leaves a partial V;
//          the four partial V's are added through LDS in fixed order and kept there as doubles.
//   step B (fp64 MFMA 16x16x4)  P[i,q] += sum_c X[i,c] V[c,q]:  wave w owns rows 16 NRB w .. of P in
//          registers for the whole kernel; K slot (s, lane group g) is column g TC/4 + s, so that a lane
//          reads four K steps of its A operand with one 16-byte LDS read.
// P is carried in fp64 (products of fp32 values are exact there): the columns of U_prev need not be
// aligned with singular vectors, so P holds components (sigma_r/sigma_1)^2 below its largest ones.
// The matrix pipe and the vector ALU of a SIMD do not run side by side on this chip, so the loops hold
// nothing but reads at immediate offsets, the widening of the A operand and the products.
//
// A workgroup owns a run of consecutive tiles and a block of 16 NBQ columns of U; it writes one fp64
// partial P (its rows x its columns) that the orthogonalisation sums in fixed order.
#include "asi_device.h"
#include "asi_kernels.h"

#include <atomic>
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int LG_NT = 512;                 // eight waves

struct LongJob {
    const void* X;
    const float* U;          // (n, r) previous factor
    double* part;            // (ncg, n, r) partial sums of P
    long long outer, inner, ncols;
    int n, r;
    int ntiles, tpw;         // column tiles of TC columns; consecutive tiles per workgroup
    int ncg, gy;             // column groups (= partial sums) x column blocks of U
    int32_t* zero;           // nullable: `nzero` int32 the kernel clears (arrival counters of later launches)
    int nzero;
};

extern __shared__ __align__(16) float lg_dyn[];

template <int NRB, int NCB, int NBQ>
struct LongShape {
    static constexpr int TC = 16 * NCB;
    static constexpr int LD = TC + 4;                 // Xs row pitch in floats: 16 bytes more than a multiple of 128
    static constexpr int NROW = 128 * NRB;
    static constexpr int VQ = 16 * NBQ;
    static constexpr int XS = NROW * LD;              // floats
    static constexpr int VP = 4 * TC * VQ;            // floats: four partial V
    static constexpr int VD = 2 * TC * VQ;            // floats: V as doubles
    static constexpr size_t lds_bytes = sizeof(float) * (size_t)(XS + VP + VD);
};

// pieces of a tile row as they travel from memory to LDS (VEC: four consecutive columns)
template <typename T, bool VEC> struct LongVec { typedef T type; };
template <> struct LongVec<float, true> { typedef v4f type; };
template <> struct LongVec<bf16_t, true> { typedef uint2 type; };
template <typename T, bool VEC, typename P>
__device__ __forceinline__ void long_store(float* dst, const P& v, bool ok) {
    if constexpr (!VEC) {
        *dst = ok ? to_f32(v) : 0.f;
    } else {
        v4f o;
        if constexpr (std::is_same<T, float>::value) {
            o = v;
        } else {
            o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
            o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        }
        const v4f z = {0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<v4f*>(dst) = ok ? o : z;
    }
}

// VEC: the inner extent is a multiple of 4 and X is aligned, so a thread moves four consecutive columns of a
// row with one 16-byte load (8 bytes for bf16) and one 16-byte LDS store: a quarter of the loader's instructions.
template <typename T, int NRB, int NCB, int NBQ, bool VEC>
__global__ __launch_bounds__(LG_NT) void k_subspace_long(Batch<LongJob> bt) {
    using SH = LongShape<NRB, NCB, NBQ>;
    constexpr int TC = SH::TC, LD = SH::LD, VQ = SH::VQ, NROW = SH::NROW;
    constexpr int HC = NCB / 2;                       // column blocks of a wave in step A
    constexpr int KSA = 8 * NRB;                      // K steps of a wave in step A (32 NRB rows)
    constexpr int W = VEC ? 4 : 1;                    // columns per piece
    constexpr int NLD = NROW * TC / W / LG_NT;        // tile pieces per thread
    constexpr int RSTEP = LG_NT / (TC / W);           // rows between a thread's consecutive pieces
    static_assert(NCB % 2 == 0 && TC % 16 == 0 && LG_NT % TC == 0, "tile shape");
    float* Xs = lg_dyn;
    float* Vp = lg_dyn + SH::XS;
    double* Vd = reinterpret_cast<double*>(lg_dyn + SH::XS + SH::VP);
    int lb;
    const LongJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const int n = jb.n, r = jb.r;
    const long long inner = jb.inner, ncols = jb.ncols;
    const int tid = threadIdx.x, lane = tid & 63, lg = lane >> 4, ll = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = wv & 3, ch = wv >> 2;              // step A: quarter of the mode index, half of the columns
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;
    const int cg = lb / jb.gy, qt = lb - cg * jb.gy;  // the column blocks of U of one column group are neighbours (one L2)
    const int q0 = qt * VQ;
    const int t_beg = cg * jb.tpw;
    const int t_end = (t_beg + jb.tpw < jb.ntiles) ? t_beg + jb.tpw : jb.ntiles;

    // rows of U this wave multiplies in step A: B operand (4 i x 16 q) of K step ks = U[32 NRB kq + 4 ks + lg][q0 + 16 nb + ll]
    float ureg[KSA][NBQ];
#pragma unroll
    for (int ks = 0; ks < KSA; ++ks)
#pragma unroll
        for (int nb = 0; nb < NBQ; ++nb) {
            const int i = 32 * NRB * kq + 4 * ks + lg, q = q0 + 16 * nb + ll;
            const bool ok = (i < n) & (q < r);
            const float u = jb.U[ok ? (long long)i * r + q : 0];
            ureg[ks][nb] = ok ? u : 0.f;
        }
    v4d pacc[NRB][NBQ];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NBQ; ++nb) pacc[rb][nb] = (v4d){0.0, 0.0, 0.0, 0.0};
    // rows n .. NROW - 1 of the tile stay zero for the whole kernel
    for (int e = tid; e < SH::XS; e += LG_NT) Xs[e] = 0.f;

    // loader: this thread's column of the tile and its first row; element offsets are 32-bit (host check)
    const int cl = W * (tid & (TC / W - 1)), r0 = tid / (TC / W);
    typename LongVec<T, VEC>::type pre[NLD];
    bool c_in = false;
    auto fetch = [&](int t) {
        const long long c = (long long)t * TC + cl;
        c_in = c < ncols;
        const long long cc = c_in ? c : 0;
        // quotient by a double division (exact below 2^52) with one correction step
        long long o = (long long)((double)cc / (double)inner);
        long long j = cc - o * inner;
        if (j < 0) { --o; j += inner; } else if (j >= inner) { ++o; j -= inner; }
        const unsigned base = (unsigned)(o * n * inner + j);
        const unsigned istep = (unsigned)inner;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int i = r0 + RSTEP * u;
            pre[u] = *reinterpret_cast<const typename LongVec<T, VEC>::type*>(X + (base + (unsigned)(i < n ? i : n - 1) * istep));   // clamped, not branched: all loads stay in flight
        }
    };
    if (t_beg < t_end) fetch(t_beg);
    for (int t = t_beg; t < t_end; ++t) {
        __syncthreads();                               // the previous tile is no longer read
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int i = r0 + RSTEP * u;
            if (i < n) long_store<T, VEC>(Xs + i * LD + cl, pre[u], c_in);
        }
        __syncthreads();
        if (t + 1 < t_end) fetch(t + 1);               // in flight during the products of this tile
        // ---- step A: partial V over this wave's rows, for its half of the columns
        {
            v4f vacc[HC][NBQ];
#pragma unroll
            for (int cb = 0; cb < HC; ++cb)
#pragma unroll
                for (int nb = 0; nb < NBQ; ++nb) vacc[cb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
            // A operand (16 columns x 4 i) of K step ks, column block cb: Xs[32 NRB kq + 4 ks + lg][16 cb + ll]
            const float* ap = Xs + (32 * NRB * kq + lg) * LD + 16 * HC * ch + ll;
#pragma unroll
            for (int ks = 0; ks < KSA; ++ks) {
                float a[HC];
#pragma unroll
                for (int cb = 0; cb < HC; ++cb) a[cb] = ap[4 * ks * LD + 16 * cb];
#pragma unroll
                for (int cb = 0; cb < HC; ++cb)
#pragma unroll
                    for (int nb = 0; nb < NBQ; ++nb)
                        vacc[cb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], ureg[ks][nb], vacc[cb][nb], 0, 0, 0);
            }
            // result layout: lane holds column 16 cb + 4 lg + v, output 16 nb + ll
            float* vp = Vp + kq * (TC * VQ) + (16 * HC * ch + 4 * lg) * VQ + ll;
#pragma unroll
            for (int cb = 0; cb < HC; ++cb)
#pragma unroll
                for (int nb = 0; nb < NBQ; ++nb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) vp[(16 * cb + v) * VQ + 16 * nb] = vacc[cb][nb][v];
        }
        __syncthreads();
        // ---- V = sum of the four partial V's (fixed order), rounded to fp32 like a stored V, kept as doubles
        for (int e = tid; e < TC * VQ; e += LG_NT) {
            const float v = ((Vp[e] + Vp[TC * VQ + e]) + Vp[2 * TC * VQ + e]) + Vp[3 * TC * VQ + e];
            Vd[e] = (double)v;
        }
        __syncthreads();
        // ---- step B: P[rows of this wave] += X V.  K slot (s, lg) is column lg TC/4 + s.
        {
            const float* xp = Xs + (16 * NRB * wv + ll) * LD + lg * (TC / 4);
            const double* vd = Vd + (lg * (TC / 4)) * VQ + ll;
#pragma unroll
            for (int s4 = 0; s4 < TC / 16; ++s4) {
                v4f xa[NRB];
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) xa[rb] = *reinterpret_cast<const v4f*>(xp + 16 * rb * LD + 4 * s4);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    double b[NBQ];
#pragma unroll
                    for (int nb = 0; nb < NBQ; ++nb) b[nb] = vd[(4 * s4 + s) * VQ + 16 * nb];
#pragma unroll
                    for (int rb = 0; rb < NRB; ++rb) {
                        const double a = (double)xa[rb][s];
#pragma unroll
                        for (int nb = 0; nb < NBQ; ++nb)
                            pacc[rb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b[nb], pacc[rb][nb], 0, 0, 0);
                    }
                }
            }
        }
    }
    // fp64 MFMA result layout: lane holds row lg + 4 v, column ll of its 16 x 16 block
    double* out = jb.part + (long long)cg * n * r;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NBQ; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * (NRB * wv + rb) + lg + 4 * v, q = q0 + 16 * nb + ll;
                if (i < n && q < r) out[(long long)i * r + q] = pacc[rb][nb][v];
            }
}

// ---- host side ---------------------------------------------------------------------------------
// shape of the instantiation that serves (n, r): rows, tile columns, columns of U per workgroup
static bool long_shape(int n, int r, int* nrb, int* ncb, int* nbq) {
    if (n <= 64 || n > 512 || r < 1 || r > 64 || r > n) return false;
    const int nb = (r + 15) / 16;
    if (n <= 128) { *nrb = 1; *ncb = 4; *nbq = nb > 3 ? 2 : nb; }
    else if (n <= 256) { *nrb = 2; *ncb = 4; *nbq = nb > 3 ? 2 : nb; }
    else { *nrb = 4; *ncb = 2; *nbq = nb > 2 ? 2 : nb; }
    return true;
}

// Every workgroup leaves a partial P of its own (n x r doubles), so the kernel pays off once the unfolding
// has enough columns to give each of 256 workgroups at least one tile: the partial sums then cost
// 2 r / (columns per workgroup) of the activation's bytes.  With fewer columns (late conv layers: 512
// channels over 3136 columns) the two-launch route, whose second product tiles the rows of P, moves less
// and is faster (measured on a 64 x 512 x 7 x 7 layer: 26 us for its two launches, 42 us fused).
bool subspace_long_supported(long long outer, int n, long long inner, int r) {
    int nrb, ncb, nbq;
    if (!long_shape(n, r, &nrb, &ncb, &nbq)) return false;
    if (outer * n * inner >= (1LL << 31)) return false;           // 32-bit element offsets inside the kernel
    return outer * inner >= 256LL * 16 * ncb;
}

static void long_geometry(long long outer, int n, long long inner, int r, LongJob* jb) {
    int nrb, ncb, nbq;
    long_shape(n, r, &nrb, &ncb, &nbq);
    const int tc = 16 * ncb;
    jb->ncols = outer * inner;
    jb->ntiles = (int)((jb->ncols + tc - 1) / tc);
    jb->gy = ((r + 15) / 16 + nbq - 1) / nbq;
    // one workgroup per CU (LDS): 256 / gy column groups
    int ncg = 256 / jb->gy;
    if (ncg < 1) ncg = 1;
    if (ncg > jb->ntiles) ncg = jb->ntiles;
    jb->tpw = (jb->ntiles + ncg - 1) / ncg;
    jb->ncg = (jb->ntiles + jb->tpw - 1) / jb->tpw;
}

int subspace_long_splits(long long outer, int n, long long inner, int r) {
    LongJob jb;
    std::memset(&jb, 0, sizeof(jb));
    long_geometry(outer, n, inner, r, &jb);
    return jb.ncg;
}

// key: [0] bf16, [1] 16-byte pieces, [4..7] NRB, [8..11] NCB, [12..15] NBQ
bool make_subspace_long(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r,
                        double* part, int nsplit, int32_t* zero, int nzero, Item* out) {
    if (!subspace_long_supported(outer, n, inner, r) || !X || !U || !part || nzero < 0 || nzero > 256) return false;
    LongJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.U = U; jb.part = part; jb.outer = outer; jb.inner = inner; jb.n = n; jb.r = r;
    jb.zero = zero; jb.nzero = zero ? nzero : 0;
    long_geometry(outer, n, inner, r, &jb);
    if (jb.ncg != nsplit) return false;
    int nrb, ncb, nbq;
    long_shape(n, r, &nrb, &ncb, &nbq);
    *out = Item();
    out->kind = IT_LONG;
    const size_t piece = xt == F32 ? 16 : 8;
    const bool vec = inner % 4 == 0 && reinterpret_cast<uintptr_t>(X) % piece == 0;
    out->key = (xt == BF16 ? 1u : 0u) | (vec ? 2u : 0u) | ((unsigned)nrb << 4) | ((unsigned)ncb << 8) | ((unsigned)nbq << 12);
    out->nblocks = jb.ncg * jb.gy;
    std::snprintf(out->label, sizeof(out->label), "k_subspace_long<%s, %d, %d, %d, %s>", xt == F32 ? "float" : "asi::bf16_t",
                  nrb, ncb, nbq, vec ? "true" : "false");
    static_assert(sizeof(LongJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

template <typename T, int NRB, int NCB, int NBQ, bool VEC>
static hipError_t launch_long_one(const Batch<LongJob>& b, dim3 grid, hipStream_t st) {
    constexpr size_t lds = LongShape<NRB, NCB, NBQ>::lds_bytes;
    static_assert(lds <= 160 * 1024, "LDS of a CU");
    if (lds > 65536) {                // more than a static array may take: allowed once per kernel
        static std::atomic<bool> allowed{false};
        if (!allowed.load()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_subspace_long<T, NRB, NCB, NBQ, VEC>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            allowed.store(true);
        }
    }
    hipLaunchKernelGGL((k_subspace_long<T, NRB, NCB, NBQ, VEC>), grid, LG_NT, lds, st, b);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_long_t(const Batch<LongJob>& b, dim3 grid, int nrb, int ncb, int nbq, bool vec, hipStream_t st) {
#define ASI_LONG_CASE(R, C, Q) if (nrb == R && ncb == C && nbq == Q) \
        return vec ? launch_long_one<T, R, C, Q, true>(b, grid, st) : launch_long_one<T, R, C, Q, false>(b, grid, st);
    ASI_LONG_CASE(1, 4, 1) ASI_LONG_CASE(1, 4, 2) ASI_LONG_CASE(1, 4, 3)
    ASI_LONG_CASE(2, 4, 1) ASI_LONG_CASE(2, 4, 2) ASI_LONG_CASE(2, 4, 3)
    ASI_LONG_CASE(4, 2, 1) ASI_LONG_CASE(4, 2, 2)
#undef ASI_LONG_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_long_items(const Item* const* items, int n, hipStream_t st) {
    Batch<LongJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int nrb = (int)((key >> 4) & 15u), ncb = (int)((key >> 8) & 15u), nbq = (int)((key >> 12) & 15u);
    const bool vec = (key & 2u) != 0;
    if (key & 1u) return launch_long_t<bf16_t>(b, grid, nrb, ncb, nbq, vec, st);
    return launch_long_t<float>(b, grid, nrb, ncb, nbq, vec, st);
}

}  // namespace asi
