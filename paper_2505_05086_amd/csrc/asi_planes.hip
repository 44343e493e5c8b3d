// Fused subspace-iteration step for the LAST TWO modes of a tensor seen as (planes, rows, cols) when
// the planes are large (33..64 rows and columns, ranks up to 32): the H and W modes of a high-resolution
// conv activation.  Both modes come from one read of the activation, and V never exists in memory.
//
// For one plane X (rows x cols), with the previous factors U_H (rows x rH) and U_W (cols x rW)  (Alg. 1):
//     mode H:   V = X^T U_H  (cols x rH),    P_H += X   V   (rows x rH)
//     mode W:   V = X   U_W  (rows x rW),    P_W += X^T V   (cols x rW)
// A tile is four consecutive planes in LDS (row pitch 68 floats).  Eight waves: wave w < 4 takes mode H of
// plane w, wave w + 4 takes mode W of the same plane; each keeps its P (fp64) and its factor (as MFMA B
// operands) in registers for the whole kernel, so the waves never exchange anything between tiles.
// Step A runs on fp32 MFMA 16x16x4, step B on fp64 MFMA 16x16x4 (products of fp32 values are exact in
// fp64, and P holds components far below its largest ones).  The result layout of step A (lane l,
// register v: row 4 (l / 16) + v, column l % 16) is the B-operand layout of step B if K slot (v, l / 16)
// of a 16-block stands for index 16 block + 4 (l / 16) + v; the A operands are read from LDS in that order
// (one 16-byte read gives a lane four K steps where the index runs along a row of the plane).
// The matrix pipe and the vector ALU of a SIMD do not run side by side, so the loops hold only reads at
// immediate offsets, the widening to fp64 and the products.
#include "asi_device.h"
#include "asi_kernels.h"

#include <atomic>
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int PN_NT = 512;                 // eight waves
constexpr int PN_PL = 4;                   // planes per tile
constexpr int PN_LD = 68;                  // row pitch in floats: 16 bytes more than a multiple of 128

struct PlanesJob {
    const void* X;
    long long planes, ntiles;
    const float* U[2];       // (rows, r[0]) and (cols, r[1])
    double* part[2];         // (nwg, rows, r[0]) and (nwg, cols, r[1])
    int rows, cols, r[2];
    int nwg;
    int32_t* zero;           // nullable: `nzero` int32 the kernel clears
    int nzero;
};

extern __shared__ __align__(16) float pn_dyn[];

// pieces of a plane row as they travel from memory to LDS
template <typename T, bool VEC> struct PlaneVec { typedef T type; };
template <> struct PlaneVec<float, true> { typedef v4f type; };
template <> struct PlaneVec<bf16_t, true> { typedef uint2 type; };
template <typename T, bool VEC, typename P>
__device__ __forceinline__ void plane_store(float* dst, const P& v, bool ok) {
    if constexpr (!VEC) {
        *dst = ok ? to_f32(v) : 0.f;
    } else if constexpr (std::is_same<T, float>::value) {
        const v4f z = {0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<v4f*>(dst) = ok ? v : z;
    } else {
        v4f o;
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        const v4f z = {0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<v4f*>(dst) = ok ? o : z;
    }
}

template <typename T, int NBM, int NBR, bool VEC>
__global__ __launch_bounds__(PN_NT) void k_subspace_planes(Batch<PlanesJob> bt) {
    constexpr int PF = 16 * NBM * PN_LD;              // floats of one plane in LDS
    constexpr int NLD = (PN_PL * 256 * NBM * NBM + PN_NT - 1) / PN_NT;    // elements per thread and tile (planes of up to 16 NBM squared)
    constexpr int RQ = 16 * NBR;
    float* Xs = pn_dyn;                               // PN_PL planes (the reduction buffer at the end), then the factors
    int lb;
    const PlanesJob& jb = bt.job[locate(bt, &lb)];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const int rows = jb.rows, cols = jb.cols, pe = rows * cols;
    const int tid = threadIdx.x, lane = tid & 63, lg = lane >> 4, ll = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wv >> 2, slot = wv & 3;          // role 0: mode H (rows), role 1: mode W (cols)
    if (jb.zero && lb == 0 && tid < jb.nzero) jb.zero[tid] = 0;

    // A tile is moved in pieces of W consecutive elements of a plane row: W = 4 (one 16-byte load, 8 bytes for
    // bf16, and one 16-byte LDS store) when rows are a multiple of 4 long and X is aligned, else single
    // elements.  The piece -> (plane, row, column) arithmetic is per piece, so the wide form needs a quarter of
    // it, and a quarter of the load and store instructions; all of them are issued by the waves that also
    // multiply, at the expense of the products.
    constexpr int W = VEC ? 4 : 1;
    constexpr int NLDW = (NLD + W - 1) / W;           // pieces per thread and tile
    const int ppr = cols / W, ppp = rows * ppr;       // pieces per row and per plane (VEC: cols % 4 == 0)
    const float inv_ppp = 1.0f / (float)ppp, inv_ppr = 1.0f / (float)ppr;
    typename PlaneVec<T, VEC>::type pre[NLDW];
    auto fetch = [&](long long t) __attribute__((always_inline)) {
        const long long p0 = t * PN_PL;
        const int np = (int)((jb.planes - p0 < PN_PL) ? jb.planes - p0 : PN_PL);
        const int count = np * ppp;
        const T* src = X + p0 * pe;
#pragma unroll
        for (int u = 0; u < NLDW; ++u) {
            const int e = u * PN_NT + tid;
            pre[u] = *reinterpret_cast<const typename PlaneVec<T, VEC>::type*>(src + (e < count ? e * W : 0));   // clamped, not branched: all loads stay in flight
        }
    };
    if (lb < jb.ntiles) fetch(lb);                    // on its way while the factors are staged

    // The factor as B operands of step A, kept in LDS in the order the lanes read it (registers are needed
    // for P): element [ks][nb][lane] is
    //   role 0: K slot (ks, lg) is row 4 ks + lg:                          U_H[4 ks + lg][16 nb + ll]
    //   role 1: K slot (v, lg) of block cb, ks = 4 cb + v, is column 16 cb + 4 lg + v:  U_W[16 cb + 4 lg + v][16 nb + ll]
    float* Us = pn_dyn + PN_PL * PF;                  // [2][4 NBM][NBR][64]
    // (all loads first, from addresses valid for every lane, then the stores: written as a loop of load and
    // store, every element paid its own round trip to memory)
    {
        constexpr int NU = 2 * 4 * NBM * NBR * 64 / PN_NT;
        static_assert(NU * PN_NT == 2 * 4 * NBM * NBR * 64, "whole passes");
        const float* U0 = jb.U[0];
        const float* U1 = jb.U[1];
        const int r0 = jb.r[0], r1 = jb.r[1];
        float ut[NU];
        bool uok[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int e = tid + PN_NT * u;
            const int l = e & 63, nb = (e >> 6) % NBR, ks = ((e >> 6) / NBR) % (4 * NBM), ro = (e >> 6) / (NBR * 4 * NBM);
            const int g = l >> 4, c = l & 15;
            const int i = ro ? 16 * (ks >> 2) + 4 * g + (ks & 3) : 4 * ks + g, q = 16 * nb + c;
            const int nn = ro ? cols : rows, rr = ro ? r1 : r0;
            uok[u] = (i < nn) & (q < rr);
            ut[u] = (ro ? U1 : U0)[uok[u] ? i * rr + q : 0];
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) Us[tid + PN_NT * u] = uok[u] ? ut[u] : 0.f;
    }
    const float* ureg = Us + role * (4 * NBM * NBR * 64) + lane;      // ureg[(ks * NBR + nb) * 64]
    v4d pacc[NBM][NBR];
#pragma unroll
    for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBR; ++nb) pacc[mb][nb] = (v4d){0.0, 0.0, 0.0, 0.0};
    // rows and columns beyond the plane stay zero for the whole kernel (a plane that fills its blocks has none:
    // the pitch's spare columns are never read)
    if (rows < 16 * NBM || cols < 16 * NBM)
        for (int e = tid; e < PN_PL * PF; e += PN_NT) Xs[e] = 0.f;

    for (long long t = lb; t < jb.ntiles; t += jb.nwg) {
        const long long p0 = t * PN_PL;
        const int np = (int)((jb.planes - p0 < PN_PL) ? jb.planes - p0 : PN_PL);
        const int count = np * ppp;
        __syncthreads();                              // the previous tile is no longer read
#pragma unroll
        for (int u = 0; u < NLDW; ++u) {
            int e = u * PN_NT + tid;                  // e < 2^15: the rounded float quotients are exact
            asm volatile("" : "+v"(e));               // (recomputed per tile: hoisted out of the loop, the offsets cost a register each)
            const int pl = (int)(((float)e + 0.5f) * inv_ppp), rem = e - pl * ppp;
            const int i = (int)(((float)rem + 0.5f) * inv_ppr), c = (rem - i * ppr) * W;
            if (e < PN_PL * ppp) plane_store<T, VEC>(Xs + pl * PF + i * PN_LD + c, pre[u], e < count);
        }
        __syncthreads();
        if (t + jb.nwg < jb.ntiles) fetch(t + jb.nwg);    // in flight during the products of this tile
        if (slot >= np) continue;                     // (uniform per wave; the barriers above are passed by all)
        const float* xp = Xs + slot * PF;
        if (role == 0) {
            // ---- mode H, step A: V[c,q] = sum_i X[i,c] U_H[i,q]; A operand (16 c x 4 i) = X[4 ks + lg][16 cb + ll]
            v4f vacc[NBM][NBR];
#pragma unroll
            for (int cb = 0; cb < NBM; ++cb)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) vacc[cb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
            const float* ap = xp + lg * PN_LD + ll;
#pragma unroll
            for (int ks = 0; ks < 4 * NBM; ++ks) {
                if (4 * ks < rows) {                  // uniform: K steps beyond the plane are skipped
                    float a[NBM], ub[NBR];
#pragma unroll
                    for (int cb = 0; cb < NBM; ++cb) a[cb] = ap[4 * ks * PN_LD + 16 * cb];
#pragma unroll
                    for (int nb = 0; nb < NBR; ++nb) ub[nb] = ureg[(ks * NBR + nb) * 64];
#pragma unroll
                    for (int cb = 0; cb < NBM; ++cb)
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb)
                            vacc[cb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], ub[nb], vacc[cb][nb], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);    // (keeps the reads of later steps from being hoisted: registers)
                }
            }
            // ---- step B: P_H[i,q] += sum_c X[i,c] V[c,q]; K slot (v, lg) of block cb = column 16 cb + 4 lg + v
            const float* bp = xp + ll * PN_LD + 4 * lg;
#pragma unroll
            for (int cb = 0; cb < NBM; ++cb) {
                if (16 * cb < cols) {
                    double b[4][NBR];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb) b[v][nb] = (double)vacc[cb][nb][v];
#pragma unroll
                    for (int rb = 0; rb < NBM; ++rb) {
                        const v4f xa = *reinterpret_cast<const v4f*>(bp + 16 * rb * PN_LD + 16 * cb);
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const double a = (double)xa[v];
#pragma unroll
                            for (int nb = 0; nb < NBR; ++nb)
                                pacc[rb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b[v][nb], pacc[rb][nb], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        } else {
            // ---- mode W, step A: V[i,q] = sum_c X[i,c] U_W[c,q]; A operand (16 i x 4 c): K slot (v, lg) of block cb
            //      = column 16 cb + 4 lg + v, so one 16-byte read of X[16 rb + ll][16 cb + 4 lg ..] gives four K steps
            v4f vacc[NBM][NBR];
#pragma unroll
            for (int rb = 0; rb < NBM; ++rb)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb) vacc[rb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};
            const float* bp = xp + ll * PN_LD + 4 * lg;
#pragma unroll
            for (int cb = 0; cb < NBM; ++cb) {
                if (16 * cb < cols) {
                    float ub[4][NBR];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb) ub[v][nb] = ureg[((4 * cb + v) * NBR + nb) * 64];
#pragma unroll
                    for (int rb = 0; rb < NBM; ++rb) {
                        const v4f xa = *reinterpret_cast<const v4f*>(bp + 16 * rb * PN_LD + 16 * cb);
#pragma unroll
                        for (int v = 0; v < 4; ++v)
#pragma unroll
                            for (int nb = 0; nb < NBR; ++nb)
                                vacc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[v], ub[v][nb], vacc[rb][nb], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            // ---- step B: P_W[c,q] += sum_i X[i,c] V[i,q]; K slot (v, lg) of block rb = row 16 rb + 4 lg + v;
            //      A operand (16 c x 4 i) = X[16 rb + 4 lg + v][16 cb + ll]
            const float* ap = xp + 4 * lg * PN_LD + ll;
#pragma unroll
            for (int rb = 0; rb < NBM; ++rb) {
                if (16 * rb < rows) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        double b[NBR];
#pragma unroll
                        for (int nb = 0; nb < NBR; ++nb) b[nb] = (double)vacc[rb][nb][v];
#pragma unroll
                        for (int cb = 0; cb < NBM; ++cb) {
                            const double a = (double)ap[(16 * rb + v) * PN_LD + 16 * cb];
#pragma unroll
                            for (int nb = 0; nb < NBR; ++nb)
                                pacc[cb][nb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b[nb], pacc[cb][nb], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    }
    // The four waves of a mode put their P side by side in LDS (in the space of the tiles) and all threads add
    // the four in a fixed order, mode H first.
    // fp64 MFMA result layout: lane holds row lg + 4 v, column ll of its 16 x 16 block.
    constexpr int RED = 16 * NBM * RQ;                // doubles of one wave's P
    static_assert(sizeof(double) * 4 * RED <= sizeof(float) * PN_PL * PF, "four partial P fit the tiles");
    double* red = reinterpret_cast<double*>(pn_dyn);
#pragma unroll
    for (int md = 0; md < 2; ++md) {
        __syncthreads();                              // the tiles (or the other mode's P) are no longer read
        if (role == md) {
#pragma unroll
            for (int mb = 0; mb < NBM; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBR; ++nb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        red[slot * RED + (16 * mb + lg + 4 * v) * RQ + 16 * nb + ll] = pacc[mb][nb][v];
        }
        __syncthreads();
        const int n = md ? cols : rows, r = jb.r[md];
        double* out = jb.part[md] + (long long)lb * n * r;
        const float inv_r = 1.0f / (float)r;
        for (int e = tid; e < n * r; e += PN_NT) {    // e < 2^11: exact
            const int i = (int)(((float)e + 0.5f) * inv_r), q = e - i * r;
            const double* p = red + i * RQ + q;
            out[e] = ((p[0] + p[RED]) + p[2 * RED]) + p[3 * RED];
        }
    }
}

// ---- host side ---------------------------------------------------------------------------------
bool subspace_planes_supported(long long planes, int rows, int cols, int r_rows, int r_cols) {
    if (rows < 33 || rows > 64 || cols < 33 || cols > 64) return false;
    if ((rows + 15) / 16 != (cols + 15) / 16) return false;               // one register shape for both modes
    if (r_rows < 1 || r_cols < 1 || r_rows > 32 || r_cols > 32 || r_rows > rows || r_cols > cols) return false;
    return planes >= 4 * 256;         // a tile of four planes for every CU; below that the general kernel spreads the work further
}
int subspace_planes_nwg(long long planes) {
    const long long ntiles = (planes + PN_PL - 1) / PN_PL;
    return (int)(ntiles < 256 ? ntiles : 256);
}

// key: [0] bf16, [1] 16-byte pieces, [4..6] NBM, [8..9] NBR
bool make_subspace_planes(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                          double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, int32_t* zero,
                          int nzero, Item* out) {
    if (!subspace_planes_supported(planes, rows, cols, r_rows, r_cols) || !X || !U_rows || !U_cols || !part_rows || !part_cols)
        return false;
    if (nzero < 0 || nzero > 256) return false;
    PlanesJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.X = X; jb.planes = planes; jb.ntiles = (planes + PN_PL - 1) / PN_PL;
    jb.U[0] = U_rows; jb.U[1] = U_cols; jb.part[0] = part_rows; jb.part[1] = part_cols;
    jb.rows = rows; jb.cols = cols; jb.r[0] = r_rows; jb.r[1] = r_cols; jb.nwg = nwg;
    jb.zero = zero; jb.nzero = zero ? nzero : 0;
    if (nwg <= 0 || nwg > jb.ntiles) return false;
    const int nbm = (rows + 15) / 16, nbr = ((r_rows > r_cols ? r_rows : r_cols) + 15) / 16;
    *out = Item();
    out->kind = IT_PLANES;
    const bool vec = cols % 4 == 0 && reinterpret_cast<uintptr_t>(X) % (xt == F32 ? 16 : 8) == 0;
    out->key = (xt == BF16 ? 1u : 0u) | (vec ? 2u : 0u) | ((unsigned)nbm << 4) | ((unsigned)nbr << 8);
    out->nblocks = nwg;
    std::snprintf(out->label, sizeof(out->label), "k_subspace_planes<%s, %d, %d, %s>", xt == F32 ? "float" : "asi::bf16_t", nbm, nbr,
                  vec ? "true" : "false");
    static_assert(sizeof(PlanesJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

template <typename T, int NBM, int NBR, bool VEC>
static hipError_t launch_planes_one(const Batch<PlanesJob>& b, dim3 grid, hipStream_t st) {
    constexpr size_t lds = sizeof(float) * ((size_t)PN_PL * 16 * NBM * PN_LD + 2 * 4 * NBM * NBR * 64);
    if (lds > 65536) {                // more than a static array may take: allowed once per kernel
        static std::atomic<bool> allowed{false};
        if (!allowed.load()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_subspace_planes<T, NBM, NBR, VEC>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            allowed.store(true);
        }
    }
    hipLaunchKernelGGL((k_subspace_planes<T, NBM, NBR, VEC>), grid, PN_NT, lds, st, b);
    return hipGetLastError();
}

hipError_t launch_planes_items(const Item* const* items, int n, hipStream_t st) {
    Batch<PlanesJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    const unsigned key = items[0]->key;
    const int nbm = (int)((key >> 4) & 7u), nbr = (int)((key >> 8) & 3u);
    const bool bf = key & 1u, vec = key & 2u;
#define ASI_PLANES_CASE(M, R)                                                                                               \
    if (nbm == M && nbr == R) {                                                                                             \
        if (vec) return bf ? launch_planes_one<bf16_t, M, R, true>(b, grid, st) : launch_planes_one<float, M, R, true>(b, grid, st);    \
        return bf ? launch_planes_one<bf16_t, M, R, false>(b, grid, st) : launch_planes_one<float, M, R, false>(b, grid, st);           \
    }
    ASI_PLANES_CASE(3, 1) ASI_PLANES_CASE(3, 2) ASI_PLANES_CASE(4, 1) ASI_PLANES_CASE(4, 2)
#undef ASI_PLANES_CASE
    return hipErrorInvalidValue;
}

}  // namespace asi
