// Orthogonalize (Alg. 1): Q factor of the thin QR of P with positive diagonal R, in fp64.
//
// Method: Cholesky-QR with a diagonal shift on the first pass (safe for cond(P) up to
// ~1e9, far beyond what a Gram matrix alone allows), followed by plain Cholesky-QR:
//     pass 0: G = P^T P + s I = R0^T R0,  Q0 = P R0^-1        cond(Q0) ~ 1e3
//     pass 1: G = Q0^T Q0     = R1^T R1,  Q  = Q0 R1^-1       |Q^T Q - I| ~ 1e-16 cond(Q0)^2
// cond(P) reaches (sigma_1/sigma_r)^2 * cond(U^T U_prev) ~ 1e8 on the benchmark tensors.  Q
// is handed back in fp32, so two passes are enough; the slow path below runs a third.  The
// product R1 R0 is upper triangular with a positive diagonal, so Q is the unique factor
// Gram-Schmidt produces.  Its diagonal is the norm each column keeps after the earlier ones
// are projected out; a column keeping less than 1e-12 ||P||_F is reported through *info.
//
// Fast path (r <= 64), two launches that serve all modes of a tensor at once:
//   gram0 : row slices of 32 rows sum the split partial sums of P -> P64 and write their slice Gram
//           (fp64 MFMA); the workgroup that arrives last at the mode's counter sums the slice Grams and
//           factors: blocked Cholesky in LDS without a shift, with the shift only if a pivot is lost;
//           it also inverts the 16x16 diagonal blocks of R
//   apply : row slices: Q0 = P R^-1 by block forward substitution (fp64 MFMA), written in fp64 and as
//           the fp32 result, plus the slice Gram of Q0; the last-arriving workgroup measures
//           |Q0^T Q0 - I| and only if that exceeds OP_DONE_TOL runs the second pass by itself
// Wide path (64 < r <= 192): separate Gram / Cholesky / apply launches on the packed triangle.
// Slow path (r > 192): one workgroup per mode, everything in global memory.
#include "asi_device.h"
#include "asi_kernels.h"

#include <atomic>
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int OP_RS = 32;              // rows per slice
constexpr int OP_RMAX = 64;
constexpr int OP_LD = OP_RMAX + 1;
constexpr double OP_EPS = 1.1102230246251565e-16;
constexpr double OP_DONE_TOL = 1e-7;   // |Q0^T Q0 - I| below which the first pass is the result


__device__ __forceinline__ void flag_info(int32_t* info, int mode1, int col1) {
    if (info) atomicCAS(info, 0, mode1 * 1000 + col1);
}

// the modes of all layers of one launch
constexpr int kMaxOrthJobs = 4 * kMaxBatch;
struct OrthBatch {
    OrthJob job[kMaxOrthJobs];
    int njobs;
};
struct PresumBatch {
    PresumJob job[kMaxOrthJobs];
    int njobs;
};
static_assert(sizeof(OrthBatch) <= 4096, "kernel argument limit");

__device__ __forceinline__ void find_job(const OrthBatch& a, int* ji, int* blk) {
    int j = 0, b = blockIdx.x;
    while (j + 1 < a.njobs && b >= a.job[j].nblk) { b -= a.job[j].nblk; ++j; }
    *ji = j; *blk = b;
}

// Packed upper triangle: element (ga <= gb) of an r x r symmetric matrix
__device__ __forceinline__ int tri_idx(int r, int ga, int gb) { return ga * r - (ga * (ga - 1)) / 2 + (gb - ga); }

// Gram of the 32 rows held in Ps (zero padded to 64 columns) -> packed upper triangle Gout (r (r+1) / 2)
__device__ void gram_from_lds(const double (*Ps)[OP_LD], int r, double* __restrict__ Gout) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lg = lane >> 4, ll = lane & 15;
    const int nb = (r + 15) / 16, npairs = nb * (nb + 1) / 2;
    const int nwaves = blockDim.x >> 6;
    for (int pr = wave; pr < npairs; pr += nwaves) {
        int ab = 0, rem = pr;
        while (rem >= nb - ab) { rem -= nb - ab; ++ab; }
        const int bb = ab + rem;
        v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < OP_RS / 4; ++ks)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[4 * ks + lg][16 * ab + ll], Ps[4 * ks + lg][16 * bb + ll], acc,
                                                       0, 0, 0);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ga = 16 * ab + lg + 4 * v, gb = 16 * bb + ll;
            if (ga < r && gb < r && ga <= gb) Gout[tri_idx(r, ga, gb)] = acc[v];
        }
    }
}

// ---- first level of the partial-sum tree -----------------------------------------------------
// When a mode arrives with more than 32 split partial sums, groups of 32 are added first
// (fixed order inside a group), so that no workgroup of gram0 has to walk hundreds of them.
__global__ __launch_bounds__(256) void k_orth_presum(PresumBatch a) { presum_block(a.job, a.njobs, blockIdx.x); }

// ---- chol -----------------------------------------------------------------------------------
__device__ __forceinline__ double bcast_lane(double x, int src) {      // src uniform
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src);
    return __hiloint2double(hi, lo);
}

// Cholesky of the 16x16 diagonal block of Gs at `base` by ONE wave, four pivots per round.
// Lane j < 16 keeps column j of the (symmetric) trailing block in registers, so row k of the
// trailing block is lane k's column.  A round eliminates its four pivots inside the 4-row
// panel, fetching the few values it needs from their lanes; every lane then publishes its four
// finished row entries in `rowbuf` (LDS serves one wave's accesses in order, so no barrier is
// needed) and applies the rank-4 update to its rows below the panel.  The rows of the next
// panel are updated first, so that the next panel's chain of reciprocals is independent of the
// rest of the update and the two are interleaved.  The code is branch free; a non-positive
// pivot is replaced by 1 and reported through `bad` (1-based index, first one wins).
// Rows are left unscaled: on return Gs[base+k][base+j], k <= j, holds R[k][j] * R[k][k], the
// diagonal the pivots R[k][k]^2, and pinvs[base+k] their reciprocals.
// Lanes 48..63 carry the columns of an identity block through the same row operations, which
// leaves the inverse of the block's unit lower triangular factor in Xb[i][j] = (L^-1)[j][i].
// e / r for 0 <= e < 2^16 and 1 <= r <= 64 without an integer division: the rounded float quotient
// of (e + 0.5) is exact in that range (the same device as in the product kernels).
__device__ __forceinline__ int small_div(int e, float inv_r) { return (int)(((float)e + 0.5f) * inv_r); }

// The matrix is reached through an accessor (ld(row, col), st(row, col, value)): a square LDS array
// for r <= 64, the packed upper triangle for wider matrices.  Only entries with row <= col are used.
struct GramSquare {
    double (*Gs)[OP_LD];
    __device__ __forceinline__ double ld(int row, int col) const { return Gs[row][col]; }
    __device__ __forceinline__ void st(int row, int col, double v) const { Gs[row][col] = v; }
};
struct GramPacked {                      // row-wise packed upper triangle of an r x r matrix, identity beyond r
    double* Gp;
    int r;
    __device__ __forceinline__ int idx(int row, int col) const { return row * r - (row * (row - 1)) / 2 + (col - row); }
    __device__ __forceinline__ double ld(int row, int col) const {
        const bool in = row <= col && col < r;
        const double v = Gp[in ? idx(row, col) : 0];
        return in ? v : (row == col ? 1.0 : 0.0);
    }
    __device__ __forceinline__ void st(int row, int col, double v) const {
        if (row <= col && col < r) Gp[idx(row, col)] = v;
    }
};
template <class GA>
__device__ void chol_block16(const GA G, double (*rowbuf)[64][4], double (*Xb)[17], double* pinvs, int base,
                             int* bad_io) {
    const int j = threadIdx.x;          // 0..63
    const bool xl = j >= 48;            // identity lane
    double col[16];
    {
        // All 16 reads are issued before any is used.  Left to itself the compiler sinks each read
        // into the branch that selects it (only lanes 0..15 keep the value) and waits for one LDS
        // round trip per row; the empty asm pins the reads in front of the selects.
        double g[16];
#pragma unroll
        for (int a2 = 0; a2 < 16; ++a2) g[a2] = G.ld(base + a2, base + (j & 15));
#pragma unroll
        for (int a2 = 0; a2 < 16; ++a2) asm volatile("" : "+v"(g[a2]));
#pragma unroll
        for (int a2 = 0; a2 < 16; ++a2) col[a2] = xl ? ((a2 == j - 48) ? 1.0 : 0.0) : (j < 16 ? g[a2] : 0.0);
    }
    int bad = *bad_io;
    double f[4];
    // Panel K0..K0+3.  Its 4x4 diagonal block (10 values, fetched from their lanes in one go) is
    // factored redundantly by every lane, which keeps the cross-lane traffic off the chain of
    // reciprocals; each lane then applies the multipliers to its own four row entries.
    // F[kk] = (row K0+kk of this lane's column) / pivot.
#define ASI_CHOL_PANEL(K0, F)                                                                       \
    {                                                                                               \
        double a_[4][4], pi_[4], m_[4][4];                                                          \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                            \
            _Pragma("unroll") for (int k2 = kk; k2 < 4; ++k2) a_[kk][k2] = bcast_lane(col[(K0) + kk], (K0) + k2); \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                          \
            double p = a_[kk][kk];                                                                  \
            const bool okp = p > 0.0;                /* false for zero, negative, NaN */            \
            bad = (!okp && bad == 0) ? base + (K0) + kk + 1 : bad;                                  \
            p = okp ? p : 1.0;                                                                      \
            double pinv = __builtin_amdgcn_rcp(p);                                                  \
            pinv = fma(fma(-p, pinv, 1.0), pinv, pinv);   /* two Newton steps: full accuracy */     \
            pinv = fma(fma(-p, pinv, 1.0), pinv, pinv);                                             \
            pi_[kk] = pinv;                                                                         \
            a_[kk][kk] = p;                          /* the pivot actually used */                  \
            _Pragma("unroll") for (int k2 = kk + 1; k2 < 4; ++k2) m_[kk][k2] = a_[kk][k2] * pinv;   \
            _Pragma("unroll") for (int k2 = kk + 1; k2 < 4; ++k2)                                   \
                _Pragma("unroll") for (int k3 = k2; k3 < 4; ++k3) a_[k2][k3] = fma(-m_[kk][k2], a_[kk][k3], a_[k2][k3]); \
        }                                                                                           \
        _Pragma("unroll") for (int k2 = 1; k2 < 4; ++k2)                                            \
            _Pragma("unroll") for (int kk = 0; kk < k2; ++kk)                                       \
                col[(K0) + k2] = fma(-m_[kk][k2], col[(K0) + kk], col[(K0) + k2]);                  \
        _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                          \
            F[kk] = col[(K0) + kk] * pi_[kk];                                                       \
            if (j == (K0) + kk) { col[(K0) + kk] = a_[kk][kk]; pinvs[base + (K0) + kk] = pi_[kk]; } \
        }                                                                                           \
    }
#define ASI_CHOL_UPDATE(A_LO, A_HI, RB)                                                             \
    {                                                                                               \
        _Pragma("unroll") for (int a0 = (A_LO); a0 < (A_HI); a0 += 4) {                             \
            double w[4][4];                                                                         \
            _Pragma("unroll") for (int g = 0; g < 4; ++g)                                           \
                _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) w[g][kk] = RB[a0 + g][kk];         \
            _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                        \
                _Pragma("unroll") for (int g = 0; g < 4; ++g)                                       \
                    col[a0 + g] = fma(-w[g][kk], f[kk], col[a0 + g]);                               \
        }                                                                                           \
    }
    ASI_CHOL_PANEL(0, f)
#pragma unroll
    for (int k0 = 0; k0 + 4 < 16; k0 += 4) {
        double (*rb)[4] = rowbuf[(k0 >> 2) & 1];
        rb[j][0] = col[k0]; rb[j][1] = col[k0 + 1]; rb[j][2] = col[k0 + 2]; rb[j][3] = col[k0 + 3];
        ASI_CHOL_UPDATE(k0 + 4, k0 + 8, rb)
        double fn[4];
        ASI_CHOL_PANEL(k0 + 4, fn)
        ASI_CHOL_UPDATE(k0 + 8, 16, rb)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) f[kk] = fn[kk];
    }
#undef ASI_CHOL_PANEL
#undef ASI_CHOL_UPDATE
    *bad_io = bad;
    // lanes 0..15 write their column of the block (entries below the diagonal are never read again),
    // lanes 48..63 their row of the inverse factor: one run of stores for both
    if (xl) {
#pragma unroll
        for (int k = 0; k < 16; ++k) Xb[j - 48][k] = col[k];
    } else if (j < 16) {
#pragma unroll
        for (int k = 0; k < 16; ++k) G.st(base + k, base + j, col[k]);
    }
}

// One workgroup (256 threads): sums the slice Grams of a mode, adds the shift (first pass) and
// factors the matrix, identity padded to a multiple of 16, by blocked right-looking Cholesky:
// wave 0 factors a diagonal block, then the four waves solve that block row and update the
// trailing blocks with fp64 MFMA.  Writes R, the inverses of R's diagonal blocks and the
// bookkeeping in scal; with `last` it reports a rank-deficient P through *info.  scal[0] = trace(P^T P), scal[1 + k] = running product of the
// R diagonals, scal[65] = first bad pivot, scal[66] = 1 when the first pass needed no second.
struct CholSmem {
    double Gs[OP_RMAX][OP_LD];
    double dinv[OP_RMAX];
    double rdiag[OP_RMAX];
    double pinvs[OP_RMAX];
    double rowbuf[2][64][4];
    double Xs[OP_RMAX / 16][16][17];
    double s_trace;
    int s_bad;
};

template <int RM>
__device__ bool chol_job(const OrthJob& jb, int pass, int last, int32_t* info, CholSmem& sm) {
    double (*Gs)[OP_LD] = sm.Gs;
    double* dinv = sm.dinv;
    double* rdiag = sm.rdiag;
    double* pinvs = sm.pinvs;
    double (*rowbuf)[64][4] = sm.rowbuf;
    double (*Xs)[16][17] = sm.Xs;
    double& s_trace = sm.s_trace;
    int& s_bad = sm.s_bad;
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int nb = (r + 15) / 16;
    // sum of the slice Grams (packed upper triangles), slice after slice in their order: a round keeps up
    // to 48 loads per thread in flight (a round is one dependent trip to memory, and a long mode has a
    // hundred slices and more): IA elements per thread x SBX slices, IA = what the rank needs of the ITS
    // elements the launch's largest rank would
    constexpr int ITS = (RM * (RM + 1) / 2 + 255) / 256;
    const int T = (r * (r + 1)) / 2;
    double sum[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) sum[it] = 0.0;
    auto sum_slices = [&](auto ia_c, auto sb_c) __attribute__((always_inline)) {
        constexpr int IA = decltype(ia_c)::value, SBX = decltype(sb_c)::value;
        for (int b0 = 0; b0 < jb.nblk; b0 += SBX) {
            double t[SBX][IA];
#pragma unroll
            for (int u = 0; u < SBX; ++u)
#pragma unroll
                for (int it = 0; it < IA; ++it) {
                    const int e = tid + 256 * it;
                    t[u][it] = ldg_f64(jb.Gpart, (long long)(b0 + u) * T + e, e < T && b0 + u < jb.nblk);
                }
#pragma unroll
            for (int u = 0; u < SBX; ++u)
#pragma unroll
                for (int it = 0; it < IA; ++it) sum[it] += t[u][it];
        }
    };
    {
        const int ia = (T + 255) / 256;
        constexpr int SB = (96 / ITS) > 16 ? 16 : (96 / ITS);
        if (ia == 1) sum_slices(std::integral_constant<int, 1>{}, std::integral_constant<int, 48>{});
        else if (ITS >= 2 && ia == 2) sum_slices(std::integral_constant<int, (ITS >= 2 ? 2 : 1)>{}, std::integral_constant<int, 24>{});
        else sum_slices(std::integral_constant<int, ITS>{}, std::integral_constant<int, SB>{});
    }
    // Gs = the summed Gram matrix, padded with the identity up to a multiple of 16
    auto scatter = [&]() {
        __syncthreads();
        for (int e = tid; e < OP_RMAX * 64; e += 256) Gs[e >> 6][e & 63] = ((e >> 6) == (e & 63)) ? 1.0 : 0.0;
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int e = tid + 256 * it;
            if (e < T) {
                // row ga of the packed triangle: largest ga with tri_idx(r, ga, ga) <= e
                int ga = (int)(((2 * r + 1) - sqrtf((float)((2 * r + 1) * (2 * r + 1) - 8 * e))) * 0.5f);
                ga = ga < 0 ? 0 : (ga > r - 1 ? r - 1 : ga);
                while (ga > 0 && tri_idx(r, ga, ga) > e) --ga;
                while (ga + 1 < r && tri_idx(r, ga + 1, ga + 1) <= e) ++ga;
                const int gb = ga + (e - tri_idx(r, ga, ga));
                Gs[ga][gb] = sum[it];
                Gs[gb][ga] = sum[it];
            }
        }
        __syncthreads();
    };
    scatter();
    int bad = 0;
    // blocked right-looking factorisation of Gs in place
    auto factor = [&]() {
        for (int P = 0; P < nb; ++P) {
            if (wave == 0) chol_block16(GramSquare{Gs}, rowbuf, Xs[P], pinvs, 16 * P, &bad);
            __syncthreads();
            if (P + 1 < nb) {
                // block row P right of the diagonal:  U_PJ = L_PP^-1 G_PJ   (unscaled rows, like the diagonal block)
                for (int J = P + 1 + wave; J < nb; J += 4) {
                    double bv[4];
    #pragma unroll
                    for (int ks = 0; ks < 4; ++ks) bv[ks] = Gs[16 * P + 4 * ks + lg][16 * J + ll];
                    v4d acc = {0.0, 0.0, 0.0, 0.0};
    #pragma unroll
                    for (int ks = 0; ks < 4; ++ks)      // A[i][k] = (L^-1)[i][k] = Xs[P][k][i]
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Xs[P][4 * ks + lg][ll], bv[ks], acc, 0, 0, 0);
    #pragma unroll
                    for (int v = 0; v < 4; ++v) Gs[16 * P + lg + 4 * v][16 * J + ll] = acc[v];
                }
                __syncthreads();
                // trailing blocks:  G_IJ -= U_PI^T diag(1/pivot) U_PJ,  P < I <= J
                int cnt = 0;
                for (int I = P + 1; I < nb; ++I)
                    for (int J = I; J < nb; ++J, ++cnt) {
                        if ((cnt & 3) != wave) continue;
                        v4d acc;
    #pragma unroll
                        for (int v = 0; v < 4; ++v) acc[v] = Gs[16 * I + lg + 4 * v][16 * J + ll];
    #pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            const int k = 16 * P + 4 * ks + lg;
                            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(-Gs[k][16 * I + ll], Gs[k][16 * J + ll] * pinvs[k], acc, 0, 0, 0);
                        }
    #pragma unroll
                        for (int v = 0; v < 4; ++v) Gs[16 * I + lg + 4 * v][16 * J + ll] = acc[v];
                    }
                __syncthreads();
            }
        }
    };
    if (pass == 1) {
        // Q0 may already be orthonormal to working accuracy (a warm-started, well-conditioned P): then
        // the second pass would only reproduce the identity, and the fp32 copy of Q0 that the solve
        // has written is the result.
        double dev = 0.0;
        const float inv_r1 = 1.0f / (float)r;
        for (int e = tid; e < r * r; e += 256) {
            const int ga = small_div(e, inv_r1), gb = e - ga * r;
            dev = fmax(dev, fabs(Gs[ga][gb] - (ga == gb ? 1.0 : 0.0)));
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) dev = fmax(dev, __shfl_xor(dev, m));
        if (lane == 0) rdiag[wave] = dev;
        __syncthreads();
        dev = fmax(fmax(rdiag[0], rdiag[1]), fmax(rdiag[2], rdiag[3]));
        __syncthreads();
        const bool done = dev <= OP_DONE_TOL;
        if (tid == 0) jb.scal[66] = done ? 1.0 : 0.0;
        if (done) {
            if (tid < 64) {
                const double floor_ = 1e-12 * sqrt(jb.scal[0]);
                const bool low = tid < r && !(jb.scal[1 + tid] > floor_);
                const unsigned long long mask = __ballot(low);
                if (tid == 0 && last && info) {
                    const double badv = jb.scal[65];
                    if (badv != 0.0) flag_info(info, jb.mode1, (int)badv);
                    if (mask) flag_info(info, jb.mode1, __ffsll((long long)mask));
                }
            }
            return false;
        }
        if (tid == 0) s_trace = jb.scal[0];
        factor();
    } else {
        // First pass.  Plain Cholesky first; if a pivot is lost (non-positive, or below 1e-12 of its
        // diagonal entry: cond(P) beyond ~1e6) the factorisation is redone with the diagonal shift
        // that makes it safe up to cond(P) ~ 1e9.
        double tr = 0.0;
        if (wave == 0) {
            const double g = (lane < r) ? Gs[lane][lane] : 0.0;
            tr = g;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) tr += __shfl_xor(tr, m);
            if (lane == 0) { s_trace = tr; jb.scal[0] = tr; }
            if (lane < r) rdiag[lane] = g;                  // the diagonal before elimination
        }
        factor();
        if (wave == 0) {
            const bool lost = lane < r && !(Gs[lane][lane] > 1e-12 * rdiag[lane]);
            const unsigned long long mask = __ballot(lost);
            if (lane == 0) s_bad = (bad != 0 || mask != 0) ? 1 : 0;
        }
        __syncthreads();
        if (s_bad) {
            scatter();
            bad = 0;
            if (wave == 0) {
                const double shift = 11.0 * ((double)n * r + (double)r * (r + 1)) * OP_EPS * tr;
                if (lane < r) Gs[lane][lane] += shift;
            }
            factor();
        }
        __syncthreads();
    }
    if (tid == 0) s_bad = bad;
    if (tid < r) {
        double p = Gs[tid][tid];
        if (!(p > 0.0)) p = 1.0;
        const double d = sqrt(p);
        dinv[tid] = 1.0 / d;
        pinvs[tid] = d;                     // the pivots' reciprocals are not needed any more
        const double rd = (pass == 0 ? 1.0 : jb.scal[1 + tid]) * d;
        rdiag[tid] = rd;
        jb.scal[1 + tid] = rd;
    }
    __syncthreads();
    {   // R = rows scaled by 1 / R[k][k], zeros below the diagonal (reads first, selects after)
        const int gb = tid & 63;
        double gv[RM / 4], dv[RM / 4], iv[RM / 4];
#pragma unroll
        for (int it = 0; it < RM / 4; ++it) {
            const int ga = (tid >> 6) + 4 * it;
            gv[it] = Gs[ga][gb]; dv[it] = pinvs[ga]; iv[it] = dinv[ga];
        }
#pragma unroll
        for (int it = 0; it < RM / 4; ++it) asm volatile("" : "+v"(gv[it]), "+v"(dv[it]), "+v"(iv[it]));
#pragma unroll
        for (int it = 0; it < RM / 4; ++it) {
            const int ga = (tid >> 6) + 4 * it;
            if (ga < r && gb < r) jb.R[ga * r + gb] = (ga < gb) ? gv[it] * iv[it] : (ga == gb ? dv[it] : 0.0);
        }
    }
    // inverse of each 16x16 diagonal block of R:  (R_bb^-1)[i][j] = (L_bb^-1)[j][i] / R[j][j]
    for (int e = tid; e < nb * 256; e += 256) {
        const int b = e >> 8, i = (e >> 4) & 15, jj = e & 15, base = 16 * b;
        const bool in = base + i < r && base + jj < r && jj >= i;
        jb.Dinv[e] = in ? Xs[b][i][jj] * dinv[base + jj] : 0.0;
    }
    if (tid < 64) {
        // first column (if any) whose accumulated R diagonal fell to the noise floor
        const double floor_ = 1e-12 * sqrt(s_trace);
        const bool low = tid < r && !(rdiag[tid] > floor_);
        const unsigned long long mask = __ballot(low);
        if (tid == 0) {
            double badv = (pass == 0) ? 0.0 : jb.scal[65];
            if (badv == 0.0 && s_bad) badv = (double)s_bad;
            jb.scal[65] = badv;
            if (last && info) {
                if (badv != 0.0) flag_info(info, jb.mode1, (int)badv);
                if (mask) flag_info(info, jb.mode1, __ffsll((long long)mask));
            }
        }
    }
    return true;
}

// ---- hand-over from the slices of a mode to its factorisation ------------------------------
// Every workgroup of a mode calls this after its global writes.  Returns true in exactly one of
// them, the one that arrives last; by then the writes of all the others are visible to it.  The
// counter must be zero before the launch and is zero again afterwards.
__device__ bool last_arrival(int32_t* ctr, int nblk, int* s_flag) {
    __threadfence();                       // this thread's writes are visible device-wide ...
    __syncthreads();                       // ... for every thread of the workgroup
    if (threadIdx.x == 0) {
        const int ticket = atomicAdd(ctr, 1);
        *s_flag = (ticket == nblk - 1);
        if (ticket == nblk - 1) *ctr = 0;
    }
    __syncthreads();
    const bool last = *s_flag != 0;
    if (last) __threadfence();             // order the reads below after the other workgroups' arrivals
    return last;
}

// ---- gram0 ----------------------------------------------------------------------------------
// RM bounds the ranks of the launch's modes: a slice has at most 32 * RM elements, ITS per thread.
template <int RM>
__global__ __launch_bounds__(256) void k_orth_gram0(OrthBatch a) {
    __shared__ __align__(16) unsigned char raw[sizeof(CholSmem)];
    __shared__ int s_last;
    double (*Ps)[OP_LD] = reinterpret_cast<double (*)[OP_LD]>(raw);                 // [OP_RS][OP_LD]
    double* red = reinterpret_cast<double*>(raw) + OP_RS * OP_LD;                     // [256]
    static_assert(sizeof(CholSmem) >= (OP_RS * OP_LD + 256) * sizeof(double), "slice buffers fit");
    int ji, blk;
    find_job(a, &ji, &blk);
    const OrthJob jb = a.job[ji];
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    if (blk == 0 && tid == 0 && jb.info) *jb.info = 0;            // nothing has reported yet
    const int i0 = blk * OP_RS;
    const int nrows = (n - i0 < OP_RS) ? n - i0 : OP_RS;
    const long long cnt = (long long)n * r;
    const int E = nrows * r;
    for (int e = tid; e < OP_RS * OP_LD; e += 256) (&Ps[0][0])[e] = 0.0;
    // Sum of the split partial sums.  A slice of 256 or more elements gives every thread ITS
    // elements and SB splits per round; a smaller one shares its splits among `nsg` thread
    // groups whose results are added in group order.  All loads of a round are in flight together.
    constexpr int ITS = RM / 8, SB = 32 / ITS;
    const bool small = E < 256;
    const int nsg = small ? 256 / E : 1;
    const int sg = small ? tid / E : 0;
    const int idx0 = small ? tid - sg * E : tid;
    const bool act0 = sg < nsg;
    double sum[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) sum[it] = 0.0;
    for (int sp0 = sg; sp0 < jb.nsplit; sp0 += SB * nsg) {
        double t[SB][ITS];
#pragma unroll
        for (int u = 0; u < SB; ++u)
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const int sp = sp0 + u * nsg, idx = idx0 + 256 * it;
                const bool ok = act0 && idx < E && (it == 0 || !small) && sp < jb.nsplit;
                t[u][it] = ldg_f64(jb.part, (long long)sp * cnt + (long long)i0 * r + idx, ok);
            }
#pragma unroll
        for (int u = 0; u < SB; ++u)
#pragma unroll
            for (int it = 0; it < ITS; ++it) sum[it] += t[u][it];
    }
    if (small && nsg > 1) {
        if (act0) red[sg * E + idx0] = sum[0];
        __syncthreads();
        if (act0 && sg == 0) {
            double s2 = 0.0;
            for (int g2 = 0; g2 < nsg; ++g2) s2 += red[g2 * E + idx0];
            sum[0] = s2;
        }
    } else {
        __syncthreads();      // the zero fill above is complete
    }
    if (act0 && sg == 0) {
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int idx = idx0 + 256 * it;
            if (idx < E && (it == 0 || !small)) {
                jb.P64[(long long)i0 * r + idx] = sum[it];
                const int pi = small_div(idx, 1.0f / (float)r);
                Ps[pi][idx - pi * r] = sum[it];
            }
        }
    }
    __syncthreads();
    gram_from_lds(Ps, r, jb.Gpart + (long long)blk * ((r * (r + 1)) / 2));
    // the workgroup that finishes a mode's last slice goes on to factor its Gram matrix
    if (!last_arrival(jb.ctr + 0, jb.nblk, &s_last)) return;
    chol_job<RM>(jb, 0, 0, jb.info, *reinterpret_cast<CholSmem*>(raw));
}

// ---- apply ----------------------------------------------------------------------------------
// 256 threads load the slice, R and the diagonal-block inverses in one round of loads; waves 0 and 1
// then solve 16 rows each.
struct ApplySmem {
    double Ps[OP_RS][OP_LD];
    double Rs[OP_RMAX][OP_LD];
    double Ds[OP_RMAX / 16][16][17];
};
union ApplyOrChol {                      // the factorisation reuses the memory of the finished solve
    ApplySmem ap;
    CholSmem ch;
};

// One 32-row slice: P64[slice] <- P64[slice] R^-1.  The first pass stores the result in fp64 for
// the second pass, its fp32 copy in Uout (the result if the first pass turns out to be enough) and
// the slice's Gram matrix; the final pass stores fp32 only.
template <int RM>
__device__ void apply_slice(const OrthJob& jb, int blk, int final_pass, ApplySmem& ap) {
    double (*Ps)[OP_LD] = ap.Ps;
    double (*Rs)[OP_LD] = ap.Rs;
    double (*Ds)[16][17] = ap.Ds;
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int nb = (r + 15) / 16;
    const int i0 = blk * OP_RS;
    const int nrows = (n - i0 < OP_RS) ? n - i0 : OP_RS;
    constexpr int PI = RM / 8, RI = RM * RM / 256, DI = RM / 16;
    const float inv_r = 1.0f / (float)r;
    double tp[PI], tr[RI], td[DI];
#pragma unroll
    for (int u = 0; u < PI; ++u) {
        const int idx = u * 256 + tid;
        tp[u] = ldg_f64(jb.P64, (long long)i0 * r + idx, idx < nrows * r);
    }
#pragma unroll
    for (int u = 0; u < RI; ++u) {
        const int e = u * 256 + tid;
        tr[u] = ldg_f64(jb.R, e, e < r * r);
    }
#pragma unroll
    for (int u = 0; u < DI; ++u) {
        const int e = u * 256 + tid;
        td[u] = ldg_f64(jb.Dinv, e, e < nb * 256);
    }
    for (int e = tid; e < OP_RS * OP_LD; e += 256) (&Ps[0][0])[e] = 0.0;
    for (int e = tid; e < OP_RMAX * OP_LD; e += 256) (&Rs[0][0])[e] = 0.0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PI; ++u) {
        const int idx = u * 256 + tid;
        const int pi = small_div(idx, inv_r);
        if (idx < nrows * r) Ps[pi][idx - pi * r] = tp[u];
    }
#pragma unroll
    for (int u = 0; u < RI; ++u) {
        const int e = u * 256 + tid;
        const int ri = small_div(e, inv_r);
        if (e < r * r) Rs[ri][e - ri * r] = tr[u];
    }
#pragma unroll
    for (int u = 0; u < DI; ++u) {
        const int e = u * 256 + tid;
        if (e < nb * 256) Ds[e >> 8][(e >> 4) & 15][e & 15] = td[u];
    }
    __syncthreads();
    // wave w < 2 owns rows 16w..16w+15 of the slice; block columns are solved left to right
    const int rw = 16 * (wave & 1);
    for (int b = 0; b < nb; ++b) {
        if (wave < 2) {
            // T = P_b - sum_{a<b} Q_a R_ab
            v4d acc = {0.0, 0.0, 0.0, 0.0};
            for (int ab = 0; ab < b; ++ab)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[rw + ll][16 * ab + 4 * ks + lg],
                                                               Rs[16 * ab + 4 * ks + lg][16 * b + ll], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) Ps[rw + lg + 4 * v][16 * b + ll] -= acc[v];
        }
        __syncthreads();
        v4d q = {0.0, 0.0, 0.0, 0.0};
        if (wave < 2) {
            // Q_b = T R_bb^-1
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                q = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[rw + ll][16 * b + 4 * ks + lg], Ds[b][4 * ks + lg][ll], q, 0, 0, 0);
        }
        __syncthreads();
        if (wave < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) Ps[rw + lg + 4 * v][16 * b + ll] = q[v];
        }
        __syncthreads();
    }
    if (final_pass) {
        for (int idx = tid; idx < nrows * r; idx += 256) {
            const int pi = small_div(idx, inv_r);
            jb.Uout[(long long)i0 * r + idx] = (float)Ps[pi][idx - pi * r];
        }
    } else {
        for (int idx = tid; idx < nrows * r; idx += 256) {
            const int pi = small_div(idx, inv_r);
            const double q0 = Ps[pi][idx - pi * r];
            jb.P64[(long long)i0 * r + idx] = q0;
            jb.Uout[(long long)i0 * r + idx] = (float)q0;
        }
        gram_from_lds(Ps, r, jb.Gpart + (long long)blk * ((r * (r + 1)) / 2));
    }
}

// Second half of the orthonormalisation in one launch: every workgroup solves its slice with the
// first-pass factor; the one that finishes a mode's last slice checks Q0^T Q0 against the identity
// and, only if that fails, factors it and solves all slices of the mode once more by itself (a
// rare, slow path: it trades a launch per call for serial work on ill-conditioned inputs).
template <int RM>
__global__ __launch_bounds__(256) void k_orth_apply(OrthBatch a) {
    __shared__ __align__(16) unsigned char raw[sizeof(ApplyOrChol)];
    __shared__ int s_last;
    ApplySmem& ap = *reinterpret_cast<ApplySmem*>(raw);
    int ji, blk;
    find_job(a, &ji, &blk);
    const OrthJob jb = a.job[ji];
    apply_slice<RM>(jb, blk, 0, ap);
    if (!last_arrival(jb.ctr + 1, jb.nblk, &s_last)) return;
    const bool again = chol_job<RM>(jb, 1, 1, jb.info, *reinterpret_cast<CholSmem*>(raw));
    if (!again) return;
    for (int b2 = 0; b2 < jb.nblk; ++b2) {
        __threadfence();                   // R, Dinv (and every slice of Q0) are read back from memory
        __syncthreads();
        apply_slice<RM>(jb, b2, 1, ap);
    }
}

// ---- wide path, 64 < r <= 192 -----------------------------------------------------------------
// Same two passes.  The Gram matrix no longer fits the statically sized LDS arrays, so
//   gramw : 128-row blocks read P64 in 32-row sub-slices and keep their block pairs in registers
//   cholw : one workgroup per mode, Gram matrix packed (upper triangle) in up to 150 KB of
//           dynamic LDS, same right-looking factorisation
//   applyw: 32-row blocks, R's off-diagonal blocks are read straight from global memory
constexpr int OW_RMAX = 192;
constexpr int OW_LD = OW_RMAX + 1;
constexpr int OW_ROWS = 64;             // rows per gramw block
constexpr int OW_MAXPAIR = 20;          // block pairs per wave: ceil(78 / 4)

__global__ __launch_bounds__(256) void k_orthw_gram(OrthBatch a) {
    __shared__ double Ps[OP_RS][OW_LD];
    int ji, blk;
    find_job(a, &ji, &blk);
    const OrthJob jb = a.job[ji];
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int nb = (r + 15) / 16, npairs = nb * (nb + 1) / 2;
    v4d acc[OW_MAXPAIR];
#pragma unroll
    for (int s = 0; s < OW_MAXPAIR; ++s) acc[s] = (v4d){0.0, 0.0, 0.0, 0.0};
    for (int e = tid; e < OP_RS * OW_LD; e += 256) (&Ps[0][0])[e] = 0.0;
    const int row_beg = blk * OW_ROWS;
    const int row_end = (row_beg + OW_ROWS < n) ? row_beg + OW_ROWS : n;
    for (int i0 = row_beg; i0 < row_end; i0 += OP_RS) {
        const int nrows = (row_end - i0 < OP_RS) ? row_end - i0 : OP_RS;
        __syncthreads();
        for (int idx0 = 0; idx0 < OP_RS * r; idx0 += 256 * 8) {
            double t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = idx0 + u * 256 + tid;
                t[u] = ldg_f64(jb.P64, (long long)i0 * r + idx, idx < nrows * r);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = idx0 + u * 256 + tid;
                if (idx < OP_RS * r) Ps[idx / r][idx % r] = t[u];      // rows past nrows become zero
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < OW_MAXPAIR; ++s) {
            const int pr = wave + 4 * s;
            if (pr < npairs) {
                int ab = 0, rem = pr;
                while (rem >= nb - ab) { rem -= nb - ab; ++ab; }
                const int bb = ab + rem;
#pragma unroll
                for (int ks = 0; ks < OP_RS / 4; ++ks)
                    acc[s] = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[4 * ks + lg][16 * ab + ll], Ps[4 * ks + lg][16 * bb + ll],
                                                                  acc[s], 0, 0, 0);
            }
        }
    }
    double* Gout = jb.Gpart + (long long)blk * r * r;
#pragma unroll
    for (int s = 0; s < OW_MAXPAIR; ++s) {
        const int pr = wave + 4 * s;
        if (pr < npairs) {
            int ab = 0, rem = pr;
            while (rem >= nb - ab) { rem -= nb - ab; ++ab; }
            const int bb = ab + rem;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int ga = 16 * ab + lg + 4 * v, gb = 16 * bb + ll;
                if (ga < r && gb < r && ga <= gb) Gout[ga * r + gb] = acc[s][v];
            }
        }
    }
}

// Sum of the slice Gram matrices of a mode and its distance from the identity, spread over the chip: the
// factorisation is one workgroup, and what it reads right after other workgroups wrote it costs it 3-5 us per
// dependent round of loads (five rounds for two partial sums of a 192 x 192 matrix: 28 us of the second pass went
// into a sum whose only use was the check that the first pass had been enough).
struct GsumBatch {
    GsumJob job[kMaxOrthJobs];
    int njobs;
};
__global__ __launch_bounds__(256) void k_orthw_gsum(GsumBatch a) {
    int j = 0, b = blockIdx.x;
    while (j + 1 < a.njobs && b >= a.job[j].nchunks) { b -= a.job[j].nchunks; ++j; }
    const GsumJob& jb = a.job[j];
    const int r = jb.r, cnt = r * r;
    const int e = b * 256 + threadIdx.x;
    double s = 0.0;
    for (int b0 = 0; b0 < jb.nblk; b0 += 32) {               // 32 slices' loads in flight, added in slice order
        double t[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) t[u] = jb.in[(long long)(b0 + u < jb.nblk ? b0 + u : jb.nblk - 1) * cnt + (e < cnt ? e : 0)];
#pragma unroll
        for (int u = 0; u < 32; ++u) s += (b0 + u < jb.nblk) ? t[u] : 0.0;
    }
    double dev = 0.0;
    if (e < cnt) {
        jb.out[e] = s;
        const int ga = e / r, gb = e - ga * r;
        if (ga <= gb) dev = fabs(s - (ga == gb ? 1.0 : 0.0));   // (only the upper triangles of the slices are written)
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dev = fmax(dev, __shfl_xor(dev, m));
    if ((threadIdx.x & 63) == 0 && dev > 0.0) atomicMax(jb.devbits, (unsigned long long)__double_as_longlong(dev));
}

extern __shared__ double ow_dyn[];

// 512 threads: with 1024 a thread may hold 128 registers, and the diagonal-block factorisation (a column
// of 16 doubles per lane plus its panels) then spills to scratch memory: 13 us per block instead of 2.
constexpr int OWC_NT = 512, OWC_NW = OWC_NT / 64;
__global__ __launch_bounds__(OWC_NT) void k_orthw_chol(OrthBatch a, int pass, int last) {
    const OrthJob jb = a.job[blockIdx.x];
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    double* Gp = ow_dyn;                              // packed upper triangle, r (r + 1) / 2
    double* dinv = ow_dyn + (r * (r + 1)) / 2;
    double* rdiag = dinv + r;
    __shared__ double s_trace;
    __shared__ int s_bad;
    auto pidx = [r](int ga, int gb) __attribute__((always_inline)) { return ga * r - (ga * (ga - 1)) / 2 + (gb - ga); };
    __shared__ int s_lost;
    __shared__ double s_red[OWC_NW];
    if (tid == 0) { s_bad = 0; s_lost = 0; }
    // Gp = sum of the slice Grams; returns this thread's share of max |G - I|.  A round keeps 32 loads
    // per thread in flight: 4 elements x 8 slices, or 16 elements x 2 slices when a tree level has
    // already added the slices up (quotient e / r by a rounded float product: exact for r * r < 2^21).
    const float inv_rf = 1.0f / (float)r;
    auto sum_gram_t = [&](auto c_c, auto u_c) __attribute__((always_inline)) {
        constexpr int C = decltype(c_c)::value, U = decltype(u_c)::value;
        double dev = 0.0;
        for (int e0 = tid; e0 < r * r; e0 += C * OWC_NT) {
            double s[C];
#pragma unroll
            for (int c = 0; c < C; ++c) s[c] = 0.0;
            for (int b0 = 0; b0 < jb.nblk; b0 += U) {
                double t[C][U];
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int e = e0 + OWC_NT * c;
                        t[c][u] = ldg_f64(jb.Gpart, (long long)(b0 + u) * r * r + e, e < r * r && b0 + u < jb.nblk);
                    }
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int u = 0; u < U; ++u) s[c] += t[c][u];
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const int e = e0 + OWC_NT * c;
                const int ga = small_div(e, inv_rf), gb = e - ga * r;
                if (e < r * r && ga <= gb) {
                    Gp[pidx(ga, gb)] = s[c];
                    dev = fmax(dev, fabs(s[c] - (ga == gb ? 1.0 : 0.0)));
                }
            }
        }
        return dev;
    };
    auto sum_gram = [&]() __attribute__((always_inline)) {
        return jb.nblk <= 2 ? sum_gram_t(std::integral_constant<int, 16>{}, std::integral_constant<int, 2>{})
                            : sum_gram_t(std::integral_constant<int, 4>{}, std::integral_constant<int, 8>{});
    };
    // Blocked right-looking factorisation in place, the scheme of the r <= 64 path on the packed
    // triangle: wave 0 factors a 16x16 diagonal block in registers (chol_block16, which also leaves
    // the inverse of the block's unit triangular factor in Xs and the pivots' reciprocals in pinvs),
    // then all waves solve the block row and update the trailing blocks on fp64 MFMA.  Rows are
    // left unscaled (row k holds R[k][j] R[k][k], the diagonal the pivots R[k][k]^2).  A pivot that is
    // not above 1e-12 of its diagonal entry (rdiag holds the diagonal before elimination) sets s_lost.
    const int nb = (r + 15) / 16;
    double* pinvs = rdiag + r;                               // nb * 16
    double (*Xs)[17] = reinterpret_cast<double (*)[17]>(pinvs + nb * 16);
    double (*rowbuf)[64][4] = reinterpret_cast<double (*)[64][4]>(pinvs + nb * 16 + 16 * 17);
    const GramPacked G{Gp, r};
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    // Second pass with a summed Gram matrix: its distance from the identity has been measured by the launch that
    // summed it, and the matrix itself is read only if the pass has to be carried out.
    const bool measured = pass != 0 && jb.devbits != nullptr;
    double dev = 0.0;
    if (measured) {
        dev = __longlong_as_double((long long)*jb.devbits);
    } else {
        dev = sum_gram();
        __syncthreads();
    }
    if (pass == 0) {
        if (tid == 0 && jb.devbits) *jb.devbits = 0ull;     // the second Gram sum starts from zero
        if (tid < r) rdiag[tid] = Gp[pidx(tid, tid)];
        __syncthreads();
        if (wave == 0) {                 // trace: lanes sum every 64th diagonal entry, then a fixed-order butterfly
            double tr = 0.0;
            for (int k = lane; k < r; k += 64) tr += rdiag[k];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) tr += __shfl_xor(tr, m);
            if (lane == 0) { s_trace = tr; jb.scal[0] = tr; }
        }
        __syncthreads();
    } else {
        // Second pass: if Q0 is orthonormal to 1e-7 already, its fp32 copy (written by the first solve)
        // is the result and the final solve returns at once.
        if (!measured) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) dev = fmax(dev, __shfl_xor(dev, m));
            if ((tid & 63) == 0) s_red[tid >> 6] = dev;
            __syncthreads();
            dev = 0.0;
            for (int w = 0; w < OWC_NW; ++w) dev = fmax(dev, s_red[w]);
        }
        const bool done = dev <= OP_DONE_TOL;
        if (tid == 0) {
            jb.scal[2 + OW_RMAX] = done ? 1.0 : 0.0;
            s_trace = jb.scal[0];
        }
        if (done && last && jb.info) {
            // first column whose accumulated diagonal fell to the noise floor: every thread looks at one column (one
            // thread walking all of them paid a round trip to memory per column: 29 us for 192 of them)
            const double floor_ = 1e-12 * sqrt(jb.scal[0]);
            const bool low = tid < r && !(jb.scal[1 + tid] > floor_);
            if (tid == 0) s_lost = 0x7fffffff;
            __syncthreads();
            if (low) atomicMin(&s_lost, tid);
            __syncthreads();
            if (tid == 0) {
                const double bad = jb.scal[1 + OW_RMAX];
                if (bad != 0.0) flag_info(jb.info, jb.mode1, (int)bad);
                if (s_lost != 0x7fffffff) flag_info(jb.info, jb.mode1, s_lost + 1);
            }
        }
        if (done) return;
        __syncthreads();
        if (tid == 0) s_lost = 0;
        if (measured) {
            sum_gram();
            __syncthreads();
        }
        if (tid < r) rdiag[tid] = Gp[pidx(tid, tid)];
        __syncthreads();
    }
    // First pass: plain Cholesky first; only if a pivot is lost is the Gram matrix summed again, shifted
    // and factored once more (the same policy as the r <= 64 path).  The factorisation is written once,
    // inside this loop: as a lambda called from three places it was not inlined, its captured pointers
    // went through scratch memory and every LDS access in it became a flat access.
    for (int attempt = 0;; ++attempt) {
        int bad = 0;
        for (int P = 0; P < nb; ++P) {
            if (wave == 0) chol_block16(G, rowbuf, Xs, pinvs, 16 * P, &bad);
            __syncthreads();
            if (tid < 16 && 16 * P + tid < r) {
                const double p = G.ld(16 * P + tid, 16 * P + tid);          // the pivot actually used
                if (!(p > 1e-12 * rdiag[16 * P + tid])) s_lost = 1;
            }
            if (P + 1 < nb) {
                // block row P right of the diagonal:  U_PJ = L_PP^-1 G_PJ
                for (int J = P + 1 + wave; J < nb; J += OWC_NW) {
                    double bv[4];
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) bv[ks] = G.ld(16 * P + 4 * ks + lg, 16 * J + ll);
                    v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)      // A[i][k] = (L^-1)[i][k] = Xs[k][i]
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Xs[4 * ks + lg][ll], bv[ks], acc, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 4; ++v) G.st(16 * P + lg + 4 * v, 16 * J + ll, acc[v]);
                }
                __syncthreads();
                // trailing blocks:  G_IJ -= U_PI^T diag(1/pivot) U_PJ,  P < I <= J.  Rows k of the panel lie
                // above both blocks, so their elements sit at roff[k] + column; a column past r reads the
                // diagonal entry instead and counts as zero.  The twelve reads of a block pair are issued
                // together (pinned: left alone, each is moved into a branch of its own and waited for there).
                int roff[4];
                double pv[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const int k = 16 * P + 4 * ks + lg;
                    roff[ks] = k * r - (k * (k + 1)) / 2;
                    pv[ks] = pinvs[k];
                }
                int cnt = 0;
                for (int I = P + 1; I < nb; ++I)
                    for (int J = I; J < nb; ++J, ++cnt) {
                        if ((cnt & (OWC_NW - 1)) != wave) continue;
                        const int ci = 16 * I + ll, cj = 16 * J + ll;
                        const bool iin = ci < r, jin = cj < r;
                        double av[4], bv[4], cv[4];
                        int cidx[4];
                        bool cin[4];
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            const int k = 16 * P + 4 * ks + lg;
                            av[ks] = Gp[roff[ks] + (iin ? ci : k)];
                            bv[ks] = Gp[roff[ks] + (jin ? cj : k)];
                        }
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int rw = 16 * I + lg + 4 * v;
                            cin[v] = rw <= cj && jin;
                            cidx[v] = cin[v] ? rw * r - (rw * (rw + 1)) / 2 + cj : 0;
                            cv[v] = Gp[cidx[v]];
                        }
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(av[ks]), "+v"(bv[ks]), "+v"(cv[ks]));
                        v4d acc;
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[v] = cin[v] ? cv[v] : 0.0;
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks)
                            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(iin ? -av[ks] : 0.0, jin ? bv[ks] * pv[ks] : 0.0, acc, 0, 0, 0);
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (cin[v]) Gp[cidx[v]] = acc[v];
                    }
                __syncthreads();
            }
        }
        if (tid == 0) s_bad = bad;
        __syncthreads();
        if (pass != 0 || attempt != 0 || !(s_lost || s_bad)) break;
        __syncthreads();
        if (tid == 0) { s_bad = 0; s_lost = 0; }
        sum_gram();
        __syncthreads();
        const double shift = 11.0 * ((double)n * r + (double)r * (r + 1)) * OP_EPS * s_trace;
        if (tid < r) Gp[pidx(tid, tid)] += shift;
        __syncthreads();
    }
    if (tid < r) {
        double p = Gp[pidx(tid, tid)];
        if (!(p > 0.0)) p = 1.0;
        const double d = sqrt(p);
        dinv[tid] = 1.0 / d;
        const double rd = (pass == 0 ? 1.0 : jb.scal[1 + tid]) * d;
        rdiag[tid] = rd;
        jb.scal[1 + tid] = rd;
    }
    __syncthreads();
    for (int e = tid; e < r * r; e += OWC_NT) {      // R, and the rows scaled in place (each entry has one owner)
        const int ga = small_div(e, inv_rf), gb = e - ga * r;
        double v = 0.0;
        if (ga < gb) {
            v = Gp[pidx(ga, gb)] * dinv[ga];
            Gp[pidx(ga, gb)] = v;
        } else if (ga == gb) {
            v = 1.0 / dinv[ga];
        }
        jb.R[e] = v;
    }
    __syncthreads();
    if (tid < nb * 16) {
        const int b = tid >> 4, i = tid & 15, base = 16 * b;
        double x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            double s = (j == i) ? 1.0 : 0.0;
#pragma unroll
            for (int k = 0; k < j; ++k) s = fma(-x[k], (base + j < r) ? Gp[pidx(base + k, base + j)] : 0.0, s);
            x[j] = (j >= i && base + j < r && base + i < r) ? s * dinv[base + j] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) jb.Dinv[(b * 16 + i) * 16 + j] = x[j];
    }
    __syncthreads();                                      // (the pivot flags are no longer read)
    if (tid == 0) s_lost = 0x7fffffff;
    __syncthreads();
    if (last && jb.info && tid < r && !(rdiag[tid] > 1e-12 * sqrt(s_trace))) atomicMin(&s_lost, tid);
    __syncthreads();
    if (tid == 0) {
        double bad = (pass == 0) ? 0.0 : jb.scal[1 + OW_RMAX];
        if (bad == 0.0 && s_bad) bad = (double)s_bad;
        jb.scal[1 + OW_RMAX] = bad;
        if (last && jb.info) {
            if (bad != 0.0) flag_info(jb.info, jb.mode1, (int)bad);
            if (s_lost != 0x7fffffff) flag_info(jb.info, jb.mode1, s_lost + 1);
        }
    }
}

__global__ __launch_bounds__(128) void k_orthw_apply(OrthBatch a, int final_pass) {
    __shared__ double Ps[OP_RS][OW_LD];
    int ji, blk;
    find_job(a, &ji, &blk);
    const OrthJob jb = a.job[ji];
    // the first pass was found to be orthonormal already: its fp32 copy is the result
    if (final_pass && jb.scal[2 + OW_RMAX] != 0.0) return;
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int nb = (r + 15) / 16;
    const int i0 = blk * OP_RS;
    const int nrows = (n - i0 < OP_RS) ? n - i0 : OP_RS;
    for (int idx0 = 0; idx0 < OP_RS * OW_LD; idx0 += 128) {
        const int e = idx0 + tid;
        if (e < OP_RS * OW_LD) (&Ps[0][0])[e] = 0.0;
    }
    __syncthreads();
    for (int idx0 = 0; idx0 < nrows * r; idx0 += 128 * 8) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = idx0 + u * 128 + tid;
            t[u] = ldg_f64(jb.P64, (long long)i0 * r + idx, idx < nrows * r);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = idx0 + u * 128 + tid;
            if (idx < nrows * r) Ps[idx / r][idx % r] = t[u];
        }
    }
    __syncthreads();
    const int rw = 16 * wave;
    const double* __restrict__ R = jb.R;
    for (int b = 0; b < nb; ++b) {
        v4d acc = {0.0, 0.0, 0.0, 0.0};
        const int cb = 16 * b + ll;
        double dv[4];                                   // B operands of R_bb^-1
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dv[ks] = jb.Dinv[(b * 16 + 4 * ks + lg) * 16 + ll];
        for (int ab0 = 0; ab0 < b; ab0 += 4) {          // 16 global loads in flight
            double rv[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const int row = 16 * (ab0 + u) + 4 * ks + lg;
                    rv[u][ks] = ldg_f64(R, (long long)row * r + cb, ab0 + u < b && cb < r);
                }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (ab0 + u < b)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[rw + ll][16 * (ab0 + u) + 4 * ks + lg], rv[u][ks], acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) Ps[rw + lg + 4 * v][16 * b + ll] -= acc[v];
        __syncthreads();
        v4d q = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            q = __builtin_amdgcn_mfma_f64_16x16x4f64(Ps[rw + ll][16 * b + 4 * ks + lg], dv[ks], q, 0, 0, 0);
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 4; ++v) Ps[rw + lg + 4 * v][16 * b + ll] = q[v];
        __syncthreads();
    }
    if (final_pass) {
        for (int idx = tid; idx < nrows * r; idx += 128) jb.Uout[(long long)i0 * r + idx] = (float)Ps[idx / r][idx % r];
    } else {
        for (int idx = tid; idx < nrows * r; idx += 128) {
            const double q0 = Ps[idx / r][idx % r];
            jb.P64[(long long)i0 * r + idx] = q0;
            jb.Uout[(long long)i0 * r + idx] = (float)q0;
        }
    }
}

// ---- slow path: one workgroup per mode, global memory, three passes ---------------------------
constexpr int ORTH_NT = 512;
constexpr int ORTH_MAXR = 1024;

__global__ __launch_bounds__(ORTH_NT) void k_orth_big(OrthBatch a) {
    __shared__ double rdiag[ORTH_MAXR];
    __shared__ double s_inv;
    __shared__ double s_trace2;
    const OrthJob jb = a.job[blockIdx.x];
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    double* __restrict__ P = jb.P64;
    double* __restrict__ G = jb.Gpart;
    int32_t* info = jb.info;
    const long long cnt = (long long)n * r;
    for (long long e = tid; e < cnt; e += ORTH_NT) {
        double s = 0.0;
        for (int sp0 = 0; sp0 < jb.nsplit; sp0 += 8) {
            double t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = ldg_f64(jb.part, (long long)(sp0 + u) * cnt + e, sp0 + u < jb.nsplit);
#pragma unroll
            for (int u = 0; u < 8; ++u) s += t[u];
        }
        P[e] = s;
    }
    for (int k = tid; k < r; k += ORTH_NT) rdiag[k] = 1.0;
    __syncthreads();
    for (int pass = 0; pass < 3; ++pass) {
        for (int e = tid; e < r * r; e += ORTH_NT) {
            const int ca = e / r, cb = e - ca * r;
            if (ca <= cb) {
                double s = 0.0;
                for (int i = 0; i < n; ++i) s = fma(P[(long long)i * r + ca], P[(long long)i * r + cb], s);
                G[ca * r + cb] = s;
            }
        }
        __syncthreads();
        if (pass == 0) {
            if (tid == 0) {
                double tr = 0.0;
                for (int k = 0; k < r; ++k) tr += G[k * r + k];
                s_trace2 = tr;
            }
            __syncthreads();
            const double shift = 11.0 * ((double)n * r + (double)r * (r + 1)) * OP_EPS * s_trace2;
            for (int k = tid; k < r; k += ORTH_NT) G[k * r + k] += shift;
            __syncthreads();
        }
        for (int k = 0; k < r; ++k) {
            if (tid == 0) {
                double p = G[k * r + k];
                if (!(p > 0.0)) {
                    flag_info(info, jb.mode1, k + 1);
                    p = 1.0;
                }
                const double d = sqrt(p);
                G[k * r + k] = d;
                rdiag[k] *= d;
                s_inv = 1.0 / d;
            }
            __syncthreads();
            for (int j = k + 1 + tid; j < r; j += ORTH_NT) G[k * r + j] *= s_inv;
            __syncthreads();
            const int m = r - k - 1;
            for (int e = tid; e < m * m; e += ORTH_NT) {
                const int ca = k + 1 + e / m, cb = k + 1 + e % m;
                if (ca <= cb) G[ca * r + cb] -= G[k * r + ca] * G[k * r + cb];
            }
            __syncthreads();
        }
        for (int i = tid; i < n; i += ORTH_NT) {
            double* row = P + (long long)i * r;
            for (int j = 0; j < r; ++j) {
                double s = row[j];
                for (int k = 0; k < j; ++k) s -= row[k] * G[k * r + j];
                row[j] = s / G[j * r + j];
            }
        }
        __syncthreads();
    }
    if (tid == 0 && info) {
        const double floor_ = 1e-12 * sqrt(s_trace2);
        for (int k = 0; k < r; ++k)
            if (!(rdiag[k] > floor_)) { flag_info(info, jb.mode1, k + 1); break; }
    }
    for (long long e = tid; e < cnt; e += ORTH_NT) jb.Uout[e] = (float)P[e];
}

// ---- host side -------------------------------------------------------------------------------
bool orth_fast_supported(int r) { return r <= OP_RMAX; }
int orth_slices(int n) { return (n + OP_RS - 1) / OP_RS; }
bool orth_wide_supported(int r) { return r > OP_RMAX && r <= OW_RMAX; }
int orth_wide_gram_blocks(int n) { return (n + OW_ROWS - 1) / OW_ROWS; }

static bool put_orth(int kind, int aux, const char* label, const OrthArgs& a, int nblocks, Item* out) {
    if (nblocks <= 0) return false;
    *out = Item();
    out->kind = kind; out->aux = aux; out->nblocks = nblocks;
    std::snprintf(out->label, sizeof(out->label), "%s", label);
    static_assert(sizeof(OrthArgs) <= kItemArgMax && sizeof(PresumArgs) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &a, sizeof(a));
    return true;
}
static int total_blocks(const OrthArgs& a) {
    int t = 0;
    for (int j = 0; j < a.njobs; ++j) t += a.job[j].nblk;
    return t;
}
static bool fast_args_ok(const OrthArgs& a) {
    if (a.njobs <= 0 || a.njobs > 4) return false;
    for (int j = 0; j < a.njobs; ++j) {
        const OrthJob& jb = a.job[j];
        if (jb.n <= 0 || jb.r <= 0 || jb.r > OP_RMAX || jb.nblk != orth_slices(jb.n)) return false;
        if (!jb.Gpart || !jb.R || !jb.Dinv || !jb.scal || !jb.P64 || !jb.Uout || !jb.part || !jb.ctr) return false;
    }
    return true;
}
// summed: the factorisation may be handed slice Grams that a tree level has already added up (fewer of them)
static bool wide_args_ok(const OrthArgs& a, bool summed = false) {
    if (a.njobs <= 0 || a.njobs > 4) return false;
    for (int j = 0; j < a.njobs; ++j) {
        const OrthJob& jb = a.job[j];
        if (jb.n <= 0 || !orth_wide_supported(jb.r)) return false;
        if (summed ? (jb.nblk < 1 || jb.nblk > orth_wide_gram_blocks(jb.n)) : jb.nblk != orth_wide_gram_blocks(jb.n)) return false;
        if (!jb.Gpart || !jb.R || !jb.Dinv || !jb.scal || !jb.P64 || !jb.Uout) return false;
    }
    return true;
}

bool make_orth_presum(const PresumArgs& a, Item* out) {
    const int blocks = presum_blocks(a);
    if (blocks <= 0) return false;
    *out = Item();
    out->kind = IT_PRESUM; out->nblocks = blocks;
    std::snprintf(out->label, sizeof(out->label), "k_orth_presum");
    std::memcpy(out->arg, &a, sizeof(a));
    return true;
}
bool make_orthw_gsum(const GsumArgs& a, Item* out) {
    if (a.njobs <= 0 || a.njobs > 4) return false;
    long long blocks = 0;
    for (int j = 0; j < a.njobs; ++j) {
        const GsumJob& jb = a.job[j];
        if (!jb.in || !jb.out || !jb.devbits || jb.nblk < 1 || !orth_wide_supported(jb.r)) return false;
        if (jb.nchunks != (jb.r * jb.r + 255) / 256) return false;
        blocks += jb.nchunks;
    }
    *out = Item();
    out->kind = IT_ORTHW_GSUM; out->nblocks = (int)blocks;
    std::snprintf(out->label, sizeof(out->label), "k_orthw_gsum");
    static_assert(sizeof(GsumArgs) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &a, sizeof(a));
    return true;
}
bool make_orth_gram0(const OrthArgs& a, Item* out) {
    return fast_args_ok(a) && put_orth(IT_GRAM0, 0, "k_orth_gram0", a, total_blocks(a), out);
}
bool make_orth_apply(const OrthArgs& a, Item* out) {
    return fast_args_ok(a) && put_orth(IT_APPLY, 0, "k_orth_apply", a, total_blocks(a), out);
}
bool make_orthw_gram(const OrthArgs& a, Item* out) {
    return wide_args_ok(a) && put_orth(IT_ORTHW_GRAM, 0, "k_orthw_gram", a, total_blocks(a), out);
}
bool make_orthw_chol(const OrthArgs& a, int pass, int last, Item* out) {
    return wide_args_ok(a, true) && put_orth(IT_ORTHW_CHOL, (pass ? 1 : 0) | (last ? 2 : 0), "k_orthw_chol", a, a.njobs, out);
}
bool make_orthw_apply(const OrthArgs& a, int final_pass, Item* out) {
    if (!wide_args_ok(a)) return false;
    OrthArgs b = a;                                // apply walks 32-row slices
    for (int j = 0; j < b.njobs; ++j) b.job[j].nblk = orth_slices(b.job[j].n);
    return put_orth(IT_ORTHW_APPLY, final_pass ? 1 : 0, "k_orthw_apply", b, total_blocks(b), out);
}
bool make_orth_big(const OrthArgs& a, Item* out) {
    if (a.njobs <= 0 || a.njobs > 4) return false;
    for (int j = 0; j < a.njobs; ++j)
        if (a.job[j].r > ORTH_MAXR || !a.job[j].Gpart || !a.job[j].P64 || !a.job[j].part || !a.job[j].Uout) return false;
    return put_orth(IT_ORTH_BIG, 0, "k_orth_big", a, a.njobs, out);
}

struct InitBatch {
    int32_t* p[kMaxBatch];
    int n;
};
__global__ void k_init_ctrl(InitBatch b) {
    if (threadIdx.x < b.n && b.p[threadIdx.x]) *b.p[threadIdx.x] = 0;
}
bool make_init_ctrl(int32_t* info, Item* out) {
    if (!info) return false;
    *out = Item();
    out->kind = IT_INIT; out->nblocks = 1;
    std::snprintf(out->label, sizeof(out->label), "k_init_ctrl");
    std::memcpy(out->arg, &info, sizeof(info));
    return true;
}

hipError_t launch_orth_items(const Item* const* items, int n, hipStream_t st, char* label_out) {
    if (n <= 0 || n > kMaxBatch) return hipErrorInvalidValue;
    const int kind = items[0]->kind, aux = items[0]->aux;
    if (kind == IT_INIT) {
        InitBatch b;
        b.n = n;
        for (int j = 0; j < kMaxBatch; ++j) b.p[j] = nullptr;
        for (int j = 0; j < n; ++j) std::memcpy(&b.p[j], items[j]->arg, sizeof(int32_t*));
        hipLaunchKernelGGL(k_init_ctrl, 1, 64, 0, st, b);
        return hipGetLastError();
    }
    long long blocks = 0;
    for (int j = 0; j < n; ++j) blocks += items[j]->nblocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    if (kind == IT_PRESUM) {
        PresumBatch b;
        b.njobs = 0;
        for (int j = 0; j < n; ++j) {
            PresumArgs a;
            std::memcpy(&a, items[j]->arg, sizeof(a));
            for (int k = 0; k < a.njobs; ++k) b.job[b.njobs++] = a.job[k];
        }
        hipLaunchKernelGGL(k_orth_presum, grid, 256, 0, st, b);
        return hipGetLastError();
    }
    if (kind == IT_ORTHW_GSUM) {
        GsumBatch b;
        b.njobs = 0;
        for (int j = 0; j < n; ++j) {
            GsumArgs a;
            std::memcpy(&a, items[j]->arg, sizeof(a));
            for (int k = 0; k < a.njobs; ++k) b.job[b.njobs++] = a.job[k];
        }
        hipLaunchKernelGGL(k_orthw_gsum, grid, 256, 0, st, b);
        return hipGetLastError();
    }
    OrthBatch b;
    b.njobs = 0;
    int rmax = 0;
    for (int j = 0; j < n; ++j) {
        OrthArgs a;
        std::memcpy(&a, items[j]->arg, sizeof(a));
        for (int k = 0; k < a.njobs; ++k) {
            b.job[b.njobs++] = a.job[k];
            rmax = a.job[k].r > rmax ? a.job[k].r : rmax;
        }
    }
    const int rm = rmax <= 16 ? 16 : (rmax <= 32 ? 32 : (rmax <= 48 ? 48 : 64));   // register shape of the fast kernels
    if (label_out && (kind == IT_GRAM0 || kind == IT_APPLY))
        std::snprintf(label_out, 96, "%s<%d>", kind == IT_GRAM0 ? "k_orth_gram0" : "k_orth_apply", rm);
    switch (kind) {
        case IT_GRAM0:
            if (rm == 16) hipLaunchKernelGGL(k_orth_gram0<16>, grid, 256, 0, st, b);
            else if (rm == 32) hipLaunchKernelGGL(k_orth_gram0<32>, grid, 256, 0, st, b);
            else if (rm == 48) hipLaunchKernelGGL(k_orth_gram0<48>, grid, 256, 0, st, b);
            else hipLaunchKernelGGL(k_orth_gram0<64>, grid, 256, 0, st, b);
            break;
        case IT_APPLY:
            if (rm == 16) hipLaunchKernelGGL(k_orth_apply<16>, grid, 256, 0, st, b);
            else if (rm == 32) hipLaunchKernelGGL(k_orth_apply<32>, grid, 256, 0, st, b);
            else if (rm == 48) hipLaunchKernelGGL(k_orth_apply<48>, grid, 256, 0, st, b);
            else hipLaunchKernelGGL(k_orth_apply<64>, grid, 256, 0, st, b);
            break;
        case IT_ORTHW_GRAM:
            hipLaunchKernelGGL(k_orthw_gram, grid, 256, 0, st, b);
            break;
        case IT_ORTHW_CHOL: {
            // packed triangle, dinv, rdiag, pivot reciprocals, inverse block factor, row exchange buffer
            const size_t nb16 = (size_t)((rmax + 15) / 16) * 16;
            const size_t lds = sizeof(double) * ((size_t)rmax * (rmax + 1) / 2 + 2 * (size_t)rmax + nb16 + 16 * 17 + 2 * 64 * 4);
            static std::atomic<size_t> lds_allowed{0};     // the attribute only ever needs to grow
            if (lds > lds_allowed.load()) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_orthw_chol),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return e;
                lds_allowed.store(lds);
            }
            hipLaunchKernelGGL(k_orthw_chol, grid, OWC_NT, lds, st, b, aux & 1, (aux >> 1) & 1);
            break;
        }
        case IT_ORTHW_APPLY:
            hipLaunchKernelGGL(k_orthw_apply, grid, 128, 0, st, b, aux);
            break;
        case IT_ORTH_BIG:
            hipLaunchKernelGGL(k_orth_big, grid, ORTH_NT, 0, st, b);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace asi
