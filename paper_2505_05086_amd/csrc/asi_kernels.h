// Host-side launchers of the ASI kernels.  All pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asi {

enum DType { F32 = 0, BF16 = 1 };

// Name of the kernel instantiation the last launcher call on this thread picked, written the
// way a profiler prints it (e.g. "k_ttm_mfma<float, false, 3>"); used to tag timing records.
void set_last_label(const char* fmt, ...);
const char* last_label();

// Y[o,q,j] = sum_i X[o,i,j] * M(i,q),  M(i,q) = Mp[i*ms_i + q*ms_q]   (Eq. 4 along one mode)
// X: (outer, n, inner) of dtype xt;  Y: (outer, r, inner) fp32;  beta != 0 adds to Y.
hipError_t launch_ttm(DType xt, const void* X, long long outer, int n, long long inner,
                      const float* Mp, long long ms_i, long long ms_q, int r,
                      float* Y, int beta, hipStream_t st);

// Two adjacent trailing modes in one pass (small extents): X is (cols, n1*n2) row-major,
//   Y[c, q1*r2 + q2] (+)= sum_{i1,i2} X[c, i1*n2 + i2] * M1(i1,q1) * M2(i2,q2),  Mk(i,q) = Mk[i*msk_i + q*msk_q]
hipError_t launch_ttm_kron(DType xt, const void* X, long long cols, int n1, int n2, const float* M1,
                           long long ms1_i, long long ms1_q, int r1, const float* M2, long long ms2_i,
                           long long ms2_q, int r2, float* Y, int beta, hipStream_t st);

// part[s][i][q] = sum_{c in split s} X[i,c] * Y[q,c]  over unfolding columns c = (o,j)
// X: (outer, n, inner) dtype xt;  Y: (outer, r, inner) fp32;  part: (nsplit, n, r) fp64
// (products of fp32 values are exact in fp64 and the sums are carried in fp64).
hipError_t launch_pair(DType xt, const void* X, long long outer, int n, long long inner,
                       const float* Y, int r, double* part, int nsplit, hipStream_t st);
int pair_splits(long long outer, int n, long long inner, int r);

// out[e] = (beta ? out[e] : 0) + sum_s part[s*count + e]
hipError_t launch_sum_partials(const float* part, int nsplit, long long count, float* out, int beta,
                               hipStream_t st);
hipError_t launch_sum_partials_f64(const double* part, int nsplit, long long count, float* out, int beta,
                                   hipStream_t st);

// Fused V/P step for a mode with n <= 64 (asi_subspace.hip): part is (nwg, n, r) fp64.
bool subspace_small_supported(int n, int r);
int subspace_small_nwg(long long outer, int n, long long inner);
hipError_t launch_subspace_small(DType xt, const void* X, long long outer, int n, long long inner, const float* U,
                                 int r, double* part, int nwg, hipStream_t st);
// The last two modes of X seen as (planes, rows, cols), both from one read of X.
bool subspace_pair_supported(int rows, int cols, int r_rows, int r_cols);
int subspace_pair_nwg(long long planes, int rows, int cols);
hipError_t launch_subspace_pair(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows,
                                int r_rows, double* part_rows, const float* U_cols, int r_cols, double* part_cols,
                                int nwg, hipStream_t st);

struct OrthJob {
    const double* part;  // (nsplit, n, r) partial sums of P
    int nsplit;
    int n, r;
    double* P64;         // (n, r) scratch
    float* Uout;         // (n, r)
    int mode1;           // 1-based mode number for *info
    // fast path (r <= 64)
    int nblk;            // row slices = orth_slices(n)
    double* Gpart;       // (nblk, r, r) slice Gram matrices
    double* R;           // (r, r)
    double* Dinv;        // (ceil(r/16), 16, 16) inverses of R's diagonal blocks
    double* scal;        // 66 doubles of bookkeeping
    // slow path (r > 64)
    double* G;           // (r, r)
};
struct OrthArgs {
    OrthJob job[4];
    int njobs;
    int32_t* info;       // nullable
};
struct PresumJob {
    const double* in;    // (nsplit, cnt)
    double* out;         // (ngroups, cnt), ngroups = ceil(nsplit / 32)
    long long cnt;
    int nsplit, nchunks, ngroups;   // nchunks = ceil(cnt / 256)
};
struct PresumArgs {
    PresumJob job[4];
    int njobs;
};
hipError_t launch_orth_presum(const PresumArgs& a, hipStream_t st);
bool orth_fast_supported(int r);
int orth_slices(int n);
hipError_t launch_orth_gram0(const OrthArgs& a, hipStream_t st);
hipError_t launch_orth_chol(const OrthArgs& a, int pass, int last, hipStream_t st);
hipError_t launch_orth_apply(const OrthArgs& a, int final_pass, hipStream_t st);
// wide path, 64 < r <= 192: nblk = orth_wide_gram_blocks(n), scal holds 2 + 192 doubles,
// P64 must already hold the summed P (launch_orth_presum with a single group does that)
bool orth_wide_supported(int r);
int orth_wide_gram_blocks(int n);
hipError_t launch_orthw_gram(const OrthArgs& a, hipStream_t st);
hipError_t launch_orthw_chol(const OrthArgs& a, int pass, int last, hipStream_t st);
hipError_t launch_orthw_apply(const OrthArgs& a, int final_pass, hipStream_t st);
hipError_t launch_orth_big(const OrthArgs& a, hipStream_t st);
hipError_t launch_init_ctrl(int32_t* info, hipStream_t st);   // *info = 0 if non-null
hipError_t launch_set_i32(int32_t* p, int32_t v, hipStream_t st);

// Step 4 of Eq. 14: T[o,j,kh,kw] = sum_{i,y,x} G1[i,o,y,x] * Zpad[i,j,y*s-p+kh*d, x*s-p+kw*d]
// G1: (r1, cout, Ho, Wo);  Z: (r1, r2, H, W);  Tpart: (nsplit, cout, r2, kh, kw), split over i.
struct CorrGeom {
    int r1, r2, cout, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, dh, dw;
};
int corr_splits(const CorrGeom& g);
hipError_t launch_corr(const float* G1, const float* Z, float* Tpart, const CorrGeom& g, int nsplit,
                       hipStream_t st);

// Step 5 of Eq. 14 with groups: dW[o,c,t] (+)= sum_j T[o,j,t] * U2[(o/og)*cg + c, j]
hipError_t launch_expand_grouped(const float* T, const float* U2, float* dW, int cout, int r2, int taps,
                                 int cg, int og, int beta, hipStream_t st);

}  // namespace asi
