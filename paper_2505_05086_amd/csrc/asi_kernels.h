// Host-side interface of the ASI kernels.  All data pointers are device pointers.
//
// Every kernel launch is prepared as an Item: the kernel instantiation (kind, key), its grid and its
// argument block for ONE layer.  Items of several layers that name the same instantiation are
// launched together (launch_items): the kernel receives the argument blocks side by side and
// each workgroup finds its layer from its block index.  A step over L layers therefore costs as
// many launches as a step over one.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

namespace asi {

enum DType { F32 = 0, BF16 = 1 };

constexpr int kMaxBatch = 8;         // layers one launch can serve
constexpr int kItemArgMax = 640;     // bytes of the largest per-layer argument block

enum ItemKind {
    IT_TTM = 1, IT_KSPLIT, IT_PAIR, IT_SMALL, IT_PRESUM, IT_GRAM0, IT_APPLY, IT_ORTHW_GRAM, IT_ORTHW_CHOL,
    IT_ORTHW_APPLY, IT_ORTH_BIG, IT_CORR_MFMA, IT_CORR, IT_SUM_F32, IT_SUM_F64, IT_EXPAND, IT_INIT, IT_TINY, IT_TTM_DUO, IT_TTM_STREAM, IT_TTM_EXPAND,
    IT_LONG, IT_PLANES, IT_SPLIT_BF16, IT_GEMM_BF16, IT_GAUSS, IT_GRAM_MODE, IT_DW_FOLD, IT_Z_PLANES, IT_CORE_PLANES, IT_ORTHW_GSUM
};

struct Item {
    int kind = 0;
    unsigned key = 0;        // instantiation within the kind
    int nblocks = 0;         // workgroups of this layer
    int aux = 0;             // kind specific (orth: final pass / pass number)
    char label[96];          // kernel instantiation the way a profiler prints it
    char role[16];           // what the launch computes ("V", "core", "dW", ...), for timing reports
    double bytes = 0, flops = 0;   // what this launch must move / compute by its definition
    alignas(16) unsigned char arg[kItemArgMax];
};

// Launches items[0..n) as ONE kernel launch, n <= kMaxBatch; they must be mergeable (same_launch).
// label_out (nullable, 96 bytes) receives the name of the instantiation that ran.
hipError_t launch_items(const Item* const* items, int n, hipStream_t st, char* label_out);
// Items of the same kernel whose instantiations differ only in size bounds (column blocks, steps)
// share the launch of the largest.
bool same_launch(const Item& a, const Item& b);

// Argument blocks side by side; workgroup `blockIdx.x` belongs to the job j with first[j] <= blockIdx.x < first[j+1].
template <typename J>
struct Batch {
    int njobs;
    int first[kMaxBatch + 1];
    J job[kMaxBatch];
};

// device side: index of the job this workgroup belongs to, and its block index inside that job
template <typename J>
__device__ __forceinline__ int locate(const Batch<J>& b, int* local) {
    int j = 0;
    const int bid = blockIdx.x;
    while (j + 1 < b.njobs && bid >= b.first[j + 1]) ++j;
    *local = bid - b.first[j];
    return j;
}
// Workgroups are handed to the 8 XCDs (each with its own L2) in round-robin order of their index, so
// neighbouring indices never share an L2.  This renumbering gives every XCD one contiguous eighth
// of a job's nb blocks instead: tiles that touch the same cache lines (adjacent column groups of an
// unfolding, the tiles of one operand) then meet in one L2 rather than each fetching the line from
// memory.  A bijection on [0, nb); only performance depends on the dispatch order.
__device__ __forceinline__ int xcd_order(int lb, int nb) {
    const int chunk = nb >> 3, rem = nb & 7, x = lb & 7, k = lb >> 3;
    return x * chunk + (x < rem ? x : rem) + k;
}
template <typename J>
__device__ __forceinline__ int locate_xcd(const Batch<J>& b, int* local) {
    const int j = locate(b, local);
    *local = xcd_order(*local, b.first[j + 1] - b.first[j]);
    return j;
}
// host side: argument blocks of items[0..n) side by side, grid = all their workgroups
template <typename J>
inline bool gather(const Item* const* items, int n, Batch<J>* b, dim3* grid) {
    if (n <= 0 || n > kMaxBatch) return false;
    long long total = 0;
    b->njobs = n;
    for (int j = 0; j < n; ++j) {
        b->first[j] = (int)total;
        memcpy(&b->job[j], items[j]->arg, sizeof(J));
        total += items[j]->nblocks;
        if (items[j]->nblocks <= 0 || total > 0x7fffffffLL) return false;
    }
    for (int j = n; j <= kMaxBatch; ++j) b->first[j] = (int)total;
    *grid = dim3((unsigned)total);
    return true;
}

// ---- m-mode product (Eq. 4 along one mode) -------------------------------------------------------
// Y[o,q,j] (+)= sum_i X[o,i,j] * M(i,q),  M(i,q) = Mp[i*ms_i + q*ms_q];  X: (outer, n, inner) of dtype xt,
// Y: (outer, r, inner) fp32.  With a second factor (kron) the matrix is the Kronecker product
// M(i,q) = M1(i / n2, q / r2) * M2(i % n2, q % r2), which contracts two adjacent trailing modes at once
// (inner must be 1).
struct KronSpec {
    const float* M2;       // second factor; element (i2, q2) at M2[i2 * ms_i + q2 * ms_q]; null = none
    long long ms_i, ms_q;
    int n2, r2;            // i = i1 * n2 + i2,  q = q1 * r2 + q2
};
struct TtmJob {
    const void* X;
    long long outer, inner;
    const float* Mp;
    long long ms_i, ms_q;
    float* Y;
    KronSpec kr;
    int n, r, beta;
    int gx, gy;            // grid of this job: column tiles x output tiles
    int tile_cols;         // tiled kernel: unfolding columns per tile (64, or whole outer indices for a short inner)
    int32_t* zero;         // nullable: `nzero` int32 the kernel clears (arrival counters of later launches)
    int nzero;
};
// stream_ok = false keeps the product on the tiled kernels (which can share a launch with a second product, make_ttm_duo)
constexpr long long kStreamMinElems = 1LL << 20;
bool make_ttm(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
              long long ms_q, int r, float* Y, int beta, Item* out, bool stream_ok = true);
// the same product by the streaming kernel (asi_ttm_stream.hip); make_ttm picks it where it is supported and faster
bool ttm_stream_supported(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp,
                          long long ms_i, long long ms_q, int r, const float* Y);
bool make_ttm_stream(DType xt, const void* X, long long outer, int n, long long inner, const float* Mp, long long ms_i,
                     long long ms_q, int r, float* Y, int beta, Item* out);
bool make_ttm_kron(DType xt, const void* X, long long cols, int n1, int n2, const float* M1, long long ms1_i,
                   long long ms1_q, int r1, const float* M2, long long ms2_i, long long ms2_q, int r2, float* Y,
                   int beta, Item* out);

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
// device side: workgroup b of the partial-sum tree's first level (groups of 32 splits, fixed order)
__device__ __forceinline__ void presum_block(const PresumJob* jobs, int njobs, int b) {
    int j = 0;
    while (j + 1 < njobs && b >= jobs[j].nchunks * jobs[j].ngroups) { b -= jobs[j].nchunks * jobs[j].ngroups; ++j; }
    const PresumJob& jb = jobs[j];
    const int g = b / jb.nchunks, chunk = b - g * jb.nchunks;
    const long long e = (long long)chunk * 256 + threadIdx.x;
    if (e >= jb.cnt) return;
    const int s0 = g * 32;
    double t[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) {
        const bool ok = s0 + u < jb.nsplit;
        const double v = jb.in[ok ? (long long)(s0 + u) * jb.cnt + e : 0];
        t[u] = ok ? v : 0.0;
    }
    double s = 0.0;
#pragma unroll
    for (int u = 0; u < 32; ++u) s += t[u];
    jb.out[(long long)g * jb.cnt + e] = s;
}

// One launch for two independent products made by make_ttm / make_ttm_kron (tagged with role, bytes, flops):
// a plain tiled product not along the last mode, and a small merged (Kronecker) product.  Returns false
// if the items do not have these forms.
bool make_ttm_duo(const Item& a, const Item& z, Item* out);

// ---- product along the last mode of a bf16 tensor on the bf16 MFMA (asi_bf16.hip) -----------------------------
// Y[c,q] = sum_i X[c,i] M[i,q]: X (ncols, n) bf16, Y (ncols, r) fp32.  The fp32 matrix is first split into two bf16
// terms laid out in operand order (make_split_bf16 -> Mb of split_bf16_elems(n, r) 16-bit elements).
bool gemm_bf16_supported(long long ncols, int n, int r);
size_t split_bf16_elems(int n, int r);
bool make_split_bf16(const float* M, long long ms_i, long long ms_q, int n, int r, unsigned short* Mb, Item* out);
// Few columns: the contraction is split over gemm_bf16_ksplit workgroups per column tile; Y then takes that
// many partial products (ksplit, ncols, r), to be summed by make_sum_partials.
int gemm_bf16_ksplit(long long ncols, int n, int r);
bool make_gemm_bf16(const void* X, long long ncols, int n, const unsigned short* Mb, int r, float* Y, int ksplit,
                    int32_t* zero, int nzero, Item* out);

// ---- pair: part[s][i][q] = sum_{c in split s} X[i,c] * Y[q,c]  over unfolding columns c = (o,j) -----
// X: (outer, n, inner) dtype xt;  Y: (outer, r, inner) fp32;  part: (nsplit, n, r) fp64
// (products of fp32 values are exact in fp64 and the sums are carried in fp64).
struct PairJob {
    const void* X;
    long long outer, inner, cols_per_split;
    const float* Y;        // null in the generating variant: Y[., q, .] is the standard-normal V of Alg. 1's t = 0
    double* part;
    int n, r;
    uint32_t seed_lo, seed_hi;   // generating variant: key of the counter-based generator, and the mode (0-based)
    int mode;
    int gx, gy, gz;        // row tiles x output tiles x splits
    int32_t* zero;         // nullable: `nzero` int32 the kernel clears
    int nzero;
    // independent work that rides along in extra workgroups: the first level of the partial-sum
    // tree of OTHER modes, whose partial sums are complete before this launch
    int pre_blocks;
    PresumArgs pre;
};
int pair_splits(long long outer, int n, long long inner, int r);
bool make_pair(DType xt, const void* X, long long outer, int n, long long inner, const float* Y, int r, double* part,
               int nsplit, int32_t* zero, int nzero, const PresumArgs* pre, Item* out);
// the same with Y = the generated standard-normal V of mode `mode` (Alg. 1, t = 0)
bool make_pair_gauss(DType xt, const void* X, long long outer, int n, long long inner, unsigned long long seed, int mode,
                     int r, double* part, int nsplit, int32_t* zero, int nzero, const PresumArgs* pre, Item* out);
// V itself, (ncols, r) row-major fp32, for inspection: the entries the generating variant multiplies by
bool make_gauss_fill(unsigned long long seed, int mode, long long ncols, int r, float* V, Item* out);
int presum_blocks(const PresumArgs& a);      // workgroups of the tree's first level, -1 if a is malformed

// ---- out[e] = (beta ? out[e] : 0) + sum_s part[s*count + e] ---------------------------------------------
struct SumJob {
    const void* part;
    float* out;
    long long count;
    int nsplit, beta;
};
bool make_sum_partials(const float* part, int nsplit, long long count, float* out, int beta, Item* it);
bool make_sum_partials_f64(const double* part, int nsplit, long long count, float* out, int beta, Item* it);

// ---- short mode with a long inner extent through its Gram matrix (asi_gram.hip): part is (nwg, n, r) fp64 ----
// P = (A_m A_m^T) U_prev: one pass accumulates the n x n Gram matrix in fp64, V is never formed
bool subspace_gram_supported(long long outer, int n, long long inner, int r);
int subspace_gram_nwg(long long outer, int n, long long inner);
bool make_subspace_gram(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r, double* part,
                        int nwg, int32_t* zero, int nzero, Item* out);
hipError_t launch_gram_items(const Item* const* items, int n, hipStream_t st);

// ---- fused V/P step for modes with n <= 64 (asi_subspace.hip): part is (nwg, n, r) fp64 ---------------
bool subspace_small_supported(int n, int r);
int subspace_small_nwg(long long outer, int n, long long inner);
bool make_subspace_small(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r,
                         double* part, int nwg, int32_t* zero, int nzero, Item* out);
// The last two modes of X seen as (planes, rows, cols), both from one read of X.
bool subspace_pair_supported(int rows, int cols, int r_rows, int r_cols);
int subspace_pair_nwg(long long planes, int rows, int cols);
bool make_subspace_pair(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                        double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, Item* out);

// ---- fused V/P step for modes with 64 < n <= 512 and r <= 64 (asi_long.hip): part is (nsplit, n, r) fp64 -------
bool subspace_long_supported(long long outer, int n, long long inner, int r);
int subspace_long_splits(long long outer, int n, long long inner, int r);
bool make_subspace_long(DType xt, const void* X, long long outer, int n, long long inner, const float* U, int r,
                        double* part, int nsplit, int32_t* zero, int nzero, Item* out);

// The last two modes of large planes (33..64 rows and columns, ranks up to 32, at least 1024 planes; asi_planes.hip):
// part_rows is (nwg, rows, r_rows), part_cols (nwg, cols, r_cols).
bool subspace_planes_supported(long long planes, int rows, int cols, int r_rows, int r_cols);
int subspace_planes_nwg(long long planes);
bool make_subspace_planes(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                          double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, int32_t* zero,
                          int nzero, Item* out);

// Both when rows, cols and both ranks are at most 8: vector-ALU kernel, no MFMA padding.
bool subspace_tiny_supported(int rows, int cols, int r_rows, int r_cols);
int subspace_tiny_nwg(long long planes);
bool make_subspace_tiny(DType xt, const void* X, long long planes, int rows, int cols, const float* U_rows, int r_rows,
                        double* part_rows, const float* U_cols, int r_cols, double* part_cols, int nwg, Item* out);

// ---- Orthogonalize (asi_orth.hip) ---------------------------------------------------------------------------
struct OrthJob {
    const double* part;  // (nsplit, n, r) partial sums of P
    double* P64;         // (n, r) scratch
    float* Uout;         // (n, r)
    int32_t* info;       // nullable
    // fast path (r <= 64) and wide path
    double* Gpart;       // (nblk, r (r+1) / 2) packed slice Gram matrices; slow path: (r, r) Gram matrix
    double* R;           // (r, r)
    double* Dinv;        // (ceil(r/16), 16, 16) inverses of R's diagonal blocks
    double* scal;        // 68 doubles of bookkeeping (wide path: 2 + 192)
    int32_t* ctr;        // 2 arrival counters, zero before the first orth launch of a call
    int nsplit;
    int n, r;
    int mode1;           // 1-based mode number for *info
    int nblk;            // row slices = orth_slices(n) (wide path: orth_wide_gram_blocks(n))
    int pad_;
    unsigned long long* devbits;   // wide path with a summed Gram matrix (make_orthw_gsum): bits of max |G - I|; else null
};
struct OrthArgs {        // the modes of one tensor that share a path
    OrthJob job[4];
    int njobs;
};
bool make_orth_presum(const PresumArgs& a, Item* out);
// Wide path, many slices: the slice Gram matrices of a mode added up into ONE matrix (slice after slice, in their
// order), and the largest deviation of its upper triangle from the identity raised into *devbits (the bit pattern of
// a non-negative double, so that an integer atomic maximum orders it; the first factorisation clears it).
struct GsumJob {
    const double* in;    // (nblk, r, r), upper triangles valid
    double* out;         // (r, r)
    unsigned long long* devbits;
    int nblk, r, nchunks;   // nchunks = ceil(r r / 256)
};
struct GsumArgs {
    GsumJob job[4];
    int njobs;
};
bool make_orthw_gsum(const GsumArgs& a, Item* out);
bool orth_fast_supported(int r);
int orth_slices(int n);
// gram0: sums the partial sums of P, slice Grams; the last workgroup of a mode factors (shifted pass)
//        and clears *info.
// apply(0): Q0 = P R0^-1, slice Grams of Q0; the last workgroup of a mode factors again.
// apply(1): U = Q0 R1^-1 in fp32.
bool make_orth_gram0(const OrthArgs& a, Item* out);
bool make_orth_apply(const OrthArgs& a, Item* out);
// wide path, 64 < r <= 192: nblk = orth_wide_gram_blocks(n), scal holds 2 + 192 doubles,
// P64 must already hold the summed P (make_orth_presum with a single group does that)
bool orth_wide_supported(int r);
int orth_wide_gram_blocks(int n);
bool make_orthw_gram(const OrthArgs& a, Item* out);
bool make_orthw_chol(const OrthArgs& a, int pass, int last, Item* out);
bool make_orthw_apply(const OrthArgs& a, int final_pass, Item* out);
bool make_orth_big(const OrthArgs& a, Item* out);
bool make_init_ctrl(int32_t* info, Item* out);   // *info = 0

// ---- step 4 of Eq. 14: T[o,j,kh,kw] = sum_{i,y,x} G1[i,o,y,x] * Zpad[i,j,y*s-p+kh*d, x*s-p+kw*d] -----------
// G1: (r1, cout, Ho, Wo);  Z: (r1, r2, H, W);  Tpart: (nsplit, cout, r2, kh, kw), split over i.
struct CorrGeom {
    int r1, r2, cout, H, W, Ho, Wo, kh, kw, sh, sw, ph, pw, dh, dw;
};
int corr_splits(const CorrGeom& g);
bool make_corr(const float* G1, const float* Z, float* Tpart, const CorrGeom& g, int nsplit, Item* out);

// ---- step 5 of Eq. 14 with groups: dW[o,c,t] (+)= sum_j T[o,j,t] * U2[(o/og)*cg + c, j] -----------------------
struct ExpandJob {
    const float* T;
    const float* U2;
    float* dW;
    int cout, r2, taps, cg, og, beta;
};
bool make_expand_grouped(const float* T, const float* U2, float* dW, int cout, int r2, int taps, int cg, int og,
                         int beta, Item* out);

// per-kind batch launchers (called by launch_items)
hipError_t launch_ttm_items(const Item* const* items, int n, hipStream_t st, char* label_out);
hipError_t launch_ttm_stream_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_ttm_expand_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_ttm_duo_items(const Item* const* items, int n, hipStream_t st, char* label_out);
hipError_t launch_pair_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_sum_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_expand_items(const Item* const* items, int n, hipStream_t st);

// ---- step 5 of Eq. 14 for an ungrouped convolution with a small core (asi_kernels.hip) ------------------------
// dW[o, c, t] (+)= sum_j T[o, j, t] U2[c, j] with T given as nsplit >= 1 partial tensors of (cout, r2, taps): one
// launch adds up the partial sums of the correlation and expands the result, and T is never written.  taps is
// 1 or 9, r2 <= 64.  False for anything else (the caller then sums and multiplies in two launches).
bool make_dw_fold(const float* Tpart, int nsplit, const float* U2, float* dW, int cout, int C, int r2, int taps, int beta,
                  Item* out);
hipError_t launch_dw_fold_items(const Item* const* items, int n, hipStream_t st);

// ---- steps 2 and 3 of Eq. 14 for large planes in one launch (asi_kernels.hip) ----------------------------------
// Z[p] = U3 S[p] U4^T for every plane p of the core: S (planes, r3, r4), U3 (H, r3), U4 (W, r4), Z (planes, H, W);
// H, W <= 64, r3, r4 <= 32 and multiples of 4, W a multiple of 4, 16-byte aligned pointers.  False otherwise (the
// caller then takes the two mode products one after the other).
bool make_z_planes(const float* S, long long planes, int r3, int r4, const float* U3, int H, const float* U4, int W, float* Z,
                   Item* out);
hipError_t launch_z_planes_items(const Item* const* items, int n, hipStream_t st);

// ---- the H and W products of the core projection for large planes in one launch (asi_kernels.hip) -----------
// Y[p] = U3^T X[p] U4 for every plane p: X (planes, H, W) fp32, U3 (H, r3), U4 (W, r4), Y (planes, r3, r4); H, W <= 64,
// r3, r4 <= 32, W a multiple of 4, X 16-byte aligned.  False otherwise (the caller takes the two mode products).
bool make_core_planes(const float* X, long long planes, int H, int W, const float* U3, int r3, const float* U4, int r4, float* Y,
                      Item* out);
hipError_t launch_core_planes_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_small_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_tiny_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_long_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_planes_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_bf16_items(const Item* const* items, int n, hipStream_t st);
hipError_t launch_orth_items(const Item* const* items, int n, hipStream_t st, char* label_out);
hipError_t launch_corr_items(const Item* const* items, int n, hipStream_t st);

}  // namespace asi
