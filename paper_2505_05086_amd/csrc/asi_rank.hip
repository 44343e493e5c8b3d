// Rank-selection front end (Sec. 3.3): what has to be measured on a stored activation before training
// starts, so that ranks can be chosen per layer under a memory budget.
//
//   mode spectrum      eigenvalues (and eigenvectors) of G = A_m A_m^T, the squared singular values and
//                      left singular vectors of the mode-m unfolding (App. A.2): k_mode_gram accumulates
//                      G in fp64 on the MFMA, split over column ranges; k_gram_reduce adds the ranges in a
//                      fixed order; a cyclic one-sided Jacobi iteration (k_jacobi_round, one launch per
//                      round of disjoint row pairs, one wave per pair) orthogonalises the rows of W = G,
//                      after which row k is lambda_k v_k^T; k_spectrum_finish sorts.
//   explained variance ranks per threshold (Sec. 3.3, Step 1): k_ev_ranks.
//   perplexity         Frobenius norm of the difference of two weight gradients (Eq. 7): k_frob_partial,
//                      k_frob_final.
//   budgeted choice    Eq. 8-9 by recursive backtracking with bounds, on the host (asi_rank_select).
//
// The compressed gradient itself comes from the library's hot path (asi_core_project and
// asi_weight_grad_* on the truncated eigenvectors).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

#include "../../include/asi.h"
#include "asi_device.h"

namespace {

using namespace asi;

typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int RK_NMAX = 512;            // longest mode the Jacobi kernel takes (8 elements per lane)
constexpr int RK_T = 64;                // Gram tile: 64 x 64 outputs, 64 unfolding columns per chunk
constexpr int RK_LD = RK_T + 4;         // LDS row pitch in floats (16 bytes more than a multiple of 128)
constexpr int RK_MAX_SPLIT = 256;
constexpr size_t RK_ALIGN = 256;
constexpr int RK_FROB_WG = 1024;

inline size_t align_up(size_t x) { return (x + RK_ALIGN - 1) / RK_ALIGN * RK_ALIGN; }

struct GramJob {
    const void* X;
    long long outer, inner, ncols;
    int n, tiles, nsplit, nchunks;
    double* part;                       // (nsplit, n, n)
};

// One 64 x 64 tile of G over the column chunks z, z + nsplit, ...  Wave w owns rows 16 w .. 16 w + 15 of the
// tile.  Both operands come from LDS tiles held row-major (mode index x columns); a 16-byte read gives a lane
// the columns 4 lg .. 4 lg + 3 of a 16-column block, which stand for K slot lg of four MFMA steps (the same
// assignment for both operands, and a sum over columns does not care about their order).
template <typename T>
__global__ __launch_bounds__(256) void k_mode_gram(GramJob jb) {
    __shared__ __align__(16) float Xi[RK_T * RK_LD];
    __shared__ __align__(16) float Xj[RK_T * RK_LD];
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int tile = blockIdx.x % (jb.tiles * jb.tiles), z = blockIdx.x / (jb.tiles * jb.tiles);
    const int bi = tile / jb.tiles, bj = tile - bi * jb.tiles;
    const int n = jb.n;
    const long long inner = jb.inner, ncols = jb.ncols;
    const bool diag = bi == bj;
    const bool last = inner == 1;       // the mode index is the contiguous one: lanes run along it
    v4d acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[b] = (v4d){0.0, 0.0, 0.0, 0.0};

    for (int ch = z; ch < jb.nchunks; ch += jb.nsplit) {
        const long long c0 = (long long)ch * RK_T;
        // tile element (row, col): 16 passes of 4 rows x 64 columns; along the last mode 64 rows x 4 columns
        float vi[16], vj[16];
        long long base0 = 0;
        bool cin0 = false;
        if (!last) {                    // this lane's column is the same in every pass
            const long long c = c0 + lane;
            cin0 = c < ncols;
            const long long cc = cin0 ? c : 0;
            const long long o = cc / inner, j = cc - o * inner;
            base0 = o * n * inner + j;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int row = last ? lane : 4 * u + wave;
            const long long c = c0 + 4 * u + wave;               // (last mode) this pass's column; its fibre starts at c n
            const bool cin = last ? c < ncols : cin0;
            const long long base = last ? (cin ? c : 0) * n : base0;
            const int ri = bi * RK_T + row, rj = bj * RK_T + row;
            const float xi = to_f32(X[base + (long long)(ri < n ? ri : 0) * inner]);
            vi[u] = (cin && ri < n) ? xi : 0.f;
            if (!diag) {
                const float xj = to_f32(X[base + (long long)(rj < n ? rj : 0) * inner]);
                vj[u] = (cin && rj < n) ? xj : 0.f;
            } else {
                vj[u] = 0.f;
            }
        }
        __syncthreads();                // the previous chunk is no longer read
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int row = last ? lane : 4 * u + wave, col = last ? 4 * u + wave : lane;
            Xi[row * RK_LD + col] = vi[u];
            if (!diag) Xj[row * RK_LD + col] = vj[u];
        }
        __syncthreads();
        const float* bsrc = diag ? Xi : Xj;
#pragma unroll
        for (int kk = 0; kk < RK_T / 16; ++kk) {
            const v4f a4 = *reinterpret_cast<const v4f*>(Xi + (16 * wave + ll) * RK_LD + 16 * kk + 4 * lg);
            v4f b4[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) b4[b] = *reinterpret_cast<const v4f*>(bsrc + (16 * b + ll) * RK_LD + 16 * kk + 4 * lg);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const double a = (double)a4[s];
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)b4[b][s], acc[b], 0, 0, 0);
            }
        }
    }
    // fp64 MFMA result layout: lane holds row lg + 4 v, column ll of its 16 x 16 block
    double* out = jb.part + (long long)z * n * n;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = bi * RK_T + 16 * wave + lg + 4 * v, j = bj * RK_T + 16 * b + ll;
            if (i < n && j < n) out[(long long)i * n + j] = acc[b][v];
        }
}

// G[e] = sum over the column ranges, in their order
__global__ __launch_bounds__(256) void k_gram_reduce(const double* __restrict__ part, int nsplit, long long cnt,
                                                     double* __restrict__ G) {
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= cnt) return;
    double s = 0.0;
    for (int z = 0; z < nsplit; ++z) s += part[(long long)z * cnt + e];
    G[e] = s;
}

__global__ void k_set_i32(int32_t* p, int32_t v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// One round of the cyclic one-sided Jacobi iteration on the rows of W (n x n, row-major): workgroup p (one
// wave) takes the p-th pair of the round-robin schedule on n2 = n rounded up to even players, and rotates its
// two rows so that they become orthogonal.  The pairs of a round are disjoint, so the waves touch disjoint
// rows; rounds are ordered by the stream.  `rotations` counts the pairs that were not yet orthogonal.
__global__ __launch_bounds__(64) void k_jacobi_round(double* __restrict__ W, int n, int round, double tol,
                                                     int32_t* __restrict__ rotations) {
    constexpr int NE = RK_NMAX / 64;
    const int n2 = (n + 1) & ~1, m = n2 - 1, p = blockIdx.x, lane = threadIdx.x;
    int a = p == 0 ? m : (round + p) % m;
    int b = p == 0 ? round : (round - p + m) % m;
    if (a > b) { const int t = a; a = b; b = t; }
    if (b >= n) return;                                  // the bye of an odd n
    double* ra = W + (long long)a * n;
    double* rb = W + (long long)b * n;
    double x[NE], y[NE];
    double al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
    for (int k = 0; k < NE; ++k) {
        const int i = lane + 64 * k;
        x[k] = i < n ? ra[i] : 0.0;
        y[k] = i < n ? rb[i] : 0.0;
        al += x[k] * x[k]; be += y[k] * y[k]; ga += x[k] * y[k];
    }
    al = wave_sum(al); be = wave_sum(be); ga = wave_sum(ga);
    if (!(fabs(ga) > tol * sqrt(al * be))) return;       // orthogonal already (or a zero row)
    const double zeta = (be - al) / (2.0 * ga);
    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
    const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
#pragma unroll
    for (int k = 0; k < NE; ++k) {
        const int i = lane + 64 * k;
        if (i < n) {
            ra[i] = c * x[k] - s * y[k];
            rb[i] = s * x[k] + c * y[k];
        }
    }
    if (lane == 0) atomicAdd(rotations, 1);
}

// After convergence row k of W is lambda_k v_k^T.  Eigenvalues in descending order (ties by row index),
// eigenvectors as the columns of an n x n row-major fp32 matrix; a column whose eigenvalue is below
// 1e-12 of the largest (a null direction, whose row carries no direction any more) is returned as zeros.
__global__ __launch_bounds__(256) void k_spectrum_finish(const double* __restrict__ W, int n, double* __restrict__ lam_out,
                                                         float* __restrict__ vec_out) {
    __shared__ double lam[RK_NMAX];
    __shared__ int order[RK_NMAX];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int k = wave; k < n; k += 4) {
        double s = 0.0;
        for (int i = lane; i < n; i += 64) { const double w = W[(long long)k * n + i]; s += w * w; }
        s = wave_sum(s);
        if (lane == 0) lam[k] = sqrt(s);
    }
    __syncthreads();
    for (int k = tid; k < n; k += 256) {
        int pos = 0;
        for (int j = 0; j < n; ++j) pos += (lam[j] > lam[k] || (lam[j] == lam[k] && j < k)) ? 1 : 0;
        order[pos] = k;
        lam_out[pos] = lam[k];
    }
    __syncthreads();
    if (!vec_out) return;
    const double lmax = lam[order[0]];
    for (long long e = tid; e < (long long)n * n; e += 256) {
        const int i = (int)(e / n), k = (int)(e - (long long)i * n);
        const int row = order[k];
        const double l = lam[row];
        vec_out[e] = (l > 1e-12 * lmax && l > 0.0) ? (float)(W[(long long)row * n + i] / l) : 0.f;
    }
}

struct EpsList { double eps[16]; int count; };
// ranks[j] = smallest r >= 1 whose leading eigenvalues hold the fraction eps[j] of their sum (Sec. 3.3, Step 1)
__global__ void k_ev_ranks(const double* __restrict__ lam, int n, EpsList el, int32_t* __restrict__ ranks) {
    const int j = threadIdx.x;
    if (j >= el.count) return;
    double total = 0.0;
    for (int k = 0; k < n; ++k) total += lam[k];
    double run = 0.0;
    int r = n;
    for (int k = 0; k < n; ++k) {
        run += lam[k];
        if (run >= el.eps[j] * total) { r = k + 1; break; }
    }
    ranks[j] = r;
}

__global__ __launch_bounds__(256) void k_frob_partial(const float* __restrict__ a, const float* __restrict__ b, long long cnt,
                                                      double* __restrict__ part) {
    __shared__ double red[4];
    double s = 0.0;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < cnt; e += (long long)gridDim.x * 256) {
        const double d = (double)a[e] - (double)b[e];
        s += d * d;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}
__global__ __launch_bounds__(64) void k_frob_final(const double* __restrict__ part, int nparts, double* __restrict__ out) {
    double s = 0.0;
    for (int k = threadIdx.x; k < nparts; k += 64) s += part[k];
    s = wave_sum(s);
    if (threadIdx.x == 0) *out = sqrt(s);
}

struct ModeShape {
    long long outer = 1, inner = 1, ncols = 1, numel = 1;
    int n = 0;
    bool bf16 = false;
};
bool parse_mode(const asi_tensor_desc* desc, int mode, ModeShape* ms, asi_status* why) {
    if (!desc || (desc->ndim != 3 && desc->ndim != 4) || mode < 0 || mode >= desc->ndim) { *why = ASI_ERR_INVALID_ARG; return false; }
    if (desc->dtype != ASI_F32 && desc->dtype != ASI_BF16) { *why = ASI_ERR_UNSUPPORTED; return false; }
    for (int m = 0; m < desc->ndim; ++m) {
        if (desc->dims[m] <= 0 || desc->dims[m] > (1LL << 30)) { *why = ASI_ERR_INVALID_ARG; return false; }
        ms->numel *= desc->dims[m];
        if (ms->numel > (1LL << 40)) { *why = ASI_ERR_UNSUPPORTED; return false; }
        if (m < mode) ms->outer *= desc->dims[m];
        if (m > mode) ms->inner *= desc->dims[m];
    }
    if (desc->dims[mode] > RK_NMAX) { *why = ASI_ERR_UNSUPPORTED; return false; }
    ms->n = (int)desc->dims[mode];
    ms->ncols = ms->outer * ms->inner;
    ms->bf16 = desc->dtype == ASI_BF16;
    return true;
}
struct GramPlan { int tiles, nchunks, nsplit; size_t part_bytes, w_bytes, bytes; };
GramPlan plan_gram(const ModeShape& ms) {
    GramPlan p;
    p.tiles = (ms.n + RK_T - 1) / RK_T;
    const long long chunks = (ms.ncols + RK_T - 1) / RK_T;
    p.nchunks = (int)(chunks > 0x7fffffffLL ? 0x7fffffffLL : chunks);
    long long want = 2048 / ((long long)p.tiles * p.tiles);
    if (want > RK_MAX_SPLIT) want = RK_MAX_SPLIT;
    if (want > chunks) want = chunks;
    if (want < 1) want = 1;
    p.nsplit = (int)want;
    p.part_bytes = align_up(sizeof(double) * (size_t)p.nsplit * ms.n * ms.n);
    p.w_bytes = align_up(sizeof(double) * (size_t)ms.n * ms.n);
    p.bytes = p.part_bytes + p.w_bytes + RK_ALIGN;      // partial Gram matrices, W, the rotation counter
    return p;
}

struct Search {
    int n, e;
    const double* P;
    const int64_t* M;
    int64_t budget;
    std::vector<double> minP;          // minP[i] = sum over layers >= i of their least perplexity
    std::vector<int64_t> minM;
    std::vector<int> cur, best;
    double best_total;
    bool found;
    void walk(int i, int64_t mem, double tot) {
        if (i == n) {
            if (!found || tot < best_total) { found = true; best_total = tot; best = cur; }
            return;
        }
        for (int j = 0; j < e; ++j) {
            const int64_t m2 = mem + M[(size_t)i * e + j];
            if (m2 + minM[i + 1] > budget) continue;                       // cannot fit whatever follows
            const double t2 = tot + P[(size_t)i * e + j];
            // cannot get below the best so far (with room for the rounding of the bound's own sum)
            if (found && t2 + minP[i + 1] > best_total + 1e-12 * fabs(best_total)) continue;
            cur[i] = j;
            walk(i + 1, m2, t2);
        }
    }
};

}  // namespace

extern "C" {

int64_t asi_activation_memory(const asi_tensor_desc* desc) {
    if (!desc || (desc->ndim != 3 && desc->ndim != 4)) return -1;
    int64_t prod = 1, sum = 0;
    for (int m = 0; m < desc->ndim; ++m) {
        if (desc->dims[m] <= 0 || desc->ranks[m] < 1 || desc->ranks[m] > desc->dims[m]) return -1;
        prod *= desc->ranks[m];
        sum += desc->dims[m] * desc->ranks[m];
    }
    return prod + sum;
}

size_t asi_mode_spectrum_workspace_bytes(const asi_tensor_desc* desc, int32_t mode) {
    ModeShape ms;
    asi_status why;
    if (!parse_mode(desc, mode, &ms, &why)) return 0;
    return plan_gram(ms).bytes;
}

asi_status asi_mode_spectrum(const asi_tensor_desc* desc, const void* A, int32_t mode, double* eigenvalues,
                             float* eigenvectors, void* ws, size_t ws_bytes, int32_t* sweeps, asi_stream_t stream) {
    ModeShape ms;
    asi_status why;
    if (!parse_mode(desc, mode, &ms, &why)) return why;
    if (!A || !eigenvalues) return ASI_ERR_INVALID_ARG;
    const GramPlan p = plan_gram(ms);
    if (!ws || reinterpret_cast<uintptr_t>(ws) % RK_ALIGN != 0 || ws_bytes < p.bytes) return ASI_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    double* part = reinterpret_cast<double*>(base);
    double* W = reinterpret_cast<double*>(base + p.part_bytes);
    int32_t* rot = reinterpret_cast<int32_t*>(base + p.part_bytes + p.w_bytes);
    const int n = ms.n;

    GramJob jb;
    jb.X = A; jb.outer = ms.outer; jb.inner = ms.inner; jb.ncols = ms.ncols; jb.n = n;
    jb.tiles = p.tiles; jb.nsplit = p.nsplit; jb.nchunks = p.nchunks; jb.part = part;
    const dim3 grid((unsigned)(p.tiles * p.tiles * p.nsplit));
    if (ms.bf16) hipLaunchKernelGGL(k_mode_gram<bf16_t>, grid, 256, 0, st, jb);
    else hipLaunchKernelGGL(k_mode_gram<float>, grid, 256, 0, st, jb);
    const long long cnt = (long long)n * n;
    hipLaunchKernelGGL(k_gram_reduce, dim3((unsigned)((cnt + 255) / 256)), 256, 0, st, part, p.nsplit, cnt, W);
    if (hipGetLastError() != hipSuccess) return ASI_ERR_HIP;

    // sweeps of n2 - 1 rounds until a whole sweep rotates nothing; the count comes back to the host after
    // every sweep (this entry point iterates to convergence and therefore waits for the stream)
    const int n2 = (n + 1) & ~1, npairs = n2 / 2;
    const double tol = 4.0 * n * 2.220446049250313e-16;     // two rows count as orthogonal below the rounding of their dot product
    int used = 0;
    bool converged = n == 1;
    for (int sweep = 0; sweep < 60 && !converged; ++sweep) {
        hipLaunchKernelGGL(k_set_i32, dim3(1), 64, 0, st, rot, 0);
        for (int round = 0; round < n2 - 1; ++round)
            hipLaunchKernelGGL(k_jacobi_round, dim3((unsigned)npairs), 64, 0, st, W, n, round, tol, rot);
        if (hipGetLastError() != hipSuccess) return ASI_ERR_HIP;
        int32_t h = -1;
        if (hipMemcpyAsync(&h, rot, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess) return ASI_ERR_HIP;
        if (hipStreamSynchronize(st) != hipSuccess) return ASI_ERR_HIP;
        used = sweep + 1;
        converged = h == 0;
    }
    if (sweeps) *sweeps = converged ? used : -1;
    hipLaunchKernelGGL(k_spectrum_finish, dim3(1), 256, 0, st, W, n, eigenvalues, eigenvectors);
    if (hipGetLastError() != hipSuccess) return ASI_ERR_HIP;
    return converged ? ASI_OK : ASI_ERR_NUMERIC;
}

asi_status asi_explained_variance_ranks(const double* eigenvalues, int32_t n, const double* eps, int32_t n_eps,
                                        int32_t* ranks, asi_stream_t stream) {
    if (!eigenvalues || !eps || !ranks || n < 1 || n_eps < 1 || n_eps > 16) return ASI_ERR_INVALID_ARG;
    EpsList el;
    el.count = n_eps;
    for (int j = 0; j < n_eps; ++j) {
        if (!(eps[j] > 0.0) || eps[j] > 1.0) return ASI_ERR_INVALID_ARG;
        el.eps[j] = eps[j];
    }
    hipLaunchKernelGGL(k_ev_ranks, dim3(1), 64, 0, static_cast<hipStream_t>(stream), eigenvalues, (int)n, el, ranks);
    return hipGetLastError() == hipSuccess ? ASI_OK : ASI_ERR_HIP;
}

asi_status asi_frobenius_diff(const float* a, const float* b, int64_t count, double* out, void* ws, size_t ws_bytes,
                              asi_stream_t stream) {
    if (!a || !b || !out || count < 1) return ASI_ERR_INVALID_ARG;
    if (!ws || reinterpret_cast<uintptr_t>(ws) % RK_ALIGN != 0 || ws_bytes < (size_t)ASI_FROBENIUS_WS_BYTES) return ASI_ERR_WORKSPACE;
    long long wg = (count + 255) / 256;
    if (wg > RK_FROB_WG) wg = RK_FROB_WG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    double* part = static_cast<double*>(ws);
    hipLaunchKernelGGL(k_frob_partial, dim3((unsigned)wg), 256, 0, st, a, b, (long long)count, part);
    hipLaunchKernelGGL(k_frob_final, dim3(1), 64, 0, st, part, (int)wg, out);
    return hipGetLastError() == hipSuccess ? ASI_OK : ASI_ERR_HIP;
}

asi_status asi_rank_select(int32_t n_layers, int32_t n_eps, const double* P, const int64_t* M, int64_t budget,
                           int32_t* choice, double* total) {
    if (n_layers < 1 || n_layers > 64 || n_eps < 1 || n_eps > 16 || !P || !M || !choice) return ASI_ERR_INVALID_ARG;
    for (size_t k = 0; k < (size_t)n_layers * n_eps; ++k)
        if (!(P[k] >= 0.0) || !std::isfinite(P[k]) || M[k] < 0) return ASI_ERR_INVALID_ARG;
    Search s;
    s.n = n_layers; s.e = n_eps; s.P = P; s.M = M; s.budget = budget;
    s.minP.assign(n_layers + 1, 0.0);
    s.minM.assign(n_layers + 1, 0);
    for (int i = n_layers - 1; i >= 0; --i) {
        double p = P[(size_t)i * n_eps];
        int64_t m = M[(size_t)i * n_eps];
        for (int j = 1; j < n_eps; ++j) {
            p = std::min(p, P[(size_t)i * n_eps + j]);
            m = std::min(m, M[(size_t)i * n_eps + j]);
        }
        s.minP[i] = s.minP[i + 1] + p;
        s.minM[i] = s.minM[i + 1] + m;
    }
    s.cur.assign(n_layers, 0);
    s.best_total = std::numeric_limits<double>::infinity();
    s.found = false;
    s.walk(0, 0, 0.0);
    if (!s.found) return ASI_ERR_INFEASIBLE;
    for (int i = 0; i < n_layers; ++i) choice[i] = s.best[i];
    if (total) *total = s.best_total;
    return ASI_OK;
}

}  // extern "C"
