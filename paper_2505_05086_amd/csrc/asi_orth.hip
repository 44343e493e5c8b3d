// Orthogonalize (Alg. 1): Q factor of the thin QR of P with positive diagonal R, computed
// in fp64 by shifted Cholesky-QR followed by two plain Cholesky-QR passes:
//   pass 0: G = P^T P + s I,  G = R^T R,  P <- P R^-1     (s makes the factorisation safe)
//   pass 1, 2: the same with s = 0.
// cond(P) reaches (sigma_1/sigma_r)^2 * cond(U^T U_prev) ~ 1e8 on the benchmark tensors, so
// the Gram matrix of P itself is numerically singular in fp64; after the shifted pass the
// condition number is ~1e3 and two further passes give orthogonality to rounding.  The
// product of the three upper-triangular factors has a positive diagonal, so the result is
// the unique Q that Gram-Schmidt produces.  That diagonal is also the norm each column keeps
// after projecting out the earlier ones; a column that keeps less than 1e-12 ||P||_F is
// reported through *info.
//
// One launch serves every mode of a tensor.  A mode gets `nred` workgroups: each sums a
// slice of the split partial sums of P into P64; the last one to finish (device counter)
// runs the three passes.  Ranks up to 64 keep the Gram matrix in LDS and use fp64 MFMA
// for it; larger ranks take a plain global-memory path.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int ORTH_NT = 512;
constexpr int ORTH_NW = ORTH_NT / 64;
constexpr int ORTH_STAGE = 10;         // Gram work items (block pair x row slice) per pass
constexpr int ORTH_RMAX = 64;          // LDS path
constexpr int ORTH_LD = ORTH_RMAX + 1;
constexpr int ORTH_MAXR = 1024;        // global path

#ifdef ASI_DEBUG_TIMING
__device__ long long g_orth_stamps[64];
#define STAMP(i) do { if (threadIdx.x == 0 && jb.mode1 == 2) g_orth_stamps[i] = wall_clock64(); } while (0)
#else
#define STAMP(i) do {} while (0)
#endif

__device__ __forceinline__ void flag_info(int32_t* info, int mode1, int col1) {
    if (info) atomicCAS(info, 0, mode1 * 1000 + col1);
}

// ---- LDS path, r <= 64 -----------------------------------------------------------------
// P <- P R^-1 by forward substitution, one row per thread, 16 columns at a time: the
// finished columns of earlier blocks are re-read from the row itself, so only two 16-wide
// register blocks are live.  Gs holds R above the diagonal, dinv the inverse diagonal.
__device__ __attribute__((noinline)) void apply_rows(double* __restrict__ P, int n, int r, const double (*Gs)[ORTH_LD],
                           const double* __restrict__ dinv) {
    const int nb = (r + 15) / 16;
    for (int i = threadIdx.x; i < n; i += ORTH_NT) {
        double* row = P + (long long)i * r;
        for (int jb = 0; jb < nb; ++jb) {
            double cur[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) cur[j] = (16 * jb + j < r) ? row[16 * jb + j] : 0.0;
            for (int pb = 0; pb < jb; ++pb) {
                double prev[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) prev[k] = row[16 * pb + k];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const double* grow = &Gs[16 * pb + k][16 * jb];
#pragma unroll
                    for (int j = 0; j < 16; ++j) cur[j] = fma(-prev[k], grow[j], cur[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                double s = cur[j];
#pragma unroll
                for (int k = 0; k < j; ++k) s = fma(-cur[k], Gs[16 * jb + k][16 * jb + j], s);
                cur[j] = s * dinv[16 * jb + j];
            }
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (16 * jb + j < r) row[16 * jb + j] = cur[j];
        }
    }
}

__device__ __attribute__((noinline)) void orth_lds(const OrthJob& jb, int32_t* info, double (*Gs)[ORTH_LD], double* stage, double* dinv,
                         double* rdiag) {
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    double* __restrict__ P = jb.P64;
    __shared__ double s_trace;
    __shared__ int s_bad;
    const int nb = (r + 15) / 16;
    const int npairs = nb * (nb + 1) / 2;          // <= 10 block pairs (ab <= bb)
    const int nks = (ORTH_NW / npairs > 0) ? ORTH_NW / npairs : 1;   // row slices per pair; npairs*nks <= 10
    for (int k = tid; k < r; k += ORTH_NT) rdiag[k] = 1.0;
    if (tid == 0) s_bad = 0;

    for (int pass = 0; pass < 3; ++pass) {
        STAMP(1 + pass * 5);
        // ---- Gram with fp64 MFMA: wave -> (block pair, row slice)
        for (int item = wave; item < npairs * nks; item += ORTH_NW) {
            const int pr = item % npairs, ks = item / npairs;
            int ab = 0, rem = pr;
            while (rem >= nb - ab) { rem -= nb - ab; ++ab; }
            const int bb = ab + rem;
            const int rows_per = ((n + nks - 1) / nks + 3) / 4 * 4;
            const int k_beg = ks * rows_per, k_end = (k_beg + rows_per < n) ? k_beg + rows_per : n;
            v4d acc = {0.0, 0.0, 0.0, 0.0};
            const int ca = 16 * ab + ll, cb = 16 * bb + ll;
            for (int k0 = k_beg; k0 < k_end; k0 += 32) {        // 16 loads in flight per lane
                double av[8], bv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int row = k0 + 4 * u + lg;
                    const bool ok = row < k_end;
                    av[u] = (ok && ca < r) ? P[(long long)row * r + ca] : 0.0;
                    bv[u] = (ok && cb < r) ? P[(long long)row * r + cb] : 0.0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av[u], bv[u], acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) stage[item * 256 + (lg + 4 * v) * 16 + ll] = acc[v];
        }
        __syncthreads();
        for (int e = tid; e < npairs * 256; e += ORTH_NT) {
            const int pr = e >> 8, ij = e & 255;
            int ab = 0, rem = pr;
            while (rem >= nb - ab) { rem -= nb - ab; ++ab; }
            const int bb = ab + rem;
            double s = 0.0;
            for (int ks = 0; ks < nks; ++ks) s += stage[(ks * npairs + pr) * 256 + ij];
            const int ga = 16 * ab + (ij >> 4), gb = 16 * bb + (ij & 15);
            if (ga < r && gb < r && ga <= gb) Gs[ga][gb] = s;
        }
        __syncthreads();
        if (pass == 0) {
            if (tid == 0) {
                double tr = 0.0;
                for (int k = 0; k < r; ++k) tr += Gs[k][k];
                s_trace = tr;
            }
            __syncthreads();
            const double shift = 11.0 * ((double)n * r + (double)r * (r + 1)) * 1.1102230246251565e-16 * s_trace;
            if (tid < r) Gs[tid][tid] += shift;
            __syncthreads();
        }
        STAMP(2 + pass * 5);
        // ---- Cholesky, right-looking; row k is left unscaled and scaled afterwards
        for (int k = 0; k < r; ++k) {
            double p = Gs[k][k];
            if (!(p > 0.0)) {            // zero or non-finite input; every thread sees the same value
                if (tid == 0 && s_bad == 0) s_bad = k + 1;
                p = 1.0;
            }
            const double pinv = 1.0 / p;
            const int m = r - k - 1;
            for (int e = tid; e < m * m; e += ORTH_NT) {
                const int ia = e / m, ib = e - ia * m;
                if (ia <= ib) {
                    const int ga = k + 1 + ia, gb = k + 1 + ib;
                    Gs[ga][gb] = fma(-Gs[k][ga] * pinv, Gs[k][gb], Gs[ga][gb]);
                }
            }
            __syncthreads();
        }
        STAMP(3 + pass * 5);
        if (tid < r) {
            double p = Gs[tid][tid];
            if (!(p > 0.0)) p = 1.0;
            const double d = sqrt(p);
            dinv[tid] = 1.0 / d;
            rdiag[tid] *= d;
        }
        __syncthreads();
        for (int e = tid; e < r * r; e += ORTH_NT) {
            const int ga = e / r, gb = e - ga * r;
            if (ga < gb) Gs[ga][gb] *= dinv[ga];       // R[ga][gb]
        }
        __syncthreads();
        // ---- P <- P R^-1, one row per thread
        STAMP(4 + pass * 5);
        apply_rows(P, n, r, Gs, dinv);
        __syncthreads();
        STAMP(5 + pass * 5);
    }
    if (tid == 0 && info) {
        if (s_bad) flag_info(info, jb.mode1, s_bad);
        const double floor_ = 1e-12 * sqrt(s_trace);
        for (int k = 0; k < r; ++k)
            if (!(rdiag[k] > floor_)) { flag_info(info, jb.mode1, k + 1); break; }
    }
    const long long cnt = (long long)n * r;
    for (long long e = tid; e < cnt; e += ORTH_NT) jb.Uout[e] = (float)P[e];
}

// ---- global-memory path, any r <= 1024 ------------------------------------------------------
__device__ __attribute__((noinline)) void orth_global(const OrthJob& jb, int32_t* info, double* rdiag) {
    const int n = jb.n, r = jb.r, tid = threadIdx.x;
    double* __restrict__ P = jb.P64;
    double* __restrict__ G = jb.G;
    __shared__ double s_inv;
    __shared__ double s_trace2;
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
            const double shift = 11.0 * ((double)n * r + (double)r * (r + 1)) * 1.1102230246251565e-16 * s_trace2;
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
    const long long cnt = (long long)n * r;
    for (long long e = tid; e < cnt; e += ORTH_NT) jb.Uout[e] = (float)P[e];
}

__global__ __launch_bounds__(ORTH_NT) void k_orth(OrthArgs a) {
    __shared__ double Gs[ORTH_RMAX][ORTH_LD];      // 33 KB
    __shared__ double stage[ORTH_STAGE * 256];     // 20 KB: Gram blocks per work item
    __shared__ double dinv[ORTH_RMAX];
    __shared__ double rdiag[ORTH_MAXR];            // running product of the R diagonals
    __shared__ int s_last;
    int ji = 0, blk = blockIdx.x;
    while (ji + 1 < a.njobs && blk >= a.job[ji].nred) { blk -= a.job[ji].nred; ++ji; }
    const OrthJob jb = a.job[ji];
    const int tid = threadIdx.x;

    // sum this block's slice of the split partial sums
    STAMP(0);
    const long long cnt = (long long)jb.n * jb.r;
    const long long per = (cnt + jb.nred - 1) / jb.nred;
    const long long e0 = blk * per, e1 = (e0 + per < cnt) ? e0 + per : cnt;
    for (long long e = e0 + tid; e < e1; e += ORTH_NT) {
        double s = 0.0;
        for (int sp = 0; sp < jb.nsplit; ++sp) s += jb.part[(long long)sp * cnt + e];
        jb.P64[e] = s;
    }
    if (jb.nred > 1) {
        __threadfence();
        __syncthreads();
        if (tid == 0) s_last = (atomicAdd(jb.counter, 1) == jb.nred - 1);
        __syncthreads();
        if (!s_last) return;
        __threadfence();
    } else {
        __syncthreads();
    }
    if (jb.r <= ORTH_RMAX) orth_lds(jb, a.info, Gs, stage, dinv, rdiag);
    else orth_global(jb, a.info, rdiag);
}

int orth_reduce_blocks(int nsplit, int n, int r) {
    const long long work = (long long)nsplit * n * r;      // partial elements to read
    long long nb = (work + (1 << 16) - 1) >> 16;           // ~64K elements per block
    const long long cnt = (long long)n * r;
    if (nb > (cnt + 255) / 256) nb = (cnt + 255) / 256;    // at least 256 outputs per block
    if (nb > 64) nb = 64;
    if (nb < 1) nb = 1;
    return (int)nb;
}

hipError_t launch_orth(const OrthArgs& a, hipStream_t st) {
    if (a.njobs <= 0 || a.njobs > 4) return hipErrorInvalidValue;
    int total = 0;
    for (int j = 0; j < a.njobs; ++j) {
        if (a.job[j].nred < 1 || a.job[j].r > ORTH_MAXR) return hipErrorInvalidValue;
        if (a.job[j].nred > 1 && !a.job[j].counter) return hipErrorInvalidValue;
        total += a.job[j].nred;
    }
    hipLaunchKernelGGL(k_orth, dim3(total), ORTH_NT, 0, st, a);
    return hipGetLastError();
}

__global__ void k_init_ctrl(int32_t* info, int* counters, int ncounters) {
    const int t = threadIdx.x;
    if (t == 0 && info) *info = 0;
    if (t < ncounters) counters[t] = 0;
}
#ifdef ASI_DEBUG_TIMING
extern "C" int asi_debug_orth_stamps(long long* out) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_orth_stamps), sizeof(long long) * 64);
}
#endif

hipError_t launch_init_ctrl(int32_t* info, int* counters, int ncounters, hipStream_t st) {
    hipLaunchKernelGGL(k_init_ctrl, 1, 64, 0, st, info, counters, ncounters);
    return hipGetLastError();
}

}  // namespace asi
