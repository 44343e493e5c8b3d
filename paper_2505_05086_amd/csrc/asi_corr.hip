// Step 4 of Eq. 14 on fp32 MFMA:
//     T[o,j,kh,kw] = sum_{i,y,x} G1[i,o,y,x] * Zpad[i,j, y*s - p + kh*d, x*s - p + kw*d]
// an implicit GEMM with M = cout (o), N = (tap, j), K = (i, y, x).  A workgroup owns 64
// output channels x 16 core channels j x all taps and walks its share of K in chunks of one
// core channel i and up to 64 output positions (whole output rows).  Per chunk it stages
//   As[k][o]           the G1 tile, so that lane (o = l%16, k = l/16) reads its A operand
//   Zs[j][row][col]    the slab of Z rows the chunk touches, with a zero halo for the padding
// and for every tap the B operand of lane (k = l/16, j = l%16) is Zs[j][zoff[k] + tapofs].
// Splits of K write partial T's that a reduction kernel sums in fixed order.
#include "asi_device.h"
#include "asi_kernels.h"

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int CR_TO = 64;            // output channels per workgroup
constexpr int CR_KC = 64;            // output positions per chunk
constexpr int CR_ZMAX = 8192;        // floats of LDS for the Z slab

struct CorrPlan {
    int ry;          // output rows per chunk
    int nyc;         // chunks per core channel i
    int rows_in;     // Z rows a chunk touches
    int wp;          // slab row length
    int slab;        // rows_in * wp
    int nchunks;     // r1 * nyc
    int cps;         // chunks per split
    int nsplit;
};

static bool corr_plan(const CorrGeom& g, CorrPlan* p) {
    const int taps = g.kh * g.kw;
    if (g.Wo > CR_KC || taps > 25) return false;
    p->ry = CR_KC / g.Wo;
    if (p->ry > g.Ho) p->ry = g.Ho;
    p->nyc = (g.Ho + p->ry - 1) / p->ry;
    p->rows_in = (p->ry - 1) * g.sh + (g.kh - 1) * g.dh + 1;
    p->wp = (g.Wo - 1) * g.sw + (g.kw - 1) * g.dw + 1;
    p->slab = p->rows_in * p->wp;
    if ((long long)p->slab * 16 > CR_ZMAX) return false;
    p->nchunks = g.r1 * p->nyc;
    const long long base = (long long)((g.cout + CR_TO - 1) / CR_TO) * ((g.r2 + 15) / 16);
    long long want = (256 + base - 1) / base;
    if (want > p->nchunks) want = p->nchunks;
    if (want < 1) want = 1;
    p->cps = (int)((p->nchunks + want - 1) / want);
    p->nsplit = (p->nchunks + p->cps - 1) / p->cps;
    return true;
}

template <int MAXT>
__global__ __launch_bounds__(256) void k_corr_mfma(const float* __restrict__ G1, const float* __restrict__ Z,
                                                   float* __restrict__ Tpart, CorrGeom g, CorrPlan pl) {
    __shared__ float As[CR_KC][CR_TO + 1];
    __shared__ float Zs[CR_ZMAX];
    __shared__ int zoff[CR_KC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lg = lane >> 4, ll = lane & 15;
    const int taps = g.kh * g.kw;
    const int o0 = blockIdx.x * CR_TO, j0 = blockIdx.y * 16, z = blockIdx.z;
    const int HoWo = g.Ho * g.Wo;

    // chunk-local position k -> offset of its window origin inside the slab (same for every chunk)
    for (int k = tid; k < CR_KC; k += 256) {
        const int yl = k / g.Wo, x = k - yl * g.Wo;
        zoff[k] = (yl < pl.ry) ? yl * g.sh * pl.wp + x * g.sw : 0;
    }
    int tapofs[MAXT];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int kh = t / g.kw, kw = t - kh * g.kw;
        tapofs[t] = (t < taps) ? kh * g.dh * pl.wp + kw * g.dw : 0;
    }
    v4f acc[MAXT];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) acc[t] = (v4f){0.f, 0.f, 0.f, 0.f};

    const int ch_beg = z * pl.cps;
    const int ch_end = (ch_beg + pl.cps < pl.nchunks) ? ch_beg + pl.cps : pl.nchunks;
    for (int ch = ch_beg; ch < ch_end; ++ch) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        const int kcv = rows * g.Wo;                       // valid positions in this chunk
        __syncthreads();                                   // previous chunk consumed
        // G1 tile: 64 channels x kcv positions, contiguous along k
        {
            const int k = tid & 63;
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int o = o0 + (tid >> 6) + 4 * u;
                t[u] = (k < kcv && o < g.cout) ? G1[((long long)i * g.cout + o) * HoWo + (long long)y0 * g.Wo + k] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) As[k][(tid >> 6) + 4 * u] = t[u];
        }
        // Z slab with zero halo: rows ylo .. ylo + rows_in - 1, columns -pw .. -pw + wp - 1
        {
            const int ylo = y0 * g.sh - g.ph;
            const int total = 16 * pl.slab;
            for (int e0 = 0; e0 < total; e0 += 256 * 8) {
                float t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256 + tid;
                    float v = 0.f;
                    if (e < total) {
                        const int jl = e / pl.slab, rem = e - jl * pl.slab;
                        const int rr = rem / pl.wp, cc = rem - rr * pl.wp;
                        const int row = ylo + rr, col = cc - g.pw, j = j0 + jl;
                        if (j < g.r2 && row >= 0 && row < g.H && col >= 0 && col < g.W)
                            v = Z[(((long long)i * g.r2 + j) * g.H + row) * g.W + col];
                    }
                    t[u] = v;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256 + tid;
                    if (e < total) Zs[e] = t[u];
                }
            }
        }
        __syncthreads();
        const float* zrow = Zs + ll * pl.slab;
        for (int ks = 0; 4 * ks < kcv; ++ks) {
            const int k = 4 * ks + lg;
            const float a = As[k][16 * wave + ll];
            const float* zp = zrow + zoff[k];
#pragma unroll
            for (int t = 0; t < MAXT; ++t)
                if (t < taps) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, zp[tapofs[t]], acc[t], 0, 0, 0);
        }
    }
    // lane holds o = o0 + 16w + 4*lg + v, j = j0 + ll
    const long long total = (long long)g.cout * g.r2 * taps;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        if (t < taps) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int o = o0 + 16 * wave + 4 * lg + v, j = j0 + ll;
                if (o < g.cout && j < g.r2) Tpart[(long long)z * total + ((long long)o * g.r2 + j) * taps + t] = acc[t][v];
            }
        }
    }
}

// one thread per T[o,j,kh,kw] and split of the r1 axis: any geometry
__global__ __launch_bounds__(256) void k_corr(const float* __restrict__ G1, const float* __restrict__ Z,
                                              float* __restrict__ Tpart, CorrGeom g, int i_per_split) {
    const int taps = g.kh * g.kw;
    const long long total = (long long)g.cout * g.r2 * taps;
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int t = (int)(e % taps);
    const int j = (int)((e / taps) % g.r2);
    const int o = (int)(e / ((long long)taps * g.r2));
    const int kh = t / g.kw, kw = t - kh * g.kw;
    const int ibeg = blockIdx.y * i_per_split;
    const int iend = (ibeg + i_per_split < g.r1) ? ibeg + i_per_split : g.r1;
    const int hoff = kh * g.dh - g.ph, woff = kw * g.dw - g.pw;
    float acc = 0.f;
    for (int i = ibeg; i < iend; ++i) {
        const float* g1p = G1 + ((long long)i * g.cout + o) * g.Ho * g.Wo;
        const float* zp = Z + ((long long)i * g.r2 + j) * g.H * g.W;
        for (int y = 0; y < g.Ho; ++y) {
            const int hh = y * g.sh + hoff;
            if (hh < 0 || hh >= g.H) continue;
            for (int x = 0; x < g.Wo; ++x) {
                const int ww = x * g.sw + woff;
                if (ww >= 0 && ww < g.W) acc = fmaf(g1p[y * g.Wo + x], zp[hh * g.W + ww], acc);
            }
        }
    }
    Tpart[(long long)blockIdx.y * total + e] = acc;
}

int corr_splits(const CorrGeom& g) {
    CorrPlan pl;
    if (corr_plan(g, &pl)) return pl.nsplit;
    const long long total = (long long)g.cout * g.r2 * g.kh * g.kw;
    const long long blocks = (total + 255) / 256;
    long long want = (2048 + blocks - 1) / blocks;
    if (want > g.r1) want = g.r1;
    if (want < 1) want = 1;
    const int ips = (int)((g.r1 + want - 1) / want);
    return (g.r1 + ips - 1) / ips;
}

hipError_t launch_corr(const float* G1, const float* Z, float* Tpart, const CorrGeom& g, int nsplit, hipStream_t st) {
    const long long total = (long long)g.cout * g.r2 * g.kh * g.kw;
    if (total <= 0 || nsplit <= 0) return hipErrorInvalidValue;
    CorrPlan pl;
    if (corr_plan(g, &pl)) {
        if (nsplit != pl.nsplit) return hipErrorInvalidValue;
        dim3 grid((unsigned)((g.cout + CR_TO - 1) / CR_TO), (unsigned)((g.r2 + 15) / 16), (unsigned)pl.nsplit);
        const int taps = g.kh * g.kw;
        if (taps == 1) hipLaunchKernelGGL((k_corr_mfma<1>), grid, 256, 0, st, G1, Z, Tpart, g, pl);
        else if (taps <= 9) hipLaunchKernelGGL((k_corr_mfma<9>), grid, 256, 0, st, G1, Z, Tpart, g, pl);
        else hipLaunchKernelGGL((k_corr_mfma<25>), grid, 256, 0, st, G1, Z, Tpart, g, pl);
        return hipGetLastError();
    }
    const int ips = (g.r1 + nsplit - 1) / nsplit;
    dim3 grid((unsigned)((total + 255) / 256), (unsigned)nsplit);
    hipLaunchKernelGGL(k_corr, grid, 256, 0, st, G1, Z, Tpart, g, ips);
    return hipGetLastError();
}

}  // namespace asi
