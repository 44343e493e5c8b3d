// Step 4 of Eq. 14 on fp32 MFMA:
//     T[o,j,kh,kw] = sum_{i,y,x} G1[i,o,y,x] * Zpad[i,j, y*s - p + kh*d, x*s - p + kw*d]
// an implicit GEMM with M = cout (o), N = (tap, j), K = (i, y, x).  A workgroup owns 64
// output channels x 16 core channels j x all taps and walks its share of K in chunks of one
// core channel i and up to 64 output positions (whole output rows).  Per chunk it stages
//   As[k][o]           the G1 tile, so that lane (o = l%16, k = l/16) reads its A operand
//   Zs[j][row][col]    the slab of Z rows the chunk touches, with a zero halo for the padding
// and for every tap the B operand of lane (k = l/16, j = l%16) is the slab entry of core channel j
// at the window origin of position k plus the tap's offset.
// Splits of K write partial T's that a reduction kernel sums in fixed order.
#include "asi_device.h"
#include "asi_kernels.h"

#include <cstdio>
#include <cstring>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int CR_TO = 64;            // output channels per workgroup
constexpr int CR_KC = 64;            // output positions per chunk
constexpr int CR_ZMAX = 4096;        // floats of LDS for the Z slab
// Waves per workgroup: 4 own 16 output channels each; with 8 the second four take every other
// K step of a chunk on accumulators of their own (summed through LDS at the end).  One wave per
// SIMD cannot overlap its operand reads and address arithmetic with its products (a step costs
// their sum, ~55-63 cycles per MFMA against 32); two waves per SIMD fill each other's gaps.
constexpr int CR_NW = 8;
constexpr int CR_NT = 64 * CR_NW;
constexpr int CR_KG = CR_NW / 4;     // K-step groups

struct CorrPlan {
    int ry;          // output rows per chunk
    int nyc;         // chunks per core channel i
    int rows_in;     // Z rows a chunk touches
    int wp;          // slab row length
    int slab;        // rows_in * wp
    int zld;         // floats between the slabs of consecutive core channels in LDS
    int nchunks;     // r1 * nyc
    int cps;         // chunks per split
    int nsplit;
};

struct CorrJob {
    const float* G1;
    const float* Z;
    float* Tpart;
    CorrGeom g;
    CorrPlan pl;
    int gx, gy, gz;      // channel tiles x core-channel tiles x splits (fallback kernel: blocks x splits x 1)
    int ips;             // fallback kernel: core channels i per split
};

static bool corr_plan(const CorrGeom& g, CorrPlan* p) {
    const int taps = g.kh * g.kw;
    if (g.Wo > CR_KC || taps > 25) return false;
    // the kernel indexes G1 and Z with 32-bit offsets
    if ((long long)g.r1 * g.cout * g.Ho * g.Wo >= (1LL << 31) || (long long)g.r1 * g.r2 * g.H * g.W >= (1LL << 31)) return false;
    p->ry = CR_KC / g.Wo;
    if (p->ry > g.Ho) p->ry = g.Ho;
    p->nyc = (g.Ho + p->ry - 1) / p->ry;
    p->rows_in = (p->ry - 1) * g.sh + (g.kh - 1) * g.dh + 1;
    p->wp = (g.Wo - 1) * g.sw + (g.kw - 1) * g.dw + 1;
    p->slab = p->rows_in * p->wp;
    if ((long long)p->slab * 16 > CR_ZMAX) return false;
    // In the multiply loop lane (j = l%16, k = l/16) reads slab j at the window origin of position k,
    // and the positions of a lane group are sw floats apart.  With unit stride a slab pitch of
    // 2 mod 32 puts the 32 lanes of a half wave on 32 different banks (a pitch that is a multiple
    // of 32, e.g. 6 rows x 16 columns, puts the 16 slabs on one bank); otherwise an odd pitch.
    p->zld = p->slab;
    while (g.sw == 1 ? (p->zld % 32 != 2) : (p->zld % 2 == 0)) ++p->zld;
    if ((long long)p->zld * 16 > CR_ZMAX) p->zld = p->slab;
    p->nchunks = g.r1 * p->nyc;
    const long long base = (long long)((g.cout + CR_TO - 1) / CR_TO) * ((g.r2 + 15) / 16);
    long long target = 256;
    long long want = (target + base - 1) / base;
    if (want > p->nchunks) want = p->nchunks;
    if (want < 1) want = 1;
    p->cps = (int)((p->nchunks + want - 1) / want);
    // A chunk is a dependent round of loads, barriers and 9 x 16 products: a workgroup that walks a
    // thousand output positions or more this way is better cut in three, so that three workgroups
    // per CU hide each other's rounds (measured on 64 x 64 planes: 252 -> 144 us; below that the extra
    // partial sums cost more than the overlap gains: 83 -> 96 us on 56 x 56 planes with twice the channels' splits).
    if ((long long)p->cps * p->ry * g.Wo >= 1024) {
        want = (3 * target + base - 1) / base;
        if (want > p->nchunks) want = p->nchunks;
        p->cps = (int)((p->nchunks + want - 1) / want);
    }
    p->nsplit = (p->nchunks + p->cps - 1) / p->cps;
    return true;
}


template <int MAXT, bool EXACT>
__global__ __launch_bounds__(CR_NT) void k_corr_mfma(Batch<CorrJob> bt) {
    // As | Zs during the K loop; afterwards the 64 x (16 x up to 9 taps) result tile
    constexpr int CR_TG = MAXT < 9 ? MAXT : 9;           // taps per pass of the result through LDS
    constexpr int CR_TS_LD = 16 * CR_TG + 1;
    constexpr int CR_LDS = (CR_TO * CR_TS_LD > CR_KC * (CR_TO + 1) + CR_ZMAX) ? CR_TO * CR_TS_LD : CR_KC * (CR_TO + 1) + CR_ZMAX;
    __shared__ float lds_raw[CR_LDS];
    float (*As)[CR_TO + 1] = reinterpret_cast<float (*)[CR_TO + 1]>(lds_raw);
    float* Zs = lds_raw + CR_KC * (CR_TO + 1);
    int lb;
    const CorrJob& jb = bt.job[locate_xcd(bt, &lb)];     // the tiles of one split share its G1 rows and Z slabs
    const float* __restrict__ G1 = jb.G1;
    const float* __restrict__ Z = jb.Z;
    float* __restrict__ Tpart = jb.Tpart;
    const CorrGeom g = jb.g;
    const CorrPlan pl = jb.pl;
    const int bz = lb / (jb.gx * jb.gy), brem = lb - bz * (jb.gx * jb.gy), by = brem / jb.gx, bx = brem - by * jb.gx;
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, kgrp = tid >> 8, lg = lane >> 4, ll = lane & 15;
    const int taps = g.kh * g.kw;
    const int o0 = bx * CR_TO, j0 = by * 16, z = bz;
    const int HoWo = g.Ho * g.Wo;

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
    const int ztotal = 16 * pl.slab;
    const float inv_slab = 1.0f / (float)pl.slab, inv_wp = 1.0f / (float)pl.wp, inv_wo = 1.0f / (float)g.Wo;
    const int row_step = g.sh * pl.wp;
    constexpr int NA = CR_KC * CR_TO / CR_NT, NZ = CR_ZMAX / CR_NT;     // loads per thread and chunk
    float a_t[NA], z_t[NZ];
    // loads of one chunk into registers: the G1 tile (64 channels x kcv positions, contiguous
    // along k) and the Z slab with its zero halo (rows ylo.., columns -pw..)
    auto fetch = [&](int ch) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        const int kcv = rows * g.Wo;
        const int k = tid & 63;
#pragma unroll
        for (int u = 0; u < NA; ++u) {
            const int o = o0 + (tid >> 6) + CR_NW * u;
            a_t[u] = ldg_f32(G1, (i * g.cout + o) * HoWo + y0 * g.Wo + k, k < kcv && o < g.cout);
        }
        const int ylo = y0 * g.sh - g.ph;
#pragma unroll
        for (int u = 0; u < NZ; ++u) {
            const int e = u * CR_NT + tid;
            // e < 4096: the rounded float quotient is exact, no integer division needed
            const int jl = (int)(((float)e + 0.5f) * inv_slab), rem = e - jl * pl.slab;
            const int rr = (int)(((float)rem + 0.5f) * inv_wp), cc = rem - rr * pl.wp;
            const int row = ylo + rr, col = cc - g.pw, j = j0 + jl;
            const bool ok = e < ztotal && j < g.r2 && row >= 0 && row < g.H && col >= 0 && col < g.W;
            const float v = ldg_f32(Z, ((i * g.r2 + j) * g.H + row) * g.W + col, ok);
            z_t[u] = v;
        }
    };
    if (ch_beg < ch_end) fetch(ch_beg);
    for (int ch = ch_beg; ch < ch_end; ++ch) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        const int kcv = rows * g.Wo;                       // valid positions in this chunk
        __syncthreads();                                   // previous chunk consumed
#pragma unroll
        for (int u = 0; u < NA; ++u) As[tid & 63][(tid >> 6) + CR_NW * u] = a_t[u];
#pragma unroll
        for (int u = 0; u < NZ; ++u) {
            const int e = u * CR_NT + tid;
            const int jl = (int)(((float)e + 0.5f) * inv_slab);
            if (e < ztotal) Zs[e + jl * (pl.zld - pl.slab)] = z_t[u];
        }
        __syncthreads();
        if (ch + 1 < ch_end) fetch(ch + 1);                // in flight while this chunk is multiplied
        // operands of step ks: the A value and one B value per tap.  The loads of step ks + 1 are
        // issued before the products of step ks, so that LDS latency is paid once per chunk and not
        // once per product.  The step count is rounded up to even: positions past the chunk's end
        // have zero A values (the loader's predicate) and read the slab origin, so they add nothing,
        // and the loop body stays free of branches.
        // steps of this wave's K group: ks = kgrp, kgrp + CR_KG, ...; their number is rounded up to even
        const int nsteps = (((kcv + 3) >> 2) + CR_KG - 1) / CR_KG;
        const int nst2 = (nsteps + 1) & ~1;
        const int zbase = ll * pl.zld;
        auto operands = [&](int st, float& a, float (&bq)[MAXT]) {
            int ks = st * CR_KG + kgrp;
            ks = ks < CR_KC / 4 ? ks : CR_KC / 4 - 1;          // only the read-ahead past the last step is clamped
            const int k = 4 * ks + lg;
            // window origin of position k inside the slab: (k / Wo) * sh * wp + (k % Wo) * sw
            // (24-bit multiplies: one instruction each, and every factor here is far below 2^23)
            const int yl = (int)(((float)k + 0.5f) * inv_wo), x = k - __mul24(yl, g.Wo);
            // (a 24-bit multiply here too: the 64-bit multiply-add the compiler would pick takes a
            // register of the next chunk's loads as its unused upper addend and waits for them)
            a = lds_raw[__mul24(k, CR_TO + 1) + 16 * wave + ll];   // As[k][..]; rows past the chunk's end are zero
            const int org = __mul24(yl, row_step) + __mul24(x, g.sw);
            const int zo = zbase + ((yl < pl.ry) ? org : 0);
#pragma unroll
            for (int t = 0; t < MAXT; ++t) bq[t] = (EXACT || t < taps) ? Zs[zo + tapofs[t]] : 0.f;
        };
        float a0, a1, b0[MAXT], b1[MAXT];
        operands(0, a0, b0);
#pragma unroll 1
        for (int st = 0; st < nst2; st += 2) {
            operands(st + 1, a1, b1);
#pragma unroll
            for (int t = 0; t < MAXT; ++t)
                if (EXACT || t < taps) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0[t], acc[t], 0, 0, 0);
            operands(st + 2, a0, b0);
#pragma unroll
            for (int t = 0; t < MAXT; ++t)
                if (EXACT || t < taps) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1[t], acc[t], 0, 0, 0);
        }
    }
    // lane holds o = o0 + 16w + 4*lg + v, j = j0 + ll
    // The result goes through LDS, up to 9 taps at a time: the K groups add their tiles there, and
    // for one output channel the (j, tap) values of this workgroup are then one contiguous run of T
    // (stored straight from the accumulators every lane of a store would hit its own cache line:
    // the taps are innermost, lanes differ in j and o).
    const long long total = (long long)g.cout * g.r2 * taps;
    const int nj = (g.r2 - j0 < 16) ? g.r2 - j0 : 16;
    float* Ts = lds_raw;
#pragma unroll
    for (int t0 = 0; t0 < MAXT; t0 += CR_TG) {
        if (t0 < taps) {
            const int tg = (taps - t0 < CR_TG) ? taps - t0 : CR_TG;
            __syncthreads();                               // the tiles (or the previous pass) are no longer read
#pragma unroll
            for (int kg = CR_KG - 1; kg >= 0; --kg) {      // the K groups add their tiles one after the other
                if (kgrp == kg) {
#pragma unroll
                    for (int tt = 0; tt < CR_TG; ++tt)
                        if (t0 + tt < MAXT && tt < tg) {
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                float* p = &Ts[(16 * wave + 4 * lg + v) * CR_TS_LD + ll * tg + tt];
                                *p = (kg == CR_KG - 1) ? acc[(t0 + tt < MAXT) ? t0 + tt : 0][v]
                                                       : *p + acc[(t0 + tt < MAXT) ? t0 + tt : 0][v];
                            }
                        }
                }
                __syncthreads();
            }
            const int rowlen = nj * tg;                    // <= 144
            const float inv_rowlen = 1.0f / (float)rowlen, inv_tg = 1.0f / (float)tg;
            for (int e = tid; e < CR_TO * rowlen; e += CR_NT) {   // e < 9216: the rounded float quotients are exact
                const int ol = (int)(((float)e + 0.5f) * inv_rowlen), c = e - ol * rowlen;
                const int jl = (int)(((float)c + 0.5f) * inv_tg), tt = c - jl * tg;
                const int o = o0 + ol;
                if (o < g.cout)
                    Tpart[(long long)z * total + ((long long)o * g.r2 + j0 + jl) * taps + t0 + tt] = Ts[ol * CR_TS_LD + c];
            }
        }
    }
}

// one thread per T[o,j,kh,kw] and split of the r1 axis: any geometry
__global__ __launch_bounds__(256) void k_corr(Batch<CorrJob> bt) {
    int lb;
    const CorrJob& jb = bt.job[locate(bt, &lb)];
    const float* __restrict__ G1 = jb.G1;
    const float* __restrict__ Z = jb.Z;
    float* __restrict__ Tpart = jb.Tpart;
    const CorrGeom g = jb.g;
    const int i_per_split = jb.ips;
    const int bsplit = lb / jb.gx, bx = lb - bsplit * jb.gx;
    const int taps = g.kh * g.kw;
    const long long total = (long long)g.cout * g.r2 * taps;
    const long long e = (long long)bx * 256 + threadIdx.x;
    if (e >= total) return;
    const int t = (int)(e % taps);
    const int j = (int)((e / taps) % g.r2);
    const int o = (int)(e / ((long long)taps * g.r2));
    const int kh = t / g.kw, kw = t - kh * g.kw;
    const int ibeg = bsplit * i_per_split;
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
    Tpart[(long long)bsplit * total + e] = acc;
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

// key: 0 = k_corr_mfma<1,true>, 1 = <9,true>, 2 = <9,false>, 3 = <25,false>; the fallback kernel has kind IT_CORR
bool make_corr(const float* G1, const float* Z, float* Tpart, const CorrGeom& g, int nsplit, Item* out) {
    const long long total = (long long)g.cout * g.r2 * g.kh * g.kw;
    if (total <= 0 || nsplit <= 0 || !G1 || !Z || !Tpart) return false;
    CorrJob jb;
    std::memset(&jb, 0, sizeof(jb));
    jb.G1 = G1; jb.Z = Z; jb.Tpart = Tpart; jb.g = g;
    *out = Item();
    if (corr_plan(g, &jb.pl)) {
        if (nsplit != jb.pl.nsplit) return false;
        jb.gx = (g.cout + CR_TO - 1) / CR_TO; jb.gy = (g.r2 + 15) / 16; jb.gz = jb.pl.nsplit;
        const int taps = g.kh * g.kw;
        out->kind = IT_CORR_MFMA;
        out->key = taps == 1 ? 0u : (taps == 9 ? 1u : (taps < 9 ? 2u : 3u));
        std::snprintf(out->label, sizeof(out->label), "k_corr_mfma<%d, %s>", taps == 1 ? 1 : (taps <= 9 ? 9 : 25),
                      (taps == 1 || taps == 9) ? "true" : "false");
    } else {
        jb.ips = (g.r1 + nsplit - 1) / nsplit;
        if ((total + 255) / 256 > 0x3fffffLL) return false;
        jb.gx = (int)((total + 255) / 256); jb.gy = nsplit; jb.gz = 1;
        out->kind = IT_CORR;
        std::snprintf(out->label, sizeof(out->label), "k_corr");
    }
    if ((long long)jb.gx * jb.gy * jb.gz > 0x3fffffffLL) return false;
    out->nblocks = jb.gx * jb.gy * jb.gz;
    static_assert(sizeof(CorrJob) <= kItemArgMax, "argument block");
    std::memcpy(out->arg, &jb, sizeof(jb));
    return true;
}

hipError_t launch_corr_items(const Item* const* items, int n, hipStream_t st) {
    Batch<CorrJob> b;
    dim3 grid;
    if (!gather(items, n, &b, &grid)) return hipErrorInvalidValue;
    if (items[0]->kind == IT_CORR) {
        hipLaunchKernelGGL(k_corr, grid, 256, 0, st, b);
        return hipGetLastError();
    }
    switch (items[0]->key) {
        case 0: hipLaunchKernelGGL((k_corr_mfma<1, true>), grid, CR_NT, 0, st, b); break;
        case 1: hipLaunchKernelGGL((k_corr_mfma<9, true>), grid, CR_NT, 0, st, b); break;
        case 2: hipLaunchKernelGGL((k_corr_mfma<9, false>), grid, CR_NT, 0, st, b); break;
        default: hipLaunchKernelGGL((k_corr_mfma<25, false>), grid, CR_NT, 0, st, b); break;
    }
    return hipGetLastError();
}

}  // namespace asi
