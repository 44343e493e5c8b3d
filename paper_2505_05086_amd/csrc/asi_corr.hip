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

#include <atomic>
#include <cstdio>
#include <cstring>
#include <type_traits>

namespace asi {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int CR_TO = 64;            // output channels per workgroup
// Output positions per chunk and the floats of LDS for the Z slab that goes with them.  Small output maps
// (a few hundred positions) take chunks of 64 in one LDS buffer: load -> barrier -> store -> barrier -> multiply.
// On large maps that order leaves the matrix pipe idle a third of the time (measured with device
// timestamps: per chunk 1.0-1.3 us of LDS stores and 1.3-2.7 us of load issue in which no wave multiplies,
// against 6-8 us of products), so they take chunks of 128 positions (whole output rows) in TWO buffers:
// half of the waves store the next chunk and issue the loads of the one after it BEFORE they multiply the
// current chunk, the other half AFTER, so that on every SIMD one wave multiplies while the other moves
// data, and a chunk costs one barrier.
constexpr int CR_KC_SMALL = 64, CR_ZMAX_SMALL = 4096;
constexpr int CR_KC_BIG = 128, CR_ZMAX_BIG = 5120;
constexpr int CR_BIG_MIN_POSITIONS = 1024;      // Ho * Wo from which the large chunks are used
// Waves per workgroup: 4 own 16 output channels each; with 8 the second four take every other
// K step of a chunk on accumulators of their own (summed through LDS at the end).  One wave per
// SIMD cannot overlap its operand reads and address arithmetic with its products (a step costs
// their sum, ~55-63 cycles per MFMA against 32); two waves per SIMD fill each other's gaps.
constexpr int CR_NW = 8;
constexpr int CR_NT = 64 * CR_NW;
constexpr int CR_KG = CR_NW / 4;     // K-step groups

struct CorrPlan {
    int kc;          // output positions a chunk can hold (CR_KC_SMALL or CR_KC_BIG)
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
    if (g.Wo > CR_KC_SMALL || taps > 25) return false;
    // the kernel indexes G1 and Z with 32-bit offsets
    if ((long long)g.r1 * g.cout * g.Ho * g.Wo >= (1LL << 31) || (long long)g.r1 * g.r2 * g.H * g.W >= (1LL << 31)) return false;
    // large chunks for large maps with 3 x 3 taps and unit column dilation, if their slab fits; otherwise chunks of 64
    int zmax = CR_ZMAX_SMALL;
    for (int big = ((long long)g.Ho * g.Wo >= CR_BIG_MIN_POSITIONS && g.kh == 3 && g.kw == 3 && g.dw == 1) ? 1 : 0; big >= 0; --big) {
        p->kc = big ? CR_KC_BIG : CR_KC_SMALL;
        zmax = big ? CR_ZMAX_BIG : CR_ZMAX_SMALL;
        p->ry = p->kc / g.Wo;
        if (p->ry > g.Ho) p->ry = g.Ho;
        p->nyc = (g.Ho + p->ry - 1) / p->ry;
        p->rows_in = (p->ry - 1) * g.sh + (g.kh - 1) * g.dh + 1;
        p->wp = (g.Wo - 1) * g.sw + (g.kw - 1) * g.dw + 1;
        p->slab = p->rows_in * p->wp;
        if ((long long)p->slab * 16 <= zmax && (!big || ((p->rows_in == 4 || p->rows_in == 6) && p->wp <= 128 && g.Wo % 4 == 0 && g.sw == 1))) break;
        if (!big) return false;
    }
    // In the multiply loop lane (j = l%16, k = l/16) reads slab j at the window origin of position k,
    // and the positions of a lane group are sw floats apart.  With unit stride a slab pitch of
    // 2 mod 32 puts the 32 lanes of a half wave on 32 different banks (a pitch that is a multiple
    // of 32, e.g. 6 rows x 16 columns, puts the 16 slabs on one bank); otherwise an odd pitch.
    p->zld = p->slab;
    while (g.sw == 1 ? (p->zld % 32 != 2) : (p->zld % 2 == 0)) ++p->zld;
    if ((long long)p->zld * 16 > zmax) p->zld = p->slab;
    p->nchunks = g.r1 * p->nyc;
    const long long base = (long long)((g.cout + CR_TO - 1) / CR_TO) * ((g.r2 + 15) / 16);
    long long target = 256;
    long long want = (target + base - 1) / base;
    // With the large chunks a CU holds one workgroup (LDS), so a workgroup beyond the 256th waits for a whole
    // round: round the split count down, not up.
    if (p->kc == CR_KC_BIG) want = target / base;
    if (want > p->nchunks) want = p->nchunks;
    if (want < 1) want = 1;
    p->cps = (int)((p->nchunks + want - 1) / want);
    // A chunk is a dependent round of loads, barriers and 9 x 16 products: a workgroup that walks a
    // thousand output positions or more this way is better cut in three, so that three workgroups
    // per CU hide each other's rounds (measured on 64 x 64 planes: 252 -> 144 us; below that the extra
    // partial sums cost more than the overlap gains: 83 -> 96 us on 56 x 56 planes with twice the channels' splits).
    if (p->kc == CR_KC_SMALL && (long long)p->cps * p->ry * g.Wo >= 1024) {
        want = (3 * target + base - 1) / base;
        if (want > p->nchunks) want = p->nchunks;
        p->cps = (int)((p->nchunks + want - 1) / want);
    }
    p->nsplit = (p->nchunks + p->cps - 1) / p->cps;
    return true;
}


extern __shared__ float cr_dyn[];

template <int MAXT>
constexpr int corr_lds_floats(int kc, int zmax) {
    // the G1 tile, the Z slabs and the table of window origins; afterwards the result tile
    return (CR_TO * (16 * (MAXT < 9 ? MAXT : 9) + 1) > kc * (CR_TO + 2) + zmax) ? CR_TO * (16 * (MAXT < 9 ? MAXT : 9) + 1)
                                                                                   : kc * (CR_TO + 2) + zmax;
}
// large chunks: two buffers of (channel-major G1 tile with a pitch of kc + 4, Z slabs), then the table
constexpr int corr_big_buf_floats() { return CR_TO * (CR_KC_BIG + 4) + CR_ZMAX_BIG; }
constexpr int corr_big_lds_floats() { return 2 * corr_big_buf_floats() + CR_KC_BIG; }

// BIG (3 x 3 taps, unit column dilation, chunks of 128 positions in two buffers): a wave owns TWO blocks of 16 output
// channels and the eight waves form four K groups.  The matrix pipe and the vector ALU of a SIMD do not
// overlap here (measured: a loop of independent 16x16x4 products runs at 33-36 cycles per product, and
// every vector instruction placed between them adds its own ~4-8 cycles, whatever the number of waves),
// so the loop carries as little else as possible: per K step one table read for the window origin,
// three address additions (one per kernel row; the three taps of a row are immediate offsets), two A
// reads and nine B reads feed eighteen products.
// BIGV: 0 = chunks of 64 in one buffer; 1..4 = the large-chunk form for slabs of ZR = 4 (1, 2) or 6 (3, 4) rows
// with a row in 64 lanes (1, 3) or 128 lanes (2, 4): the loader's loop bounds are compile-time constants, so
// it has no branches (as uniform run-time tests they cost 200 scalar branches and 1000 scalar instructions
// per chunk and wave, 1.4 us of the 3.3 us a wave spent on a chunk).
template <int MAXT, bool EXACT, int BIGV>
__global__ __launch_bounds__(CR_NT) void k_corr_mfma(Batch<CorrJob> bt) {
    constexpr bool BIG = BIGV != 0;
    constexpr int ZR = BIGV >= 3 ? 6 : 4;                // BIG: rows of a slab
    constexpr bool ZW64 = (BIGV & 1) != 0;               // BIG: a slab row fits 64 lanes
    constexpr int CR_KC = BIG ? CR_KC_BIG : CR_KC_SMALL, CR_ZMAX = BIG ? CR_ZMAX_BIG : CR_ZMAX_SMALL;
    constexpr int OB = BIG ? 2 : 1;                      // blocks of 16 output channels per wave
    constexpr int NWO = 4 / OB;                          // waves side by side along the output channels
    constexpr int KG = CR_NW / NWO;                      // K groups: waves that share channels and split the K steps
    static_assert(!BIG || (MAXT == 9 && EXACT), "the large-chunk form is written for 3 x 3 taps");
    // As | Zs | korg during the K loop; afterwards the 64 x (16 x up to 9 taps) result tile
    constexpr int CR_TG = MAXT < 9 ? MAXT : 9;           // taps per pass of the result through LDS
    constexpr int CR_TS_LD = 16 * CR_TG + 1;
    float* lds_raw = cr_dyn;                             // corr_lds_floats<MAXT>(CR_KC, CR_ZMAX) floats (BIG: corr_big_lds_floats())
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
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6, wo = wid % NWO, lg = lane >> 4, ll = lane & 15;
    const int kgrp_s = __builtin_amdgcn_readfirstlane(wid / NWO);      // the same for a whole wave: a scalar
    const int taps = g.kh * g.kw;
    const int o0 = bx * CR_TO, j0 = by * 16, z = bz;
    const int HoWo = g.Ho * g.Wo;

    int tapofs[MAXT];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int kh = t / g.kw, kw = t - kh * g.kw;
        tapofs[t] = (t < taps) ? kh * g.dh * pl.wp + kw * g.dw : 0;
    }
    v4f acc[OB][MAXT];
#pragma unroll
    for (int ob = 0; ob < OB; ++ob)
#pragma unroll
        for (int t = 0; t < MAXT; ++t) acc[ob][t] = (v4f){0.f, 0.f, 0.f, 0.f};

    const int ch_beg = z * pl.cps;
    const int ch_end = (ch_beg + pl.cps < pl.nchunks) ? ch_beg + pl.cps : pl.nchunks;
    const int ztotal = 16 * pl.slab;
    const float inv_slab = 1.0f / (float)pl.slab, inv_wp = 1.0f / (float)pl.wp, inv_wo = 1.0f / (float)g.Wo;
    const int row_step = g.sh * pl.wp;
    // loads per thread and chunk.  BIG: a thread serves one slab column of CR_ZRMAX rows of four slabs
    constexpr int NA = CR_KC * CR_TO / CR_NT, NZ = BIG ? 1 : CR_ZMAX / CR_NT;
    static_assert(NA <= 32 && NZ <= 32, "one mask bit per load");
    float a_t[NA], z_t[NZ];
    unsigned amask = 0, zmask = 0;     // which of the loaded values belong to the chunk (set by fetch, used by the next store)
    // Loads of one chunk into registers: the G1 tile (64 channels x kcv positions, contiguous along k)
    // and the Z slab with its zero halo (rows ylo.., columns -pw..).  Every load goes to an address
    // that is valid whatever the lane (a lane outside the tile or in the halo reads a clamped position)
    // and its result is only masked when it is stored to LDS: a load guarded by a test of its own is
    // compiled into a conditional block that waits for it, and the loads of a chunk would then run one
    // after the other instead of together.
    // BIG: every quantity that depends on the row of the tile or slab a load belongs to is the same for
    // a whole wave (rows are dealt out by tid / 256 resp. tid / 128), so it is kept in scalar registers
    // and a load costs no vector arithmetic; what depends on the lane (position, slab column) is fixed
    // for the kernel.  The vector instructions of fetch and store run at the expense of the products.
    // G1 tile (BIG): a thread moves four consecutive positions of one channel with a 16-byte load; a wave
    // covers two channel rows of 128 positions (chunks are whole output rows and Wo is a multiple of 4, so
    // the pieces are aligned and lie wholly inside or outside the chunk); the 8 waves serve 16 channels per
    // load.  The lane's offset inside the tile of one core channel is fixed for the kernel; what changes with
    // the chunk is one scalar base.  In LDS the tile is held channel-major, Ab[o][k] with a pitch of
    // CR_KC + 4 floats: the store is one 16-byte write, and the A operand of lane (o = l % 16, k = l / 16)
    // sits 4 (l % 16) + l / 16 banks from the block's origin, one bank per lane.
    // Z slabs (BIG): a slab row takes 64 lanes when it fits (128 otherwise), so that no wave is idle;
    // group rgz of lanes serves `spg` of the 16 slabs, up to CR_ZRMAX rows each; every quantity that
    // depends on the slab or its row is the same for a whole wave and lives in scalar registers.
    constexpr int AP = CR_KC + 4;                                         // BIG: pitch of the channel-major G1 tile
    constexpr int NA4 = CR_TO * CR_KC / 4 / CR_NT;                        // BIG: 16-byte loads of G1 per thread
    constexpr int BUF = BIG ? corr_big_buf_floats() : 0;                  // BIG: floats of one buffer
    constexpr int SPG = ZW64 ? 2 : 4;                                     // BIG: slabs per lane group
    constexpr int NZB = SPG * ZR;                                         // BIG: Z loads per thread and chunk
    const int rgz = __builtin_amdgcn_readfirstlane(ZW64 ? (tid >> 6) : (tid >> 7));
    const int zcc = ZW64 ? (tid & 63) : (tid & 127);                      // slab column of this lane
    const bool zc_in = zcc < pl.wp, zc_ok = zc_in & (zcc - g.pw >= 0) & (zcc - g.pw < g.W);
    const int zcolc = min(max(zcc - g.pw, 0), g.W - 1);
    const int k4 = 4 * (tid & (CR_KC / 4 - 1));                           // first of this thread's four positions
    const int arow_l = tid / (CR_KC / 4);                                 // its channel row within a load (0 .. 15)
    // what does not change from chunk to chunk: the offsets of the thread's G1 pieces inside the tile of one
    // core channel, the (clamped) slabs of its lane group, its LDS addresses
    unsigned aoff_b[BIG ? NA4 : 1];                                       // byte offsets (the tile of one core channel is below 2^31 bytes: host check)
    int zjc[BIG ? SPG : 1];
    const unsigned zcol_b = 4u * (unsigned)zcolc;
#pragma unroll
    for (int u = 0; u < (BIG ? NA4 : 1); ++u) {
        const int ol = arow_l + 16 * u;
        aoff_b[u] = 4u * (unsigned)((o0 + ol < g.cout ? ol : 0) * HoWo);
    }
#pragma unroll
    for (int jj = 0; jj < (BIG ? SPG : 1); ++jj) {
        const int j = j0 + SPG * rgz + jj;
        zjc[jj] = j < g.r2 ? j : g.r2 - 1;                                // scalar
    }
    const int zst0 = SPG * rgz * pl.zld + zcc;                            // LDS offset of (first slab of the group, row 0, this column)
    v4f a4[BIG ? NA4 : 1];
    float ztb[BIG ? NZB : 1];
    int kcv_f = 0, ylo_f = 0;          // BIG: positions and first slab row of the chunk in the registers
    auto fetch_big = [&](int ch) __attribute__((always_inline)) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        kcv_f = rows * g.Wo;
        ylo_f = y0 * g.sh - g.ph;
        int rowc[ZR];                                                     // scalar: the slab's rows, clamped into the map
#pragma unroll
        for (int rr = 0; rr < ZR; ++rr) {
            const int row = ylo_f + rr;
            rowc[rr] = row < 0 ? 0 : (row > g.H - 1 ? g.H - 1 : row);
        }
#pragma unroll
        for (int jj = 0; jj < SPG; ++jj) {
            const int pbase = (i * g.r2 + zjc[BIG ? jj : 0]) * g.H;       // scalar
#pragma unroll
            for (int rr = 0; rr < ZR; ++rr) {
                // a uniform row pointer and an unsigned lane offset: the load takes its address from a scalar
                // pair plus a 32-bit register, no vector instruction builds it
                const char* zrow = reinterpret_cast<const char*>(Z + (unsigned)((pbase + rowc[rr]) * g.W));
                ztb[BIG ? jj * ZR + rr : 0] = *reinterpret_cast<const float*>(zrow + zcol_b);
            }
        }
        // a piece past the chunk's positions reads the chunk's first piece instead
        const char* abase = reinterpret_cast<const char*>(G1 + (unsigned)((i * g.cout + o0) * HoWo + y0 * g.Wo));  // scalar
        const unsigned kc4_b = k4 < kcv_f ? 4u * (unsigned)k4 : 0u;
#pragma unroll
        for (int u = 0; u < NA4; ++u) a4[BIG ? u : 0] = *reinterpret_cast<const v4f*>(abase + (aoff_b[BIG ? u : 0] + kc4_b));
    };
    auto store_big = [&](float* buf) __attribute__((always_inline)) {
        const bool kin = k4 < kcv_f;
        const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NA4; ++u) {
            const int ol = arow_l + 16 * u;
            const bool oin = o0 + ol < g.cout;
            *reinterpret_cast<v4f*>(buf + ol * AP + k4) = (kin & oin) ? a4[BIG ? u : 0] : zero4;
        }
        if (zc_in) {                                                      // one masked region for all slab stores
            float* zb = buf + CR_TO * AP + zst0;
#pragma unroll
            for (int jj = 0; jj < SPG; ++jj) {
                const bool jin = j0 + SPG * rgz + jj < g.r2;                                  // scalar
#pragma unroll
                for (int rr = 0; rr < ZR; ++rr) {
                    const int row = ylo_f + rr;
                    const bool rin = jin & (row >= 0) & (row < g.H);                         // scalar
                    zb[jj * pl.zld + rr * pl.wp] = (rin & zc_ok) ? ztb[BIG ? jj * ZR + rr : 0] : 0.f;
                }
            }
        }
    };
    auto fetch = [&](int ch) __attribute__((always_inline)) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        const int kcv = rows * g.Wo;
        // Z slab first.  Row, column and core channel are clamped one by one (no select between two
        // address expressions, no 64-bit multiply-add: both make the compiler wait for earlier loads).
        const int ylo = y0 * g.sh - g.ph;
        const int zbase = i * g.r2;
        zmask = 0;
#pragma unroll
        for (int u = 0; u < NZ; ++u) {
            const int e = u * CR_NT + tid;
            // e < 8192, slab <= 512: the rounded float quotient is exact, no integer division needed
            const int jl = (int)(((float)e + 0.5f) * inv_slab), rem = e - __mul24(jl, pl.slab);
            const int rr = (int)(((float)rem + 0.5f) * inv_wp), cc = rem - __mul24(rr, pl.wp);
            const int row = ylo + rr, col = cc - g.pw, j = j0 + jl;
            const bool ok = (e < ztotal) & (j < g.r2) & (row >= 0) & (row < g.H) & (col >= 0) & (col < g.W);
            const int jc = min(j, g.r2 - 1), rowc = min(max(row, 0), g.H - 1), colc = min(max(col, 0), g.W - 1);
            z_t[u] = Z[__mul24(__mul24(zbase + jc, g.H) + rowc, g.W) + colc];
            zmask |= ok ? (1u << u) : 0u;
        }
        // G1 tile: lane k of a wave walks the positions, the rows (channels) are CR_NT / CR_KC apart
        const int k = tid & (CR_KC - 1);
        const bool kin = k < kcv;
        const int abase = __mul24(i, g.cout) * HoWo + y0 * g.Wo + (kin ? k : 0);
        amask = 0;
#pragma unroll
        for (int u = 0; u < NA; ++u) {
            const int o = o0 + tid / CR_KC + (CR_NT / CR_KC) * u;
            const bool oin = o < g.cout;
            a_t[u] = G1[abase + __mul24(oin ? o : o0, HoWo)];
            amask |= (kin & oin) ? (1u << u) : 0u;
        }
    };
    // korg[k]: offset of the window origin of output position k inside a slab, (k / Wo) * sh * wp + (k % Wo) * sw
    // (0 for positions beyond the rows of a chunk; their A values are zero).  The same for every chunk.
    int* korg = reinterpret_cast<int*>(lds_raw + (BIG ? 2 * BUF : CR_KC * (CR_TO + 1) + CR_ZMAX));
    for (int k = tid; k < CR_KC; k += CR_NT) {
        const int yl = (int)(((float)k + 0.5f) * inv_wo), x = k - yl * g.Wo;     // k < 2^14: exact
        korg[k] = (yl < pl.ry) ? yl * row_step + x * g.sw : 0;
    }
    // per-lane constants of the operand reads: As[4 ks + lg][16 (OB wo + ob) + ll] (BIG: Ab[16 (OB wo + ob) + ll][4 ks + lg]),
    // slab ll of Zs
    const int a_lane = BIG ? (16 * OB * wo + ll) * AP + lg : lg * (CR_TO + 1) + 16 * OB * wo + ll, zlane = ll * pl.zld;
    const int khstep = g.dh * pl.wp;                       // slab offset of one kernel row
    auto chunk_positions = [&](int ch) __attribute__((always_inline)) {
        const int i = ch / pl.nyc, yc = ch - i * pl.nyc;
        const int y0 = yc * pl.ry;
        const int rows = (g.Ho - y0 < pl.ry) ? g.Ho - y0 : pl.ry;
        return rows * g.Wo;                                // valid positions in this chunk
    };
    // The products of one chunk held in LDS at (Ab, Zb).
    // Operands of step ks: one A value per channel block and one B value per tap.  The reads of step
    // ks + 1 are issued before the products of step ks, so that LDS latency is paid once per chunk
    // and not once per product.  Steps are taken in pairs; positions past the chunk's end have zero A
    // values (the loader's mask) and read the slab origin, so a step past the end adds nothing (the large
    // chunks skip its products with a uniform branch) and the loop body stays free of vector tests.
    // The step index is the same for a whole wave, so the A address is a per-lane constant plus a scalar,
    // and the window origin of a position comes from the table korg: no vector multiply is left in the
    // loop (besides their cost, the 64-bit multiply-add the compiler picks for some of them takes an
    // unrelated register - one of the next chunk's pending loads - as its unused upper addend and waits
    // for that load).
    auto multiply = [&](int kcv, const float* Ab, const float* Zb) __attribute__((always_inline)) {
        const int nsteps = (((kcv + 3) >> 2) + KG - 1) / KG;   // steps of this wave's K group: ks = kgrp, kgrp + KG, ...
        const int nst2 = (nsteps + 1) & ~1;
        int org = korg[4 * kgrp_s + lg];                   // origin of this lane's position in step 0
        auto operands = [&](int st, float (&a)[OB], float (&bq)[MAXT]) __attribute__((always_inline)) {
            int ks = st * KG + kgrp_s;
            ks = ks < CR_KC / 4 ? ks : CR_KC / 4 - 1;          // only the read-ahead past the last step is clamped
            const float* ap = Ab + a_lane + ks * (BIG ? 4 : 4 * (CR_TO + 1));
#pragma unroll
            for (int ob = 0; ob < OB; ++ob) a[ob] = ap[BIG ? 16 * ob * AP : 16 * ob];   // positions past the chunk's end are zero
            const int zo = zlane + org;
            if constexpr (BIG) {
                const float* z0 = Zb + zo;
                const float* z1 = z0 + khstep;
                const float* z2 = z1 + khstep;
                bq[0] = z0[0]; bq[1] = z0[1]; bq[2] = z0[2];
                bq[3] = z1[0]; bq[4] = z1[1]; bq[5] = z1[2];
                bq[6] = z2[0]; bq[7] = z2[1]; bq[8] = z2[2];
            } else {
#pragma unroll
                for (int t = 0; t < MAXT; ++t) bq[t] = (EXACT || t < taps) ? Zb[zo + tapofs[t]] : 0.f;
            }
            int kn = ks + KG;
            kn = kn < CR_KC / 4 ? kn : CR_KC / 4 - 1;
            org = korg[4 * kn + lg];                           // for the next step of this wave
        };
        float a0[OB], a1[OB], b0[MAXT], b1[MAXT];
        operands(0, a0, b0);
        // (scheduling fences: left alone, the compiler moves each read down next to the product that uses
        // it, and the product then waits for the LDS round trip)
#pragma unroll 1
        for (int st = 0; st < nst2; st += 2) {
            operands(st + 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < MAXT; ++t)
                if (EXACT || t < taps) {
#pragma unroll
                    for (int ob = 0; ob < OB; ++ob)
                        acc[ob][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[ob], b0[t], acc[ob][t], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
            operands(st + 2, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (!BIG || st + 1 < nsteps) {                      // uniform
#pragma unroll
                for (int t = 0; t < MAXT; ++t)
                    if (EXACT || t < taps) {
#pragma unroll
                        for (int ob = 0; ob < OB; ++ob)
                            acc[ob][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[ob], b1[t], acc[ob][t], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // BIG: the same products with a quarter of the LDS instructions.  The K steps of a chunk are taken in
    // blocks of 16 positions (four steps); K slot (s, lane group g) of a block stands for position
    // 16 kb + 4 g + s, so that a lane's A operands of the four steps are ONE 16-byte read of the channel-major
    // tile, and its B operands for the three taps of a kernel row over the four steps are SIX consecutive
    // slab entries (positions of a group of four lie in one output row because Wo is a multiple of 4; with
    // unit stride they are neighbours in the slab), read as three 8-byte pieces (slab pitch, row length and
    // window origins are all even).  Per block and wave: 2 + 9 + 1 LDS reads for 72 products, against 48 for
    // the step-by-step form, whose reads cost the SIMD about as many issue cycles as its products.
    const int a_lane4 = (16 * OB * wo + ll) * AP + 4 * lg;
    auto multiply_big = [&](int kcv, const float* Ab, const float* Zb) __attribute__((always_inline)) {
        const int nblk = (kcv + 15) >> 4;                              // blocks of 16 positions in this chunk
        const int nbw = nblk > kgrp_s ? (nblk - kgrp_s + KG - 1) / KG : 0;   // blocks of this wave: kgrp, kgrp + KG, ..
        auto operands = [&](int kb, v4f (&a)[OB], float (&b)[3][6]) __attribute__((always_inline)) {
            kb = kb < CR_KC / 16 ? kb : CR_KC / 16 - 1;                // only the read-ahead past the last block is clamped
            const float* ap = Ab + a_lane4 + 16 * kb;
#pragma unroll
            for (int ob = 0; ob < OB; ++ob) a[ob] = *reinterpret_cast<const v4f*>(ap + 16 * ob * AP);
            const float* z0 = Zb + zlane + korg[16 * kb + 4 * lg];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const float2* zr = reinterpret_cast<const float2*>(z0 + kh * khstep);
                const float2 p0 = zr[0], p1 = zr[1], p2 = zr[2];
                b[kh][0] = p0.x; b[kh][1] = p0.y; b[kh][2] = p1.x; b[kh][3] = p1.y; b[kh][4] = p2.x; b[kh][5] = p2.y;
            }
        };
        auto products = [&](const v4f (&a)[OB], const float (&b)[3][6]) __attribute__((always_inline)) {
#pragma unroll
            for (int sst = 0; sst < 4; ++sst)
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int ob = 0; ob < OB; ++ob)
                        acc[ob][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ob][sst], b[t / 3][t % 3 + sst], acc[ob][t], 0, 0, 0);
        };
        // operands of block it + 1 are read before the products of block it
        v4f a0[OB], a1[OB];
        float b0[3][6], b1[3][6];
        operands(kgrp_s, a0, b0);
#pragma unroll 1
        for (int it = 0; it < nbw; it += 2) {
            operands(kgrp_s + (it + 1) * KG, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            products(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (it + 2 < nbw) operands(kgrp_s + (it + 2) * KG, a0, b0);   // uniform
            __builtin_amdgcn_sched_barrier(0);
            if (it + 1 < nbw) products(a1, b1);                        // uniform
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if constexpr (BIG) {
        // Two buffers.  Iteration ch: every wave stores chunk ch + 1 (in its registers) to the other buffer,
        // issues the loads of chunk ch + 2 and multiplies chunk ch; one barrier per chunk orders both hazards:
        // the other buffer was last read by the products of chunk ch - 1 (finished before the previous
        // barrier), and chunk ch + 1 is complete before iteration ch + 1.  (Letting half of the waves
        // multiply first, so that each SIMD always has a multiplying wave, changed nothing: a SIMD issues the
        // loader's instructions of one wave and the products of the other one after the other, not side by side.)
        if (ch_beg < ch_end) {
            fetch_big(ch_beg);
            store_big(lds_raw);
        }
        if (ch_beg + 1 < ch_end) fetch_big(ch_beg + 1);
        __syncthreads();                                   // chunk ch_beg and the table korg are in LDS
#pragma unroll 1
        for (int ch = ch_beg; ch < ch_end; ++ch) {
            const int cur = (ch - ch_beg) & 1;
            float* bcur = lds_raw + cur * BUF;
            if (ch + 1 < ch_end) store_big(lds_raw + (cur ^ 1) * BUF);
            if (ch + 2 < ch_end) fetch_big(ch + 2);
            multiply_big(chunk_positions(ch), bcur, bcur + CR_TO * AP);
            __syncthreads();
        }
    } else {
        if (ch_beg < ch_end) fetch(ch_beg);
        for (int ch = ch_beg; ch < ch_end; ++ch) {
            __syncthreads();                               // previous chunk consumed
#pragma unroll
            for (int u = 0; u < NA; ++u)
                As[tid & (CR_KC - 1)][tid / CR_KC + (CR_NT / CR_KC) * u] = ((amask >> u) & 1u) ? a_t[u] : 0.f;
#pragma unroll
            for (int u = 0; u < NZ; ++u) {
                const int e = u * CR_NT + tid;
                const int jl = (int)(((float)e + 0.5f) * inv_slab);
                if (e < ztotal) Zs[e + jl * (pl.zld - pl.slab)] = ((zmask >> u) & 1u) ? z_t[u] : 0.f;
            }
            __syncthreads();
            if (ch + 1 < ch_end) fetch(ch + 1);            // in flight while this chunk is multiplied
            multiply(chunk_positions(ch), lds_raw, Zs);
        }
    }
    // lane holds o = o0 + 16 (OB wo + ob) + 4*lg + v, j = j0 + ll
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
            // The K groups add their tiles in LDS in a fixed order.  Four groups use two tiles: groups 2 and 3
            // write, groups 0 and 1 add to them, and the store below adds the two tiles (two rounds instead of four).
            constexpr int NTS = KG == 4 ? 2 : 1;           // result tiles in LDS
            constexpr int TS_SZ = CR_TO * CR_TS_LD;
            static_assert(NTS * TS_SZ <= (BIG ? corr_big_lds_floats() : corr_lds_floats<MAXT>(CR_KC, CR_ZMAX)),
                          "result tiles fit the K-loop buffers");
#pragma unroll
            for (int round = 0; round < KG / NTS; ++round) {
                const int kg_lo = (KG / NTS - 1 - round) * NTS;    // groups kg_lo .. kg_lo + NTS - 1 take this round
                if (kgrp_s >= kg_lo && kgrp_s < kg_lo + NTS) {
                    float* Tg = Ts + (kgrp_s - kg_lo) * TS_SZ;
#pragma unroll
                    for (int ob = 0; ob < OB; ++ob)
#pragma unroll
                        for (int tt = 0; tt < CR_TG; ++tt)
                            if (t0 + tt < MAXT && tt < tg) {
#pragma unroll
                                for (int v = 0; v < 4; ++v) {
                                    float* p = &Tg[(16 * (OB * wo + ob) + 4 * lg + v) * CR_TS_LD + ll * tg + tt];
                                    const float mine = acc[ob][(t0 + tt < MAXT) ? t0 + tt : 0][v];
                                    *p = (round == 0) ? mine : *p + mine;
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
                    Tpart[(long long)z * total + ((long long)o * g.r2 + j0 + jl) * taps + t0 + tt] =
                        NTS == 2 ? Ts[ol * CR_TS_LD + c] + Ts[TS_SZ + ol * CR_TS_LD + c] : Ts[ol * CR_TS_LD + c];
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

// key: low nibble 0 = k_corr_mfma<1,true,0>, 1 = <9,true,0>, 2 = <9,false,0>, 3 = <25,false,0>; high nibble = BIGV of <9,true,BIGV> (large chunks);
// the fallback kernel has kind IT_CORR
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
        // large chunks: instantiation by slab rows (4 or 6) and lanes per slab row (64 or 128)
        const int bigv = jb.pl.kc == CR_KC_BIG ? (jb.pl.rows_in == 4 ? 1 : 3) + (jb.pl.wp <= 64 ? 0 : 1) : 0;
        out->key = (taps == 1 ? 0u : (taps == 9 ? 1u : (taps < 9 ? 2u : 3u))) | ((unsigned)bigv << 4);
        std::snprintf(out->label, sizeof(out->label), "k_corr_mfma<%d, %s, %d>", taps == 1 ? 1 : (taps <= 9 ? 9 : 25),
                      (taps == 1 || taps == 9) ? "true" : "false", bigv);
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
    // LDS is dynamic: the large-chunk instantiations need more than the 64 KB a static array may take,
    // which has to be allowed once per kernel (the flags are only ever set, so a race between threads is harmless)
#define ASI_CORR_LAUNCH(MAXT, EXACT, BIG)                                                                          \
    do {                                                                                                           \
        constexpr size_t lds = sizeof(float) * (BIG ? corr_big_lds_floats()                                        \
                                                    : corr_lds_floats<MAXT>(CR_KC_SMALL, CR_ZMAX_SMALL));          \
        if (lds > 65536) {                                                                                         \
            static std::atomic<bool> allowed{false};                                                               \
            if (!allowed.load()) {                                                                                 \
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_corr_mfma<MAXT, EXACT, BIG>),   \
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
                if (e != hipSuccess) return e;                                                                     \
                allowed.store(true);                                                                               \
            }                                                                                                      \
        }                                                                                                          \
        hipLaunchKernelGGL((k_corr_mfma<MAXT, EXACT, BIG>), grid, CR_NT, lds, st, b);                              \
    } while (0)
    switch (items[0]->key) {
        case 0: ASI_CORR_LAUNCH(1, true, 0); break;
        case 1: ASI_CORR_LAUNCH(9, true, 0); break;
        case 2: ASI_CORR_LAUNCH(9, false, 0); break;
        case 3: ASI_CORR_LAUNCH(25, false, 0); break;
        case 0x11: ASI_CORR_LAUNCH(9, true, 1); break;
        case 0x21: ASI_CORR_LAUNCH(9, true, 2); break;
        case 0x31: ASI_CORR_LAUNCH(9, true, 3); break;
        case 0x41: ASI_CORR_LAUNCH(9, true, 4); break;
        default: return hipErrorInvalidValue;
    }
#undef ASI_CORR_LAUNCH
    return hipGetLastError();
}

}  // namespace asi
