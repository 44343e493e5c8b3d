// C ABI of the ASI library: argument validation, workspace carving and launch
// sequencing.  No kernel code lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/asi.h"
#include "asi_kernels.h"

namespace {

using namespace asi;

constexpr size_t kAlign = 256;
constexpr int kMaxRank = 1024;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align_up(count * sizeof(T));
        return p;
    }
};

struct Shape {
    int d = 0;
    long long n[4] = {1, 1, 1, 1};
    int r[4] = {1, 1, 1, 1};
    long long numel = 1;
    DType dt = F32;
    long long outer(int m) const { long long o = 1; for (int k = 0; k < m; ++k) o *= n[k]; return o; }
    long long inner(int m) const { long long o = 1; for (int k = m + 1; k < d; ++k) o *= n[k]; return o; }
};

bool parse_desc(const asi_tensor_desc* desc, Shape* s, asi_status* why) {
    if (!desc) { *why = ASI_ERR_INVALID_ARG; return false; }
    if (desc->ndim != 3 && desc->ndim != 4) { *why = ASI_ERR_INVALID_ARG; return false; }
    if (desc->dtype != ASI_F32 && desc->dtype != ASI_BF16) { *why = ASI_ERR_UNSUPPORTED; return false; }
    s->d = desc->ndim;
    s->dt = desc->dtype == ASI_F32 ? F32 : BF16;
    s->numel = 1;
    for (int m = 0; m < s->d; ++m) {
        if (desc->dims[m] <= 0 || desc->dims[m] > (1LL << 30)) { *why = ASI_ERR_INVALID_ARG; return false; }
        s->n[m] = desc->dims[m];
        s->numel *= desc->dims[m];
        if (s->numel > (1LL << 40)) { *why = ASI_ERR_UNSUPPORTED; return false; }
    }
    for (int m = 0; m < s->d; ++m) {
        const long long b = s->numel / s->n[m];
        const long long rmax = std::min(s->n[m], b);
        if (desc->ranks[m] < 1 || desc->ranks[m] > rmax) { *why = ASI_ERR_INVALID_ARG; return false; }
        if (desc->ranks[m] > kMaxRank) { *why = ASI_ERR_UNSUPPORTED; return false; }
        s->r[m] = desc->ranks[m];
    }
    return true;
}

// ---- compress ---------------------------------------------------------------
struct CompressPlan {
    float* V = nullptr;
    unsigned short* Ub = nullptr;    // a factor split into bf16 terms (bf16 tensors, product along the last mode)
    bool bfv[4] = {};                // V of this mode comes from the bf16 MFMA kernel
    int bfks[4] = {1, 1, 1, 1};      // ... with the contraction split over this many workgroups per column tile
    float* Vpart = nullptr;          // ... whose partial products are summed into V
    double* part[4] = {};
    double* part2[4] = {};          // first level of the partial-sum tree (nsplit > 32)
    int nsplit2[4] = {};
    double* P64[4] = {};
    double* Gpart[4] = {};
    double* Gsum[4] = {};           // wide path, many slices: the slice Grams added up by a tree level
    int ngsum[4] = {};
    double* R[4] = {};
    double* Dinv[4] = {};
    double* scal[4] = {};
    int32_t* ctr8 = nullptr;         // arrival counters, two per mode
    int nsplit[4] = {};
    int nblk[4] = {};
    bool fused[4] = {};
    bool gramm[4] = {};              // short mode, long inner extent: P = (A_m A_m^T) U_prev (asi_gram.hip)
    bool longm[4] = {};              // long fibres: V and P from one LDS tile of complete fibres (asi_long.hip)
    bool paired = false;             // the last two modes of a 4-mode tensor share one kernel
    bool tiny = false;               // ... the vector-ALU kernel for tiny planes
    bool planes = false;             // ... the kernel for large planes (asi_planes.hip)
    bool fast_orth[4] = {};
    bool wide_orth[4] = {};
    size_t bytes = 0;
};

// cold: the first iteration of Alg. 1 (t = 0).  V is generated inside the P kernel of every mode, so no
// mode takes a fused V/P kernel and no V is stored.
CompressPlan plan_compress(const Shape& s, void* ws, bool cold = false) {
    CompressPlan p;
    Carver c(ws);
    size_t vmax = 0;
    for (int m = 0; m < s.d; ++m) {
        p.fused[m] = !cold && subspace_small_supported((int)s.n[m], s.r[m]);
        p.gramm[m] = p.fused[m] && subspace_gram_supported(s.outer(m), (int)s.n[m], s.inner(m), s.r[m]);
        p.longm[m] = !cold && !p.fused[m] && subspace_long_supported(s.outer(m), (int)s.n[m], s.inner(m), s.r[m]);
        if (!cold && !p.fused[m] && !p.longm[m]) vmax = std::max(vmax, (size_t)(s.numel / s.n[m]) * s.r[m]);
    }
    p.V = c.take<float>(vmax);
    size_t ubmax = 0;
    for (int m = 0; m < s.d; ++m) {
        p.bfv[m] = !cold && s.dt == BF16 && !p.fused[m] && !p.longm[m] && m == s.d - 1 &&
                   gemm_bf16_supported(s.numel / s.n[m], (int)s.n[m], s.r[m]);
        if (p.bfv[m]) ubmax = std::max(ubmax, split_bf16_elems((int)s.n[m], s.r[m]));
    }
    p.Ub = c.take<unsigned short>(ubmax);
    size_t vpmax = 0;
    for (int m = 0; m < s.d; ++m) {
        if (!p.bfv[m]) continue;
        p.bfks[m] = gemm_bf16_ksplit(s.numel / s.n[m], (int)s.n[m], s.r[m]);
        if (p.bfks[m] > 1) vpmax = std::max(vpmax, (size_t)p.bfks[m] * (size_t)(s.numel / s.n[m]) * s.r[m]);
    }
    p.Vpart = c.take<float>(vpmax);
    p.ctr8 = c.take<int32_t>(8);
    p.tiny = !cold && s.d == 4 && subspace_tiny_supported((int)s.n[2], (int)s.n[3], s.r[2], s.r[3]);
    p.planes = !cold && s.d == 4 && subspace_planes_supported(s.n[0] * s.n[1], (int)s.n[2], (int)s.n[3], s.r[2], s.r[3]);
    p.paired = p.tiny || p.planes || (!cold && s.d == 4 && subspace_pair_supported((int)s.n[2], (int)s.n[3], s.r[2], s.r[3]));
    for (int m = 0; m < s.d; ++m) {
        const size_t n = (size_t)s.n[m], r = (size_t)s.r[m];
        if (p.tiny && m >= 2) p.nsplit[m] = subspace_tiny_nwg(s.n[0] * s.n[1]);
        else if (p.planes && m >= 2) p.nsplit[m] = subspace_planes_nwg(s.n[0] * s.n[1]);
        else if (p.paired && m >= 2) p.nsplit[m] = subspace_pair_nwg(s.n[0] * s.n[1], (int)s.n[2], (int)s.n[3]);
        else if (p.gramm[m]) p.nsplit[m] = subspace_gram_nwg(s.outer(m), (int)n, s.inner(m));
        else if (p.longm[m]) p.nsplit[m] = subspace_long_splits(s.outer(m), (int)n, s.inner(m), (int)r);
        else p.nsplit[m] = p.fused[m] ? subspace_small_nwg(s.outer(m), (int)n, s.inner(m))
                                      : pair_splits(s.outer(m), (int)n, s.inner(m), (int)r);
        p.part[m] = c.take<double>((size_t)p.nsplit[m] * n * r);
        if (p.nsplit[m] > 32) {
            p.nsplit2[m] = (p.nsplit[m] + 31) / 32;
            p.part2[m] = c.take<double>((size_t)p.nsplit2[m] * n * r);
        }
        p.P64[m] = c.take<double>(n * r);
        p.fast_orth[m] = orth_fast_supported((int)r);
        if (p.fast_orth[m]) {
            p.nblk[m] = orth_slices((int)n);
            p.Gpart[m] = c.take<double>((size_t)p.nblk[m] * r * r);
            p.R[m] = c.take<double>(r * r);
            p.Dinv[m] = c.take<double>(((r + 15) / 16) * 256);
            p.scal[m] = c.take<double>(68);
        } else if (orth_wide_supported((int)r)) {
            p.wide_orth[m] = true;
            p.nblk[m] = orth_wide_gram_blocks((int)n);
            p.Gpart[m] = c.take<double>((size_t)p.nblk[m] * r * r);
            // The factorisation is one workgroup; summing megabytes of slice Grams there runs at the
            // bandwidth of one CU (110 us for 24 slices of 192 x 192), so a tree level does it first.
            if ((size_t)p.nblk[m] * r * r >= (size_t)1 << 16) {
                p.ngsum[m] = 1;                       // one summed matrix (k_orthw_gsum)
                p.Gsum[m] = c.take<double>((size_t)r * r);
            }
            p.R[m] = c.take<double>(r * r);
            p.Dinv[m] = c.take<double>(((r + 15) / 16) * 256);
            p.scal[m] = c.take<double>(200);
        } else {
            p.Gpart[m] = c.take<double>(r * r);      // slow path: the Gram matrix itself
        }
    }
    p.bytes = c.off;
    return p;
}

// ---- core projection ----------------------------------------------------------
// The products are ordered by a cost that follows their measured time (see core_cost).  For small spatial extents the H and W
// modes are contracted together by one pass with the Kronecker product of their factors, so
// the tensor is treated as (B, C, H*W) with three "super modes".
// merged products pay off while the contraction fits one or two K chunks of the kernel; a longer
// one is a chain of dependent chunks on few workgroups and two separate products are faster
constexpr int kKronMaxN = 64, kKronMaxR = 64, kKronMaxOut = 256;

struct CorePlan {
    int d = 0;                       // super modes
    long long n[4] = {1, 1, 1, 1};
    int r[4] = {1, 1, 1, 1};
    bool kron = false;               // the last super mode is (H, W) merged
    int order[4] = {0, 1, 2, 3};
    float* buf[2] = {};
    unsigned short* Ub = nullptr;    // split factor of a first product along the last mode of a bf16 tensor
    bool bf_last = false;            // such a product is available (bf16 MFMA kernel)
    int bf_ks = 1;                   // ... with its contraction split over this many workgroups per column tile
    float* part = nullptr;           // ... whose partial products are summed into the product's output
    size_t bytes = 0;
};

bool kron_ok(long long n_a, long long n_b, int r_a, int r_b) {
    return n_a * n_b <= kKronMaxN && (long long)r_a * r_b <= kKronMaxR;
}

// Cost of the products taken in the order perm.  Every product is one pass over its input, so the
// elements read and written count first and the multiply-adds count at the rate the product
// kernels sustain relative to their data movement (about 64 per element moved).  Counting
// multiply-adds alone would start with the cheap halvings along H and W, i.e. with the largest
// number of full passes; this measure starts with the mode that shrinks the tensor most.
double core_cost(const CorePlan& p, const int* perm) {
    long long cur[4];
    for (int m = 0; m < 4; ++m) cur[m] = p.n[m];
    double cost = 0.0;
    for (int k = 0; k < p.d; ++k) {
        const int m = perm[k];
        double in = 1.0;
        for (int q = 0; q < p.d; ++q) in *= (double)cur[q];
        const double out = in / (double)cur[m] * p.r[m];
        // first product along the last mode of a bf16 tensor: half the bytes per element, and the bf16 MFMA
        // (two terms) multiplies at eight times the fp32 rate
        if (k == 0 && p.bf_last && m == p.d - 1) cost += 0.5 * in + out + in * p.r[m] / 512.0;
        else cost += in + out + in * p.r[m] / 64.0;
        cur[m] = p.r[m];
    }
    return cost;
}

void core_shape(const Shape& s, CorePlan* p) {
    p->kron = s.d == 4 && kron_ok(s.n[2], s.n[3], s.r[2], s.r[3]);
    p->d = p->kron ? 3 : s.d;
    for (int m = 0; m < p->d; ++m) { p->n[m] = s.n[m]; p->r[m] = s.r[m]; }
    if (p->kron) { p->n[2] = s.n[2] * s.n[3]; p->r[2] = s.r[2] * s.r[3]; }
    p->bf_last = s.dt == BF16 && !p->kron &&
                 gemm_bf16_supported(s.numel / s.n[s.d - 1], (int)s.n[s.d - 1], s.r[s.d - 1]);
}

// order: the order of the products, or null for the cheapest.  The two intermediate buffers are
// sized for any order, so that a batch may impose a common one.
CorePlan plan_core(const Shape& s, void* ws, const int* order = nullptr) {
    CorePlan p;
    core_shape(s, &p);
    int perm[4] = {0, 1, 2, 3};
    double best = -1.0;
    size_t need[2] = {0, 0};
    do {
        const double cost = core_cost(p, perm);
        if (!order && (best < 0 || cost < best)) { best = cost; std::memcpy(p.order, perm, sizeof(perm)); }
        long long cur[4];
        for (int m = 0; m < 4; ++m) cur[m] = p.n[m];
        for (int k = 0; k + 1 < p.d; ++k) {   // the last product writes S itself
            cur[perm[k]] = p.r[perm[k]];
            size_t sz = 1;
            for (int q = 0; q < p.d; ++q) sz *= (size_t)cur[q];
            need[k & 1] = std::max(need[k & 1], sz);
        }
    } while (std::next_permutation(perm, perm + p.d));
    if (order) std::memcpy(p.order, order, sizeof(int) * 4);
    Carver c(ws);
    p.buf[0] = c.take<float>(need[0]);
    p.buf[1] = c.take<float>(need[1]);
    p.Ub = c.take<unsigned short>(p.bf_last ? split_bf16_elems((int)s.n[s.d - 1], s.r[s.d - 1]) : 0);
    if (p.bf_last) p.bf_ks = gemm_bf16_ksplit(s.numel / s.n[s.d - 1], (int)s.n[s.d - 1], s.r[s.d - 1]);
    p.part = c.take<float>(p.bf_ks > 1 ? (size_t)p.bf_ks * (size_t)(s.numel / s.n[s.d - 1]) * s.r[s.d - 1] : 0);
    p.bytes = c.off;
    return p;
}

// ---- conv2d weight gradient ------------------------------------------------------
struct ConvGeom {
    CorrGeom g;
    int C, B, groups;
};

bool parse_conv(const Shape& s, const asi_conv2d_desc* cv, ConvGeom* out) {
    if (!cv || s.d != 4) return false;
    if (cv->cout <= 0 || cv->cout > (1 << 24) || cv->kh <= 0 || cv->kw <= 0 || cv->kh > 64 || cv->kw > 64) return false;
    if (cv->stride_h <= 0 || cv->stride_w <= 0 || cv->dil_h <= 0 || cv->dil_w <= 0) return false;
    if (cv->pad_h < 0 || cv->pad_w < 0 || cv->groups <= 0) return false;
    const long long C = s.n[1];
    if (C % cv->groups != 0 || cv->cout % cv->groups != 0) return false;
    const long long H = s.n[2], W = s.n[3];
    const long long eh = H + 2LL * cv->pad_h - (long long)cv->dil_h * (cv->kh - 1) - 1;
    const long long ew = W + 2LL * cv->pad_w - (long long)cv->dil_w * (cv->kw - 1) - 1;
    if (eh < 0 || ew < 0) return false;
    CorrGeom& g = out->g;
    g.r1 = s.r[0]; g.r2 = s.r[1];
    g.cout = (int)cv->cout;
    g.H = (int)H; g.W = (int)W;
    g.Ho = (int)(eh / cv->stride_h + 1); g.Wo = (int)(ew / cv->stride_w + 1);
    g.kh = cv->kh; g.kw = cv->kw; g.sh = cv->stride_h; g.sw = cv->stride_w;
    g.ph = cv->pad_h; g.pw = cv->pad_w; g.dh = cv->dil_h; g.dw = cv->dil_w;
    out->C = (int)C; out->B = (int)s.n[0]; out->groups = cv->groups;
    return true;
}

struct ConvPlan {
    float *G1 = nullptr, *Z1 = nullptr, *Z = nullptr, *Tpart = nullptr, *T = nullptr;
    float* S1 = nullptr;             // r1 = B: the core expanded along the batch mode (see build_conv)
    int nsplit = 1;
    size_t bytes = 0;
};

ConvPlan plan_conv(const Shape& s, const ConvGeom& cg, void* ws) {
    ConvPlan p;
    const CorrGeom& g = cg.g;
    Carver c(ws);
    p.G1 = c.take<float>((size_t)g.r1 * g.cout * g.Ho * g.Wo);
    if (g.r1 == cg.B) p.S1 = c.take<float>((size_t)cg.B * g.r2 * s.r[2] * s.r[3]);
    if ((long long)s.r[2] * s.r[3] > kKronMaxN || (long long)g.H * g.W > kKronMaxOut)
        p.Z1 = c.take<float>((size_t)g.r1 * g.r2 * g.H * s.r[3]);      // else Z comes from one merged pass
    p.Z = c.take<float>((size_t)g.r1 * g.r2 * g.H * g.W);
    p.nsplit = corr_splits(g);
    const size_t tsz = (size_t)g.cout * g.r2 * g.kh * g.kw;
    p.T = c.take<float>(tsz);
    p.Tpart = p.nsplit > 1 ? c.take<float>(tsz * p.nsplit) : p.T;
    p.bytes = c.off;
    return p;
}

// ---- linear weight gradient --------------------------------------------------------
struct LinPlan {
    float *G1 = nullptr, *G2 = nullptr, *T = nullptr;
    float* S1 = nullptr;             // r1 = B: the core expanded along the batch mode (see build_linear)
    double* Tpart = nullptr;
    int nsplit = 1;
    size_t bytes = 0;
};

LinPlan plan_linear(const Shape& s, long long dout, void* ws) {
    LinPlan p;
    Carver c(ws);
    p.G1 = c.take<float>((size_t)s.r[0] * s.n[1] * dout);
    p.G2 = c.take<float>((size_t)s.r[0] * s.r[1] * dout);
    if (s.r[0] == s.n[0]) p.S1 = c.take<float>((size_t)s.n[0] * s.r[1] * s.r[2]);
    p.nsplit = pair_splits((long long)s.r[0] * s.r[1], (int)dout, 1, s.r[2]);
    p.T = c.take<float>((size_t)dout * s.r[2]);
    p.Tpart = c.take<double>((size_t)p.nsplit * dout * s.r[2]);
    p.bytes = c.off;
    return p;
}

bool ws_ok(const void* ws, size_t have, size_t need) {
    return ws && (reinterpret_cast<uintptr_t>(ws) % kAlign) == 0 && have >= need;
}

// ---- per-kernel timing for benchmarks (off by default) -----------------------------
// When enabled, every launch is bracketed by two HIP events on the launch stream and
// tagged with the bytes and flops the step must move / compute by its definition.
struct ProfRec {
    std::string site;
    double bytes, flops, wgs;
    hipEvent_t e0, e1;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof;

inline double esize(DType t) { return t == F32 ? 4.0 : 2.0; }

// ---- the launches of one layer, in order --------------------------------------------
struct Program {
    std::vector<Item> items;
    Item* add(const char* role, double bytes, double flops) {
        items.emplace_back();
        return &items.back();
    }
};
// finishes the item appended last
inline void tag(Program& pg, const char* role, double bytes, double flops) {
    Item& it = pg.items.back();
    std::snprintf(it.role, sizeof(it.role), "%s", role);
    it.bytes = bytes; it.flops = flops;
}
#define ASI_ADD(pg, role, bytes, flops, make_call)         \
    do {                                                   \
        (pg).items.emplace_back();                         \
        Item* it__ = &(pg).items.back();                   \
        if (!(make_call)) return ASI_ERR_UNSUPPORTED;      \
        tag((pg), (role), (bytes), (flops));               \
    } while (0)

// mode product with its accounting: reads X and M once, writes (or updates) Y once
asi_status add_ttm(Program& pg, const char* role, DType xt, const void* X, long long outer, int n, long long inner,
                   const float* Mp, long long ms_i, long long ms_q, int r, float* Y, int beta, bool stream_ok = true) {
    const double cols = (double)outer * (double)inner;
    ASI_ADD(pg, role, cols * n * esize(xt) + 4.0 * n * r + 4.0 * cols * r * (beta ? 2 : 1), 2.0 * cols * n * r,
            make_ttm(xt, X, outer, n, inner, Mp, ms_i, ms_q, r, Y, beta, it__, stream_ok));
    return ASI_OK;
}
// two trailing modes at once (Kronecker product of their matrices)
asi_status add_ttm_kron(Program& pg, const char* role, DType xt, const void* X, long long cols, int n1, int n2,
                        const float* M1, long long ms1_i, long long ms1_q, int r1, const float* M2, long long ms2_i,
                        long long ms2_q, int r2, float* Y) {
    const double n = (double)n1 * n2, r = (double)r1 * r2;
    ASI_ADD(pg, role, cols * n * esize(xt) + 4.0 * (n1 * r1 + n2 * r2) + 4.0 * cols * r, 2.0 * cols * n * r,
            make_ttm_kron(xt, X, cols, n1, n2, M1, ms1_i, ms1_q, r1, M2, ms2_i, ms2_q, r2, Y, 0, it__));
    return ASI_OK;
}
asi_status add_pair(Program& pg, const char* role, DType xt, const void* X, long long outer, int n, long long inner,
                    const float* Y, int r, double* part, int nsplit, int32_t* zero, int nzero,
                    const PresumArgs* ride = nullptr, double ride_bytes = 0.0) {
    const double cols = (double)outer * (double)inner;
    ASI_ADD(pg, role, cols * n * esize(xt) + 4.0 * cols * r + 8.0 * n * r * nsplit + ride_bytes, 2.0 * cols * n * r,
            make_pair(xt, X, outer, n, inner, Y, r, part, nsplit, zero, nzero, ride, it__));
    return ASI_OK;
}
// P = A_m V with the generated V of Alg. 1's first iteration: nothing of V is read
asi_status add_pair_gauss(Program& pg, const char* role, DType xt, const void* X, long long outer, int n, long long inner,
                          unsigned long long seed, int mode, int r, double* part, int nsplit, int32_t* zero, int nzero,
                          const PresumArgs* ride, double ride_bytes) {
    const double cols = (double)outer * (double)inner;
    ASI_ADD(pg, role, cols * n * esize(xt) + 8.0 * n * r * nsplit + ride_bytes, 2.0 * cols * n * r,
            make_pair_gauss(xt, X, outer, n, inner, seed, mode, r, part, nsplit, zero, nzero, ride, it__));
    return ASI_OK;
}
#define ASI_TRYS(expr)                                 \
    do {                                               \
        asi_status s__ = (expr);                       \
        if (s__ != ASI_OK) return s__;                 \
    } while (0)

// Runs the programs of `count` layers: position by position, the items that can share a
// launch (same kernel instantiation up to size bounds) go out together.
asi_status flush(std::vector<Program>& progs, hipStream_t st, const char* phase) {
    size_t maxlen = 0;
    for (auto& pg : progs) maxlen = std::max(maxlen, pg.items.size());
    for (size_t pos = 0; pos < maxlen; ++pos) {
        std::vector<const Item*> pending;
        for (auto& pg : progs)
            if (pos < pg.items.size()) pending.push_back(&pg.items[pos]);
        while (!pending.empty()) {
            const Item* group[kMaxBatch];
            int n = 0;
            std::vector<const Item*> rest;
            for (const Item* it : pending) {
                if (n < kMaxBatch && (n == 0 || same_launch(*group[0], *it))) group[n++] = it;
                else rest.push_back(it);
            }
            ProfRec rec;
            const bool prof = g_prof_on;
            if (prof) {
                if (hipEventCreate(&rec.e0) != hipSuccess || hipEventCreate(&rec.e1) != hipSuccess) return ASI_ERR_HIP;
                (void)hipEventRecord(rec.e0, st);
            }
            char label[96];
            if (launch_items(group, n, st, label) != hipSuccess) return ASI_ERR_HIP;
            if (prof) {
                (void)hipEventRecord(rec.e1, st);
                // "phase|kernel instantiation:role", e.g. "core|k_ttm_mfma<float, false, 3, 0>:core"
                rec.site = std::string(phase) + "|" + label + (group[0]->role[0] ? std::string(":") + group[0]->role : std::string());
                rec.bytes = rec.flops = rec.wgs = 0;
                for (int j = 0; j < n; ++j) { rec.bytes += group[j]->bytes; rec.flops += group[j]->flops; rec.wgs += group[j]->nblocks; }
                std::lock_guard<std::mutex> lk(g_prof_mu);
                g_prof.push_back(rec);
            }
            pending.swap(rest);
        }
    }
    return ASI_OK;
}

// ---- builders: validate one layer's arguments and append its launches -----------------------------
// seed: null for the warm-start branch (U_prev given); else the first iteration, V drawn from *seed
asi_status build_compress(const asi_tensor_desc* desc, const void* A, const float* const* U_prev, float* const* U_out,
                          void* ws, size_t ws_bytes, int32_t* info, const unsigned long long* seed, Program& pg) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    const bool cold = seed != nullptr;
    if (!A || (!cold && !U_prev) || !U_out) return ASI_ERR_INVALID_ARG;
    for (int m = 0; m < s.d; ++m)
        if ((!cold && !U_prev[m]) || !U_out[m]) return ASI_ERR_INVALID_ARG;
    CompressPlan p = plan_compress(s, ws, cold);
    if (!ws_ok(ws, ws_bytes, p.bytes)) return ASI_ERR_WORKSPACE;

    OrthArgs fast, wide, slow;
    GsumArgs gsum;                   // wide modes with many slices: tree level over the slice Grams
    std::memset(&gsum, 0, sizeof(gsum));
    double gsum_b = 0;
    std::memset(&fast, 0, sizeof(fast));
    std::memset(&wide, 0, sizeof(wide));
    std::memset(&slow, 0, sizeof(slow));
    PresumArgs pre, pre2;            // pre2, second tree level: wide modes need the finished sum in P64
    std::memset(&pre, 0, sizeof(pre));
    std::memset(&pre2, 0, sizeof(pre2));
    double wide_b = 0, wide_f = 0, pre2_b = 0, chol_b = 0, chol_f = 0, wchol_b = 0, wchol_f = 0;
    double fast_b = 0, fast_f = 0, slow_b = 0, slow_f = 0, pre_b = 0;
    // Launch order of the subspace steps: the modes served by one kernel first, then the modes that
    // take two (V, then P).  The last P launch also carries the first level of the partial-sum tree of
    // the modes before it (independent work in extra workgroups), which saves a launch of its own.
    int order[4], nord = 0, last_two = -1;
    for (int m = 0; m < s.d; ++m)
        if (p.fused[m] || p.longm[m] || (p.paired && m >= 2)) order[nord++] = m;
    for (int m = 0; m < s.d; ++m)
        if (!(p.fused[m] || p.longm[m] || (p.paired && m >= 2))) { order[nord++] = m; last_two = m; }
    PresumJob prejob[4];
    bool preneed[4] = {false, false, false, false};
    for (int m = 0; m < s.d; ++m) {
        if (!p.part2[m]) continue;
        PresumJob& pj = prejob[m];
        pj.in = p.part[m]; pj.out = p.part2[m]; pj.cnt = (long long)s.n[m] * s.r[m]; pj.nsplit = p.nsplit[m];
        pj.nchunks = (int)((pj.cnt + 255) / 256); pj.ngroups = p.nsplit2[m];
        preneed[m] = true;
    }
    bool zero_given = false;
    for (int k = 0; k < nord; ++k) {
        const int m = order[k];
        const long long outer = s.outer(m), inner = s.inner(m);
        const int n = (int)s.n[m], r = s.r[m];
        if (p.paired && m == 2) {
            // H and W modes: both subspace steps from one read of the activation's planes
            const double tot = (double)s.numel;
            if (p.planes)
                ASI_ADD(pg, "", tot * esize(s.dt) + 8.0 * (n * r + (double)s.n[3] * s.r[3]) * p.nsplit[m], 4.0 * tot * (r + s.r[3]),
                        make_subspace_planes(s.dt, A, s.n[0] * s.n[1], n, (int)s.n[3], U_prev[2], r, p.part[2], U_prev[3], s.r[3],
                                             p.part[3], p.nsplit[m], nullptr, 0, it__));
            else if (p.tiny)
                ASI_ADD(pg, "", tot * esize(s.dt) + 8.0 * (n * r + (double)s.n[3] * s.r[3]) * p.nsplit[m], 4.0 * tot * (r + s.r[3]),
                        make_subspace_tiny(s.dt, A, s.n[0] * s.n[1], n, (int)s.n[3], U_prev[2], r, p.part[2], U_prev[3], s.r[3],
                                           p.part[3], p.nsplit[m], it__));
            else
                ASI_ADD(pg, "", tot * esize(s.dt) + 8.0 * (n * r + (double)s.n[3] * s.r[3]) * p.nsplit[m], 4.0 * tot * (r + s.r[3]),
                        make_subspace_pair(s.dt, A, s.n[0] * s.n[1], n, (int)s.n[3], U_prev[2], r, p.part[2], U_prev[3], s.r[3],
                                           p.part[3], p.nsplit[m], it__));
        } else if (p.paired && m == 3) {
            // done together with mode 3
        } else if (p.longm[m]) {
            // long fibres (64 < n <= 512): V and P from one LDS tile of complete fibres, V never stored
            int32_t* zero = zero_given ? nullptr : p.ctr8;
            zero_given = true;
            const double cols = (double)outer * (double)inner;
            ASI_ADD(pg, "", cols * n * esize(s.dt) + 4.0 * n * r + 8.0 * n * r * p.nsplit[m], 4.0 * cols * n * r,
                    make_subspace_long(s.dt, A, outer, n, inner, U_prev[m], r, p.part[m], p.nsplit[m], zero, 8, it__));
        } else if (p.gramm[m]) {
            // short mode, long inner extent: the Gram matrix of the unfolding in one pass, then G U_prev
            int32_t* zero = zero_given ? nullptr : p.ctr8;
            zero_given = true;
            const double cols = (double)outer * (double)inner;
            // flops by the step's definition (two products of 2 cols n r), not the Gram matrix's own count
            ASI_ADD(pg, "", cols * n * esize(s.dt) + 4.0 * n * r + 8.0 * n * r * p.nsplit[m], 4.0 * cols * n * r,
                    make_subspace_gram(s.dt, A, outer, n, inner, U_prev[m], r, p.part[m], p.nsplit[m], zero, 8, it__));
        } else if (p.fused[m]) {
            // short fibres: V and P from one LDS tile of complete fibres, V never stored
            int32_t* zero = zero_given ? nullptr : p.ctr8;       // one early kernel clears the arrival counters
            zero_given = true;
            const double cols = (double)outer * (double)inner;
            ASI_ADD(pg, "", cols * n * esize(s.dt) + 4.0 * n * r + 8.0 * n * r * p.nsplit[m], 4.0 * cols * n * r,
                    make_subspace_small(s.dt, A, outer, n, inner, U_prev[m], r, p.part[m], p.nsplit[m], zero, 8, it__));
        } else {
            int32_t* zero = zero_given ? nullptr : p.ctr8;
            zero_given = true;
            // V = A_m^T U_prev, kept as a tensor with mode m of size r (first iteration: generated, not kept)
            if (cold) {
            } else if (p.bfv[m]) {
                const double cols = (double)outer;
                ASI_ADD(pg, "V", 4.0 * n * r + 2.0 * (double)split_bf16_elems(n, r), 0.0,
                        make_split_bf16(U_prev[m], r, 1, n, r, p.Ub, it__));
                const int ks = p.bfks[m];
                ASI_ADD(pg, "V", cols * n * 2.0 + 2.0 * (double)split_bf16_elems(n, r) + 4.0 * cols * r * ks, 2.0 * cols * n * r,
                        make_gemm_bf16(A, outer, n, p.Ub, r, ks > 1 ? p.Vpart : p.V, ks, nullptr, 0, it__));
                if (ks > 1)
                    ASI_ADD(pg, "V", 4.0 * cols * r * (ks + 1), cols * r * ks,
                            make_sum_partials(p.Vpart, ks, (long long)outer * r, p.V, 0, it__));
            } else {
                ASI_TRYS(add_ttm(pg, "V", s.dt, A, outer, n, inner, U_prev[m], r, 1, r, p.V, 0));
            }
            // P = A_m V, split over the unfolding's columns
            PresumArgs ride;
            std::memset(&ride, 0, sizeof(ride));
            double ride_b = 0;
            if (m == last_two)
                for (int k2 = 0; k2 < k; ++k2) {
                    const int m2 = order[k2];
                    if (!preneed[m2]) continue;
                    ride.job[ride.njobs++] = prejob[m2];
                    ride_b += 8.0 * s.n[m2] * s.r[m2] * (p.nsplit[m2] + p.nsplit2[m2]);
                    preneed[m2] = false;
                }
            if (cold)
                ASI_TRYS(add_pair_gauss(pg, "P", s.dt, A, outer, n, inner, *seed, m, r, p.part[m], p.nsplit[m], zero, 8,
                                        ride.njobs ? &ride : nullptr, ride_b));
            else
                ASI_TRYS(add_pair(pg, "P", s.dt, A, outer, n, inner, p.V, r, p.part[m], p.nsplit[m], zero, 8,
                                  ride.njobs ? &ride : nullptr, ride_b));
        }
    }
    for (int m = 0; m < s.d; ++m)
        if (preneed[m]) {
            pre.job[pre.njobs++] = prejob[m];
            pre_b += 8.0 * s.n[m] * s.r[m] * (p.nsplit[m] + p.nsplit2[m]);
        }
    for (int m = 0; m < s.d; ++m) {
        const int n = (int)s.n[m], r = s.r[m];
        OrthArgs& oa = p.fast_orth[m] ? fast : (p.wide_orth[m] ? wide : slow);
        OrthJob& j = oa.job[oa.njobs++];
        j.part = p.part[m]; j.nsplit = p.nsplit[m]; j.n = n; j.r = r;
        if (p.part2[m]) { j.part = p.part2[m]; j.nsplit = p.nsplit2[m]; }     // the tree's first level has run
        j.P64 = p.P64[m]; j.Uout = U_out[m]; j.mode1 = m + 1; j.info = info;
        j.nblk = p.nblk[m]; j.Gpart = p.Gpart[m]; j.R = p.R[m]; j.Dinv = p.Dinv[m]; j.scal = p.scal[m];
        j.ctr = p.ctr8 + 2 * m;
        if (p.wide_orth[m] && p.Gsum[m]) {
            GsumJob& gj = gsum.job[gsum.njobs++];
            gj.in = p.Gpart[m]; gj.out = p.Gsum[m]; gj.nblk = p.nblk[m]; gj.r = r;
            gj.nchunks = (r * r + 255) / 256;
            gj.devbits = reinterpret_cast<unsigned long long*>(p.scal[m] + 196);     // (the wide path's bookkeeping ends at 194)
            j.devbits = gj.devbits;
            gsum_b += 8.0 * r * r * (p.nblk[m] + 1);
        }
        if (p.wide_orth[m]) {
            PresumJob& pj = pre2.job[pre2.njobs++];
            pj.in = j.part; pj.out = p.P64[m]; pj.cnt = (long long)n * r; pj.nsplit = j.nsplit;
            pj.nchunks = (int)((pj.cnt + 255) / 256); pj.ngroups = 1;
            pre2_b += 8.0 * n * r * (j.nsplit + 1);
        }
        // Cholesky: reads the slice Grams, writes R and the diagonal-block inverses; r^3/3 flops
        const double cb = 8.0 * ((double)(p.Gsum[m] ? p.ngsum[m] : p.nblk[m]) * r * r + (double)r * r + 256.0 * ((r + 15) / 16));
        const double cf = (double)r * r * r / 3.0;
        if (p.fast_orth[m]) { chol_b += cb; chol_f += cf; }
        if (p.wide_orth[m]) { wchol_b += cb; wchol_f += cf; }
        (p.fast_orth[m] ? fast_b : (p.wide_orth[m] ? wide_b : slow_b)) += 8.0 * n * r;
        (p.fast_orth[m] ? fast_f : (p.wide_orth[m] ? wide_f : slow_f)) += 2.0 * (double)n * r * r;
    }
    if (info && !fast.njobs) ASI_ADD(pg, "", 4.0, 0.0, make_init_ctrl(info, it__));     // otherwise gram0 clears it
    if (pre.njobs) ASI_ADD(pg, "", pre_b, pre_b / 8.0, make_orth_presum(pre, it__));
    if (fast.njobs) {
        // Orthogonalize: Cholesky-QR (with a diagonal shift if the plain factorisation loses a pivot),
        // then a second Cholesky-QR pass unless the first result is orthonormal to 1e-7 already.
        // Each launch ends with the factorisation of its Gram matrices in the last workgroup of a
        // mode; the second pass, when needed, is carried out by that workgroup too.
        ASI_ADD(pg, "", fast_b + chol_b, fast_f + chol_f, make_orth_gram0(fast, it__));
        ASI_ADD(pg, "", 2.5 * fast_b + chol_b, 2 * fast_f + chol_f, make_orth_apply(fast, it__));
    }
    if (wide.njobs) {
        ASI_ADD(pg, "", pre2_b, pre2_b / 8.0, make_orth_presum(pre2, it__));
        OrthArgs wchol = wide;           // the factorisation reads the summed Grams where a tree level made them
        for (int j = 0; j < wchol.njobs; ++j) {
            const int m = wchol.job[j].mode1 - 1;
            if (p.Gsum[m]) { wchol.job[j].Gpart = p.Gsum[m]; wchol.job[j].nblk = p.ngsum[m]; }
        }
        ASI_ADD(pg, "", wide_b, wide_f, make_orthw_gram(wide, it__));
        if (gsum.njobs) ASI_ADD(pg, "", gsum_b, gsum_b / 8.0, make_orthw_gsum(gsum, it__));
        ASI_ADD(pg, "", wchol_b, wchol_f, make_orthw_chol(wchol, 0, 0, it__));
        ASI_ADD(pg, "", 2 * wide_b, wide_f, make_orthw_apply(wide, 0, it__));
        ASI_ADD(pg, "", wide_b, wide_f, make_orthw_gram(wide, it__));
        if (gsum.njobs) ASI_ADD(pg, "", gsum_b, gsum_b / 8.0, make_orthw_gsum(gsum, it__));
        ASI_ADD(pg, "", wchol_b, wchol_f, make_orthw_chol(wchol, 1, 1, it__));
        ASI_ADD(pg, "", 1.5 * wide_b, wide_f, make_orthw_apply(wide, 1, it__));
    }
    if (slow.njobs) ASI_ADD(pg, "", 6 * slow_b, 9 * slow_f, make_orth_big(slow, it__));
    return ASI_OK;
}

asi_status build_core(const asi_tensor_desc* desc, const void* A, const float* const* U, float* S, void* ws,
                      size_t ws_bytes, const int* order, Program& pg) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    if (!A || !U || !S) return ASI_ERR_INVALID_ARG;
    for (int m = 0; m < s.d; ++m)
        if (!U[m]) return ASI_ERR_INVALID_ARG;
    CorePlan p = plan_core(s, ws, order);
    if (!ws_ok(ws, ws_bytes, p.bytes)) return ASI_ERR_WORKSPACE;

    long long cur[4];
    for (int m = 0; m < 4; ++m) cur[m] = p.n[m];
    const void* src = A;
    DType sdt = s.dt;
    int pp = 0;                                         // which of the two buffers the next intermediate goes to
    for (int k = 0; k < p.d; ++k) {
        const int m = p.order[k];
        long long outer = 1, inner = 1;
        for (int q = 0; q < m; ++q) outer *= cur[q];
        for (int q = m + 1; q < p.d; ++q) inner *= cur[q];
        // The H and W products of an fp32 intermediate with large planes, when the order has them side by side:
        // one launch, plane by plane (the intermediate is a few MB and each product alone is a chain of round trips).
        if (!p.kron && p.d == 4 && k >= 1 && k + 1 < p.d && sdt == F32 && m + p.order[k + 1] == 5 && m >= 2 && p.order[k + 1] >= 2) {
            float* dst2 = (k + 2 == p.d) ? S : p.buf[pp];
            pg.items.emplace_back();
            if (make_core_planes(static_cast<const float*>(src), cur[0] * cur[1], (int)cur[2], (int)cur[3], U[2], p.r[2], U[3],
                                 p.r[3], dst2, &pg.items.back())) {
                const double planes = (double)cur[0] * (double)cur[1], H = (double)cur[2], W = (double)cur[3];
                tag(pg, "core", 4.0 * (planes * (H * W + (double)p.r[2] * p.r[3]) + H * p.r[2] + W * p.r[3]),
                    2.0 * planes * (H * W * p.r[3] + H * p.r[2] * p.r[3]));
                cur[2] = p.r[2]; cur[3] = p.r[3];
                src = dst2; pp ^= 1; ++k;
                continue;
            }
            pg.items.pop_back();
        }
        float* dst = (k + 1 == p.d) ? S : p.buf[pp];
        pp ^= 1;
        if (k == 0 && p.bf_last && m == p.d - 1) {
            // the bf16 activation along its last mode: split factor, then the bf16 MFMA product
            const int n = (int)cur[m], r = p.r[m];
            const double cols = (double)outer;
            ASI_ADD(pg, "core", 4.0 * n * r + 2.0 * (double)split_bf16_elems(n, r), 0.0,
                    make_split_bf16(U[m], r, 1, n, r, p.Ub, it__));
            const int ks = p.bf_ks;
            ASI_ADD(pg, "core", cols * n * 2.0 + 2.0 * (double)split_bf16_elems(n, r) + 4.0 * cols * r * ks, 2.0 * cols * n * r,
                    make_gemm_bf16(src, outer, n, p.Ub, r, ks > 1 ? p.part : dst, ks, nullptr, 0, it__));
            if (ks > 1)
                ASI_ADD(pg, "core", 4.0 * cols * r * (ks + 1), cols * r * ks,
                        make_sum_partials(p.part, ks, (long long)outer * r, dst, 0, it__));
        } else if (p.kron && m == 2) {
            // (.., H, W) -> (.., r3, r4):  M(h*W + w, a*r4 + b) = U3[h,a] * U4[w,b]
            ASI_TRYS(add_ttm_kron(pg, "core", sdt, src, outer, (int)s.n[2], (int)s.n[3], U[2], s.r[2], 1, s.r[2], U[3],
                                  s.r[3], 1, s.r[3], dst));
        } else {
            ASI_TRYS(add_ttm(pg, "core", sdt, src, outer, (int)cur[m], inner, U[m], p.r[m], 1, p.r[m], dst, 0));
        }
        cur[m] = p.r[m];
        src = dst;
        sdt = F32;
    }
    return ASI_OK;
}

asi_status build_conv(const asi_tensor_desc* desc, const float* S, const float* const* U, const void* grad_out,
                      const asi_conv2d_desc* conv, float* dW, int accumulate, void* ws, size_t ws_bytes, Program& pg) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    if (s.d != 4 || !conv) return ASI_ERR_INVALID_ARG;
    ConvGeom cg;
    if (!parse_conv(s, conv, &cg)) return ASI_ERR_INVALID_ARG;
    if (!S || !U || !grad_out || !dW) return ASI_ERR_INVALID_ARG;
    for (int m = 0; m < 4; ++m)
        if (!U[m]) return ASI_ERR_INVALID_ARG;
    ConvPlan p = plan_conv(s, cg, ws);
    if (!ws_ok(ws, ws_bytes, p.bytes)) return ASI_ERR_WORKSPACE;
    const CorrGeom& g = cg.g;
    const int r3 = s.r[2], r4 = s.r[3];
    const int taps = g.kh * g.kw;

    // With r1 = B the batch factor is square: G1 would be as large as grad_out, and forming it saves the
    // correlation nothing.  The same sum with the parentheses moved expands the small core instead,
    //     T = sum_i (sum_b U1[b,i] dY[b]) * Z[i] = sum_b dY[b] * Z'[b],   Z' from S1 = S x_1 U1   (B, r2, r3, r4),
    // and the correlation reads grad_out itself (fp32 data, aligned for its 16-byte loads).
    const bool expand_core = p.S1 && s.dt == F32 && reinterpret_cast<uintptr_t>(grad_out) % 16 == 0;
    const float* Sz = S;
    const float* G1 = p.G1;
    if (expand_core) {
        // 1'. S1[b,...] = sum_i U1[b,i] S[i,...]
        ASI_TRYS(add_ttm(pg, "S1", F32, S, 1, g.r1, (long long)g.r2 * r3 * r4, U[0], 1, g.r1, cg.B, p.S1, 0));
        Sz = p.S1;
        G1 = static_cast<const float*>(grad_out);
    } else {
        // 1. G1 = grad_out x_1 U1^T                                   (r1, cout, Ho, Wo)
        // (where Z comes from one merged product it can share G1's launch: G1 then stays on the tiled kernel)
        ASI_TRYS(add_ttm(pg, "G1", s.dt, grad_out, 1, cg.B, (long long)g.cout * g.Ho * g.Wo, U[0], g.r1, 1, g.r1, p.G1, 0,
                         p.Z1 != nullptr));
    }
    if (!p.Z1) {
        // 2+3. Z = S x_3 U3 x_4 U4 in one pass:  M(a*r4 + b, h*W + w) = U3[h,a] * U4[w,b]   (r1, r2, H, W)
        ASI_TRYS(add_ttm_kron(pg, "Z", F32, Sz, (long long)g.r1 * g.r2, r3, r4, U[2], 1, r3, g.H, U[3], 1, r4, g.W, p.Z));
        // G1 and Z do not depend on each other: one launch for both when their kernels allow it
        Item duo;
        const size_t ni = pg.items.size();
        if (!expand_core && make_ttm_duo(pg.items[ni - 2], pg.items[ni - 1], &duo)) {
            pg.items.pop_back();
            pg.items.back() = duo;
        }
    } else if (pg.items.emplace_back(),
               make_z_planes(Sz, (long long)g.r1 * g.r2, r3, r4, U[2], g.H, U[3], g.W, p.Z, &pg.items.back())) {
        // 2+3. Z[p] = U3 S[p] U4^T plane by plane, both products in one launch (planes of up to 64 x 64, ranks up to 32)
        const double planes = (double)g.r1 * g.r2;
        tag(pg, "Z", 4.0 * (planes * ((double)r3 * r4 + (double)g.H * g.W) + (double)g.H * r3 + (double)g.W * r4),
            2.0 * planes * ((double)g.H * r3 * r4 + (double)g.H * g.W * r4));
    } else {
        pg.items.pop_back();
        // 2. Z1 = S x_3 U3                                        (r1, r2, H, r4)
        ASI_TRYS(add_ttm(pg, "Z1", F32, Sz, (long long)g.r1 * g.r2, r3, r4, U[2], 1, r3, g.H, p.Z1, 0));
        // 3. Z = Z1 x_4 U4                                        (r1, r2, H, W)
        ASI_TRYS(add_ttm(pg, "Z", F32, p.Z1, (long long)g.r1 * g.r2 * g.H, r4, 1, U[3], 1, r4, g.W, p.Z, 0));
    }
    // 4. T = correlation of Zpad with G1 over (r1, Ho, Wo)        (cout, r2, kh, kw)
    const double tsz = (double)g.cout * g.r2 * taps;
    ASI_ADD(pg, "", 4.0 * ((double)g.r1 * g.cout * g.Ho * g.Wo + (double)g.r1 * g.r2 * g.H * g.W + tsz * p.nsplit),
            2.0 * g.r1 * g.Ho * g.Wo * tsz, make_corr(G1, p.Z, p.Tpart, g, p.nsplit, it__));
    // 5. dW = T x_(r2) U2, per group                              (cout, C/groups, kh, kw)
    // An ungrouped convolution with 1 or 9 taps and r2 <= 64 sums the partial T's and expands the result in one
    // launch (T itself is then never written); anything else sums first and multiplies in a second launch.
    if (cg.groups == 1) {
        pg.items.emplace_back();
        if (make_dw_fold(p.Tpart, p.nsplit, U[1], dW, g.cout, cg.C, g.r2, taps, accumulate ? 1 : 0, &pg.items.back())) {
            tag(pg, "dW", 4.0 * (tsz * p.nsplit + (double)cg.C * g.r2 + (double)g.cout * cg.C * taps * (accumulate ? 2 : 1)),
                2.0 * (double)g.cout * taps * g.r2 * cg.C + tsz * p.nsplit);
            return ASI_OK;
        }
        pg.items.pop_back();
    }
    if (p.nsplit > 1)
        ASI_ADD(pg, "", 4.0 * tsz * (p.nsplit + 1), tsz * p.nsplit,
                make_sum_partials(p.Tpart, p.nsplit, (long long)g.cout * g.r2 * taps, p.T, 0, it__));
    if (cg.groups == 1) {
        ASI_TRYS(add_ttm(pg, "dW", F32, p.T, g.cout, g.r2, taps, U[1], 1, g.r2, cg.C, dW, accumulate ? 1 : 0));
    } else {
        const double dwsz = (double)g.cout * (cg.C / cg.groups) * taps;
        ASI_ADD(pg, "", 4.0 * ((double)g.cout * g.r2 * taps + (double)cg.C * g.r2 + dwsz), 2.0 * dwsz * g.r2,
                make_expand_grouped(p.T, U[1], dW, g.cout, g.r2, taps, cg.C / cg.groups, g.cout / cg.groups,
                                    accumulate ? 1 : 0, it__));
    }
    return ASI_OK;
}

asi_status build_linear(const asi_tensor_desc* desc, const float* S, const float* const* U, const void* grad_out,
                        int64_t dout, float* dW, int accumulate, void* ws, size_t ws_bytes, Program& pg) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    if (s.d != 3 || dout <= 0 || dout > (1 << 24)) return ASI_ERR_INVALID_ARG;
    if (!S || !U || !grad_out || !dW) return ASI_ERR_INVALID_ARG;
    for (int m = 0; m < 3; ++m)
        if (!U[m]) return ASI_ERR_INVALID_ARG;
    LinPlan p = plan_linear(s, dout, ws);
    if (!ws_ok(ws, ws_bytes, p.bytes)) return ASI_ERR_WORKSPACE;
    const int B = (int)s.n[0], N = (int)s.n[1], D = (int)s.n[2];
    const int r1 = s.r[0], r2 = s.r[1], r3 = s.r[2];

    const float* Sz = S;
    if (p.S1) {
        // r1 = B: U1 is square and G1 would be as large as grad_out.  The sum over the batch mode is moved to
        // the small core instead: S1[b,j,k] = sum_i U1[b,i] S[i,j,k], and step 2 reads grad_out itself.
        ASI_TRYS(add_ttm(pg, "S1", F32, S, 1, r1, (long long)r2 * r3, U[0], 1, r1, B, p.S1, 0));
        ASI_TRYS(add_ttm(pg, "G2", s.dt, grad_out, B, N, dout, U[1], r2, 1, r2, p.G2, 0));
        Sz = p.S1;
    } else {
        // 1. G1[i,n,o] = sum_b U1[b,i] dY[b,n,o]
        ASI_TRYS(add_ttm(pg, "G1", s.dt, grad_out, 1, B, (long long)N * dout, U[0], r1, 1, r1, p.G1, 0));
        // 2. G2[i,j,o] = sum_n U2[n,j] G1[i,n,o]
        ASI_TRYS(add_ttm(pg, "G2", F32, p.G1, r1, N, dout, U[1], r2, 1, r2, p.G2, 0));
    }
    // 3. T[o,k] = sum_{i,j} G2[i,j,o] S[i,j,k]
    ASI_TRYS(add_pair(pg, "T", F32, p.G2, (long long)r1 * r2, (int)dout, 1, Sz, r3, p.Tpart, p.nsplit, nullptr, 0));
    const double tsz = (double)dout * r3;
    ASI_ADD(pg, "", tsz * (8.0 * p.nsplit + 4.0), tsz * p.nsplit,
            make_sum_partials_f64(p.Tpart, p.nsplit, (long long)dout * r3, p.T, 0, it__));
    // 4. dW[o,d] = sum_k T[o,k] U3[d,k]
    ASI_TRYS(add_ttm(pg, "dW", F32, p.T, dout, r3, 1, U[2], 1, r3, D, dW, accumulate ? 1 : 0));
    return ASI_OK;
}

bool batch_count_ok(int32_t count) { return count >= 1 && count <= kMaxBatch; }

// ---- scratch memory of the entry point that allocates nothing -----------------------------------
// A file-scope device array: every GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a stand-in for the symbol; the device address of the current
// GPU's copy is asked for once per device (hipGetSymbolAddress) and used from then on.
static __device__ __align__(256) unsigned char scratch[ASI_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

asi_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ASI_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ASI_ERR_HIP;
        if (reinterpret_cast<uintptr_t>(p) % kAlign != 0) return ASI_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ASI_OK;
}

}  // namespace

extern "C" {

int32_t asi_version(void) { return 1002; }

int32_t asi_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    const int32_t was = g_prof_on ? 1 : 0;
    for (auto& r : g_prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    g_prof.clear();
    g_prof_on = on != 0;
    return was;
}

int64_t asi_profile_report(char* buf, int64_t buflen) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    struct Agg { long long count = 0; double ms = 0, bytes = 0, flops = 0, wgs = 0; };
    std::map<std::string, Agg> agg;
    for (auto& r : g_prof) {
        if (hipEventSynchronize(r.e1) != hipSuccess) return -1;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) return -1;
        Agg& a = agg[r.site];
        a.count += 1; a.ms += ms; a.bytes += r.bytes; a.flops += r.flops; a.wgs += r.wgs;
    }
    std::string out;
    char line[320];
    for (auto& kv : agg) {
        std::snprintf(line, sizeof(line), "%s,%lld,%.6f,%.1f,%.1f,%.0f\n", kv.first.c_str(), kv.second.count,
                      kv.second.ms, kv.second.bytes, kv.second.flops, kv.second.wgs);
        out += line;
    }
    if (buf && buflen > 0) {
        const size_t ncopy = std::min((size_t)buflen - 1, out.size());
        std::memcpy(buf, out.data(), ncopy);
        buf[ncopy] = 0;
    }
    return (int64_t)out.size() + 1;
}

const char* asi_status_string(asi_status s) {
    switch (s) {
        case ASI_OK: return "ASI_OK";
        case ASI_ERR_INVALID_ARG: return "ASI_ERR_INVALID_ARG";
        case ASI_ERR_UNSUPPORTED: return "ASI_ERR_UNSUPPORTED";
        case ASI_ERR_WORKSPACE: return "ASI_ERR_WORKSPACE";
        case ASI_ERR_HIP: return "ASI_ERR_HIP";
        case ASI_ERR_NUMERIC: return "ASI_ERR_NUMERIC";
        case ASI_ERR_INFEASIBLE: return "ASI_ERR_INFEASIBLE";
    }
    return "ASI_ERR_UNKNOWN";
}

size_t asi_workspace_bytes(const asi_tensor_desc* desc, const asi_conv2d_desc* conv, int64_t dout) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return 0;
    size_t need = std::max(plan_compress(s, nullptr).bytes, plan_core(s, nullptr).bytes);
    need = std::max(need, plan_compress(s, nullptr, true).bytes);
    if (conv) {
        ConvGeom cg;
        if (!parse_conv(s, conv, &cg)) return 0;
        need = std::max(need, plan_conv(s, cg, nullptr).bytes);
    }
    if (dout > 0) {
        if (s.d != 3 || dout > (1 << 24)) return 0;
        need = std::max(need, plan_linear(s, dout, nullptr).bytes);
    }
    return std::max(need, kAlign);
}

asi_status asi_compress_batch(int32_t count, const asi_tensor_desc* descs, const void* const* A,
                              const float* const* const* U_prev, float* const* const* U_out, void* const* ws,
                              const size_t* ws_bytes, int32_t* const* info, asi_stream_t stream) {
    if (!batch_count_ok(count)) return ASI_ERR_UNSUPPORTED;
    if (!descs || !A || !U_prev || !U_out || !ws || !ws_bytes) return ASI_ERR_INVALID_ARG;
    std::vector<Program> progs(count);
    for (int l = 0; l < count; ++l)
        ASI_TRYS(build_compress(&descs[l], A[l], U_prev[l], U_out[l], ws[l], ws_bytes[l], info ? info[l] : nullptr, nullptr,
                                progs[l]));
    return flush(progs, static_cast<hipStream_t>(stream), "compress");
}

asi_status asi_compress_cold(const asi_tensor_desc* desc, const void* A, uint64_t seed, float* const* U_out, void* ws,
                             size_t ws_bytes, int32_t* info, asi_stream_t stream) {
    std::vector<Program> progs(1);
    const unsigned long long sd = seed;
    ASI_TRYS(build_compress(desc, A, nullptr, U_out, ws, ws_bytes, info, &sd, progs[0]));
    return flush(progs, static_cast<hipStream_t>(stream), "cold");
}

asi_status asi_cold_start_matrix(const asi_tensor_desc* desc, int32_t mode, uint64_t seed, float* V, asi_stream_t stream) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    if (mode < 0 || mode >= s.d || !V) return ASI_ERR_INVALID_ARG;
    std::vector<Program> progs(1);
    const double cnt = (double)(s.numel / s.n[mode]) * s.r[mode];
    ASI_ADD(progs[0], "", 4.0 * cnt, 0.0, make_gauss_fill(seed, mode, s.numel / s.n[mode], s.r[mode], V, it__));
    return flush(progs, static_cast<hipStream_t>(stream), "cold");
}

asi_status asi_core_project_batch(int32_t count, const asi_tensor_desc* descs, const void* const* A,
                                  const float* const* const* U, float* const* S, void* const* ws,
                                  const size_t* ws_bytes, asi_stream_t stream) {
    if (!batch_count_ok(count)) return ASI_ERR_UNSUPPORTED;
    if (!descs || !A || !U || !S || !ws || !ws_bytes) return ASI_ERR_INVALID_ARG;
    // Layers with the same mode structure take their products in one common order (the cheapest in
    // total), so that product k of every layer can share a launch.
    int common[4] = {0, 1, 2, 3};
    bool have_common = count > 1;
    CorePlan first;
    std::vector<CorePlan> shapes(count);
    for (int l = 0; l < count && have_common; ++l) {
        Shape s;
        asi_status why;
        if (!parse_desc(&descs[l], &s, &why)) { have_common = false; break; }
        core_shape(s, &shapes[l]);
        if (shapes[l].d != shapes[0].d || shapes[l].kron != shapes[0].kron) have_common = false;
    }
    if (have_common) {
        int perm[4] = {0, 1, 2, 3};
        double best = -1.0;
        do {
            double cost = 0.0;
            for (int l = 0; l < count; ++l) cost += core_cost(shapes[l], perm);
            if (best < 0 || cost < best) { best = cost; std::memcpy(common, perm, sizeof(perm)); }
        } while (std::next_permutation(perm, perm + shapes[0].d));
    }
    std::vector<Program> progs(count);
    for (int l = 0; l < count; ++l)
        ASI_TRYS(build_core(&descs[l], A[l], U[l], S[l], ws[l], ws_bytes[l], have_common ? common : nullptr, progs[l]));
    return flush(progs, static_cast<hipStream_t>(stream), "core");
}

asi_status asi_weight_grad_conv2d_batch(int32_t count, const asi_tensor_desc* descs, const float* const* S,
                                        const float* const* const* U, const void* const* grad_out,
                                        const asi_conv2d_desc* convs, float* const* dW, const int32_t* accumulate,
                                        void* const* ws, const size_t* ws_bytes, asi_stream_t stream) {
    if (!batch_count_ok(count)) return ASI_ERR_UNSUPPORTED;
    if (!descs || !S || !U || !grad_out || !convs || !dW || !ws || !ws_bytes) return ASI_ERR_INVALID_ARG;
    std::vector<Program> progs(count);
    for (int l = 0; l < count; ++l)
        ASI_TRYS(build_conv(&descs[l], S[l], U[l], grad_out[l], &convs[l], dW[l], accumulate ? accumulate[l] : 0, ws[l],
                            ws_bytes[l], progs[l]));
    return flush(progs, static_cast<hipStream_t>(stream), "dW");
}

asi_status asi_weight_grad_linear_batch(int32_t count, const asi_tensor_desc* descs, const float* const* S,
                                        const float* const* const* U, const void* const* grad_out, const int64_t* dout,
                                        float* const* dW, const int32_t* accumulate, void* const* ws,
                                        const size_t* ws_bytes, asi_stream_t stream) {
    if (!batch_count_ok(count)) return ASI_ERR_UNSUPPORTED;
    if (!descs || !S || !U || !grad_out || !dout || !dW || !ws || !ws_bytes) return ASI_ERR_INVALID_ARG;
    std::vector<Program> progs(count);
    for (int l = 0; l < count; ++l)
        ASI_TRYS(build_linear(&descs[l], S[l], U[l], grad_out[l], dout[l], dW[l], accumulate ? accumulate[l] : 0, ws[l],
                              ws_bytes[l], progs[l]));
    return flush(progs, static_cast<hipStream_t>(stream), "dW");
}

asi_status asi_compress(const asi_tensor_desc* desc, const void* A, const float* const* U_prev,
                        float* const* U_out, void* ws, size_t ws_bytes, int32_t* info, asi_stream_t stream) {
    if (!desc) return ASI_ERR_INVALID_ARG;
    return asi_compress_batch(1, desc, &A, &U_prev, &U_out, &ws, &ws_bytes, &info, stream);
}

asi_status asi_compress_static(const asi_tensor_desc* desc, const void* A, const float* const* U_prev,
                               float* const* U_out, int32_t* info, asi_stream_t stream) {
    Shape s;
    asi_status why;
    if (!parse_desc(desc, &s, &why)) return why;
    // the limit is checked before anything touches the device
    if (plan_compress(s, nullptr).bytes > (size_t)ASI_STATIC_SCRATCH_BYTES) return ASI_ERR_WORKSPACE;
    void* ws = nullptr;
    ASI_TRYS(static_scratch(&ws));
    // Everything the kernels expect to start from zero (the arrival counters) is cleared by the first
    // kernel of the call itself, so what the previous call left in the array does not matter.
    return asi_compress(desc, A, U_prev, U_out, ws, (size_t)ASI_STATIC_SCRATCH_BYTES, info, stream);
}

asi_status asi_core_project(const asi_tensor_desc* desc, const void* A, const float* const* U, float* S,
                            void* ws, size_t ws_bytes, asi_stream_t stream) {
    if (!desc) return ASI_ERR_INVALID_ARG;
    return asi_core_project_batch(1, desc, &A, &U, &S, &ws, &ws_bytes, stream);
}

asi_status asi_weight_grad_conv2d(const asi_tensor_desc* desc, const float* S, const float* const* U,
                                  const void* grad_out, const asi_conv2d_desc* conv, float* dW, int accumulate,
                                  void* ws, size_t ws_bytes, asi_stream_t stream) {
    if (!desc || !conv) return ASI_ERR_INVALID_ARG;
    const int32_t acc = accumulate;
    return asi_weight_grad_conv2d_batch(1, desc, &S, &U, &grad_out, conv, &dW, &acc, &ws, &ws_bytes, stream);
}

asi_status asi_weight_grad_linear(const asi_tensor_desc* desc, const float* S, const float* const* U,
                                  const void* grad_out, int64_t dout, float* dW, int accumulate, void* ws,
                                  size_t ws_bytes, asi_stream_t stream) {
    if (!desc) return ASI_ERR_INVALID_ARG;
    const int32_t acc = accumulate;
    return asi_weight_grad_linear_batch(1, desc, &S, &U, &grad_out, &dout, &dW, &acc, &ws, &ws_bytes, stream);
}

}  // extern "C"
