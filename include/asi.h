/*
 * asi.h - C ABI of the MI355X (gfx950) library for the hot path of Activation
 * Subspace Iteration (ASI, arxiv 2505.05086).
 *
 * Per training step and per fine-tuned layer the method
 *   (1) runs one warm-started subspace-iteration step on every mode unfolding
 *       of the stored activation and orthonormalises the result (Alg. 1),
 *   (2) projects the activation onto those factors to get the Tucker core
 *       (Alg. 1's core update; Eq. 3, Eq. 4),
 *   (3) in the backward pass computes the conv2d / linear weight gradient from
 *       core + factors without rebuilding the activation (App. A.3, Eq. 14).
 * Before training, the ranks of every layer are chosen from measurements on a
 * batch of activations (Sec. 3.3): the entry points at the end of this header.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is caller-owned DEVICE memory on the current HIP
 *     device.  The library allocates nothing, keeps no state between calls and
 *     only enqueues kernels on `stream`; it never synchronises with the host
 *     (one exception, stated there: asi_mode_spectrum).
 *   - Activation `A` and output gradient `grad_out`: dense row-major, (B,C,H,W)
 *     or (B,N,D); element type given by asi_tensor_desc.dtype (fp32, or bf16
 *     with fp32 accumulation).
 *   - Factor U_m: row-major (dims[m] x ranks[m]) fp32.  Core S: row-major
 *     (ranks[0] x ... x ranks[ndim-1]) fp32.  dW: (Cout, C/groups, kh, kw) or
 *     (Dout, Din) fp32.
 *   - `ws` is scratch of at least asi_workspace_bytes() bytes, 256-byte aligned.
 *     Calls that share one workspace must be ordered on one stream.
 *   - Synchronous argument errors are returned as a status and enqueue nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef ASI_H
#define ASI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ASI_OK = 0,
    ASI_ERR_INVALID_ARG = 1,   /* null pointer, bad ndim/dims/ranks, bad conv geometry */
    ASI_ERR_UNSUPPORTED = 2,   /* unknown dtype, size beyond an implementation limit */
    ASI_ERR_WORKSPACE = 3,     /* ws null, misaligned or smaller than asi_workspace_bytes() */
    ASI_ERR_HIP = 4,           /* a HIP runtime call failed (launch error) */
    ASI_ERR_NUMERIC = 5,       /* an iteration did not converge (asi_mode_spectrum); elsewhere numeric
                                  breakdown is reported through *info */
    ASI_ERR_INFEASIBLE = 6     /* asi_rank_select: no choice of ranks fits the budget */
} asi_status;

typedef enum { ASI_F32 = 0, ASI_BF16 = 1 } asi_dtype;   /* element type of A and grad_out */

/* One stored activation and its target ranks (Alg. 1 inputs).
 * ndim = 4: dims = (B, C, H, W); ndim = 3: dims = (B, N, D).
 * 1 <= ranks[m] <= min(dims[m], numel / dims[m]) (Alg. 1's rank range); ranks[m] <= 1024. */
typedef struct {
    int32_t ndim;
    int64_t dims[4];
    int32_t ranks[4];
    int32_t dtype;             /* asi_dtype */
} asi_tensor_desc;

/* Geometry of the convolution whose weight gradient is wanted (Sec. 3.1 notation:
 * C' = cout, D = kh = kw in the paper; general stride / padding / dilation / groups here). */
typedef struct {
    int64_t cout;
    int32_t kh, kw;
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    int32_t dil_h, dil_w;
    int32_t groups;            /* must divide both C and cout */
} asi_conv2d_desc;

typedef void* asi_stream_t;    /* hipStream_t */

/* Scratch bytes that cover every entry point for this layer: asi_compress and
 * asi_core_project always; asi_weight_grad_conv2d if conv != NULL;
 * asi_weight_grad_linear if dout > 0.  Returns 0 if desc (or conv) is invalid. */
size_t asi_workspace_bytes(const asi_tensor_desc* desc, const asi_conv2d_desc* conv, int64_t dout);

/* Alg. 1, warm-start branch, for every mode m of A:
 *     V = A_m^T U_prev[m];   P = A_m V;   U_out[m] = Orthogonalize(P)
 * where A_m is the mode-m unfolding of the ORIGINAL activation (Sec. 3.2) and
 * U_prev[m] is the factor kept from the previous training step.  Orthogonalize
 * returns the Q factor of the thin QR of P with positive diagonal R (what
 * Gram-Schmidt produces, App. A.1), so U_out^T U_out = I.
 *   A          in  device, dims per desc, dtype per desc
 *   U_prev[m]  in  device fp32 (dims[m] x ranks[m]), m < ndim; any full-rank matrix
 *   U_out[m]   out device fp32 (dims[m] x ranks[m]); may alias U_prev[m]
 *   info       out device int32 (nullable).  Set to 0 when the call starts executing;
 *              if P of mode m (1-based) is numerically rank deficient at column
 *              j (1-based) it becomes m*1000 + j and U_out[m] is unspecified.
 *              Read it after synchronising the stream. */
asi_status asi_compress(const asi_tensor_desc* desc, const void* A,
                        const float* const* U_prev, float* const* U_out,
                        void* ws, size_t ws_bytes, int32_t* info, asi_stream_t stream);

/* Alg. 1, first iteration (t = 0), for every mode m of A:
 *     V ~ N(0, 1)^(b_m x ranks[m]);   P = A_m V;   U_out[m] = Orthogonalize(P)
 * V is not stored: entry V[c, q] of mode m (0-based; c = column of the mode-m unfolding in the row-major
 * order of the remaining modes) is a pure function of (seed, m, c, q).  With g = q / 4 and k = q % 4,
 * Philox4x32-10 keyed by (seed mod 2^32, seed div 2^32) on the counter (c mod 2^32, c div 2^32, g, m) gives
 * words x0..x3; u_i = ((x_i >> 9) + 0.5) / 2^23; V[c, 4g + {0,1}] = sqrt(-2 ln u0) * {cos, sin}(2 pi u1) and
 * V[c, 4g + {2,3}] the same from (u2, u3), evaluated in fp64 and rounded to fp32.  Arguments, workspace (asi_workspace_bytes
 * covers it) and error behaviour as asi_compress, without U_prev. */
asi_status asi_compress_cold(const asi_tensor_desc* desc, const void* A, uint64_t seed,
                             float* const* U_out, void* ws, size_t ws_bytes, int32_t* info,
                             asi_stream_t stream);

/* The V that asi_compress_cold multiplies by for one mode, written out for inspection:
 *   V  out device fp32 (b_mode x ranks[mode]) row-major, b_mode = numel / dims[mode]. */
asi_status asi_cold_start_matrix(const asi_tensor_desc* desc, int32_t mode, uint64_t seed, float* V,
                            asi_stream_t stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): asi_compress with the library's own scratch memory in
 * place of `ws`.  The scratch is a static device array of ASI_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends; the call allocates and frees nothing.  Same
 * arguments, results (bit for bit) and error behaviour as asi_compress, plus ASI_ERR_WORKSPACE when
 * the layer needs more scratch than the array holds (asi_workspace_bytes(desc, NULL, 0) is an upper
 * bound of that need) — then nothing is enqueued.  The array belongs to the current device; all calls
 * on one GPU share it, so calls that overlap in time on one GPU (two streams, two threads) race:
 * order them on one stream.  What a call leaves in the array is of no use to the next; the kernels
 * clear what they need cleared. */
#define ASI_STATIC_SCRATCH_BYTES (16u << 20)
asi_status asi_compress_static(const asi_tensor_desc* desc, const void* A,
                               const float* const* U_prev, float* const* U_out,
                               int32_t* info, asi_stream_t stream);

/* Core tensor S = A x_1 U[0]^T x_2 U[1]^T ... x_d U[d-1]^T (Alg. 1's core update with
 * Eq. 4's m-mode product; the order of the products does not change the result).
 *   U[m]  in  device fp32 (dims[m] x ranks[m])
 *   S     out device fp32, row-major (ranks[0] x ... x ranks[ndim-1]) */
asi_status asi_core_project(const asi_tensor_desc* desc, const void* A,
                            const float* const* U, float* S,
                            void* ws, size_t ws_bytes, asi_stream_t stream);

/* Weight gradient of a conv2d layer from the compressed activation, in the order
 * the five terms of C_ASI describe (App. A.3, Eq. 14):
 *     G1 = grad_out x_1 U1^T;  Z = S x_3 U3 x_4 U4;
 *     T[o,j,kh,kw] = sum_{i,h',w'} G1[i,o,h',w'] * Zpad[i,j,h'*s-p+kh*dil, w'*s-p+kw*dil];
 *     dW[o,c,kh,kw] = sum_j T[o,j,kh,kw] * U2[g(o)*C/groups + c, j].
 * The result equals Eq. 1 applied to the reconstruction S x_1 U1 ... x_4 U4.
 *   desc      4-mode descriptor of the activation that was compressed
 *   grad_out  in  device (B, cout, H', W'), dtype per desc,
 *             H' = floor((H + 2 pad_h - dil_h (kh-1) - 1) / stride_h) + 1
 *   dW        out device fp32 (cout, C/groups, kh, kw); overwritten, or added to
 *             when accumulate != 0 */
asi_status asi_weight_grad_conv2d(const asi_tensor_desc* desc, const float* S,
                                  const float* const* U, const void* grad_out,
                                  const asi_conv2d_desc* conv, float* dW, int accumulate,
                                  void* ws, size_t ws_bytes, asi_stream_t stream);

/* Weight gradient of a linear layer (Sec. 3.1 footnote: the fully-connected case
 * follows the same construction) for a 3-mode activation (B, N, Din):
 *     G1 = grad_out x_1 U1^T;  G2 = G1 x_2 U2^T;
 *     T[o,k] = sum_{i,j} G2[i,j,o] S[i,j,k];   dW[o,d] = sum_k T[o,k] U3[d,k].
 *   grad_out  in  device (B, N, dout), dtype per desc
 *   dW        out device fp32 (dout, Din); overwritten, or added to when accumulate != 0 */
asi_status asi_weight_grad_linear(const asi_tensor_desc* desc, const float* S,
                                  const float* const* U, const void* grad_out,
                                  int64_t dout, float* dW, int accumulate,
                                  void* ws, size_t ws_bytes, asi_stream_t stream);

/* Batched forms of the four operations above: the same computation for `count` layers
 * (1 <= count <= 8) in as many kernel launches as ONE layer needs, because every kernel
 * serves the argument blocks of all layers side by side (launches of different layers are
 * merged when they use the same kernel; layers of one network stage usually do).  Per-step
 * cost on MI355X is dominated by the number of dependent launches, not by their size.
 * Every array argument is a HOST array of length count whose element l holds what the
 * single-layer call takes for layer l (descs and convs are arrays of structs; accumulate may
 * be NULL = all zero; info may be NULL or hold NULL entries).  Each layer has its own
 * workspace.  The factors are bit-identical to those of `count` single-layer calls; the core
 * projection may take its m-mode products in another order (one order for the whole batch, so
 * that the layers' products share launches), which changes S and dW at rounding level only.
 * If any layer's arguments are rejected nothing is enqueued and that status is returned;
 * count outside the range gives ASI_ERR_UNSUPPORTED. */
asi_status asi_compress_batch(int32_t count, const asi_tensor_desc* descs, const void* const* A,
                              const float* const* const* U_prev, float* const* const* U_out,
                              void* const* ws, const size_t* ws_bytes, int32_t* const* info,
                              asi_stream_t stream);
asi_status asi_core_project_batch(int32_t count, const asi_tensor_desc* descs, const void* const* A,
                                  const float* const* const* U, float* const* S,
                                  void* const* ws, const size_t* ws_bytes, asi_stream_t stream);
asi_status asi_weight_grad_conv2d_batch(int32_t count, const asi_tensor_desc* descs, const float* const* S,
                                        const float* const* const* U, const void* const* grad_out,
                                        const asi_conv2d_desc* convs, float* const* dW,
                                        const int32_t* accumulate, void* const* ws, const size_t* ws_bytes,
                                        asi_stream_t stream);
asi_status asi_weight_grad_linear_batch(int32_t count, const asi_tensor_desc* descs, const float* const* S,
                                        const float* const* const* U, const void* const* grad_out,
                                        const int64_t* dout, float* const* dW,
                                        const int32_t* accumulate, void* const* ws, const size_t* ws_bytes,
                                        asi_stream_t stream);

/* ---- Rank selection (Sec. 3.3): measurements made once, before training, to choose the ranks ---- */

/* Eq. 5: elements kept for one layer, prod_m ranks[m] + sum_m dims[m] * ranks[m]; -1 if desc is invalid. */
int64_t asi_activation_memory(const asi_tensor_desc* desc);

/* Scratch bytes of asi_mode_spectrum for this mode (desc->ranks is not read); 0 if the descriptor or
 * the mode is invalid or dims[mode] exceeds the limit of 512. */
size_t asi_mode_spectrum_workspace_bytes(const asi_tensor_desc* desc, int32_t mode);

/* Spectrum of one mode (App. A.2; Sec. 3.3, Step 1): the eigenvalues of A_m A_m^T, i.e. the squared
 * singular values of the mode-m unfolding, and its eigenvectors, the principal components of the mode.
 *   A             in  device, dims per desc, dtype per desc (desc->ranks is not read)
 *   eigenvalues   out device fp64 (dims[mode]), descending
 *   eigenvectors  out device fp32 (dims[mode] x dims[mode]) row-major, column k = k-th principal component,
 *                 nullable; its first r columns are the factor of a truncated HOSVD of rank r.  A column
 *                 whose eigenvalue is below 1e-12 of the largest is returned as zeros.
 *   sweeps        out HOST int32 (nullable): Jacobi sweeps used, -1 if 60 sweeps did not converge
 * Unlike every other entry point this one WAITS for the stream: it iterates to convergence and reads
 * the iteration's state after every sweep.  dims[mode] <= 512 (ASI_ERR_UNSUPPORTED beyond);
 * ASI_ERR_NUMERIC if the iteration did not converge (the outputs then hold its last state). */
asi_status asi_mode_spectrum(const asi_tensor_desc* desc, const void* A, int32_t mode, double* eigenvalues,
                             float* eigenvectors, void* ws, size_t ws_bytes, int32_t* sweeps,
                             asi_stream_t stream);

/* Sec. 3.3, Step 1: for each threshold eps[j] (HOST array, 0 < eps <= 1, n_eps <= 16) the smallest
 * r >= 1 with sum_{k <= r} lambda_k >= eps[j] * sum_k lambda_k.
 *   eigenvalues in  device fp64 (n), descending (asi_mode_spectrum's output)
 *   ranks       out device int32 (n_eps) */
asi_status asi_explained_variance_ranks(const double* eigenvalues, int32_t n, const double* eps, int32_t n_eps,
                                        int32_t* ranks, asi_stream_t stream);

/* Eq. 7, the perplexity of a layer at one threshold: *out = || a - b ||_F in fp64.
 *   a, b  in  device fp32 (count): the exact weight gradient and the one computed from the compressed
 *             activation (asi_weight_grad_* on the truncated eigenvectors and their core)
 *   out   out device fp64 (1)
 *   ws    scratch of at least ASI_FROBENIUS_WS_BYTES bytes, 256-byte aligned */
#define ASI_FROBENIUS_WS_BYTES 8192
asi_status asi_frobenius_diff(const float* a, const float* b, int64_t count, double* out, void* ws,
                              size_t ws_bytes, asi_stream_t stream);

/* Eq. 8-9: one threshold index per layer, choice[i] in [0, n_eps), that minimises sum_i P[i, choice[i]]
 * subject to sum_i M[i, choice[i]] <= budget, by recursive backtracking (exhaustive up to bounds that
 * cannot change the result; among equal totals the lexicographically first choice).  HOST code on
 * HOST arrays: P, M row-major (n_layers x n_eps), P >= 0 finite, M >= 0 (Eq. 5, in elements);
 * n_layers <= 64, n_eps <= 16.  total (nullable) receives the minimum.  ASI_ERR_INFEASIBLE if no
 * choice fits the budget (choice is then untouched). */
asi_status asi_rank_select(int32_t n_layers, int32_t n_eps, const double* P, const int64_t* M, int64_t budget,
                           int32_t* choice, double* total);

/* Static, human-readable name of a status code. */
const char* asi_status_string(asi_status s);

/* Library ABI version (major*1000 + minor). */
int32_t asi_version(void);

/* Benchmark aid, off by default, not thread-safe against concurrent launches.
 * asi_profile_enable(on): drops earlier records; while on, every kernel launch of the
 * entry points above is bracketed by two HIP events on its stream and tagged with the
 * bytes and flops that step must move / compute by its definition.  Returns the previous
 * setting.
 * asi_profile_report(buf, buflen): waits for the recorded events and writes one text
 * line per launch site, "site,launches,total_ms,total_bytes,total_flops,total_workgroups\n", NUL-terminated
 * (site = "phase|kernel instantiation[:role]", phase one of compress / core / dW; it may contain commas)
 * and truncated to buflen (host memory).  Returns the bytes a full report needs, or -1
 * if an event could not be read. */
int32_t asi_profile_enable(int32_t on);
int64_t asi_profile_report(char* buf, int64_t buflen);

#ifdef __cplusplus
}
#endif
#endif /* ASI_H */
