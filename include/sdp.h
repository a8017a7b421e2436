/*
 * sdp.h -- C ABI of the Subnetwork-Data-Parallel (SDP) masked-MLP hot path for
 * AMD MI355X (gfx950).
 *
 * SDP (the paper's Sec. 3) trains, on each of n = K workers, a structurally
 * complete subnetwork chosen by a fixed binary mask matrix m in {0,1}^{K x F}
 * (Sec. 3.1).  This library instantiates the neuron-level variant (Sec. 3.2)
 * on a bias-free SwiGLU transformer MLP
 *
 *     G = X W1^T,  U = X W3^T,  A = silu(G) * U,  Y = A W2^T,   silu(z) = z / (1 + e^-z)
 *
 * where hidden neuron j owns row j of W1 and W3 and column j of W2.
 *
 * Conventions common to every entry point
 *   - Layout: all matrices are dense row-major.  The three weights are stored
 *     NEURON-MAJOR, [F][d] each: W1[j][:], W3[j][:] and W2T[j][:] (= column j of
 *     W2) are the d parameters of neuron j.  Weight gradients use the same layout.
 *   - Pointers are DEVICE pointers unless a parameter says "host".  The caller
 *     owns all memory; the library keeps no pointer after a call returns and
 *     allocates no device memory.  Scratch comes from the caller's workspace
 *     `ws` (device, 256-byte aligned), at least the matching
 *     *_workspace_bytes() large.
 *   - Every call only enqueues work on `stream` (a hipStream_t, NULL = the
 *     default stream) and returns; outputs are complete once the stream reaches
 *     that point.  Outputs are fully overwritten, never accumulated into.
 *   - dtype SDP_F32: all tensors fp32.  dtype SDP_BF16: all tensors bf16,
 *     products accumulated in fp32, intermediates that feed a later
 *     contraction rounded once to bf16 (round to nearest even).
 *   - Errors: argument errors are found on the host before any launch and
 *     returned as a negative sdp_status; nothing is enqueued in that case.
 *     No call aborts or throws.
 */
#ifndef SDP_H
#define SDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SDP_OK = 0,
    SDP_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, unknown enum value, misaligned pointer */
    SDP_ERR_SHAPE = -2,       /* sizes inconsistent with each other or beyond a stated limit          */
    SDP_ERR_WORKSPACE = -3,   /* ws is NULL or ws_bytes too small                                      */
    SDP_ERR_UNCOVERED = -4,   /* require_cover set but K * p < F: some neuron cannot be covered        */
    SDP_ERR_UNSUPPORTED = -5, /* combination not implemented                                           */
    SDP_ERR_HIP = -6          /* a HIP runtime call failed (launch, copy)                              */
} sdp_status;

typedef enum { SDP_F32 = 0, SDP_BF16 = 1 } sdp_dtype;
typedef enum { SDP_MASK_FORWARD = 0, SDP_MASK_BACKWARD = 1 } sdp_mode;
typedef enum { SDP_DW_COMPACT = 0, SDP_DW_SCATTER = 1 } sdp_dw_layout;
/* values of the `require_cover` argument of the samplers */
typedef enum { SDP_MASKS_UNIFORM = 0, SDP_MASKS_UNIFORM_COVER = 1, SDP_MASKS_BALANCED = 2 } sdp_mask_sampler;

#define SDP_MAX_WORKERS 64 /* largest K accepted anywhere */

const char* sdp_status_string(int status);

/* ---------------------------------------------------------------------------------------------
 * Masks (Sec. 3.1: m_{k,j} = 1 iff worker k is responsible for coordinate j; App. A: exact row
 * budget sum_j m_{k,j} = p, column loads c_j = sum_k m_{k,j}).
 *
 * sdp_make_masks draws the K x F mask matrix on the host from `seed`, copies it to the device and
 * derives its index form there (see sdp_index_masks).  Sampler: worker k takes p distinct neurons
 * uniformly (partial Fisher-Yates on the counter-based stream k); with require_cover != 0 every
 * neuron left with load 0 is then given to a worker that hands back a neuron of load >= 2, so all
 * row sums stay p and every c_j >= 1.  require_cover = SDP_MASKS_BALANCED (2) selects the balanced
 * construction of App. A (Algorithm "Structured Mask Construction") instead: worker i draws its p
 * neurons with weights max(t - c_j, 1e-6), t = ceil(K p / F), c_j the loads of the workers before it
 * (successive weighted draws on stream 2^20 + i), then under-loaded neurons j (ascending) are handed
 * to the first worker that lacks j and holds a neuron loaded above t, which gives up its most
 * loaded such neuron; row sums are p throughout, loads end within one of K p / F whenever K p is a
 * multiple of F.  The draw is a pure function of (K, F, p, seed, require_cover).
 *   mask  [K][F] u8 out     idx [K][p] i32 out     pos [K][F] i32 out     cov [F] u8 out
 *   ws: sdp_index_masks_workspace_bytes(K, F).
 * The call synchronises `stream` before returning (the host staging buffer is freed).
 * Errors: INVALID_ARG (null, K < 1, K > SDP_MAX_WORKERS, F < 1, p < 0, require_cover not 0..2),
 * SHAPE (p > F), UNCOVERED (require_cover = 1 and K p < F), WORKSPACE, HIP.
 * ------------------------------------------------------------------------------------------- */
int sdp_make_masks(int K, int F, int p, uint64_t seed, int require_cover, uint8_t* mask, int32_t* idx,
                   int32_t* pos, uint8_t* cov, void* ws, size_t ws_bytes, void* stream);

/* Host-only variant of the sampler: fills mask_host[K][F]; no device work. */
int sdp_sample_masks_host(int K, int F, int p, uint64_t seed, int require_cover, uint8_t* mask_host);

/* ---------------------------------------------------------------------------------------------
 * Mask -> index compaction (prefix sum over each worker's mask row) and coverage counts: the index
 * form of the mask matrix of Sec. 3.1, with the row sums and the column loads c_j = sum_k m_{k,j} of
 * App. A (the load of a column is the divisor of the gated average of every parameter it owns).
 *   mask  [K][F] u8 in, any non-zero byte counts as 1
 *   idx   [K][idx_ld] i32 out: idx[k][i] = i-th active neuron of worker k, ascending; entries
 *         from count[k] on are -1; active neurons of rank >= idx_ld are dropped
 *   pos   [K][F] i32 out: rank of neuron j in worker k's active set, or -1 if m_{k,j} = 0
 *   count [K] i32 out (may be NULL): row sums
 *   cov   [F] u8 out: c_j, the number of workers covering neuron j, which is the count of
 *         every parameter in neuron row j
 * Limits: 1 <= K <= SDP_MAX_WORKERS, 1 <= F < 2^31, 1 <= idx_ld <= F.
 * ------------------------------------------------------------------------------------------- */
size_t sdp_index_masks_workspace_bytes(int K, int64_t F);
int sdp_index_masks(int K, int64_t F, const uint8_t* mask, int32_t* idx, int64_t idx_ld, int32_t* pos,
                    int32_t* count, uint8_t* cov, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * sdp_index_masks for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * results as sdp_index_masks without `ws`: the table of per-chunk counts that long rows need lives in a
 * fixed array of the library, SDP_INDEX_STATIC_MAX_COUNTS int32 (256 KiB), which every GPU the library
 * runs on holds until the process ends.  The call allocates nothing and frees nothing.
 * Limit: rows of more than 32768 columns need K * ceil(F / 2048) <= SDP_INDEX_STATIC_MAX_COUNTS
 * (K = 8 workers: F up to 16.7 million columns), else SDP_ERR_SHAPE and nothing is enqueued; shorter rows
 * use no table and have no such limit.  Other errors as for sdp_index_masks (no WORKSPACE).
 * All calls on one GPU share that array: two calls that may run at the same time on one GPU (different
 * streams, or different host threads) race and must be ordered by the caller.  The array keeps the
 * previous call's contents; every entry a call reads it has written itself, so nothing needs clearing.
 * ------------------------------------------------------------------------------------------- */
#define SDP_INDEX_STATIC_MAX_COUNTS 65536
int sdp_index_masks_static(int K, int64_t F, const uint8_t* mask, int32_t* idx, int64_t idx_ld, int32_t* pos,
                           int32_t* count, uint8_t* cov, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Distance to uniform masking (Thm. 3.1): rho^2 = || (1/K) 1 - m / c ||_Frob^2 over the K x F mask
 * matrix, with the column's own load c_j as c (the gated average divides column j by c_j); it is 0
 * iff every worker holds every neuron and enters the step-size bound and the variance term of the
 * backward-masking rate.  A column of load c > 0 contributes 1/c - 1/K, an uncovered column 1/K, so
 * the value follows from the histogram of loads, which is counted on the device in integers (the
 * result does not depend on the order of the atomics) and finished on the host in fp64.
 *   cov  [F] u8 device in: the loads c_j written by sdp_index_masks / sdp_make_masks
 *   hist [SDP_MAX_WORKERS + 2] u64 device out: hist[c] = number of neurons of load c for c <= SDP_MAX_WORKERS;
 *        the last entry counts bytes of cov above SDP_MAX_WORKERS (always an error)
 *   rho2_host: host out
 * The call synchronises `stream`.  Multiply by the row length to get the figure over all parameters
 * of a neuron-major matrix.
 * Errors: INVALID_ARG (null, K out of range, F < 1, a load above K in cov), SHAPE (F >= 2^31), HIP.
 * ------------------------------------------------------------------------------------------- */
int sdp_mask_rho2(int K, int64_t F, const uint8_t* cov, uint64_t* hist, double* rho2_host, void* stream);

/* ---------------------------------------------------------------------------------------------
 * One worker's MLP forward under either regime of Sec. 3.1.
 *   SDP_MASK_FORWARD  (m_fwd = m): the block is evaluated at the gated parameters, i.e. as the
 *     smaller dense MLP made of the worker's p active neurons idx_k[0..p) (Sec. 3.2):
 *     G = X W1[S]^T, U = X W3[S]^T [T][p];  Y = (silu(G) * U) W2T[S]  [T][d].
 *   SDP_MASK_BACKWARD (m_fwd = all ones): the dense block over all F neurons; idx_k is ignored
 *     and p is ignored; G, U are [T][F].
 *   X [T][d] in;  W1, W3, W2T [F][d] in;  idx_k [p] i32 in (strictly ascending, in [0, F))
 *   Y [T][d] out; G_save, U_save [T][n] out with n = p (forward) or F (backward): pre-activations
 *   kept for sdp_masked_mlp_bwd.
 *   ws: sdp_masked_mlp_fwd_workspace_bytes(mode, dtype, T, d, F, p).
 * Limits: d, F, p multiples of 8 for SDP_BF16 (16-byte rows); pointers 16-byte aligned.
 * The index values are trusted (they come from sdp_index_masks); an index outside [0, F) is
 * undefined behaviour.
 * ------------------------------------------------------------------------------------------- */
size_t sdp_masked_mlp_fwd_workspace_bytes(int mode, int dtype, int T, int d, int F, int p);
int sdp_masked_mlp_fwd(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* W1,
                       const void* W3, const void* W2T, const int32_t* idx_k, void* Y, void* G_save,
                       void* U_save, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * One worker's MLP backward for upstream gradient dY = dL/dY (Sec. 3.1).
 *   SDP_MASK_FORWARD : gradients of the compact network: dX [T][d] through the p active neurons;
 *     dW1, dW3, dW2T for the active neurons only (all others are exactly zero by Sec. 3.1 and are
 *     not materialised).
 *   SDP_MASK_BACKWARD: dX through the full block (all F neurons); the weight gradient is
 *     computed ONLY on the worker's mask (m_bwd = m): rows idx_k of the dense dW1, dW3, dW2T.
 *   G_save, U_save: what sdp_masked_mlp_fwd stored for the same mode and shapes.
 *   dw_layout SDP_DW_COMPACT: dW1, dW3, dW2T are [p][d], row i belongs to neuron idx_k[i].
 *   dw_layout SDP_DW_SCATTER: they are full [F][d] buffers; row idx_k[i] is written, rows off the
 *     mask are left untouched (sdp_coverage_grad_avg never reads them).
 *   ws: sdp_masked_mlp_bwd_workspace_bytes(mode, dtype, T, d, F, p).
 * Limits as for the forward call, and additionally T a multiple of 8 for SDP_BF16.
 * ------------------------------------------------------------------------------------------- */
size_t sdp_masked_mlp_bwd_workspace_bytes(int mode, int dtype, int T, int d, int F, int p);
int sdp_masked_mlp_bwd(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* dY,
                       const void* W1, const void* W3, const void* W2T, const int32_t* idx_k,
                       const void* G_save, const void* U_save, void* dX, void* dW1, void* dW3, void* dW2T,
                       int dw_layout, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * One worker's attention block with head-level masks (Sec. 4.1: the neuron-level variant masks
 * attention heads on W_Q, W_K, W_V and W_O), under either regime of Sec. 3.1:
 *   SDP_MASK_FORWARD  (m_fwd = m_bwd = m): the block is evaluated at the gated parameters, i.e. as the
 *     smaller dense block made of the worker's ph held heads head_idx_k[0..ph) -- the projections shrink
 *     to those heads' rows and the attention core runs on those heads only (n = ph below).
 *   SDP_MASK_BACKWARD (m_fwd = all ones): the dense block over all H heads; head_idx_k and ph are
 *     ignored by the forward call (n = H below).
 * Bias-free causal self-attention over Bt sequences of S tokens (token
 * t = b S + s, T = Bt S), H heads of width hd, logits scaled by 1 / sqrt(hd), no positional rotation
 * (the paper does not state one), every weight neuron-major as in the MLP:
 *   Wqkv [3][H hd][d] in: W_Q, W_K, W_V stacked; row h hd + r of each = feature r of head h
 *   WoT  [H hd][d]    in: row j = column j of W_O
 *   Q = X Wq[S]^T, K = X Wk[S]^T, V = X Wv[S]^T;  P_h = softmax over s' <= s of Q_h K_h^T / sqrt(hd);
 *   O_h = P_h V_h;  Y = sum over the n heads of O_h WoT_h   (S = the held heads, or all of them).
 *   X [T][d] in;  head_idx_k [ph] i32 in (strictly ascending, in [0, H); trusted like idx_k above)
 *   Y [T][d] out
 *   QKV_save [T][3 n hw] out: Q | K | V of the n heads (head i of the list at columns i hw of each)
 *   O_save [T][n hw] out;  LSE_save [Bt][n][S] fp32 out: log2 of the softmax denominators, logits in
 *   base 2 -- kept for sdp_masked_attn_bwd.
 *   hw = sdp_masked_attn_saved_head_width(dtype, hd): the columns a head takes in the saved tensors.  It is hd,
 *   except for SDP_BF16 with hd < 64 (the paper's 500M / 1B models have hd = 50), where every head is padded to
 *   64 columns of which the last 64 - hd hold zeros, so that the block runs on the MFMA core.
 *   ws: sdp_masked_attn_fwd_workspace_bytes(...).
 * Limits: hd <= 128 (else UNSUPPORTED); for SDP_BF16 d a multiple of 8 (16-byte rows), and hd a multiple of 8 when
 * above 64; Bt, H <= 65535; pointers 16-byte aligned.  bf16 with hd <= 64 runs the MFMA attention core; fp32,
 * and bf16 with wider heads, run a plain fp32-arithmetic core.  Errors as for the MLP calls.
 * ------------------------------------------------------------------------------------------- */
int sdp_masked_attn_saved_head_width(int dtype, int hd);
size_t sdp_masked_attn_fwd_workspace_bytes(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph);
int sdp_masked_attn_fwd(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X,
                        const void* Wqkv, const void* WoT, const int32_t* head_idx_k, void* Y, void* QKV_save,
                        void* O_save, float* LSE_save, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Backward of the same block for upstream gradient dY.
 *   SDP_MASK_FORWARD : dX [T][d] through the held heads, and the weight gradients of the held heads
 *     (all others are exactly zero by Sec. 3.1 and are not materialised).
 *   SDP_MASK_BACKWARD: dX through the full block (all H heads); the weight gradient is computed ONLY
 *     for the worker's held heads (m_bwd = m): their rows of the dense dW_Q, dW_K, dW_V, dW_O.
 *   dw_layout SDP_DW_COMPACT: dWqkv [3][ph hd][d], dWoT [ph hd][d]; row i hd + r belongs to head
 *     head_idx_k[i].
 *   dw_layout SDP_DW_SCATTER: full [3][H hd][d] and [H hd][d] buffers; the held heads' rows are
 *     written, all other rows are left untouched.
 *   QKV_save, O_save, LSE_save: what sdp_masked_attn_fwd stored for the same mode, shapes and heads.
 *   ws: sdp_masked_attn_bwd_workspace_bytes(...).
 * ------------------------------------------------------------------------------------------- */
size_t sdp_masked_attn_bwd_workspace_bytes(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph);
int sdp_masked_attn_bwd(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X,
                        const void* dY, const void* Wqkv, const void* WoT, const int32_t* head_idx_k,
                        const void* QKV_save, const void* O_save, const float* LSE_save, void* dX, void* dWqkv,
                        void* dWoT, int dw_layout, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Block-level masking (Sec. 3.2, block-level variant: the masked block computes m B(x) + x; the
 * backward-masked variant runs the block in the forward pass and leaves it out of the backward pass).
 * One worker's pass through one residual transformer block under its mask bit m for that block.  The block
 * is attention followed by the SwiGLU MLP, each behind its own skip connection, without normalisation layers
 * (the paper's block is "Attention + MLP"; it states no more):
 *     Hm = X + Attn(X),   Y = Hm + MLP(Hm),   i.e.  B(X) = Y - X
 * with the dense forms of sdp_masked_attn_fwd (all H heads) and sdp_masked_mlp_fwd (all F neurons); the skip
 * connections are added in the epilogues of the contractions that produce the sums.
 *   mode SDP_MASK_FORWARD  (m_fwd = m_bwd = m):  m = 1 the dense block;  m = 0 the block is skipped, Y = X
 *     (only X and Y are looked at; every other pointer may be null), and in the backward call dX = dY and no
 *     weight gradient is written: the block's parameters get none (Sec. 3.1).
 *   mode SDP_MASK_BACKWARD (m_fwd = all ones, m_bwd = m):  the forward call runs the dense block whatever m is.
 *     Backward with m = 1: the dense backward pass.  Backward with m = 0: no weight gradient of the block is
 *     computed or written; dX follows dx_rule:
 *       SDP_BLOCK_DX_THROUGH  dX = dY carried through the block and its skip connections: the gradient at the full
 *                             parameters, which is what Sec. 3.1's backward masking aggregates for the blocks below
 *       SDP_BLOCK_DX_SKIP     dX = dY: the whole backward pass of the block is omitted, the gradient takes the
 *                             skip connection alone (the cost model of the 1.5 x iteration multiplier in Sec. 4)
 *   X, dY [T][d] in, T = Bt S;  Wqkv [3][H hd][d], WoT [H hd][d], W1, W3, W2T [F][d] in
 *   Y [T][d] out;  saved for the backward call: Hm_save [T][d], QKV_save [T][3 H hw], O_save [T][H hw] (hw =
 *   sdp_masked_attn_saved_head_width(dtype, hd)),
 *   LSE_save [Bt][H][S] fp32, G_save, U_save [T][F]
 *   dX [T][d] out;  dWqkv [3][H hd][d], dWoT [H hd][d], dW1, dW3, dW2T [F][d] out (m = 1 only; may be null otherwise)
 *   ws: sdp_block_fwd_workspace_bytes / sdp_block_bwd_workspace_bytes.
 * Limits as for the attention and MLP calls (bf16: d and F multiples of 8, hd any value up to 64 (narrower heads are
 * padded to 64 inside, as in the attention calls) or a multiple of 8 up to 128, T a multiple of 8 in the backward call).  Y, Hm_save and X must be three different buffers, dX and dY two.
 * Errors: INVALID_ARG (null, misaligned, aliasing, m not 0 / 1, unknown mode / dx_rule), SHAPE, WORKSPACE, UNSUPPORTED, HIP.
 * ------------------------------------------------------------------------------------------- */
typedef enum { SDP_BLOCK_DX_THROUGH = 0, SDP_BLOCK_DX_SKIP = 1 } sdp_block_dx_rule;
size_t sdp_block_fwd_workspace_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F);
size_t sdp_block_bwd_workspace_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F);
int sdp_block_fwd(int mode, int m, int dtype, int Bt, int S, int d, int H, int hd, int F, const void* X,
                  const void* Wqkv, const void* WoT, const void* W1, const void* W3, const void* W2T, void* Y,
                  void* Hm_save, void* QKV_save, void* O_save, float* LSE_save, void* G_save, void* U_save, void* ws,
                  size_t ws_bytes, void* stream);
int sdp_block_bwd(int mode, int m, int dx_rule, int dtype, int Bt, int S, int d, int H, int hd, int F, const void* X,
                  const void* dY, const void* Wqkv, const void* WoT, const void* W1, const void* W3, const void* W2T,
                  const void* Hm_save, const void* QKV_save, const void* O_save, const float* LSE_save,
                  const void* G_save, const void* U_save, void* dX, void* dWqkv, void* dWoT, void* dW1, void* dW3,
                  void* dW2T, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Gated average of K workers' gradients (Sec. 3.1, eq. "average"), normalised per coordinate by
 * the number of workers that cover it:
 *     out[r][e] = (1 / c_r) * sum_{k : mask[k][r] != 0} g_k[r][e],   c_r = sum_k mask[k][r],
 * the mask being constant along a neuron row of D parameters.  The mask SELECTS: rows a worker
 * does not cover are never read (they may hold anything).  c_r = 0 gives out = 0.  The sum is
 * taken in fp32 in worker order k = 0..K-1, then divided once; the result does not depend on
 * launch geometry.
 *   g     HOST array of K DEVICE pointers, each [R][D] of gdtype (SDP_F32 or SDP_BF16)
 *   mask  [K][R] u8 in;   out [R][D] fp32 out;   cov [R] u8 out (may be NULL)
 * Limits: 1 <= K <= SDP_MAX_WORKERS, R >= 0, D >= 1; buffers 16-byte aligned.
 * ------------------------------------------------------------------------------------------- */
int sdp_coverage_grad_avg(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                          float* out, uint8_t* cov, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The same pass with the optimizer fused in (the paper trains with AdamW, App. "Hyperparameters for
 * LLM Architecture": beta1 = 0.9, beta2 = 0.95, weight decay 0.1; Sec. 3.2: parameters, gradients and
 * optimizer state exist only for covered coordinates): for every row r with c_r >= 1 and every
 * parameter e of it, with ghat = grad_scale * (1 / c_r) * sum_{k covers r} g_k[r][e],
 *     theta <- theta (1 - lr wd);  m <- beta1 m + (1 - beta1) ghat;  v <- beta2 v + (1 - beta2) ghat^2;
 *     theta <- theta - lr / (1 - beta1^t) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps)
 * (decoupled weight decay, bias-corrected moments, t = step >= 1), all in fp32.  Rows with c_r = 0 are
 * left untouched: no gradient reached them, and neither decay nor moment update is applied.
 * grad_scale (host value) times *grad_scale_dev (device value, if given) scales the gradient: a loss scale
 * and / or the clipping coefficient (1 = none).  The averaged gradient itself is not stored.
 *   g, mask, cov   as for sdp_coverage_grad_avg
 *   theta, m, v    [R][D] fp32, updated in place (each row read and written once)
 *   theta_bf16     [R][D] bf16 out, may be NULL: the updated parameters rounded to nearest even, i.e.
 *                  the weights of the next step's bf16 contractions (covered rows only)
 * Errors: INVALID_ARG (null, misaligned, K or D out of range, lr < 0, beta outside [0, 1), eps <= 0,
 * weight_decay < 0, step < 1, non-finite grad_scale), SHAPE (R D > 2^40).
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay, grad_scale;
    int step; /* t, counted from 1 */
    const float* grad_scale_dev; /* device, may be NULL: a second factor of the gradient's scale, read by the
                                    kernel (e.g. the coefficient sdp_clip_scale wrote), so that clipping needs
                                    no round trip to the host; 4-byte aligned */
} sdp_adamw_params;
int sdp_coverage_avg_adamw(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                           float* theta, float* m, float* v, void* theta_bf16, uint8_t* cov,
                           const sdp_adamw_params* hp, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Squared l2 norm of the coverage-normalised average, sum over all rows and parameters of
 * ((1 / c_r) sum_{k covers r} g_k[r][e])^2, without storing the average: the quantity that global
 * gradient clipping (App. "Hyperparameters for LLM Architecture": clipping at 1.0) measures before the
 * update; min(1, clip / sqrt(norm^2)) is the grad_scale of sdp_coverage_avg_adamw.  Same streaming
 * pass as the average (only covered rows are read); each element is averaged in fp32 exactly as
 * sdp_coverage_grad_avg would store it, squares are summed in fp64 in a fixed order (no atomics: the
 * result is a pure function of the inputs).  Rows nobody covers contribute 0.
 *   g, mask   as for sdp_coverage_grad_avg
 *   sqnorm    device, one fp64 value out (8-byte aligned)
 *   ws        sdp_coverage_grad_sqnorm_workspace_bytes(R, D) bytes, 16-byte aligned
 * R = 0 writes 0.  Errors: INVALID_ARG, SHAPE (R D > 2^40), WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t sdp_coverage_grad_sqnorm_workspace_bytes(int64_t R, int D);
int sdp_coverage_grad_sqnorm(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                             double* sqnorm, void* ws, size_t ws_bytes, void* stream);

/* Clipping coefficient of global-norm clipping from the squared norms of n parameter groups (each from
 * sdp_coverage_grad_sqnorm): *scale = min(1, max_norm / (sqrt(sum_i sqnorm[i]) + 1e-6)), the usual form
 * (the paper states only the threshold, 1.0).  sqnorm: device [n] fp64; scale: device fp32 out, to be passed
 * as grad_scale_dev.  Errors: INVALID_ARG (null, misaligned, n < 1, max_norm not positive and finite). */
int sdp_clip_scale(int n, const double* sqnorm, float max_norm, float* scale, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SDP_H */
