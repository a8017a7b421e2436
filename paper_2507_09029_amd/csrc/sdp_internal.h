// Internal declarations shared by the translation units of libsdp_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sdp.h"
#include "sdp_measure.h"

namespace sdp {

// ---- per-kernel event timing (sdp_profile_*) -------------------------------------------------
bool profiling_on();
bool profiling_wants(const char* name); // on, and `name` passes the filter
void profile_begin(const char* name, hipStream_t s);
// start / stop events for a launch that records them itself (hipExtLaunchKernel); false = not timed
bool profile_launch_events(const char* name, hipEvent_t* start, hipEvent_t* stop);
void profile_end(hipStream_t s);

struct ProfileScope {
    hipStream_t s;
    bool on;
    ProfileScope(const char* name, hipStream_t stream) : s(stream), on(name && profiling_on() && profiling_wants(name)) {
        if (on) profile_begin(name, s);
    }
    ~ProfileScope() {
        if (on) profile_end(s);
    }
};

inline int hip_status(hipError_t e) { return e == hipSuccess ? SDP_OK : SDP_ERR_HIP; }
inline int launch_status() { return hip_status(hipGetLastError()); }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- contraction descriptor --------------------------------------------------------------------
// C[M][N] = sum_k A(m,k) * B(k,n), fp32 accumulation, all matrices row-major.
//   A(m,k) = a_km ? A[k * lda + m] : A[ra(m) * lda + k]  (a_km: A is stored depth-major, [K][M])
//   B(k,n) = B[rb(n) * ldb + k]                           (B is stored [N][K], rows contiguous along k)
// rb is the identity when b_gather is null, else a lookup in an int32 table (active-neuron rows); ra likewise
// with a_gather (not together with a_km).
// A second operand pair (A2, B2) with the same shapes and strides is used by two of the epilogues.
enum Epilogue {
    EPI_STORE = 0,       // C[rc(m) * ldc + n] = acc      (rc: optional row scatter; rc(m) < 0 drops row m)
    EPI_DUAL_ACC = 1,    // as STORE with acc = A.B + A2.B2
    EPI_SWIGLU_FWD = 2,  // g = A.B, u = A.B2: G = g, U = u, Act = silu(g) * u, all [M][N] (ld = ldc)
    EPI_SWIGLU_BWD = 3   // da = A.B; with g = Gin[m][n], u = Uin[m][n]  (ld = ldg):
                         //   dU = da silu(g), dG = da u silu'(g), act = silu(g) u, all [M][N] (ld = ldc);
                         //   plain kernel: with cidx != null also the column-compacted copies [M][pc]
                         //   (ld = ldcc): column c of Cc / Cc2 / Cc3 is column cidx[c] of dG / dU / act
};

constexpr int kMaxBatch = 4;

struct GemmDesc {
    int M = 0, N = 0, K = 0;
    const void* A = nullptr;
    const void* A2 = nullptr;
    int64_t lda = 0;
    int a_km = 0;
    const int32_t* a_gather = nullptr;
    int64_t a_rows = 0; // number of rows of the stored A (bounds the gathered row index); 0 = M
    const void* B = nullptr;
    const void* B2 = nullptr;
    int64_t ldb = 0;
    const int32_t* b_gather = nullptr;
    int64_t b_rows = 0; // number of rows of the stored B (bounds the gathered row index); 0 = N
    int epilogue = EPI_STORE;
    // outputs
    void* C = nullptr;  // STORE / DUAL_ACC: C.  SWIGLU_FWD: G.  SWIGLU_BWD: dG
    void* C2 = nullptr; // SWIGLU_FWD: U.  SWIGLU_BWD: dU
    void* C3 = nullptr; // SWIGLU_FWD / SWIGLU_BWD: Act
    int64_t ldc = 0;
    const int32_t* c_scatter = nullptr;
    // STORE / DUAL_ACC of a single problem: optional residual, C = acc + R[m][n] (added in fp32 before the
    // result is rounded; R is indexed like C without the row scatter; R may be C itself: an element is read
    // before it is written, by the same lane)
    const void* R = nullptr;
    int64_t ldr = 0;
    // SWIGLU_BWD inputs and optional compact copies
    const void* Gin = nullptr;
    const void* Uin = nullptr;
    int64_t ldg = 0;
    void* Cc = nullptr;
    void* Cc2 = nullptr;
    void* Cc3 = nullptr;
    int64_t ldcc = 0;
    const int32_t* cidx = nullptr;
    int pc = 0;
    // with cidx and Ct (MFMA kernel): crank[n], n < N: the number of listed columns below n if n is listed, else
    // -1 - that number (see column_ranks); spares the kernel a search of cidx per wave
    const int32_t* crank = nullptr;
    // SWIGLU_BWD, MFMA kernel only: neuron-major copies Ct / Ct2 / Ct3 of dG / dU / act, [rows][ldct] with
    // Ct[r(n)][m] = dG[m][n]; r(n) = n, or with cidx the rank of n in cidx (columns not listed are dropped).
    // With Ct set, C3 may be null (act is then not stored row-major).
    void* Ct = nullptr;
    void* Ct2 = nullptr;
    void* Ct3 = nullptr;
    int64_t ldct = 0;
    const char* name = "gemm";
    // batched launch of up to kMaxBatch problems with the same shape, strides and scatter (the
    // weight-gradient contractions): nbatch > 0 selects Ab/Bb/Cb instead of A/B/C
    int nbatch = 0;
    const void* Ab[4] = {nullptr, nullptr, nullptr, nullptr};
    const void* Bb[4] = {nullptr, nullptr, nullptr, nullptr};
    void* Cb[4] = {nullptr, nullptr, nullptr, nullptr};
    int force_tile = 0; // 0 = choose; 256 / 192 / 128 force a tile shape (tuning and tests)
    // batched launches only: optional fp32 scratch of gemm_split_ws_bytes(M, N, K, nbatch) bytes.  With it, a
    // launch that has few tiles and a deep K cuts the depth into ranges that run as extra problems, and a second
    // kernel sums the ranges' partial results (gemm_choose_ksplit decides; 1 = no cut).
    void* split_ws = nullptr;
    int ksplit = 1; // set by gemm_mfma_bf16
    // batched launches only: optional fp32 scratch of gemm_tail_ws_bytes(M, N, K, nbatch) bytes.  With it, a launch
    // whose tiles fill the CUs more than once but leave the last round partly empty cuts the depth of that last
    // round's tiles into ranges (gemm_choose_tail), which a second small kernel adds up.
    void* tail_ws = nullptr;
    const char* tail_name = "dw_tail_reduce"; // profile name of that second kernel
};

// tags that give each call site of the MFMA contraction its own kernel symbol
enum GemmOp { OP_GATE_UP = 0, OP_DOWN = 1, OP_DACT = 2, OP_DX = 3, OP_DW = 4, OP_DW_SPLIT = 5, OP_DW_TAIL = 6 };

// Plain LDS-tiled FMA contraction, any shape; element type float or bf16 (dtype as sdp_dtype).
int gemm_simple(int dtype, const GemmDesc& g, hipStream_t s);
// bf16 MFMA contraction; returns SDP_ERR_UNSUPPORTED when the shape / alignment does not fit.
int gemm_mfma_bf16(const GemmDesc& g, hipStream_t s);
bool gemm_mfma_supported(const GemmDesc& g);
// depth ranges a batched launch of nbatch problems of shape M x N x K would be cut into, and the scratch that takes
int gemm_choose_ksplit(int M, int N, int K, int nbatch);
size_t gemm_split_ws_bytes(int M, int N, int K, int nbatch);
// scratch of the tail cut of a batched launch (0 when none is taken)
size_t gemm_tail_ws_bytes(int M, int N, int K, int nbatch);

// ---- attention core -----------------------------------------------------------------------------
// Causal attention of n heads of width hd over Bt sequences of S tokens, on the saved projections:
// qkv [Bt S][ldq] = Q | K | V (head i at columns i hd of each part), o / dO [Bt S][ldo], lse / delta [Bt][n][S].
struct AttnCoreDesc {
    const void* qkv = nullptr;
    int64_t ldq = 0;
    const void* o = nullptr; // backward: the forward's output
    void* o_out = nullptr;   // forward
    const void* dO = nullptr;
    int64_t ldo = 0;
    float* lse = nullptr;
    float* delta = nullptr;
    void* dqkv = nullptr;
    int Bt = 0, S = 0, n = 0, hd = 0;
};
// plain core: fp32 or bf16 storage, fp32 arithmetic, hd <= 128 (SDP_ERR_UNSUPPORTED beyond)
bool attn_plain_supported(const AttnCoreDesc& c);
int attn_plain_fwd(int dtype, const AttnCoreDesc& c, hipStream_t s);
int attn_plain_bwd(int dtype, const AttnCoreDesc& c, hipStream_t s);

// ---- one worker's MLP / attention passes with the options the block-level calls need ----------------
// As sdp_masked_mlp_fwd / _bwd and sdp_masked_attn_fwd / _bwd after argument checks, plus:
//   residual     [T][d] or null: added to the output Y (forward) in the contraction's epilogue
//   dx_residual  [T][d] or null: added to dX likewise (the gradient that arrives over the skip connection)
//   want_dw      false: the weight gradients and everything only they need (transposed copies) are left out
//   idx_k / head_idx_k null (forward masking with p = F; backward masking of heads): every neuron / head, in order
int mlp_fwd_impl(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* W1, const void* W3,
                 const void* W2T, const int32_t* idx_k, void* Y, void* G_save, void* U_save, const void* residual,
                 void* ws, hipStream_t s);
int mlp_bwd_impl(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* dY, const void* W1,
                 const void* W3, const void* W2T, const int32_t* idx_k, const void* G_save, const void* U_save, void* dX,
                 void* dW1, void* dW3, void* dW2T, int dw_layout, const void* dx_residual, bool want_dw, void* ws,
                 hipStream_t s);
int attn_fwd_impl(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X, const void* Wqkv,
                  const void* WoT, const int32_t* head_idx_k, void* Y, void* QKV_save, void* O_save, float* LSE_save,
                  const void* residual, void* ws, hipStream_t s);
int attn_bwd_impl(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X, const void* dY,
                  const void* Wqkv, const void* WoT, const int32_t* head_idx_k, const void* QKV_save, const void* O_save,
                  const float* LSE_save, void* dX, void* dWqkv, void* dWoT, int dw_layout, const void* dx_residual,
                  bool want_dw, void* ws, hipStream_t s);

// out[c][r] = in[rows ? rows[r] : r][c] for r < R, c < C: (gathered) transpose, element size 2 or 4.
int transpose_rows(int elem_bytes, const void* in, int64_t ld_in, const int32_t* rows, int R, int C, void* out,
                   int64_t ld_out, const char* name, hipStream_t s);

// Several such transposes as one launch (16-bit elements with 8-element aligned shapes; otherwise one launch each).
constexpr int kMaxTransposeJobs = 4;
struct TransposeJob {
    const void* in;
    void* out;
    int64_t ld_in, ld_out;
    const int32_t* rows; // optional gather of input rows
    int R, C;
};
int transpose_batch(int elem_bytes, const TransposeJob* jobs, int n, const char* name, hipStream_t s);

// crank[n] for n < N from the ascending list cidx[0 .. pc): the number of listed columns below n if n is listed,
// else -1 - that number
int column_ranks(const int32_t* cidx, int pc, int N, int32_t* crank, hipStream_t s);

} // namespace sdp
