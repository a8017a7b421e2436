// One worker's masked SwiGLU MLP forward and backward (the paper's Sec. 3.1 regimes applied to the
// neuron-level masks of Sec. 3.2), expressed as a fixed sequence of contractions C = A . B^T whose
// operands are all read depth-contiguous.
//
// With n = p and S = idx_k under forward masking, n = F and S = all neurons under backward masking:
//   forward   wt      : W2c = W2T[S]^T                       ([d][n], gather + transpose, HBM-bound)
//             gate_up : [G | U] = X . [W1 | W3][S]^T         (T x n, depth d; rows of W1, W3 gathered in
//                        the operand load)  + SwiGLU epilogue -> Act
//             down    : Y  = Act . W2c^T                     (T x d, depth n)
//   backward  wt      : W1c = W1[S]^T, W3c = W3[S]^T ([d][n]);  XT = X^T, dYT = dY^T ([d][T])
//             dact    : dA = dY . W2T[S]^T                   (T x n, depth d; rows of W2T gathered)
//                        + SwiGLU-backward epilogue -> dG, dU [T][n] and, transposed, dG^T, dU^T,
//                        Act^T [p][T] (neuron-major; under backward masking only the worker's p
//                        columns are kept, row = rank of the neuron in idx_k)
//             dw      : dW1[S] = dG^T . X, dW3[S] = dU^T . X, dW2T[S] = Act^T . dY   (p x d, depth T),
//                        one batched launch over the neuron-major copies and XT, dYT
//             dx      : dX = dG . W1c^T + dU . W3c^T         (T x d, depth 2n)
// Under backward masking the weight-gradient contraction reads only the p kept rows: the gradient is
// computed on the worker's mask and nowhere else.  fp32 tensors and bf16 shapes the MFMA kernel does
// not take go through the plain kernel, which reads dG, dU, Act depth-major as they are (and, under
// backward masking, their column-compacted copies [T][p]).
#include "sdp_internal.h"

namespace {

using namespace sdp;

size_t esize(int dtype) { return dtype == SDP_F32 ? 4 : 2; }

// Leading dimension of the token-contiguous copies X^T, dY^T [d][T]: T plus 64 elements, so that
// consecutive rows do not sit a power of two apart (rows 2^k bytes apart fall onto the same memory
// channels, and a depth step touches one 128-byte piece of each of 192-256 rows).
int64_t ld_tokens(int T) { return (int64_t)T + 64; }

int check_common(int mode, int dtype, int T, int d, int F, int p) {
    if (mode != SDP_MASK_FORWARD && mode != SDP_MASK_BACKWARD) return SDP_ERR_INVALID_ARG;
    if (dtype != SDP_F32 && dtype != SDP_BF16) return SDP_ERR_INVALID_ARG;
    if (T < 1 || d < 1 || F < 1) return SDP_ERR_INVALID_ARG;
    if (p < 1 || p > F) return SDP_ERR_SHAPE;
    if ((int64_t)T * F >= ((int64_t)1 << 40)) return SDP_ERR_SHAPE;
    if (dtype == SDP_BF16 && (d % 8 || F % 8 || p % 8)) return SDP_ERR_SHAPE;
    return SDP_OK;
}

// one thread per column n: lower bound of n in the ascending list
__global__ __launch_bounds__(256) void column_ranks_kernel(const int32_t* __restrict__ cidx, int pc, int N,
                                                           int32_t* __restrict__ crank) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    int lo = 0, hi = pc;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (cidx[mid] < n) lo = mid + 1; else hi = mid;
    }
    crank[n] = lo < pc && cidx[lo] == n ? lo : -1 - lo;
}

int run(int dtype, const GemmDesc& g, hipStream_t s) {
    if (dtype == SDP_BF16 && gemm_mfma_supported(g)) return gemm_mfma_bf16(g, s);
    return gemm_simple(dtype, g, s);
}

} // namespace

int sdp::column_ranks(const int32_t* cidx, int pc, int N, int32_t* crank, hipStream_t s) {
    if (!cidx || !crank || pc < 0 || N < 1) return SDP_ERR_INVALID_ARG;
    ProfileScope ps("mlp_column_ranks", s);
    column_ranks_kernel<<<(unsigned)((N + 255) / 256), 256, 0, s>>>(cidx, pc, N, crank);
    return launch_status();
}

extern "C" size_t sdp_masked_mlp_fwd_workspace_bytes(int mode, int dtype, int T, int d, int F, int p) {
    if (check_common(mode, dtype, T, d, F, mode == SDP_MASK_BACKWARD ? F : p) != SDP_OK) return 0;
    const size_t n = mode == SDP_MASK_FORWARD ? p : F;
    return round_up((size_t)T * n * esize(dtype), 256) + round_up((size_t)d * n * esize(dtype), 256);
}

extern "C" size_t sdp_masked_mlp_bwd_workspace_bytes(int mode, int dtype, int T, int d, int F, int p) {
    if (check_common(mode, dtype, T, d, F, p) != SDP_OK) return 0;
    const size_t n = mode == SDP_MASK_FORWARD ? p : F;
    const size_t e = esize(dtype);
    size_t bytes = 3 * round_up((size_t)T * n * e, 256) + 2 * round_up((size_t)d * n * e, 256) +
                   2 * round_up((size_t)d * ld_tokens(T) * e, 256);
    if (mode == SDP_MASK_BACKWARD) bytes += 3 * round_up((size_t)T * p * e, 256);
    bytes += 3 * round_up((size_t)p * ld_tokens(T) * e, 256); // neuron-major copies of dG, dU, Act on the mask
    if (mode == SDP_MASK_BACKWARD) bytes += round_up((size_t)F * sizeof(int32_t), 256); // rank of every neuron in the list
    if (dtype == SDP_BF16) bytes += round_up(gemm_tail_ws_bytes(p, d, T, 3), 256); // depth ranges of the weight gradients' last round
    return bytes;
}

extern "C" int sdp_masked_mlp_fwd(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* W1,
                                  const void* W3, const void* W2T, const int32_t* idx_k, void* Y, void* G_save,
                                  void* U_save, void* ws, size_t ws_bytes, void* stream) {
    if (mode == SDP_MASK_BACKWARD) p = F;
    int rc = check_common(mode, dtype, T, d, F, p);
    if (rc != SDP_OK) return rc;
    if (!X || !W1 || !W3 || !W2T || !Y || !G_save || !U_save) return SDP_ERR_INVALID_ARG;
    if (mode == SDP_MASK_FORWARD && !idx_k) return SDP_ERR_INVALID_ARG;
    for (const void* q : {X, W1, W3, W2T, (const void*)Y, (const void*)G_save, (const void*)U_save})
        if (!aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < sdp_masked_mlp_fwd_workspace_bytes(mode, dtype, T, d, F, p))
        return SDP_ERR_WORKSPACE;
    return mlp_fwd_impl(mode, dtype, T, d, F, p, X, W1, W3, W2T, idx_k, Y, G_save, U_save, nullptr, ws,
                        (hipStream_t)stream);
}

int sdp::mlp_fwd_impl(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* W1, const void* W3,
                      const void* W2T, const int32_t* idx_k, void* Y, void* G_save, void* U_save, const void* residual,
                      void* ws, hipStream_t s) {
    if (mode == SDP_MASK_BACKWARD) p = F;
    int rc;
    const int n = mode == SDP_MASK_FORWARD ? p : F;
    const int32_t* gather = mode == SDP_MASK_FORWARD ? idx_k : nullptr;
    const size_t e = esize(dtype);
    char* w = (char*)ws;
    void* Act = w;
    void* W2c = w + round_up((size_t)T * n * e, 256);

    rc = transpose_rows((int)e, W2T, d, gather, n, d, W2c, n, "mlp_wt_fwd", s);
    if (rc != SDP_OK) return rc;

    GemmDesc gu;
    gu.name = "mlp_gate_up";
    gu.M = T, gu.N = n, gu.K = d;
    gu.A = X, gu.lda = d;
    gu.B = W1, gu.B2 = W3, gu.ldb = d, gu.b_gather = gather, gu.b_rows = F;
    gu.epilogue = EPI_SWIGLU_FWD;
    gu.C = G_save, gu.C2 = U_save, gu.C3 = Act, gu.ldc = n;
    rc = run(dtype, gu, s);
    if (rc != SDP_OK) return rc;

    GemmDesc dn;
    dn.name = "mlp_down";
    dn.M = T, dn.N = d, dn.K = n;
    dn.A = Act, dn.lda = n;
    dn.B = W2c, dn.ldb = n;
    dn.epilogue = EPI_STORE;
    dn.C = Y, dn.ldc = d;
    dn.R = residual, dn.ldr = d;
    return run(dtype, dn, s);
}

extern "C" int sdp_masked_mlp_bwd(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* dY,
                                  const void* W1, const void* W3, const void* W2T, const int32_t* idx_k,
                                  const void* G_save, const void* U_save, void* dX, void* dW1, void* dW3, void* dW2T,
                                  int dw_layout, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_common(mode, dtype, T, d, F, p);
    if (rc != SDP_OK) return rc;
    if (dtype == SDP_BF16 && T % 8) return SDP_ERR_SHAPE;
    if (dw_layout != SDP_DW_COMPACT && dw_layout != SDP_DW_SCATTER) return SDP_ERR_INVALID_ARG;
    if (!X || !dY || !W1 || !W3 || !W2T || !idx_k || !G_save || !U_save || !dX || !dW1 || !dW3 || !dW2T)
        return SDP_ERR_INVALID_ARG;
    for (const void* q : {X, dY, W1, W3, W2T, G_save, U_save, (const void*)dX, (const void*)dW1, (const void*)dW3,
                          (const void*)dW2T})
        if (!aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < sdp_masked_mlp_bwd_workspace_bytes(mode, dtype, T, d, F, p))
        return SDP_ERR_WORKSPACE;
    return mlp_bwd_impl(mode, dtype, T, d, F, p, X, dY, W1, W3, W2T, idx_k, G_save, U_save, dX, dW1, dW3, dW2T, dw_layout,
                        nullptr, true, ws, (hipStream_t)stream);
}

int sdp::mlp_bwd_impl(int mode, int dtype, int T, int d, int F, int p, const void* X, const void* dY, const void* W1,
                      const void* W3, const void* W2T, const int32_t* idx_k, const void* G_save, const void* U_save,
                      void* dX, void* dW1, void* dW3, void* dW2T, int dw_layout, const void* dx_residual, bool want_dw,
                      void* ws, hipStream_t s) {
    int rc;
    const int n = mode == SDP_MASK_FORWARD ? p : F;
    const int32_t* gather = mode == SDP_MASK_FORWARD ? idx_k : nullptr;
    const size_t e = esize(dtype);
    const size_t act_b = round_up((size_t)T * n * e, 256), wt_b = round_up((size_t)d * n * e, 256);
    const size_t xt_b = round_up((size_t)d * ld_tokens(T) * e, 256), cmp_b = round_up((size_t)T * p * e, 256);
    char* w = (char*)ws;
    void *dG = w, *dU = w + act_b, *Act = w + 2 * act_b;
    w += 3 * act_b;
    void *W1c = w, *W3c = w + wt_b;
    w += 2 * wt_b;
    void *XT = w, *dYT = w + xt_b;
    w += 2 * xt_b;
    void *dGc = dG, *dUc = dU, *Actc = Act; // forward masking: the tensors are compact already
    if (mode == SDP_MASK_BACKWARD) {
        dGc = w, dUc = w + cmp_b, Actc = w + 2 * cmp_b;
        w += 3 * cmp_b;
    }
    const size_t nm_b = round_up((size_t)p * ld_tokens(T) * e, 256);
    void *dGn = w, *dUn = w + nm_b, *Actn = w + 2 * nm_b; // [p][T(+pad)]: neuron-major
    w += 3 * nm_b;
    int32_t* ranks = (int32_t*)w; // backward masking: [F]
    if (mode == SDP_MASK_BACKWARD) w += round_up((size_t)F * sizeof(int32_t), 256);
    void* tail_ws = dtype == SDP_BF16 && gemm_tail_ws_bytes(p, d, T, 3) > 0 ? w : nullptr;

    // the four operand copies of the backward pass as one launch (X^T, dY^T only feed the weight gradients)
    const TransposeJob tj[4] = {{W1, W1c, d, n, gather, n, d},
                                {W3, W3c, d, n, gather, n, d},
                                {X, XT, d, ld_tokens(T), nullptr, T, d},
                                {dY, dYT, d, ld_tokens(T), nullptr, T, d}};
    rc = transpose_batch((int)e, tj, want_dw ? 4 : 2, "mlp_tr_bwd", s);
    if (rc != SDP_OK) return rc;

    // weight-gradient contraction (set up first: whether it can take the MFMA path decides what the
    // activation-gradient kernel writes)
    const void* rhs[3] = {XT, XT, dYT};
    void* outp[3] = {dW1, dW3, dW2T};
    void* nmaj[3] = {dGn, dUn, Actn};
    GemmDesc dw;
    dw.name = "mlp_dw";
    dw.M = p, dw.N = d, dw.K = T;
    dw.ldb = ld_tokens(T);
    dw.epilogue = EPI_STORE;
    dw.ldc = d;
    dw.c_scatter = dw_layout == SDP_DW_SCATTER ? idx_k : nullptr;
    dw.nbatch = 3;
    dw.lda = ld_tokens(T), dw.a_km = 0;
    dw.tail_ws = tail_ws, dw.tail_name = "mlp_dw_reduce";
    for (int i = 0; i < 3; ++i) dw.Ab[i] = nmaj[i], dw.Bb[i] = rhs[i], dw.Cb[i] = outp[i];

    GemmDesc da;
    da.name = "mlp_dact";
    da.M = T, da.N = n, da.K = d;
    da.A = dY, da.lda = d;
    da.B = W2T, da.ldb = d, da.b_gather = gather, da.b_rows = F;
    da.epilogue = EPI_SWIGLU_BWD;
    da.Gin = G_save, da.Uin = U_save, da.ldg = n;
    da.C = dG, da.C2 = dU, da.ldc = n;
    // bf16, aligned shapes: the epilogue also writes dG, dU and act transposed (neuron-major [p][T],
    // under backward masking only the worker's p columns), which is the layout in which the batched
    // weight-gradient contraction reads both operands depth-contiguous; act is not stored row-major.
    da.Ct = dGn, da.Ct2 = dUn, da.Ct3 = Actn, da.ldct = ld_tokens(T);
    if (mode == SDP_MASK_BACKWARD) da.cidx = idx_k, da.pc = p, da.crank = ranks;
    const bool fused = want_dw && dtype == SDP_BF16 && p % 8 == 0 && T % 8 == 0 && gemm_mfma_supported(dw) && gemm_mfma_supported(da);
    if (!fused) {
        da.Ct = da.Ct2 = da.Ct3 = nullptr, da.cidx = nullptr, da.pc = 0, da.crank = nullptr;
        // without weight gradients nothing reads act: the MFMA kernel then skips its store, the plain one writes it anyway
        if (want_dw || dtype != SDP_BF16 || !gemm_mfma_supported(da)) da.C3 = Act;
        if (mode == SDP_MASK_BACKWARD && want_dw) {
            da.Cc = dGc, da.Cc2 = dUc, da.Cc3 = Actc, da.ldcc = p;
            da.cidx = idx_k, da.pc = p;
        }
    }
    if (fused && mode == SDP_MASK_BACKWARD) {
        rc = column_ranks(idx_k, p, F, ranks, s);
        if (rc != SDP_OK) return rc;
    }
    rc = run(dtype, da, s);
    if (rc != SDP_OK) return rc;

    if (fused) {
        rc = gemm_mfma_bf16(dw, s);
        if (rc != SDP_OK) return rc;
    }
    GemmDesc dx;
    dx.name = "mlp_dx";
    dx.M = T, dx.N = d, dx.K = n;
    dx.A = dG, dx.A2 = dU, dx.lda = n;
    dx.B = W1c, dx.B2 = W3c, dx.ldb = n;
    dx.epilogue = EPI_DUAL_ACC;
    dx.C = dX, dx.ldc = d;
    dx.R = dx_residual, dx.ldr = d;
    rc = run(dtype, dx, s);
    if (rc != SDP_OK) return rc;

    if (fused || !want_dw) return SDP_OK;
    // plain path: read the left operands depth-major ([T][p]) as they are
    const void* lhs[3] = {dGc, dUc, Actc};
    dw.nbatch = 0;
    dw.lda = p, dw.a_km = 1;
    for (int i = 0; i < 3; ++i) {
        dw.A = lhs[i], dw.B = rhs[i], dw.C = outp[i];
        rc = gemm_simple(dtype, dw, s);
        if (rc != SDP_OK) return rc;
    }
    return SDP_OK;
}
