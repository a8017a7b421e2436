// Block-level masking (the paper's Sec. 3.2, block-level variant): one worker's pass through one residual
// transformer block under a block mask bit m,
//     masked block:  m B(x) + x,      B(x) = Attn(x) + MLP(x + Attn(x))
// (attention and MLP each behind its own skip connection, no normalisation layers), composed from the dense
// forms of the attention and MLP passes of this library.  The skip connections are not passes of their own:
// the residual is added in the epilogue of the contraction that produces the sum (the attention output
// projection, the MLP down projection, and in the backward pass the two dX contractions).
//
//   forward masking (m_fwd = m_bwd = m):   m = 1 the dense block;  m = 0 the block is skipped: Y = X, dX = dY, the
//     block's parameters get no gradient (one 16-byte-wide copy each way; nothing else runs)
//   backward masking (m_fwd = 1, m_bwd = m):   the forward pass always runs the block;  m = 1 the dense backward
//     pass;  m = 0 the block's weight gradients are not computed, and dX is either carried through the block
//     (dX_RULE_THROUGH: dact, dX contractions and the attention core's backward run, no weight-gradient launch,
//     none of the transposed copies that only feed it) or through the skip connection alone (dX_RULE_SKIP)
#include "sdp_internal.h"

namespace {

using namespace sdp;

size_t esize(int dtype) { return dtype == SDP_F32 ? 4 : 2; }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// dst = src, n16 pieces of 16 bytes (both 16-byte aligned), then `tail` single bytes
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16,
                                                   int tail) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
    if (blockIdx.x == 0 && (int)threadIdx.x < tail)
        ((unsigned char*)(dst + n16))[threadIdx.x] = ((const unsigned char*)(src + n16))[threadIdx.x];
}

int copy_tokens(const void* src, void* dst, size_t bytes, const char* name, hipStream_t s) {
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t blocks = (n16 + 255) / 256;
    ProfileScope ps(name, s);
    copy_kernel<<<(unsigned)(blocks < 1 ? 1 : (blocks < 4096 ? blocks : 4096)), 256, 0, s>>>((const u32x4*)src, (u32x4*)dst, n16,
                                                                                             (int)(bytes % 16));
    return launch_status();
}

int check_block(int mode, int m, int dtype, int Bt, int S, int d, int H, int hd, int F) {
    if (mode != SDP_MASK_FORWARD && mode != SDP_MASK_BACKWARD) return SDP_ERR_INVALID_ARG;
    if (m != 0 && m != 1) return SDP_ERR_INVALID_ARG;
    if (dtype != SDP_F32 && dtype != SDP_BF16) return SDP_ERR_INVALID_ARG;
    if (Bt < 1 || S < 1 || d < 1 || H < 1 || hd < 1 || F < 1) return SDP_ERR_INVALID_ARG;
    if (Bt > 65535 || H > 65535) return SDP_ERR_SHAPE;
    if ((int64_t)Bt * S >= ((int64_t)1 << 31) || (int64_t)H * hd >= ((int64_t)1 << 24)) return SDP_ERR_SHAPE;
    if ((int64_t)Bt * S * F >= ((int64_t)1 << 40)) return SDP_ERR_SHAPE;
    if (hd > 128) return SDP_ERR_UNSUPPORTED;
    // as for the attention block alone: heads up to 64 wide are padded to 64 inside, wider ones need 16-byte rows
    if (dtype == SDP_BF16 && (d % 8 || (hd > 64 && hd % 8) || F % 8)) return SDP_ERR_SHAPE;
    return SDP_OK;
}

// the two halves run one after the other: their workspaces share one region
size_t fwd_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F) {
    const size_t a = sdp_masked_attn_fwd_workspace_bytes(SDP_MASK_BACKWARD, dtype, Bt, S, d, H, hd, H);
    const size_t b = sdp_masked_mlp_fwd_workspace_bytes(SDP_MASK_FORWARD, dtype, Bt * S, d, F, F);
    return a > b ? a : b;
}
size_t bwd_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F) {
    const size_t a = sdp_masked_attn_bwd_workspace_bytes(SDP_MASK_BACKWARD, dtype, Bt, S, d, H, hd, H);
    const size_t b = sdp_masked_mlp_bwd_workspace_bytes(SDP_MASK_FORWARD, dtype, Bt * S, d, F, F);
    return round_up((size_t)Bt * S * d * esize(dtype), 256) + (a > b ? a : b); // dHm first
}

} // namespace

extern "C" size_t sdp_block_fwd_workspace_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F) {
    if (check_block(SDP_MASK_FORWARD, 1, dtype, Bt, S, d, H, hd, F) != SDP_OK) return 0;
    return fwd_bytes(dtype, Bt, S, d, H, hd, F);
}

extern "C" size_t sdp_block_bwd_workspace_bytes(int dtype, int Bt, int S, int d, int H, int hd, int F) {
    if (check_block(SDP_MASK_FORWARD, 1, dtype, Bt, S, d, H, hd, F) != SDP_OK) return 0;
    return bwd_bytes(dtype, Bt, S, d, H, hd, F);
}

extern "C" int sdp_block_fwd(int mode, int m, int dtype, int Bt, int S, int d, int H, int hd, int F, const void* X,
                             const void* Wqkv, const void* WoT, const void* W1, const void* W3, const void* W2T, void* Y,
                             void* Hm_save, void* QKV_save, void* O_save, float* LSE_save, void* G_save, void* U_save,
                             void* ws, size_t ws_bytes, void* stream) {
    int rc = check_block(mode, m, dtype, Bt, S, d, H, hd, F);
    if (rc != SDP_OK) return rc;
    if (!X || !Y || !aligned16(X) || !aligned16(Y)) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int T = Bt * S;
    if (mode == SDP_MASK_FORWARD && m == 0) // the skipped block is the identity; nothing of it is touched
        return copy_tokens(X, Y, (size_t)T * d * esize(dtype), "block_skip_fwd", s);
    if (!Wqkv || !WoT || !W1 || !W3 || !W2T || !Hm_save || !QKV_save || !O_save || !LSE_save || !G_save || !U_save)
        return SDP_ERR_INVALID_ARG;
    for (const void* q : {Wqkv, WoT, W1, W3, W2T, (const void*)Hm_save, (const void*)QKV_save, (const void*)O_save,
                          (const void*)LSE_save, (const void*)G_save, (const void*)U_save})
        if (!aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (Y == X || Hm_save == X || Hm_save == Y) return SDP_ERR_INVALID_ARG; // the residuals are read while the sums are written
    if (!ws || !aligned16(ws) || ws_bytes < fwd_bytes(dtype, Bt, S, d, H, hd, F)) return SDP_ERR_WORKSPACE;
    // Hm = X + Attn(X): the dense attention block with X added in the output projection's epilogue
    rc = attn_fwd_impl(SDP_MASK_BACKWARD, dtype, Bt, S, d, H, hd, H, X, Wqkv, WoT, nullptr, Hm_save, QKV_save, O_save,
                       LSE_save, X, ws, s);
    if (rc != SDP_OK) return rc;
    // Y = Hm + MLP(Hm): all F neurons in order (no index list), Hm added in the down projection's epilogue
    return mlp_fwd_impl(SDP_MASK_FORWARD, dtype, T, d, F, F, Hm_save, W1, W3, W2T, nullptr, Y, G_save, U_save, Hm_save, ws, s);
}

extern "C" int sdp_block_bwd(int mode, int m, int dx_rule, int dtype, int Bt, int S, int d, int H, int hd, int F,
                             const void* X, const void* dY, const void* Wqkv, const void* WoT, const void* W1,
                             const void* W3, const void* W2T, const void* Hm_save, const void* QKV_save,
                             const void* O_save, const float* LSE_save, const void* G_save, const void* U_save, void* dX,
                             void* dWqkv, void* dWoT, void* dW1, void* dW3, void* dW2T, void* ws, size_t ws_bytes,
                             void* stream) {
    int rc = check_block(mode, m, dtype, Bt, S, d, H, hd, F);
    if (rc != SDP_OK) return rc;
    if (dx_rule != SDP_BLOCK_DX_THROUGH && dx_rule != SDP_BLOCK_DX_SKIP) return SDP_ERR_INVALID_ARG;
    if (!dY || !dX || !aligned16(dY) || !aligned16(dX)) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int T = Bt * S;
    const bool want_dw = m == 1;
    if (!want_dw && (mode == SDP_MASK_FORWARD || dx_rule == SDP_BLOCK_DX_SKIP)) // only the skip connection carries gradient
        return copy_tokens(dY, dX, (size_t)T * d * esize(dtype), "block_skip_bwd", s);
    if (dtype == SDP_BF16 && T % 8) return SDP_ERR_SHAPE;
    if (!X || !Wqkv || !WoT || !W1 || !W3 || !W2T || !Hm_save || !QKV_save || !O_save || !LSE_save || !G_save || !U_save)
        return SDP_ERR_INVALID_ARG;
    if (want_dw && (!dWqkv || !dWoT || !dW1 || !dW3 || !dW2T)) return SDP_ERR_INVALID_ARG;
    for (const void* q : {X, Wqkv, WoT, W1, W3, W2T, Hm_save, QKV_save, O_save, (const void*)LSE_save, G_save, U_save,
                          (const void*)dWqkv, (const void*)dWoT, (const void*)dW1, (const void*)dW3, (const void*)dW2T})
        if (q && !aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (dX == dY) return SDP_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < bwd_bytes(dtype, Bt, S, d, H, hd, F)) return SDP_ERR_WORKSPACE;
    void* dHm = ws;
    void* sub = (char*)ws + round_up((size_t)T * d * esize(dtype), 256);
    // dHm = dY + (dL/dHm through the MLP): the incoming gradient is added in the epilogue of the MLP's dX contraction
    rc = mlp_bwd_impl(SDP_MASK_FORWARD, dtype, T, d, F, F, Hm_save, dY, W1, W3, W2T, nullptr, G_save, U_save, dHm, dW1, dW3,
                      dW2T, SDP_DW_COMPACT, dY, want_dw, sub, s);
    if (rc != SDP_OK) return rc;
    // dX = dHm + (dL/dX through the attention half)
    return attn_bwd_impl(SDP_MASK_BACKWARD, dtype, Bt, S, d, H, hd, H, X, dHm, Wqkv, WoT, nullptr, QKV_save, O_save, LSE_save,
                         dX, dWqkv, dWoT, SDP_DW_COMPACT, dHm, want_dw, sub, s);
}
