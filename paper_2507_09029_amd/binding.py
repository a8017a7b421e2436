"""ctypes binding of the C ABI in include/sdp.h.

Argument marshalling only: every function here checks tensor dtypes / devices, passes raw device
pointers and torch's current HIP stream to the library call of the same name and raises SdpError on
a negative status.  PyTorch supplies device memory and streams; no step of the path runs in torch.
There is no fallback: if libsdp_hip.so is missing or fails to load, importing `lib()` raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsdp_hip.so")

F32, BF16 = 0, 1
MASK_FORWARD, MASK_BACKWARD = 0, 1
DW_COMPACT, DW_SCATTER = 0, 1
MAX_WORKERS = 64

_MODES = {"fm": MASK_FORWARD, "bm": MASK_BACKWARD, MASK_FORWARD: MASK_FORWARD, MASK_BACKWARD: MASK_BACKWARD}
_DTYPES = {torch.float32: F32, torch.bfloat16: BF16}


class SdpError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {lib().sdp_status_string(status).decode()} ({status})")


_lib = None


def library_path():
    return _LIB_PATH


def lib():
    """Loads libsdp_hip.so (building it first if it is absent and hipcc is available)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build

        _build.build_library()
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
    L.sdp_status_string.restype = ctypes.c_char_p
    L.sdp_status_string.argtypes = [i32]
    L.sdp_make_masks.restype = i32
    L.sdp_make_masks.argtypes = [i32, i32, i32, u64, i32, vp, vp, vp, vp, vp, sz, vp]
    L.sdp_sample_masks_host.restype = i32
    L.sdp_sample_masks_host.argtypes = [i32, i32, i32, u64, i32, vp]
    L.sdp_index_masks_workspace_bytes.restype = sz
    L.sdp_index_masks_workspace_bytes.argtypes = [i32, i64]
    L.sdp_index_masks.restype = i32
    L.sdp_index_masks.argtypes = [i32, i64, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    L.sdp_profile_launch_shape.restype = i32
    L.sdp_profile_launch_shape.argtypes = [ctypes.c_char_p] + [ctypes.POINTER(ctypes.c_int)] * 4
    L.sdp_index_masks_static.restype = i32
    L.sdp_index_masks_static.argtypes = [i32, i64, vp, vp, i64, vp, vp, vp, vp]
    L.sdp_mask_rho2.restype = i32
    L.sdp_mask_rho2.argtypes = [i32, i64, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.sdp_masked_mlp_fwd_workspace_bytes.restype = sz
    L.sdp_masked_mlp_fwd_workspace_bytes.argtypes = [i32] * 6
    L.sdp_masked_mlp_bwd_workspace_bytes.restype = sz
    L.sdp_masked_mlp_bwd_workspace_bytes.argtypes = [i32] * 6
    L.sdp_masked_mlp_fwd.restype = i32
    L.sdp_masked_mlp_fwd.argtypes = [i32] * 6 + [vp] * 9 + [sz, vp]
    L.sdp_masked_mlp_bwd.restype = i32
    L.sdp_masked_mlp_bwd.argtypes = [i32] * 6 + [vp] * 12 + [i32, vp, sz, vp]
    L.sdp_masked_attn_saved_head_width.restype = i32
    L.sdp_masked_attn_saved_head_width.argtypes = [i32, i32]
    L.sdp_masked_attn_fwd_workspace_bytes.restype = sz
    L.sdp_masked_attn_fwd_workspace_bytes.argtypes = [i32] * 8
    L.sdp_masked_attn_bwd_workspace_bytes.restype = sz
    L.sdp_masked_attn_bwd_workspace_bytes.argtypes = [i32] * 8
    L.sdp_masked_attn_fwd.restype = i32
    L.sdp_masked_attn_fwd.argtypes = [i32] * 8 + [vp] * 9 + [sz, vp]
    L.sdp_masked_attn_bwd.restype = i32
    L.sdp_masked_attn_bwd.argtypes = [i32] * 8 + [vp] * 11 + [i32, vp, sz, vp]
    L.sdp_block_fwd_workspace_bytes.restype = sz
    L.sdp_block_fwd_workspace_bytes.argtypes = [i32] * 7
    L.sdp_block_bwd_workspace_bytes.restype = sz
    L.sdp_block_bwd_workspace_bytes.argtypes = [i32] * 7
    L.sdp_block_fwd.restype = i32
    L.sdp_block_fwd.argtypes = [i32] * 9 + [vp] * 14 + [sz, vp]
    L.sdp_block_bwd.restype = i32
    L.sdp_block_bwd.argtypes = [i32] * 10 + [vp] * 20 + [sz, vp]
    L.sdp_coverage_grad_avg.restype = i32
    L.sdp_coverage_grad_avg.argtypes = [i32, i64, i32, i32, ctypes.POINTER(vp), vp, vp, vp, vp]
    L.sdp_coverage_grad_sqnorm_workspace_bytes.restype = sz
    L.sdp_coverage_grad_sqnorm_workspace_bytes.argtypes = [i64, i32]
    L.sdp_coverage_grad_sqnorm.restype = i32
    L.sdp_coverage_grad_sqnorm.argtypes = [i32, i64, i32, i32, ctypes.POINTER(vp), vp, vp, vp, sz, vp]
    L.sdp_clip_scale.restype = i32
    L.sdp_clip_scale.argtypes = [i32, vp, ctypes.c_float, vp, vp]
    L.sdp_coverage_avg_adamw.restype = i32
    L.sdp_coverage_avg_adamw.argtypes = [i32, i64, i32, i32, ctypes.POINTER(vp), vp, vp, vp, vp, vp, vp, vp, vp]
    L.sdp_profile_enable.restype = i32
    L.sdp_profile_enable.argtypes = [i32]
    L.sdp_profile_filter.restype = i32
    L.sdp_profile_filter.argtypes = [ctypes.c_char_p]
    L.sdp_profile_reset.restype = i32
    L.sdp_profile_reset.argtypes = []
    L.sdp_profile_read.restype = i32
    L.sdp_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    L.sdp_probe_mfma_operand_bytes.restype = sz
    L.sdp_probe_mfma_operand_bytes.argtypes = []
    L.sdp_probe_mfma_sink_bytes.restype = sz
    L.sdp_probe_mfma_sink_bytes.argtypes = [i32]
    L.sdp_probe_mfma_tflops.restype = i32
    L.sdp_probe_mfma_tflops.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.sdp_probe_mfma_shape_tflops.restype = i32
    L.sdp_probe_mfma_shape_tflops.argtypes = [i32, vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.sdp_probe_hbm_gbs.restype = i32
    L.sdp_probe_hbm_gbs.argtypes = [i32, vp, vp, sz, i32, ctypes.POINTER(ctypes.c_double), vp]
    _lib = L
    return L


def _check(status, what):
    if status < 0:
        raise SdpError(status, what)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _sampler(require_cover):
    """False / True -> uniform sampler without / with coverage repair; "balanced" (or 2) -> App. A's construction."""
    if require_cover == "balanced":
        return 2
    return int(require_cover) if isinstance(require_cover, int) and not isinstance(require_cover, bool) else int(bool(require_cover))


def sample_masks_host(K, F, p, seed, require_cover=True):
    """The library's host sampler alone: uint8 [K][F] CPU tensor."""
    mask = torch.zeros((K, F), dtype=torch.uint8)
    _check(lib().sdp_sample_masks_host(K, F, p, seed, _sampler(require_cover), mask.data_ptr()), "sdp_sample_masks_host")
    return mask


def index_masks_workspace_bytes(K, F):
    return int(lib().sdp_index_masks_workspace_bytes(K, F))


def make_masks(K, F, p, seed, require_cover=True, device="cuda"):
    """-> (mask u8 [K][F], idx i32 [K][p], pos i32 [K][F], cov u8 [F]) on the GPU."""
    mask = torch.empty((K, F), dtype=torch.uint8, device=device)
    idx = torch.empty((K, max(p, 0)), dtype=torch.int32, device=device)
    pos = torch.empty((K, F), dtype=torch.int32, device=device)
    cov = torch.empty((F,), dtype=torch.uint8, device=device)
    ws = _ws(index_masks_workspace_bytes(K, F), device)
    st = lib().sdp_make_masks(K, F, p, seed, _sampler(require_cover), mask.data_ptr(), idx.data_ptr(), pos.data_ptr(),
                              cov.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_make_masks")
    return mask, idx, pos, cov


def index_masks(mask, idx_ld=None, ws=None):
    """mask u8 [K][F] (GPU) -> (idx i32 [K][idx_ld], pos i32 [K][F], count i32 [K], cov u8 [F])."""
    mptr = _dev(mask, torch.uint8, "mask")
    K, F = mask.shape
    if idx_ld is None:
        idx_ld = F
    idx = torch.empty((K, idx_ld), dtype=torch.int32, device=mask.device)
    pos = torch.empty((K, F), dtype=torch.int32, device=mask.device)
    count = torch.empty((K,), dtype=torch.int32, device=mask.device)
    cov = torch.empty((F,), dtype=torch.uint8, device=mask.device)
    if ws is None:
        ws = _ws(index_masks_workspace_bytes(K, F), mask.device)
    st = lib().sdp_index_masks(K, F, mptr, idx.data_ptr(), idx_ld, pos.data_ptr(), count.data_ptr(), cov.data_ptr(),
                               ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_index_masks")
    return idx, pos, count, cov


def index_masks_static(mask, idx_ld=None, out=None):
    """index_masks without a workspace: the library's fixed table holds the chunk counts (no allocation inside the call).

    `out` = (idx, pos, count, cov) preallocated tensors makes the whole call allocation-free."""
    mptr = _dev(mask, torch.uint8, "mask")
    K, F = mask.shape
    if idx_ld is None:
        idx_ld = F
    if out is None:
        out = (torch.empty((K, idx_ld), dtype=torch.int32, device=mask.device),
               torch.empty((K, F), dtype=torch.int32, device=mask.device),
               torch.empty((K,), dtype=torch.int32, device=mask.device),
               torch.empty((F,), dtype=torch.uint8, device=mask.device))
    idx, pos, count, cov = out
    st = lib().sdp_index_masks_static(K, F, mptr, _dev(idx, torch.int32, "idx"), idx_ld, _dev(pos, torch.int32, "pos"),
                                      _dev(count, torch.int32, "count"), _dev(cov, torch.uint8, "cov"), _stream())
    _check(st, "sdp_index_masks_static")
    return idx, pos, count, cov


def mask_rho2(K, cov):
    """cov u8 [F] (GPU), K workers -> (rho^2 as a float, load histogram i64 [65] on the GPU: loads 0 .. 64)."""
    cptr = _dev(cov, torch.uint8, "cov")
    hist = torch.empty((MAX_WORKERS + 2,), dtype=torch.int64, device=cov.device)  # last bin: bytes above 64
    out = ctypes.c_double(0.0)
    st = lib().sdp_mask_rho2(K, cov.numel(), cptr, hist.data_ptr(), ctypes.byref(out), _stream())
    _check(st, "sdp_mask_rho2")
    return out.value, hist[: MAX_WORKERS + 1]


def masked_mlp_fwd_workspace_bytes(mode, dtype, T, d, F, p):
    return int(lib().sdp_masked_mlp_fwd_workspace_bytes(_MODES[mode], _DTYPES[dtype], T, d, F, p))


def masked_mlp_bwd_workspace_bytes(mode, dtype, T, d, F, p):
    return int(lib().sdp_masked_mlp_bwd_workspace_bytes(_MODES[mode], _DTYPES[dtype], T, d, F, p))


def masked_mlp_fwd(mode, X, W1, W3, W2T, idx_k, out=None, ws=None):
    """One worker's forward. Returns (Y [T][d], G_save, U_save [T][n]); n = p ('fm') or F ('bm')."""
    m = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    F = W1.shape[0]
    p = int(idx_k.numel()) if idx_k is not None else F
    n = p if m == MASK_FORWARD else F
    for name, w in (("W1", W1), ("W3", W3), ("W2T", W2T)):
        if tuple(w.shape) != (F, d):
            raise ValueError(f"{name}: expected shape {(F, d)}")
    if out is None:
        out = (torch.empty((T, d), dtype=dt, device=X.device), torch.empty((T, n), dtype=dt, device=X.device),
               torch.empty((T, n), dtype=dt, device=X.device))
    Y, G, U = out
    if ws is None:
        ws = _ws(masked_mlp_fwd_workspace_bytes(m, dt, T, d, F, p), X.device)
    st = lib().sdp_masked_mlp_fwd(
        m, _DTYPES[dt], T, d, F, p, _dev(X, dt, "X"), _dev(W1, dt, "W1"), _dev(W3, dt, "W3"), _dev(W2T, dt, "W2T"),
        _dev(idx_k, torch.int32, "idx_k") if idx_k is not None else None, _dev(Y, dt, "Y"), _dev(G, dt, "G_save"),
        _dev(U, dt, "U_save"), ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_masked_mlp_fwd")
    return Y, G, U


def masked_mlp_bwd(mode, X, dY, W1, W3, W2T, idx_k, G_save, U_save, dw_layout="compact", out=None, ws=None):
    """One worker's backward. Returns (dX [T][d], dW1, dW3, dW2T); [p][d] compact or [F][d] scattered."""
    m = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    F = W1.shape[0]
    p = int(idx_k.numel())
    lay = {"compact": DW_COMPACT, "scatter": DW_SCATTER}[dw_layout]
    if out is None:
        rows = p if lay == DW_COMPACT else F
        out = (torch.empty((T, d), dtype=dt, device=X.device),) + tuple(
            torch.empty((rows, d), dtype=dt, device=X.device) for _ in range(3))
    dX, dW1, dW3, dW2T = out
    if ws is None:
        ws = _ws(masked_mlp_bwd_workspace_bytes(m, dt, T, d, F, p), X.device)
    st = lib().sdp_masked_mlp_bwd(
        m, _DTYPES[dt], T, d, F, p, _dev(X, dt, "X"), _dev(dY, dt, "dY"), _dev(W1, dt, "W1"), _dev(W3, dt, "W3"),
        _dev(W2T, dt, "W2T"), _dev(idx_k, torch.int32, "idx_k"), _dev(G_save, dt, "G_save"), _dev(U_save, dt, "U_save"),
        _dev(dX, dt, "dX"), _dev(dW1, dt, "dW1"), _dev(dW3, dt, "dW3"), _dev(dW2T, dt, "dW2T"), lay,
        ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_masked_mlp_bwd")
    return dX, dW1, dW3, dW2T


def masked_attn_fwd_workspace_bytes(mode, dtype, Bt, S, d, H, hd, ph):
    return int(lib().sdp_masked_attn_fwd_workspace_bytes(_MODES[mode], _DTYPES[dtype], Bt, S, d, H, hd, ph))


def masked_attn_bwd_workspace_bytes(mode, dtype, Bt, S, d, H, hd, ph):
    return int(lib().sdp_masked_attn_bwd_workspace_bytes(_MODES[mode], _DTYPES[dtype], Bt, S, d, H, hd, ph))


def attn_saved_head_width(dtype, hd):
    """Columns a head takes in QKV_save / O_save: hd, or 64 for bf16 heads narrower than 64 (padded with zeros)."""
    return int(lib().sdp_masked_attn_saved_head_width(_DTYPES[dtype], hd))


def attn_unpad(t, hd, parts=1):
    """View of a saved tensor [T][parts n hw] without the padding columns: [T][parts n hd] (a copy when padded)."""
    T, cols = t.shape
    hw = attn_saved_head_width(t.dtype, hd)
    if hw == hd:
        return t
    return t.reshape(T, cols // hw, hw)[:, :, :hd].reshape(T, -1)


def masked_attn_fwd(mode, Bt, S, hd, X, Wqkv, WoT, head_idx_k, out=None, ws=None):
    """One worker's head-masked attention forward ('fm': the held heads only; 'bm': the dense block).

    X [Bt S][d]; Wqkv [3][H hd][d]; WoT [H hd][d]; head_idx_k int32 [ph].  With n = ph ('fm') or H ('bm') and
    hw = attn_saved_head_width(dtype, hd): returns (Y [T][d], QKV_save [T][3 n hw], O_save [T][n hw],
    LSE_save fp32 [Bt][n][S]).
    """
    m = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    E_all = WoT.shape[0]
    H = E_all // hd
    ph = int(head_idx_k.numel()) if head_idx_k is not None else H
    n = ph if m == MASK_FORWARD else H
    if T != Bt * S or tuple(Wqkv.shape) != (3, E_all, d) or tuple(WoT.shape) != (E_all, d) or H * hd != E_all:
        raise ValueError("attention shapes do not fit together")
    hw = attn_saved_head_width(dt, hd)
    if out is None:
        out = (torch.empty((T, d), dtype=dt, device=X.device), torch.empty((T, 3 * n * hw), dtype=dt, device=X.device),
               torch.empty((T, n * hw), dtype=dt, device=X.device),
               torch.empty((Bt, n, S), dtype=torch.float32, device=X.device))
    Y, QKV, O, LSE = out
    if ws is None:
        ws = _ws(masked_attn_fwd_workspace_bytes(m, dt, Bt, S, d, H, hd, ph), X.device)
    st = lib().sdp_masked_attn_fwd(
        m, _DTYPES[dt], Bt, S, d, H, hd, ph, _dev(X, dt, "X"), _dev(Wqkv, dt, "Wqkv"), _dev(WoT, dt, "WoT"),
        _dev(head_idx_k, torch.int32, "head_idx_k") if head_idx_k is not None else None, _dev(Y, dt, "Y"),
        _dev(QKV, dt, "QKV_save"), _dev(O, dt, "O_save"), _dev(LSE, torch.float32, "LSE_save"), ws.data_ptr(), ws.numel(),
        _stream())
    _check(st, "sdp_masked_attn_fwd")
    return Y, QKV, O, LSE


def masked_attn_bwd(mode, Bt, S, hd, X, dY, Wqkv, WoT, head_idx_k, QKV_save, O_save, LSE_save, dw_layout="compact",
                    out=None, ws=None):
    """One worker's head-masked attention backward.

    Returns (dX [T][d], dWqkv, dWoT): [3][ph hd][d] and [ph hd][d] compact, or full-size buffers with the held
    heads' rows written (scatter).  'bm': dX through all heads, weight gradients of the held heads only.
    """
    m = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    E_all = WoT.shape[0]
    H = E_all // hd
    ph = int(head_idx_k.numel())
    lay = {"compact": DW_COMPACT, "scatter": DW_SCATTER}[dw_layout]
    if out is None:
        rows = ph * hd if lay == DW_COMPACT else E_all
        out = (torch.empty((T, d), dtype=dt, device=X.device), torch.empty((3, rows, d), dtype=dt, device=X.device),
               torch.empty((rows, d), dtype=dt, device=X.device))
    dX, dWqkv, dWoT = out
    if ws is None:
        ws = _ws(masked_attn_bwd_workspace_bytes(m, dt, Bt, S, d, H, hd, ph), X.device)
    st = lib().sdp_masked_attn_bwd(
        m, _DTYPES[dt], Bt, S, d, H, hd, ph, _dev(X, dt, "X"), _dev(dY, dt, "dY"), _dev(Wqkv, dt, "Wqkv"), _dev(WoT, dt, "WoT"),
        _dev(head_idx_k, torch.int32, "head_idx_k"), _dev(QKV_save, dt, "QKV_save"), _dev(O_save, dt, "O_save"),
        _dev(LSE_save, torch.float32, "LSE_save"), _dev(dX, dt, "dX"), _dev(dWqkv, dt, "dWqkv"), _dev(dWoT, dt, "dWoT"),
        lay, ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_masked_attn_bwd")
    return dX, dWqkv, dWoT


BLOCK_DX_THROUGH, BLOCK_DX_SKIP = 0, 1
_DX_RULES = {"through": BLOCK_DX_THROUGH, "skip": BLOCK_DX_SKIP, BLOCK_DX_THROUGH: BLOCK_DX_THROUGH, BLOCK_DX_SKIP: BLOCK_DX_SKIP}


def block_fwd_workspace_bytes(dtype, Bt, S, d, H, hd, F):
    return int(lib().sdp_block_fwd_workspace_bytes(_DTYPES[dtype], Bt, S, d, H, hd, F))


def block_bwd_workspace_bytes(dtype, Bt, S, d, H, hd, F):
    return int(lib().sdp_block_bwd_workspace_bytes(_DTYPES[dtype], Bt, S, d, H, hd, F))


def _opt(t, dtype, name):
    return _dev(t, dtype, name) if t is not None else None


def block_fwd(mode, m, Bt, S, hd, X, Wqkv, WoT, W1, W3, W2T, out=None, ws=None):
    """One worker's forward through one residual block (attention + MLP) under its block mask bit m.

    'fm' with m = 0 skips the block: returns (Y = X, None): nothing is saved.  Otherwise returns
    (Y [T][d], saved) with saved = (Hm, QKV, O, LSE, G, U) for block_bwd."""
    md = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    E = WoT.shape[0]
    H = E // hd
    F = W1.shape[0]
    dev = X.device
    if md == MASK_FORWARD and not m:
        Y = torch.empty_like(X) if out is None else out
        st = lib().sdp_block_fwd(md, 0, _DTYPES[dt], Bt, S, d, H, hd, F, _dev(X, dt, "X"), None, None, None, None, None,
                                 _dev(Y, dt, "Y"), None, None, None, None, None, None, None, 0, _stream())
        _check(st, "sdp_block_fwd")
        return Y, None
    Es = H * attn_saved_head_width(dt, hd)
    if out is None:
        out = (torch.empty((T, d), dtype=dt, device=dev), torch.empty((T, d), dtype=dt, device=dev),
               torch.empty((T, 3 * Es), dtype=dt, device=dev), torch.empty((T, Es), dtype=dt, device=dev),
               torch.empty((Bt, H, S), dtype=torch.float32, device=dev), torch.empty((T, F), dtype=dt, device=dev),
               torch.empty((T, F), dtype=dt, device=dev))
    Y, Hm, QKV, O, LSE, G, U = out
    if ws is None:
        ws = _ws(block_fwd_workspace_bytes(dt, Bt, S, d, H, hd, F), dev)
    st = lib().sdp_block_fwd(md, int(bool(m)), _DTYPES[dt], Bt, S, d, H, hd, F, _dev(X, dt, "X"), _dev(Wqkv, dt, "Wqkv"),
                             _dev(WoT, dt, "WoT"), _dev(W1, dt, "W1"), _dev(W3, dt, "W3"), _dev(W2T, dt, "W2T"), _dev(Y, dt, "Y"),
                             _dev(Hm, dt, "Hm_save"), _dev(QKV, dt, "QKV_save"), _dev(O, dt, "O_save"),
                             _dev(LSE, torch.float32, "LSE_save"), _dev(G, dt, "G_save"), _dev(U, dt, "U_save"),
                             ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_block_fwd")
    return Y, (Hm, QKV, O, LSE, G, U)


def block_bwd(mode, m, Bt, S, hd, X, dY, Wqkv, WoT, W1, W3, W2T, saved, dx_rule="through", out=None, ws=None):
    """Backward of block_fwd.  Returns (dX, grads) with grads = (dWqkv, dWoT, dW1, dW3, dW2T) when m = 1 and None
    otherwise (a masked block gets no weight gradient; under 'bm' dX then follows dx_rule)."""
    md = _MODES[mode]
    dt = X.dtype
    T, d = X.shape
    E = WoT.shape[0]
    H = E // hd
    F = W1.shape[0]
    dev = X.device
    rule = _DX_RULES[dx_rule]
    if not m and (md == MASK_FORWARD or rule == BLOCK_DX_SKIP):
        dX = torch.empty_like(dY) if out is None else out[0]
        st = lib().sdp_block_bwd(md, 0, rule, _DTYPES[dt], Bt, S, d, H, hd, F, None, _dev(dY, dt, "dY"), *([None] * 11),
                                 _dev(dX, dt, "dX"), *([None] * 5), None, 0, _stream())
        _check(st, "sdp_block_bwd")
        return dX, None
    Hm, QKV, O, LSE, G, U = saved
    if out is None:
        out = (torch.empty((T, d), dtype=dt, device=dev),)
        if m:
            out += (torch.empty((3, E, d), dtype=dt, device=dev), torch.empty((E, d), dtype=dt, device=dev),
                    torch.empty((F, d), dtype=dt, device=dev), torch.empty((F, d), dtype=dt, device=dev),
                    torch.empty((F, d), dtype=dt, device=dev))
    dX = out[0]
    g = tuple(out[1:6]) if m else (None,) * 5
    if ws is None:
        ws = _ws(block_bwd_workspace_bytes(dt, Bt, S, d, H, hd, F), dev)
    st = lib().sdp_block_bwd(md, int(bool(m)), rule, _DTYPES[dt], Bt, S, d, H, hd, F, _dev(X, dt, "X"), _dev(dY, dt, "dY"),
                             _dev(Wqkv, dt, "Wqkv"), _dev(WoT, dt, "WoT"), _dev(W1, dt, "W1"), _dev(W3, dt, "W3"),
                             _dev(W2T, dt, "W2T"), _dev(Hm, dt, "Hm_save"), _dev(QKV, dt, "QKV_save"), _dev(O, dt, "O_save"),
                             _dev(LSE, torch.float32, "LSE_save"), _dev(G, dt, "G_save"), _dev(U, dt, "U_save"),
                             _dev(dX, dt, "dX"), *[_opt(t, dt, "dW") for t in g], ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_block_bwd")
    return dX, (g if m else None)


def coverage_grad_avg(grads, mask, out=None, cov=None):
    """grads: K GPU tensors [R][D] (fp32 or bf16); mask u8 [K][R] -> (out fp32 [R][D], cov u8 [R])."""
    K = len(grads)
    if K < 1 or K > MAX_WORKERS:
        raise SdpError(-1, "sdp_coverage_grad_avg")
    dt = grads[0].dtype
    R, D = grads[0].shape
    ptrs = (ctypes.c_void_p * K)(*[_dev(g, dt, f"grads[{i}]") for i, g in enumerate(grads)])
    for g in grads:
        if tuple(g.shape) != (R, D):
            raise ValueError("all gradient buffers must share one shape")
    if tuple(mask.shape) != (K, R):
        raise ValueError("mask must be [K][R]")
    if out is None:
        out = torch.empty((R, D), dtype=torch.float32, device=grads[0].device)
    if cov is None:
        cov = torch.empty((R,), dtype=torch.uint8, device=grads[0].device)
    st = lib().sdp_coverage_grad_avg(K, R, D, _DTYPES[dt], ptrs, _dev(mask, torch.uint8, "mask"),
                                     _dev(out, torch.float32, "out"), _dev(cov, torch.uint8, "cov"), _stream())
    _check(st, "sdp_coverage_grad_avg")
    return out, cov


def coverage_grad_sqnorm(grads, mask, out=None, ws=None):
    """Squared l2 norm of the coverage-normalised average of `grads` -> fp64 tensor with one element, on the GPU."""
    K = len(grads)
    if K < 1 or K > MAX_WORKERS:
        raise SdpError(-1, "sdp_coverage_grad_sqnorm")
    dt = grads[0].dtype
    R, D = grads[0].shape
    ptrs = (ctypes.c_void_p * K)(*[_dev(g, dt, f"grads[{i}]") for i, g in enumerate(grads)])
    for g in grads:
        if tuple(g.shape) != (R, D):
            raise ValueError("all gradient buffers must share one shape")
    if tuple(mask.shape) != (K, R):
        raise ValueError("mask must be [K][R]")
    if out is None:
        out = torch.empty((1,), dtype=torch.float64, device=grads[0].device)
    if ws is None:
        ws = _ws(int(lib().sdp_coverage_grad_sqnorm_workspace_bytes(R, D)), grads[0].device)
    st = lib().sdp_coverage_grad_sqnorm(K, R, D, _DTYPES[dt], ptrs, _dev(mask, torch.uint8, "mask"),
                                        _dev(out, torch.float64, "sqnorm"), ws.data_ptr(), ws.numel(), _stream())
    _check(st, "sdp_coverage_grad_sqnorm")
    return out


class AdamWParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("grad_scale", ctypes.c_float), ("step", ctypes.c_int),
                ("grad_scale_dev", ctypes.c_void_p)]


def clip_scale(sqnorms, max_norm, out=None):
    """sqnorms: fp64 GPU tensor [n] of squared norms -> fp32 GPU tensor [1]: min(1, max_norm / (sqrt(sum) + 1e-6))."""
    if out is None:
        out = torch.empty((1,), dtype=torch.float32, device=sqnorms.device)
    st = lib().sdp_clip_scale(sqnorms.numel(), _dev(sqnorms, torch.float64, "sqnorms"), max_norm,
                              _dev(out, torch.float32, "scale"), _stream())
    _check(st, "sdp_clip_scale")
    return out


def coverage_avg_adamw(grads, mask, theta, m, v, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0,
                       theta_bf16=None, cov=None, grad_scale_dev=None):
    """Coverage average fused with AdamW on covered rows: theta, m, v (fp32 [R][D]) are updated in place.

    theta_bf16 (optional bf16 [R][D]) receives the updated parameters of covered rows.  Returns cov u8 [R].
    """
    K = len(grads)
    if K < 1 or K > MAX_WORKERS:
        raise SdpError(-1, "sdp_coverage_avg_adamw")
    dt = grads[0].dtype
    R, D = grads[0].shape
    ptrs = (ctypes.c_void_p * K)(*[_dev(g, dt, f"grads[{i}]") for i, g in enumerate(grads)])
    for t, name in ((theta, "theta"), (m, "m"), (v, "v")):
        if tuple(t.shape) != (R, D):
            raise ValueError(f"{name} must be [R][D]")
    if tuple(mask.shape) != (K, R):
        raise ValueError("mask must be [K][R]")
    if cov is None:
        cov = torch.empty((R,), dtype=torch.uint8, device=grads[0].device)
    hp = AdamWParams(lr, beta1, beta2, eps, weight_decay, grad_scale, step,
                     _dev(grad_scale_dev, torch.float32, "grad_scale_dev") if grad_scale_dev is not None else None)
    lowp = _dev(theta_bf16, torch.bfloat16, "theta_bf16") if theta_bf16 is not None else None
    st = lib().sdp_coverage_avg_adamw(K, R, D, _DTYPES[dt], ptrs, _dev(mask, torch.uint8, "mask"),
                                      _dev(theta, torch.float32, "theta"), _dev(m, torch.float32, "m"),
                                      _dev(v, torch.float32, "v"), lowp, _dev(cov, torch.uint8, "cov"), ctypes.byref(hp), _stream())
    _check(st, "sdp_coverage_avg_adamw")
    return cov


def profile_enable(on=True):
    _check(lib().sdp_profile_enable(int(bool(on))), "sdp_profile_enable")


def profile_filter(name=None):
    """Time only launches of kernel `name` (None: every kernel)."""
    _check(lib().sdp_profile_filter(name.encode() if name else None), "sdp_profile_filter")


def profile_reset():
    _check(lib().sdp_profile_reset(), "sdp_profile_reset")


def profile_read(cap=64):
    """-> {kernel name: (launches, total ms)} since the last reset (waits for the recorded events)."""
    names = (ctypes.c_char_p * cap)()
    calls = (ctypes.c_int64 * cap)()
    ms = (ctypes.c_double * cap)()
    n = lib().sdp_profile_read(cap, names, calls, ms)
    _check(n, "sdp_profile_read")
    return {names[i].decode(): (int(calls[i]), float(ms[i])) for i in range(n)}


def profile_launch_shape(name):
    """-> {"tile": "BMxBN", "group_m": g, "stacked": bool} of the last MFMA contraction launched under `name` while
    timing was on, or None if there was none."""
    v = [ctypes.c_int(0) for _ in range(4)]
    st = lib().sdp_profile_launch_shape(name.encode(), *[ctypes.byref(x) for x in v])
    if st != 0:
        return None
    return {"tile": f"{v[0].value}x{v[1].value}", "group_m": v[2].value, "stacked": bool(v[3].value)}


def probe_mfma_tflops(operands, blocks=1024, iters=500, shape=16):
    """Sustained bf16 MFMA rate (TFLOP/s) on the values of `operands` (bf16 tensor on the GPU); shape 16 =
    v_mfma_f32_16x16x32_bf16 (what the contractions use), 32 = v_mfma_f32_32x32x16_bf16."""
    L = lib()
    need = L.sdp_probe_mfma_operand_bytes()
    _dev(operands, torch.bfloat16, "operands")
    if operands.numel() * 2 < need:
        raise ValueError(f"operands: need at least {need} bytes")
    sink = torch.empty(L.sdp_probe_mfma_sink_bytes(blocks), dtype=torch.uint8, device=operands.device)
    out = ctypes.c_double(0.0)
    _check(L.sdp_probe_mfma_shape_tflops(shape, operands.data_ptr(), blocks, iters, sink.data_ptr(), ctypes.byref(out), _stream()),
           "sdp_probe_mfma_shape_tflops")
    return out.value


def probe_hbm_gbs(src, dst=None, launches=5):
    """GB/s a plain streaming kernel sustains over `src` (any contiguous GPU tensor): read-only if dst is None, else
    a copy into dst (same size)."""
    L = lib()
    if not (isinstance(src, torch.Tensor) and src.is_cuda and src.is_contiguous()):
        raise TypeError("src: expected a contiguous tensor on the GPU")
    nbytes = src.numel() * src.element_size()
    if dst is None:
        sink = torch.zeros(16, dtype=torch.uint8, device=src.device)
        target, copy = sink, 0
    else:
        if not (isinstance(dst, torch.Tensor) and dst.is_cuda and dst.is_contiguous()
                and dst.numel() * dst.element_size() >= nbytes):
            raise TypeError("dst: expected a contiguous GPU tensor at least as large as src")
        target, copy = dst, 1
    out = ctypes.c_double(0.0)
    _check(L.sdp_probe_hbm_gbs(copy, src.data_ptr(), target.data_ptr(), nbytes, launches, ctypes.byref(out), _stream()),
           "sdp_probe_hbm_gbs")
    return out.value
