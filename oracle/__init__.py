"""TEST INFRASTRUCTURE ONLY: ctypes front end of the plain fp64 CPU oracle.

The oracle states, from the paper's definitions (Sec. 3.1 gate / average,
Sec. 3.2 neuron-level masks, App. A column loads), what the masked SwiGLU MLP
path computes.  It shares nothing with the GPU library and must never be
imported by it: only tests, the smoke check and the benchmark's cpu_baseline
leg use this module.

All floating-point inputs are widened exactly to fp64 before the C code sees
them; no intermediate is rounded.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdp_oracle.c")
_LIB = os.path.join(_HERE, "libsdp_oracle.so")


def build(force=False):
    """Compile the C oracle with gcc (fp64, -O2, OpenMP on outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None

_u8p = ctypes.POINTER(ctypes.c_uint8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_mix64.restype = ctypes.c_uint64
        L.orc_mix64.argtypes = [ctypes.c_uint64]
        L.orc_rand64.restype = ctypes.c_uint64
        L.orc_rand64.argtypes = [ctypes.c_uint64] * 3
        L.orc_rand_below.restype = ctypes.c_uint64
        L.orc_rand_below.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64), ctypes.c_uint64]
        L.orc_make_masks.restype = ctypes.c_int
        L.orc_make_masks.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_int, _u8p]
        L.orc_make_masks_balanced.restype = ctypes.c_int
        L.orc_make_masks_balanced.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint64, _u8p]
        L.orc_avg_adamw.restype = None
        L.orc_avg_adamw.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), _u8p, _f64p, _f64p, _f64p, _u8p] + [ctypes.c_double] * 6 + [ctypes.c_int]
        L.orc_index_masks.restype = None
        L.orc_index_masks.argtypes = [ctypes.c_int, ctypes.c_int64, _u8p, _i32p, ctypes.c_int64, _i32p, _i32p, _u8p]
        L.orc_mlp_fwd.restype = None
        L.orc_mlp_fwd.argtypes = [ctypes.c_int64] * 3 + [_f64p] * 8
        L.orc_mlp_bwd.restype = None
        L.orc_mlp_bwd.argtypes = [ctypes.c_int64] * 3 + [_f64p] * 14
        L.orc_worker_step.restype = ctypes.c_int64
        L.orc_worker_step.argtypes = [ctypes.c_int] + [ctypes.c_int64] * 3 + [_u8p] + [_f64p] * 12
        L.orc_gated_average.restype = None
        L.orc_gated_average.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.POINTER(ctypes.c_void_p), _u8p, _f64p, _u8p,
        ]
        L.orc_gated_average_sqnorm.restype = ctypes.c_double
        L.orc_gated_average_sqnorm.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), _u8p,
        ]
        L.orc_clip_scale.restype = ctypes.c_double
        L.orc_clip_scale.argtypes = [ctypes.c_int, _f64p, ctypes.c_double]
        L.orc_attn_fwd.restype = None
        L.orc_attn_fwd.argtypes = [ctypes.c_int64] * 5 + [_f64p] * 10
        L.orc_attn_bwd.restype = None
        L.orc_attn_bwd.argtypes = [ctypes.c_int64] * 5 + [_f64p] * 18
        L.orc_attn_worker_step.restype = ctypes.c_int64
        L.orc_attn_worker_step.argtypes = [ctypes.c_int] + [ctypes.c_int64] * 5 + [_u8p] + [_f64p] * 19
        L.orc_rho2.restype = ctypes.c_double
        L.orc_rho2.argtypes = [ctypes.c_int, ctypes.c_int64, _u8p]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def mix64(z):
    return int(lib().orc_mix64(ctypes.c_uint64(z & (2**64 - 1))))


def rand64(seed, stream, ctr):
    return int(lib().orc_rand64(seed, stream, ctr))


def rand_below(seed, stream, ctr, n):
    """Returns (value, next counter)."""
    c = ctypes.c_uint64(ctr)
    v = lib().orc_rand_below(seed, stream, ctypes.byref(c), n)
    return int(v), int(c.value)


def make_masks(K, F, p, seed, require_cover=True):
    """Mask matrix m[K][F] (uint8) with row sums p; see orc_make_masks."""
    mask = np.zeros((K, F), dtype=np.uint8)
    rc = lib().orc_make_masks(K, F, p, seed, int(bool(require_cover)), _p(mask, _u8p))
    if rc != 0:
        raise ValueError(f"orc_make_masks failed with {rc}")
    return mask


def make_masks_balanced(K, F, p, seed):
    """Balanced mask matrix m[K][F] (uint8), row sums p, loads near ceil(K p / F); see orc_make_masks_balanced."""
    mask = np.zeros((K, F), dtype=np.uint8)
    rc = lib().orc_make_masks_balanced(K, F, p, seed, _p(mask, _u8p))
    if rc != 0:
        raise ValueError(f"orc_make_masks_balanced failed with {rc}")
    return mask


def index_masks(mask, idx_ld=None):
    """(idx[K][idx_ld], pos[K][F], count[K], cov[F]) of a 0/1 mask matrix."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, F = mask.shape
    if idx_ld is None:
        idx_ld = int(mask.astype(np.int64).sum(axis=1).max()) if K else 0
    idx = np.empty((K, idx_ld), dtype=np.int32)
    pos = np.empty((K, F), dtype=np.int32)
    count = np.empty((K,), dtype=np.int32)
    cov = np.empty((F,), dtype=np.uint8)
    lib().orc_index_masks(K, F, _p(mask, _u8p), _p(idx, _i32p), idx_ld, _p(pos, _i32p), _p(count, _i32p), _p(cov, _u8p))
    return idx, pos, count, cov


def mlp_fwd(X, W1, W3, W2T):
    """Dense SwiGLU MLP forward -> dict(G, U, A, Y), all fp64."""
    X, W1, W3, W2T = map(_f64, (X, W1, W3, W2T))
    T, d = X.shape
    F = W1.shape[0]
    assert W1.shape == (F, d) and W3.shape == (F, d) and W2T.shape == (F, d)
    G = np.empty((T, F)); U = np.empty((T, F)); A = np.empty((T, F)); Y = np.empty((T, d))
    lib().orc_mlp_fwd(T, d, F, *[_p(a, _f64p) for a in (X, W1, W3, W2T, G, U, A, Y)])
    return dict(G=G, U=U, A=A, Y=Y)


def mlp_bwd(X, dY, W1, W3, W2T, G, U, A):
    """Dense SwiGLU MLP backward -> dict(dG, dU, dX, dW1, dW3, dW2T), all fp64."""
    X, dY, W1, W3, W2T, G, U, A = map(_f64, (X, dY, W1, W3, W2T, G, U, A))
    T, d = X.shape
    F = W1.shape[0]
    dG = np.empty((T, F)); dU = np.empty((T, F)); dX = np.empty((T, d))
    dW1 = np.empty((F, d)); dW3 = np.empty((F, d)); dW2T = np.empty((F, d))
    lib().orc_mlp_bwd(T, d, F, *[_p(a, _f64p) for a in (X, dY, W1, W3, W2T, G, U, A, dG, dU, dX, dW1, dW3, dW2T)])
    return dict(dG=dG, dU=dU, dX=dX, dW1=dW1, dW3=dW3, dW2T=dW2T)


def worker_step(mode, mask_k, X, dY, W1, W3, W2T):
    """One worker's forward + backward under forward ('fm') or backward ('bm') masking.

    Returns full-size fp64 arrays G, U [T][F]; Y, dX [T][d]; dW1, dW3, dW2T [F][d]
    and `nonzero_off_mask` (count of off-mask gradient entries that were not
    exactly zero before any gradient masking; the paper's Sec. 3.1 remark says
    it is 0 under forward masking).
    """
    m = {"fm": 0, "bm": 1}[mode]
    mask_k = np.ascontiguousarray(mask_k, dtype=np.uint8)
    X, dY, W1, W3, W2T = map(_f64, (X, dY, W1, W3, W2T))
    T, d = X.shape
    F = W1.shape[0]
    assert mask_k.shape == (F,)
    G = np.empty((T, F)); U = np.empty((T, F)); Y = np.empty((T, d)); dX = np.empty((T, d))
    dW1 = np.empty((F, d)); dW3 = np.empty((F, d)); dW2T = np.empty((F, d))
    nz = lib().orc_worker_step(
        m, T, d, F, _p(mask_k, _u8p),
        *[_p(a, _f64p) for a in (X, dY, W1, W3, W2T, G, U, Y, dX, dW1, dW3, dW2T)],
    )
    return dict(G=G, U=U, Y=Y, dX=dX, dW1=dW1, dW3=dW3, dW2T=dW2T, nonzero_off_mask=int(nz))


def gated_average(g_list, mask):
    """Coverage-normalised average of K gradient buffers [R][D].

    `g_list` holds K numpy arrays of dtype float32, float64 or uint16 (bf16
    bit patterns); `mask` is uint8 [K][R].  Returns (out fp64 [R][D], cov u8 [R]).
    """
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, R = mask.shape
    assert len(g_list) == K
    g_list = [np.ascontiguousarray(g) for g in g_list]
    D = g_list[0].shape[1]
    dt = g_list[0].dtype
    gtype = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}[dt]
    for g in g_list:
        assert g.shape == (R, D) and g.dtype == dt
    ptrs = (ctypes.c_void_p * K)(*[g.ctypes.data for g in g_list])
    out = np.empty((R, D), dtype=np.float64)
    cov = np.empty((R,), dtype=np.uint8)
    lib().orc_gated_average(K, R, D, gtype, ptrs, _p(mask, _u8p), _p(out, _f64p), _p(cov, _u8p))
    return out, cov


def gated_average_sqnorm(g_list, mask):
    """Squared l2 norm of the coverage-normalised average (fp64); see orc_gated_average_sqnorm."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, R = mask.shape
    assert len(g_list) == K
    g_list = [np.ascontiguousarray(g) for g in g_list]
    D = g_list[0].shape[1]
    dt = g_list[0].dtype
    gtype = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}[dt]
    for g in g_list:
        assert g.shape == (R, D) and g.dtype == dt
    ptrs = (ctypes.c_void_p * K)(*[g.ctypes.data for g in g_list])
    return float(lib().orc_gated_average_sqnorm(K, R, D, gtype, ptrs, _p(mask, _u8p)))


def clip_scale(sqnorms, max_norm):
    """Coefficient of global-norm clipping from the groups' squared norms; see orc_clip_scale."""
    sq = np.ascontiguousarray(sqnorms, dtype=np.float64).reshape(-1)
    return float(lib().orc_clip_scale(sq.size, _p(sq, _f64p), float(max_norm)))


def avg_adamw(g_list, mask, theta, m, v, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0):
    """Gated average followed by AdamW on covered rows; see orc_avg_adamw.

    theta, m, v: arrays [R][D] of any float dtype (widened exactly); returns new fp64 (theta, m, v, cov).
    """
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, R = mask.shape
    g_list = [np.ascontiguousarray(g) for g in g_list]
    D = g_list[0].shape[1]
    dt = g_list[0].dtype
    gtype = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}[dt]
    for g in g_list:
        assert g.shape == (R, D) and g.dtype == dt
    th, mm, vv = (np.array(a, dtype=np.float64, order="C", copy=True) for a in (theta, m, v))
    assert th.shape == mm.shape == vv.shape == (R, D)
    ptrs = (ctypes.c_void_p * K)(*[g.ctypes.data for g in g_list])
    cov = np.empty((R,), dtype=np.uint8)
    lib().orc_avg_adamw(K, R, D, gtype, ptrs, _p(mask, _u8p), _p(th, _f64p), _p(mm, _f64p), _p(vv, _f64p), _p(cov, _u8p),
                        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), float(grad_scale), int(step))
    return th, mm, vv, cov


def rho2(mask):
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, F = mask.shape
    return float(lib().orc_rho2(K, F, _p(mask, _u8p)))


def attn_fwd(Bt, S, hd, X, Wq, Wk, Wv, WoT):
    """Dense causal multi-head attention block forward -> dict(Q, K, V, O, Y), fp64; see orc_attn_fwd."""
    X, Wq, Wk, Wv, WoT = map(_f64, (X, Wq, Wk, Wv, WoT))
    T, d = X.shape
    E = Wq.shape[0]
    assert T == Bt * S and E % hd == 0
    for w in (Wq, Wk, Wv, WoT):
        assert w.shape == (E, d)
    Q = np.empty((T, E)); K = np.empty((T, E)); V = np.empty((T, E)); O = np.empty((T, E)); Y = np.empty((T, d))
    lib().orc_attn_fwd(Bt, S, d, E // hd, hd, *[_p(a, _f64p) for a in (X, Wq, Wk, Wv, WoT, Q, K, V, O, Y)])
    return dict(Q=Q, K=K, V=V, O=O, Y=Y)


def attn_bwd(Bt, S, hd, X, dY, Wq, Wk, Wv, WoT, Q, K, V, O):
    """Dense attention block backward -> dict(dQ, dK, dV, dX, dWq, dWk, dWv, dWoT), fp64; see orc_attn_bwd."""
    X, dY, Wq, Wk, Wv, WoT, Q, K, V, O = map(_f64, (X, dY, Wq, Wk, Wv, WoT, Q, K, V, O))
    T, d = X.shape
    E = Wq.shape[0]
    dQ = np.empty((T, E)); dK = np.empty((T, E)); dV = np.empty((T, E)); dX = np.empty((T, d))
    dWq = np.empty((E, d)); dWk = np.empty((E, d)); dWv = np.empty((E, d)); dWoT = np.empty((E, d))
    lib().orc_attn_bwd(Bt, S, d, E // hd, hd,
                       *[_p(a, _f64p) for a in (X, dY, Wq, Wk, Wv, WoT, Q, K, V, O, dQ, dK, dV, dX, dWq, dWk, dWv, dWoT)])
    return dict(dQ=dQ, dK=dK, dV=dV, dX=dX, dWq=dWq, dWk=dWk, dWv=dWv, dWoT=dWoT)


def attn_worker_step(Bt, S, hd, head_mask, X, dY, Wq, Wk, Wv, WoT, mode="fm"):
    """One worker's attention forward + backward with heads masked forward ('fm') or backward ('bm')
    (Sec. 3.1 applied to the head masks of Sec. 4.1).

    Returns full-size fp64 arrays Q, K, V, O [T][H hd]; Y, dX [T][d]; dWq, dWk, dWv, dWoT [H hd][d] and
    `nonzero_off_mask` (gradient entries of unheld heads that are not exactly zero before any masking of the
    gradient; must be 0 under forward masking).
    """
    head_mask = np.ascontiguousarray(head_mask, dtype=np.uint8)
    X, dY, Wq, Wk, Wv, WoT = map(_f64, (X, dY, Wq, Wk, Wv, WoT))
    T, d = X.shape
    E = Wq.shape[0]
    H = E // hd
    assert head_mask.shape == (H,) and T == Bt * S
    names = ["Q", "K", "V", "O", "Y", "dQ", "dK", "dV", "dX", "dWq", "dWk", "dWv", "dWoT"]
    shapes = [(T, E)] * 4 + [(T, d)] + [(T, E)] * 3 + [(T, d)] + [(E, d)] * 4
    out = {n: np.empty(s) for n, s in zip(names, shapes)}
    nz = lib().orc_attn_worker_step({"fm": 0, "bm": 1}[mode], Bt, S, d, H, hd, _p(head_mask, _u8p),
                                    *[_p(a, _f64p) for a in (X, dY, Wq, Wk, Wv, WoT)],
                                    *[_p(out[n], _f64p) for n in names])
    out["nonzero_off_mask"] = int(nz)
    return out


def block_fwd(Bt, S, hd, X, Wq, Wk, Wv, WoT, W1, W3, W2T):
    """Dense residual transformer block (attention + MLP, each behind its own skip connection, no normalisation):
    Hm = X + Attn(X), Y = Hm + MLP(Hm); with B(X) = Y - X this is the paper's block "B(x) + x" (Sec. 3.2,
    block-level variant).  Returns the attention and MLP intermediates too."""
    a = attn_fwd(Bt, S, hd, X, Wq, Wk, Wv, WoT)
    Hm = _f64(X) + a["Y"]
    f = mlp_fwd(Hm, W1, W3, W2T)
    return dict(Hm=Hm, Y=Hm + f["Y"], attn=a, mlp=f)


def block_bwd(Bt, S, hd, X, dY, Wq, Wk, Wv, WoT, W1, W3, W2T, fwd):
    """Backward of block_fwd for upstream dY: the skip connections add the incoming gradient to what comes back
    through each half.  Returns dX and the seven weight gradients."""
    dY = _f64(dY)
    f, a = fwd["mlp"], fwd["attn"]
    bm = mlp_bwd(fwd["Hm"], dY, W1, W3, W2T, f["G"], f["U"], f["A"])
    dHm = dY + bm["dX"]
    ba = attn_bwd(Bt, S, hd, X, dHm, Wq, Wk, Wv, WoT, a["Q"], a["K"], a["V"], a["O"])
    return dict(dX=dHm + ba["dX"], dHm=dHm, dWq=ba["dWq"], dWk=ba["dWk"], dWv=ba["dWv"], dWoT=ba["dWoT"],
                dW1=bm["dW1"], dW3=bm["dW3"], dW2T=bm["dW2T"])


BLOCK_WEIGHTS = ("Wq", "Wk", "Wv", "WoT", "W1", "W3", "W2T")


def block_step(mode, m, Bt, S, hd, X, dY, Wq, Wk, Wv, WoT, W1, W3, W2T, dx_rule="through"):
    """One worker's forward + backward through one residual block under a block-level mask bit m (Sec. 3.2):

    mode 'fm' (block-level forward masking): the masked computation is m B(x) + x.  m = 0 skips the block: Y = X,
      the gradient passes the skip connection unchanged (dX = dY) and the block's weights get no gradient.
    mode 'bm' (block-level backward masking): the forward pass always runs the block (m_fwd is all ones); with
      m = 0 the block is left out of the backward pass: its weight gradients are not computed.  What then reaches
      the layers below is a reading: 'through' sends the gradient through the block as well as the skip
      connection (the gradient at the full parameters that Sec. 3.1's backward masking aggregates), 'skip' sends
      it through the skip connection alone (the whole backward pass of the block omitted, the cost model behind
      the 1.5 x iteration multiplier of Sec. 4).
    Weight gradients that are not computed are returned as exact zeros, `computed` says which case ran."""
    W = (Wq, Wk, Wv, WoT, W1, W3, W2T)
    zero = {"d" + n: np.zeros_like(_f64(w)) for n, w in zip(BLOCK_WEIGHTS, W)}
    if mode == "fm" and not m:
        return dict(Y=_f64(X).copy(), dX=_f64(dY).copy(), computed="skipped", **zero)
    f = block_fwd(Bt, S, hd, X, *W)
    b = block_bwd(Bt, S, hd, X, dY, *W, f)
    if m:
        return dict(Y=f["Y"], dX=b["dX"], computed="full", **{k: b[k] for k in zero})
    assert mode == "bm" and dx_rule in ("through", "skip")
    return dict(Y=f["Y"], dX=b["dX"] if dx_rule == "through" else _f64(dY).copy(), computed="forward only", **zero)
