"""The bf16 path's arithmetic with nothing but its rounding points: test infrastructure that explains the error the
bf16 kernels show against the fp64 oracle.

Every function here computes, in fp64 on the CPU, exactly what the oracle computes (with `on=False` the results
agree with the oracle to fp64 rounding: tests/test_rounding_model.py), and with `on=True` rounds to bf16 (nearest
even) at the places where the GPU path stores a value as bf16 or feeds it to a matrix instruction as a bf16
operand, and nowhere else:

  MLP        G, U stored; Act stored; dG, dU stored; Y, dX stored; dW1, dW3, dW2T stored.
  attention  Q, K, V stored; the probabilities as operand of P V, the row sum taken over the rounded values;
             O stored; Y stored; dO stored; in the backward pass the probabilities (recomputed from the stored
             log-sum-exp) as operand of P^T dO and the logit gradients dZ = P (dP - delta) as operand of dZ K and
             dZ^T Q; dQ, dK, dV stored; dX stored; the four weight gradients stored.
  block      the two halves chained, the skip connections added before the rounding of Hm, Y, dHm, dX.

Accumulation stays exact (the kernels accumulate in fp32, whose error is far below bf16's), as do exp and the
sigmoid.  If the GPU result agrees with this model much more closely than with the oracle, the kernels add no
error of their own beyond the roundings listed; the model's own distance from the oracle is then the error the
bf16 storage format alone causes.
"""
import numpy as np
import torch


def _t(x):
    return torch.as_tensor(np.asarray(x, dtype=np.float64))


def rb(x, on=True):
    """Round an fp64 tensor to bf16 (nearest even) and widen back; identity when `on` is false."""
    if not on:
        return x
    return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def mlp_model(mode, mask_k, X, dY, W1, W3, W2T, on=True, residual=None, dx_residual=None):
    """One worker's masked MLP forward + backward.  Returns full-size arrays like oracle.worker_step (rows of the
    weight gradients off the mask are zero)."""
    X, dY, W1, W3, W2T = map(_t, (X, dY, W1, W3, W2T))
    F = W1.shape[0]
    S = np.flatnonzero(np.asarray(mask_k))
    run = S if mode == "fm" else np.arange(F)  # neurons the forward pass and dX run on
    w1, w3, w2 = W1[run], W3[run], W2T[run]
    G = rb(X @ w1.T, on)
    U = rb(X @ w3.T, on)
    sig = torch.sigmoid(G)
    silu = G * sig
    Act = rb(silu * U, on)
    Yacc = Act @ w2
    Y = rb(Yacc + (_t(residual) if residual is not None else 0.0), on)
    dA = dY @ w2.T
    dU = rb(dA * silu, on)
    dG = rb(dA * U * (sig * (1 + G * (1 - sig))), on)
    dXacc = dG @ w1 + dU @ w3
    dX = rb(dXacc + (_t(dx_residual) if dx_residual is not None else 0.0), on)
    # weight gradients on the mask: columns S of the (possibly dense) dG, dU, Act
    pos = {int(j): i for i, j in enumerate(run)}
    cols = [pos[int(j)] for j in S]
    out = {n: torch.zeros((F, X.shape[1]), dtype=torch.float64) for n in ("dW1", "dW3", "dW2T")}
    out["dW1"][S] = rb(dG[:, cols].T @ X, on)
    out["dW3"][S] = rb(dU[:, cols].T @ X, on)
    out["dW2T"][S] = rb(Act[:, cols].T @ dY, on)
    Gf = torch.zeros((X.shape[0], F), dtype=torch.float64)
    Uf = torch.zeros_like(Gf)
    Gf[:, run], Uf[:, run] = G, U
    res = dict(G=Gf, U=Uf, Y=Y, dX=dX, **out)
    return {k: v.numpy() for k, v in res.items()}


def attn_model(Bt, S, hd, head_mask, X, dY, Wq, Wk, Wv, WoT, mode="fm", on=True, residual=None, dx_residual=None):
    """One worker's head-masked attention forward + backward.  Returns full-size arrays like
    oracle.attn_worker_step (Q, K, V, O columns and weight-gradient rows of heads that did not run are zero)."""
    X, dY, Wq, Wk, Wv, WoT = map(_t, (X, dY, Wq, Wk, Wv, WoT))
    T, d = X.shape
    E_all = Wq.shape[0]
    H = E_all // hd
    held = np.flatnonzero(np.asarray(head_mask))
    run = held if mode == "fm" else np.arange(H)
    rows = np.concatenate([np.arange(h * hd, (h + 1) * hd) for h in run])
    hrows = np.concatenate([np.arange(h * hd, (h + 1) * hd) for h in held])
    n = len(run)
    wq, wk, wv, wo = Wq[rows], Wk[rows], Wv[rows], WoT[rows]
    Q, K, V = rb(X @ wq.T, on), rb(X @ wk.T, on), rb(X @ wv.T, on)

    def heads(z):
        return z.reshape(Bt, S, n, hd).permute(0, 2, 1, 3)  # [Bt][n][S][hd]

    def unheads(z):
        return z.permute(0, 2, 1, 3).reshape(T, n * hd)

    q, k, v = heads(Q), heads(K), heads(V)
    scale = 1.0 / np.sqrt(hd)
    z = (q @ k.transpose(-1, -2)) * scale
    causal = torch.tril(torch.ones((S, S), dtype=torch.bool))
    z = z.masked_fill(~causal, -np.inf)
    mx = z.max(dim=-1, keepdim=True).values
    p_un = rb(torch.exp(z - mx), on)                     # operand of P V; a power-of-two change of reference does not change the rounding
    l = p_un.sum(dim=-1, keepdim=True)
    O = rb(unheads((p_un @ v) / l), on)
    lse = mx + torch.log(l)                              # what the backward pass normalises with
    Yacc = O @ wo
    Y = rb(Yacc + (_t(residual) if residual is not None else 0.0), on)
    # backward
    dO = rb(dY @ wo.T, on)
    do, o = heads(dO), heads(O)
    delta = (do * o).sum(dim=-1, keepdim=True)
    p = torch.exp(z - lse)                               # recomputed, fp32 on the GPU
    dp = do @ v.transpose(-1, -2)
    dz = p * (dp - delta)
    dz_b, p_b = rb(dz, on), rb(p, on)
    dq = rb(unheads(dz_b @ k) * scale, on)
    dk = rb(unheads(dz_b.transpose(-1, -2) @ q) * scale, on)
    dv = rb(unheads(p_b.transpose(-1, -2) @ do), on)
    dXacc = dq @ wq + dk @ wk + dv @ wv
    dX = rb(dXacc + (_t(dx_residual) if dx_residual is not None else 0.0), on)
    pos = {int(r): i for i, r in enumerate(rows)}
    hc = [pos[int(r)] for r in hrows]
    res = {}
    for name, val in (("Q", Q), ("K", K), ("V", V), ("O", O)):
        full = torch.zeros((T, E_all), dtype=torch.float64)
        full[:, rows] = val
        res[name] = full
    for name, lhs, rhs in (("dWq", dq, X), ("dWk", dk, X), ("dWv", dv, X), ("dWoT", O, dY)):
        full = torch.zeros((E_all, d), dtype=torch.float64)
        full[hrows] = rb(lhs[:, hc].T @ rhs, on)
        res[name] = full
    res.update(Y=Y, dX=dX)
    return {k_: v_.numpy() for k_, v_ in res.items()}


def block_model(mode, m, Bt, S, hd, X, dY, Wq, Wk, Wv, WoT, W1, W3, W2T, dx_rule="through", on=True):
    """One worker's pass through one residual block under its block mask bit (see oracle.block_step)."""
    names = ("Wq", "Wk", "Wv", "WoT", "W1", "W3", "W2T")
    W = dict(zip(names, (Wq, Wk, Wv, WoT, W1, W3, W2T)))
    zero = {"d" + n_: np.zeros_like(np.asarray(w, dtype=np.float64)) for n_, w in W.items()}
    Xn, dYn = np.asarray(X, dtype=np.float64), np.asarray(dY, dtype=np.float64)
    if mode == "fm" and not m:
        return dict(Y=Xn.copy(), dX=dYn.copy(), **zero)
    H = np.asarray(Wq).shape[0] // hd
    F = np.asarray(W1).shape[0]
    allh, alln = np.ones(H, dtype=np.uint8), np.ones(F, dtype=np.uint8)
    # forward: Hm = X + Attn(X), Y = Hm + MLP(Hm)
    a_f = attn_model(Bt, S, hd, allh, Xn, np.zeros_like(Xn), Wq, Wk, Wv, WoT, mode="bm", on=on, residual=Xn)
    Hm = a_f["Y"]
    mm = mlp_model("bm", alln, Hm, dYn, W1, W3, W2T, on=on, residual=Hm, dx_residual=dYn)
    Y = mm["Y"]
    if not m and dx_rule == "skip":
        return dict(Y=Y, dX=dYn.copy(), Hm=Hm, **zero)
    dHm = mm["dX"]
    a_b = attn_model(Bt, S, hd, allh, Xn, dHm, Wq, Wk, Wv, WoT, mode="bm", on=on, residual=Xn, dx_residual=dHm)
    out = dict(Y=Y, dX=a_b["dX"], Hm=Hm)
    if m:
        out.update(dWq=a_b["dWq"], dWk=a_b["dWk"], dWv=a_b["dWv"], dWoT=a_b["dWoT"], dW1=mm["dW1"], dW3=mm["dW3"], dW2T=mm["dW2T"])
    else:
        out.update(zero)
    return out
