"""Seeded synthetic inputs shared, as data, by the CPU oracle and the GPU path.

This module holds none of the method's arithmetic: it only names the workload
shapes and draws input tensors (activations, upstream gradients, weights,
per-worker gradient buffers) from fixed seeds with torch's generators.  Masks
are NOT produced here: each side builds them from (K, F, p, seed) on its own.

The tensors stand in for a LLaMA-style MLP block's activations and weights
during pre-training; cost and correctness of the path depend on shapes, value
scale and the mask structure, not on token content.
"""
from dataclasses import dataclass

import numpy as np
import torch

BASE_SEED = 20250709


@dataclass(frozen=True)
class MlpWorkload:
    name: str
    dtype: str  # "f32" | "bf16"
    T: int  # tokens per worker batch
    d: int  # d_model
    F: int  # d_ff (hidden neurons)
    p: int  # active neurons per worker
    K: int  # simulated workers
    mode: str  # "fm" forward masking | "bm" backward masking
    mask_seed: int = BASE_SEED

    @property
    def active_flop_per_worker(self):
        if self.mode == "fm":
            return 18 * self.T * self.d * self.p
        return 12 * self.T * self.d * self.F + 6 * self.T * self.d * self.p


@dataclass(frozen=True)
class AvgWorkload:
    name: str
    K: int
    R: int  # neuron rows
    D: int  # parameters per row
    p: int  # covered rows per worker
    mask_seed: int = BASE_SEED + 5
    sigma: float = 1e-3

    @property
    def algorithmic_bytes(self):
        # covered rows read as bf16, every output row written as fp32, masks read, counts written
        return self.K * self.p * self.D * 2 + self.R * self.D * 4 + self.K * self.R + self.R


@dataclass(frozen=True)
class AttnWorkload:
    """Head-masked causal self-attention block: Bt sequences of S tokens, H heads of width hd, ph held per worker."""
    name: str
    Bt: int
    S: int
    d: int
    H: int
    hd: int
    ph: int
    K: int
    mask_seed: int = BASE_SEED + 7
    dtype: str = "bf16"

    @property
    def T(self):
        return self.Bt * self.S

    @property
    def active_flop_per_worker(self):
        # projections (forward 2, backward 4 flop per multiply-add pair): Q, K, V, O on the held heads;
        # core: causal half of 2 S^2 hd products, 2 forward (Q K^T, P V) and 5 backward
        E = self.ph * self.hd
        proj = 6 * self.T * self.d * 4 * E
        core = 7 * self.Bt * self.ph * self.S * self.S * self.hd
        return proj + core


ATTN_500M = AttnWorkload("attn_bf16_fm_500M", 4, 2048, 1536, 24, 64, 12, 4)
# the paper's own 500M width (App. "Hyperparameters for LLM Architecture": hidden 1200, 24 heads, i.e. head width 50)
ATTN_500M_HD50 = AttnWorkload("attn_bf16_fm_500M_paper_width", 4, 2048, 1200, 24, 50, 12, 4)

CONFIG1 = MlpWorkload("config1_f32_fm", "f32", 256, 256, 1024, 512, 4, "fm")
CONFIG2 = MlpWorkload("config2_bf16_fm_500M", "bf16", 8192, 1536, 4096, 2048, 4, "fm")
CONFIG3 = MlpWorkload("config3_bf16_fm_1B", "bf16", 16384, 2048, 5504, 4128, 8, "fm")
CONFIG4 = MlpWorkload("config4_bf16_bm_1B", "bf16", 16384, 2048, 5504, 4128, 8, "bm")
CONFIG5 = AvgWorkload("config5_avg_1B", 8, 488282, 2048, round(0.69 * 488282))

MLP_CONFIGS = {c.name: c for c in (CONFIG1, CONFIG2, CONFIG3, CONFIG4)}


def _gen(stream):
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED * 1000 + stream)
    return g


def _draw(shape, std, stream, dtype):
    x = torch.randn(shape, generator=_gen(stream), dtype=torch.float32) * std
    if dtype == "bf16":
        return x.to(torch.bfloat16)  # rounded once, to nearest even: these bits are the input
    return x


def mlp_weights(w, stream_base=0):
    """W1, W3, W2T, each [F][d] neuron-major, N(0, 0.02^2)."""
    return tuple(_draw((w.F, w.d), 0.02, stream_base + 1 + i, w.dtype) for i in range(3))


def mlp_batch(w, k, stream_base=0, rows=None):
    """Worker k's activations X_k and upstream gradient dY_k, [T][d], N(0, 1)."""
    T = w.T if rows is None else rows
    X = _draw((T, w.d), 1.0, stream_base + 100 + 2 * k, w.dtype)
    dY = _draw((T, w.d), 1.0, stream_base + 101 + 2 * k, w.dtype)
    return X, dY


def attn_weights(w, stream_base=0):
    """Wqkv [3][H hd][d] (W_Q, W_K, W_V stacked, neuron-major) and WoT [H hd][d], N(0, 0.02^2)."""
    E = w.H * w.hd
    return _draw((3, E, w.d), 0.02, stream_base + 11, w.dtype), _draw((E, w.d), 0.02, stream_base + 12, w.dtype)


def attn_batch(w, k, stream_base=0):
    """Worker k's block input X_k and upstream gradient dY_k, [Bt S][d], N(0, 1)."""
    X = _draw((w.T, w.d), 1.0, stream_base + 300 + 2 * k, w.dtype)
    dY = _draw((w.T, w.d), 1.0, stream_base + 301 + 2 * k, w.dtype)
    return X, dY


def to_f64(t):
    """Exact widening of an fp32 / bf16 torch tensor to a numpy fp64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bf16_bits(t):
    """bf16 torch tensor -> numpy uint16 bit patterns (no value change)."""
    assert t.dtype == torch.bfloat16
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)


def grad_buffers(K, R, D, sigma, dtype, stream_base=500, device="cpu", poison_mask=None):
    """K per-worker gradient buffers [R][D] ~ N(0, sigma^2).

    On `device` other than cpu the device generator is used (values then differ
    from the cpu draw; callers copy what they need back to the host).  With
    `poison_mask` (uint8 [K][R] torch tensor), rows a worker does not cover are
    overwritten with NaN, which a correct average never reads.
    """
    out = []
    for k in range(K):
        if device == "cpu":
            g = torch.randn((R, D), generator=_gen(stream_base + k), dtype=torch.float32) * sigma
        else:
            gen = torch.Generator(device=device)
            gen.manual_seed(BASE_SEED * 1000 + stream_base + k)
            g = torch.randn((R, D), generator=gen, dtype=torch.float32, device=device) * sigma
        g = g.to(torch.bfloat16) if dtype == "bf16" else g
        if poison_mask is not None:
            off = poison_mask[k].to(g.device) == 0
            g[off] = float("nan")
        out.append(g)
    return out
