"""The flop counts behind the benchmark's metric against the two iteration multipliers the paper prints for
FLOP matching (tests/golden/flop_matching_multipliers.txt, Sec. 4): they fix the 1 : 2 split between forward
and backward cost and the proportionality of the masked part to the coverage ratio."""
import os

from workloads import MlpWorkload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "flop_matching_multipliers.txt")


def _golden():
    rows = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, cov, mult = line.split()
            rows[name] = (float(cov), float(mult))
    return rows


def test_active_flops_reproduce_the_printed_multipliers():
    g = _golden()
    T, d, F = 512, 256, 1024
    dense = MlpWorkload("dense", "bf16", T, d, F, F, 8, "fm").active_flop_per_worker
    assert dense == 18 * T * d * F  # three contractions forward, six backward, 2 T d F flops each
    # forward masking: the whole step shrinks with the coverage ratio
    cov, mult = g["forward_masking"]
    fm = MlpWorkload("fm", "bf16", T, d, F, int(cov * F), 8, "fm").active_flop_per_worker
    assert abs(dense / fm - mult) < 1e-12
    # full forward, backward masked as a whole (the paper's block-level example): forward 1/3 of the dense step,
    # backward 2/3 of it times the coverage ratio
    cov, mult = g["full_forward_masked_bwd"]
    fwd, bwd = dense / 3, 2 * dense / 3
    assert abs(dense / (fwd + cov * bwd) - mult) < 1e-12
    # neuron-level backward masking keeps the dense dX (the gradient is taken at the full parameters) and masks
    # only the weight gradients, which are half of the backward cost: between the two
    bm = MlpWorkload("bm", "bf16", T, d, F, int(cov * F), 8, "bm").active_flop_per_worker
    assert bm == fwd + bwd / 2 + cov * bwd / 2
    assert fwd + cov * bwd < bm < dense
