"""Helpers for the GPU parity tests: moving seeded inputs to the device and the tolerance rules."""
from __future__ import annotations

import numpy as np

from paper_2601_07667_amd import asl, synth

# Score tolerance: bf16 inputs, fp32 accumulate vs the float64 oracle.
RTOL, ATOL = 2e-3, 1e-5


def to_dev(x: np.ndarray, dtype: str, dev):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev)
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def params_of(sh: synth.Shape, flags: int = 0, scale: float = 0.0):
    return asl.make_params(sh.Hq, sh.Hk, sh.d, sh.N, sh.W, sh.S, sh.budget,
                           dtype=asl.ASL_BF16 if sh.dtype == "bf16" else asl.ASL_F32,
                           scale=scale, flags=flags)


def ctx_for(sh: synth.Shape):
    return asl.Asl(sh.N, sh.Hk, sh.Hq * sh.W)


def assert_scores_close(gpu: np.ndarray, ora: np.ndarray, what: str = ""):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ora)
    tol = ATOL + RTOL * np.abs(ora)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst at {i}: "
                             f"gpu={gpu[i]:.9g} oracle={ora[i]:.9g}")
    worst = float((err / tol).max()) if err.size else 0.0
    if what:
        note_margin(f"{what} score error", worst)
    return worst


# Worst observed margins of the chained checks, as fractions of the allowed tolerance, keyed by
# the `what` label; printed by report_margins() so that a run shows how far inside the band it is.
MARGINS = {}


def note_margin(what: str, frac: float) -> None:
    MARGINS[what] = max(MARGINS.get(what, 0.0), float(frac))


def report_margins(prefix: str = "") -> None:
    for what, frac in sorted(MARGINS.items()):
        if what.startswith(prefix):
            print(f"margin {what}: {frac:.3g} of the tolerance", flush=True)


def check_topk_within_tolerance(gpu_idx: np.ndarray, ora_scores: np.ndarray, k: int, what: str = ""):
    """Chained top-k rule: every index on which GPU and oracle disagree must have an oracle score
    within the score tolerance (1e-5 + 2e-3 |kth|) of the oracle's k-th largest score."""
    from oracle import asl_oracle as orc
    ora_idx = orc.topk_indices(ora_scores, k)
    g = np.asarray(gpu_idx[:k], dtype=np.int64)
    assert np.all(np.diff(g) > 0), f"{what}: gpu top-k not strictly ascending"
    assert g.min() >= 0 and g.max() < ora_scores.shape[0]
    diff = np.setxor1d(g, ora_idx)
    if diff.size:
        kth = np.sort(ora_scores)[::-1][k - 1]
        tol = ATOL + RTOL * abs(kth)
        worst = np.abs(ora_scores[diff] - kth).max()
        note_margin(f"{what} boundary gap", worst / tol)
        assert worst <= tol, f"{what}: {diff.size} differing indices, worst score gap {worst} > {tol}"
    return diff.size
