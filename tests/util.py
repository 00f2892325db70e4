"""Shared helpers for the GPU parity tests (plumbing only)."""
import numpy as np
import torch

import oracle
from paper_2501_13629_amd import inputs

TOL = {"f32": 1e-4, "bf16": 2e-2}  # max-abs error against the float64 oracle


def dev(t):
    return None if t is None else t.cuda()


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def max_abs(gpu: torch.Tensor, ref: np.ndarray) -> float:
    g = f64(gpu)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), "non-finite values in the GPU output"
    return float(np.max(np.abs(g - ref))) if g.size else 0.0


def check(gpu: torch.Tensor, ref: np.ndarray, dtype: str, what: str = ""):
    err = max_abs(gpu, ref)
    assert err <= TOL[dtype], "%s: max-abs error %.3e exceeds %.1e" % (what, err, TOL[dtype])
    return err


def check_lse(gpu: torch.Tensor, ref: np.ndarray, what: str = ""):
    g = f64(gpu)
    both_inf = np.isneginf(g) & np.isneginf(ref)
    with np.errstate(invalid="ignore"):
        diff = np.where(both_inf, 0.0, np.abs(g - ref))
    assert np.all(np.isfinite(diff)) and diff.max(initial=0.0) <= 2e-3, "%s: lse error %s" % (what, diff.max(initial=0.0))


def oracle_decode(d, scale=None, T=None):
    sl = None if d.get("seqlens") is None else d["seqlens"].numpy()
    return oracle.decode(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]), inputs.as_numpy(d["v"]), seqlens=sl,
                         scale=scale, T=T)
