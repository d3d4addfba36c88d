"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

MAX_REL = 2e-2   # max|O_gpu - O_ref| / max|O_ref|, per head   (acceptance bar of the target)
MEAN_REL = 5e-3  # mean|O_gpu - O_ref| / mean|O_ref|, per head


def to_f64(x: torch.Tensor) -> np.ndarray:
    """[B,H,n,d] (or [BH,...]) tensor -> float64 numpy with batch and head flattened"""
    a = x.detach().float().cpu().numpy().astype(np.float64)
    if a.ndim == 4:
        a = a.reshape(a.shape[0] * a.shape[1], a.shape[2], a.shape[3])
    return a


def rel_errors(got: np.ndarray, ref: np.ndarray, rows=None):
    """per-head (max_rel, mean_rel); got/ref are [BH, n, d]; rows optionally restricts the tokens"""
    if rows is not None:
        got, ref = got[:, rows], ref[:, rows]
    out = []
    for h in range(ref.shape[0]):
        d = np.abs(got[h] - ref[h])
        out.append((d.max() / np.abs(ref[h]).max(), d.mean() / np.abs(ref[h]).mean()))
    return out


def assert_close(got, ref, rows=None, what=""):
    assert np.isfinite(got if rows is None else got[:, rows]).all(), f"{what}: non-finite output"
    for h, (mx, mean) in enumerate(rel_errors(got, ref, rows)):
        assert mx <= MAX_REL and mean <= MEAN_REL, f"{what}: head {h}: max_rel={mx:.3e} mean_rel={mean:.3e}"
