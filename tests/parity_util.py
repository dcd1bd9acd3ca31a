"""Error norms and host/device shuttling shared by the GPU parity tests."""
import numpy as np
import torch

TOL_F32 = 1e-5        # float32 coefficients, and half storage against the oracle on the stored bits
TOL_HALF = 2e-2       # half storage against the oracle on the float32 master

ORACLE_DTYPE = {"f32": 0, "f16": 1, "bf16": 2}


def bits(t: torch.Tensor) -> np.ndarray:
    """Stored coefficient tensor -> numpy array the oracle reads (float32, or uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


def rowwise_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """Worst row of  max_j |got - want| / max_j |want|  (rows = leading axis)."""
    got = got.reshape(got.shape[0], -1).astype(np.float64)
    want = want.reshape(want.shape[0], -1)
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    bad = ~np.isfinite(num)
    if bad.any():
        return float("inf")
    return float((num / den).max()) if got.size else 0.0


def output_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """Error of a [batch][n_out] result: row by row where a row has enough entries (eight) for its
    largest one to set a scale; over the whole tensor for layers with fewer outputs, where a row is
    one or a few sums that may cancel to nothing."""
    if want.shape[-1] >= 8:
        return rowwise_rel_err(got, want)
    err = np.abs(got.astype(np.float64) - want)
    if not np.isfinite(err).all():
        return float("inf")
    return float(err.max() / max(np.abs(want).max(), 1e-30)) if got.size else 0.0


def pair_slice_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """grad_coef slices [G+1][G+1][n_out] of one pair: max-norm relative error."""
    den = max(np.abs(want).max(), 1e-30)
    return float(np.abs(got.astype(np.float64) - want).max() / den)
