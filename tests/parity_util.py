"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np

TOL_F32 = 1e-4    # max relative error, float32 path
TOL_BF16 = 2e-2   # bf16 inputs, float32 accumulation


def slice_rel_err(got: np.ndarray, ref: np.ndarray, lead: int = 1) -> float:
    """Largest, over the leading `lead` index dimensions, of max|got - ref| / max|ref| within the
    slice.  A slice whose reference is identically zero must be identically zero."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    n = int(np.prod(ref.shape[:lead])) if lead else 1
    g = np.asarray(got, dtype=np.float64).reshape(n, -1)
    r = np.asarray(ref, dtype=np.float64).reshape(n, -1)
    assert np.isfinite(g).all(), "non-finite values in the GPU result"
    num = np.abs(g - r).max(axis=1)
    den = np.abs(r).max(axis=1)
    zero = den == 0.0
    assert (num[zero] == 0.0).all(), "a slice that must be exactly zero is not"
    out = np.zeros(n)
    out[~zero] = num[~zero] / den[~zero]
    return float(out.max()) if n else 0.0


def hidden_margin(Ws, bs, X, act_fn):
    """Smallest |pre-activation| over all hidden units (numpy float64 forward)."""
    a = np.asarray(X, dtype=np.float64)
    m = np.inf
    for l in range(len(Ws) - 1):
        z = a @ np.asarray(Ws[l], dtype=np.float64) + np.asarray(bs[l], dtype=np.float64)
        m = min(m, float(np.abs(z).min()))
        a = act_fn(z)
    return m
