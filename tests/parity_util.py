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


def outer_elem_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Element-wise measure for stacked outer products, shape [..., I, J] with every [I, J] slice of
    the reference a rank-one matrix a_i g_j: the largest |got - ref|_ij / (R_i + C_j), where
    R_i = max_j |ref_ij| and C_j = max_i |ref_ij| are the largest entry of the element's row and of
    its column.  A factor computed with an error that is small against the factor's largest entry
    (what fixed-order float32 sums deliver) gives |err_ij| <= eps_a max|a| |g_j| + eps_g |a_i| max|g|
    = eps_a C_j + eps_g R_i, so this ratio is bounded by the relative error of the factors; unlike the
    per-slice measure it holds an entry in a small row AND a small column to that small scale.
    (An entry-by-entry relative error is ill-posed here: a hidden activation or cotangent that is a
    sum of O(1) terms cancelling to 1e-6 carries O(1e-7) absolute round-off, unbounded against
    itself.)  Entries whose row and column are zero in the reference must be exactly zero."""
    assert got.shape == ref.shape and ref.ndim >= 3, (got.shape, ref.shape)
    g = np.asarray(got, dtype=np.float64).reshape((-1,) + ref.shape[-2:])
    r = np.abs(np.asarray(ref, dtype=np.float64).reshape(g.shape))
    err = np.abs(g - np.asarray(ref, dtype=np.float64).reshape(g.shape))
    scale = r.max(axis=2, keepdims=True) + r.max(axis=1, keepdims=True)
    dead = scale == 0.0
    assert (err[dead] == 0.0).all(), "an entry that must be exactly zero is not"
    scale[dead] = 1.0
    err /= scale
    return float(err.max())


def hidden_margin(Ws, bs, X, act_fn):
    """Smallest |pre-activation| over all hidden units (numpy float64 forward)."""
    a = np.asarray(X, dtype=np.float64)
    m = np.inf
    for l in range(len(Ws) - 1):
        z = a @ np.asarray(Ws[l], dtype=np.float64) + np.asarray(bs[l], dtype=np.float64)
        m = min(m, float(np.abs(z).min()))
        a = act_fn(z)
    return m
