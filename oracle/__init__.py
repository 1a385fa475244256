"""float64 CPU oracle (test infrastructure, not product code).

Only ``tests/``, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may import
this package.  It is independent of the HIP library: it neither imports nor is imported by it.

The arithmetic lives in ``pfg_oracle.c`` (dense networks; plain C, literal loops over examples and
seed rows), ``lstm_oracle.c`` (the unrolled LSTM, wrapped by ``oracle.lstm``), ``conv_oracle.c`` (the small
convolutional network, wrapped by ``oracle.conv``) and ``cond_oracle.c`` (a loop body with a
conditional, wrapped by ``oracle.cond``); this module only
builds them with gcc, loads the first through ctypes and marshals numpy arrays.
Every array that crosses this boundary is float64 (labels: int32).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pfg_oracle.c")
_LIB = os.path.join(_HERE, "libpfg_oracle.so")

ACT = {"identity": 0, "relu": 1, "tanh": 2, "gelu": 3}
HEAD = {"logits": 0, "softmax": 1}

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_int32_p = ctypes.POINTER(ctypes.c_int32)


class _Net(ctypes.Structure):
    _fields_ = [
        ("L", ctypes.c_int32),
        ("dims", _c_int32_p),
        ("W", ctypes.POINTER(_c_double_p)),
        ("b", ctypes.POINTER(_c_double_p)),
        ("act", ctypes.c_int32),
    ]


def compile_source(src: str, lib: str) -> None:
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-o", lib, src, "-lm"]
    subprocess.run(cmd, check=True)


def build(force: bool = False) -> str:
    """Compile the C oracles with gcc (OpenMP only parallelises the outermost pfor index)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    from . import cond, conv, lstm
    lstm.build(force)
    conv.build(force)
    cond.build(force)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # PFG_ORACLE_LIB: a deliberately broken build, used only by the mutation test that
        # checks the pins have teeth
        path = os.environ.get("PFG_ORACLE_LIB") or build()
        lib = ctypes.CDLL(path)
        lib.pfgo_act.restype = ctypes.c_double
        lib.pfgo_act.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.pfgo_act_deriv.restype = ctypes.c_double
        lib.pfgo_act_deriv.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.pfgo_act_deriv2.restype = ctypes.c_double
        lib.pfgo_act_deriv2.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.pfgo_loss.restype = ctypes.c_double
        lib.pfgo_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dp(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_c_double_p) if a is not None else _c_double_p()


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


class Net:
    """A dense network held as float64 arrays: W_l [d_{l-1}, d_l] row-major, b_l [d_l] or None."""

    def __init__(self, Ws: Sequence[np.ndarray], bs: Optional[Sequence[Optional[np.ndarray]]],
                 act: str):
        self.Ws = [_f64(W) for W in Ws]
        self.L = len(self.Ws)
        assert self.L >= 1
        self.bs = [None] * self.L if bs is None else [None if b is None else _f64(b) for b in bs]
        self.dims = [self.Ws[0].shape[0]] + [W.shape[1] for W in self.Ws]
        for l, W in enumerate(self.Ws):
            assert W.shape == (self.dims[l], self.dims[l + 1])
            assert self.bs[l] is None or self.bs[l].shape == (self.dims[l + 1],)
        self.act = act
        self._dims_arr = np.asarray(self.dims, dtype=np.int32)
        self._Wp = (_c_double_p * self.L)(*[_dp(W) for W in self.Ws])
        self._bp = (_c_double_p * self.L)(*[_dp(b) for b in self.bs])
        self.c = _Net(self.L, self._dims_arr.ctypes.data_as(_c_int32_p), self._Wp, self._bp,
                      ACT[act])


def num_threads() -> int:
    return int(_load().pfgo_num_threads())


def act(name: str, z: float) -> float:
    return float(_load().pfgo_act(ACT[name], float(z)))


def act_deriv(name: str, z: float) -> float:
    return float(_load().pfgo_act_deriv(ACT[name], float(z)))


def act_deriv2(name: str, z: float) -> float:
    return float(_load().pfgo_act_deriv2(ACT[name], float(z)))


def forward(net: Net, x) -> np.ndarray:
    """Logits of one example."""
    x = _f64(x)
    assert x.shape == (net.dims[0],)
    y = np.empty(net.dims[-1], dtype=np.float64)
    _load().pfgo_forward(ctypes.byref(net.c), _dp(x), _dp(y))
    return y


def loss(net: Net, x, label: int) -> float:
    x = _f64(x)
    assert x.shape == (net.dims[0],) and 0 <= int(label) < net.dims[-1]
    return float(_load().pfgo_loss(ctypes.byref(net.c), _dp(x), ctypes.c_int(int(label))))


def softmax(y) -> np.ndarray:
    y = _f64(y)
    p = np.empty_like(y)
    _load().pfgo_softmax(_dp(y), ctypes.c_int(y.size), _dp(p))
    return p


def _ptr_array(arrs: List[Optional[np.ndarray]]):
    return (_c_double_p * len(arrs))(*[_dp(a) for a in arrs])


def per_example_grads(net: Net, X, labels, want_dW: Optional[Sequence[bool]] = None):
    """pfor over examples of body = gradients(loss of one example).

    Returns (dW list of [B, d_{l-1}, d_l] or None, db list of [B, d_l], loss [B])."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.dims[0])
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (B,) and (labels >= 0).all() and (labels < net.dims[-1]).all()
    want = [True] * net.L if want_dW is None else list(want_dW)
    dW = [np.empty((B, net.dims[l], net.dims[l + 1])) if want[l] else None for l in range(net.L)]
    db = [np.empty((B, net.dims[l + 1])) for l in range(net.L)]
    ls = np.empty(B)
    _load().pfgo_per_example_grads(ctypes.byref(net.c), _dp(X),
                                   labels.ctypes.data_as(_c_int32_p), ctypes.c_int64(B),
                                   _ptr_array(dW), _ptr_array(db), _dp(ls))
    return dW, db, ls


def body_per_example_grads(net: Net, x, label: int):
    """One iteration of the per-example-gradient parfor (one example)."""
    x = _f64(x)
    dW = [np.empty((net.dims[l], net.dims[l + 1])) for l in range(net.L)]
    db = [np.empty((net.dims[l + 1],)) for l in range(net.L)]
    ls = ctypes.c_double(0.0)
    _load().pfgo_body_per_example_grads(ctypes.byref(net.c), _dp(x), ctypes.c_int(int(label)),
                                        _ptr_array(dW), _ptr_array(db), ctypes.byref(ls))
    return dW, db, float(ls.value)


def _seed_args(net: Net, B: int, seeds, S: Optional[int]):
    dL = net.dims[-1]
    if seeds is None:
        S = dL if S is None else S
        assert S == dL, "identity seeds need S == d_L"
        return None, S, 0
    seeds = _f64(seeds)
    if seeds.ndim == 2:
        assert seeds.shape[1] == dL
        return seeds, seeds.shape[0], 0
    assert seeds.ndim == 3 and seeds.shape[0] == B and seeds.shape[2] == dL
    return seeds, seeds.shape[1], seeds.shape[1] * dL


def jacobian_input(net: Net, X, seeds=None, S: Optional[int] = None) -> np.ndarray:
    """J[b, s, :] = gradient of <seed row s, y_b> with respect to x_b.  seeds: None (identity),
    [S, d_L] shared by every example, or [B, S, d_L]."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.dims[0])
    seeds, S, stride = _seed_args(net, B, seeds, S)
    J = np.empty((B, S, net.dims[0]))
    _load().pfgo_jacobian_input(ctypes.byref(net.c), _dp(X), ctypes.c_int64(B), _dp(seeds),
                                ctypes.c_int64(S), ctypes.c_int64(stride), _dp(J))
    return J


def body_jacobian_input_row(net: Net, x, seed_row) -> np.ndarray:
    """One iteration of the Jacobian parfor: gradient of <seed_row, y(x)> with respect to x."""
    x = _f64(x)
    seed_row = _f64(seed_row)
    assert seed_row.shape == (net.dims[-1],)
    row = np.empty(net.dims[0])
    _load().pfgo_body_jacobian_input_row(ctypes.byref(net.c), _dp(x), _dp(seed_row), _dp(row))
    return row


def jacobian_weights(net: Net, X, head: str = "logits", seeds=None, S: Optional[int] = None,
                     want_JW: Optional[Sequence[bool]] = None):
    """JW_l[b, k] = gradient of scalar k of example b (see pfg_oracle.c) w.r.t. W_l; Jb_l likewise.

    Returns (JW list of [B, S, d_{l-1}, d_l] or None, Jb list of [B, S, d_l])."""
    X = _f64(X)
    B = X.shape[0]
    seeds, S, stride = _seed_args(net, B, seeds, S)
    want = [True] * net.L if want_JW is None else list(want_JW)
    JW = [np.empty((B, S, net.dims[l], net.dims[l + 1])) if want[l] else None
          for l in range(net.L)]
    Jb = [np.empty((B, S, net.dims[l + 1])) for l in range(net.L)]
    _load().pfgo_jacobian_weights(ctypes.byref(net.c), _dp(X), ctypes.c_int64(B),
                                  ctypes.c_int(HEAD[head]), _dp(seeds), ctypes.c_int64(S),
                                  ctypes.c_int64(stride), _ptr_array(JW), _ptr_array(Jb))
    return JW, Jb


def per_example_grad_norms(net: Net, X, labels):
    """(sq_layers [B, L], norm [B]): squared gradient norm of every layer (weights plus the bias,
    where the layer has one) and the norm over all parameters, for each example's own loss."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.dims[0])
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (B,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < net.dims[-1]
    sq = np.empty((B, net.L))
    norm = np.empty(B)
    _load().pfgo_per_example_grad_norms(ctypes.byref(net.c), _dp(X),
                                        labels.ctypes.data_as(_c_int32_p), ctypes.c_int64(B),
                                        _dp(sq), _dp(norm))
    return sq, norm


def body_hessian_input_dir(net: Net, x, seed_row, j: int) -> np.ndarray:
    """One iteration of the Hessian parfor: d J[s, :] / d x[j] for one example and one seed row."""
    x = _f64(x)
    seed_row = _f64(seed_row)
    assert x.shape == (net.dims[0],) and seed_row.shape == (net.dims[-1],)
    assert 0 <= int(j) < net.dims[0]
    col = np.empty(net.dims[0])
    _load().pfgo_body_hessian_input_dir(ctypes.byref(net.c), _dp(x), _dp(seed_row),
                                        ctypes.c_int(int(j)), _dp(col))
    return col


def hessian_input(net: Net, X, seeds=None, S: Optional[int] = None) -> np.ndarray:
    """H[b, s, i, j] = d^2 <seed row s, y_b> / d x_b[i] d x_b[j], as [B, S, d_0, d_0]."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.dims[0])
    seeds, S, stride = _seed_args(net, B, seeds, S)
    H = np.empty((B, S, net.dims[0], net.dims[0]))
    _load().pfgo_hessian_input(ctypes.byref(net.c), _dp(X), ctypes.c_int64(B), _dp(seeds),
                               ctypes.c_int64(S), ctypes.c_int64(stride), _dp(H))
    return H


def softmax_jacobian_row(y, k: int) -> np.ndarray:
    y = _f64(y)
    row = np.empty_like(y)
    _load().pfgo_softmax_jacobian_row(_dp(y), ctypes.c_int(y.size), ctypes.c_int(int(k)),
                                      _dp(row))
    return row


def pfor_add_sub(a, b):
    """The worked example of Section 4: body(i) = (a[i] + b[i], a[i] - b[i]), stacked."""
    a, b = _f64(a), _f64(b)
    assert a.shape == b.shape and a.ndim == 2
    s, d = np.empty_like(a), np.empty_like(a)
    _load().pfgo_pfor_add_sub(_dp(a), _dp(b), ctypes.c_int64(a.shape[0]),
                              ctypes.c_int64(a.shape[1]), _dp(s), _dp(d))
    return s, d
