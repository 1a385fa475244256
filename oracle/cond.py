"""float64 CPU oracle for a parallel-for whose body holds a conditional (test infrastructure, not
product code).

The arithmetic lives in ``cond_oracle.c``; this module builds it with gcc, loads it through ctypes
and marshals numpy arrays (all float64).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
CPU-baseline leg of ``bench.py`` may import it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import Net, _Net, _c_double_p, _c_int32_p, _dp, _f64, compile_source

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cond_oracle.c")
_LIB = os.path.join(_HERE, "libcond_oracle.so")

PER_ITERATION = -1     # the condition depends on the iteration; 0 / 1: a loop-invariant value


class _Cond(ctypes.Structure):
    _fields_ = [("pre", ctypes.POINTER(_Net)), ("w", _c_double_p), ("c0", ctypes.c_double),
                ("then_net", ctypes.POINTER(_Net)), ("else_net", ctypes.POINTER(_Net))]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # PFG_COND_ORACLE_LIB: a deliberately broken build, used only by the mutation test
        lib = ctypes.CDLL(os.environ.get("PFG_COND_ORACLE_LIB") or build())
        lib.condo_score.restype = ctypes.c_double
        lib.condo_body.restype = ctypes.c_int
        _lib = lib
    return _lib


class Cond:
    """body(x): t = phi_pre(pre(x)); if t . w + c0 > 0: then_net(t) else: else_net(t).
    pre, then_net and else_net are ``oracle.Net`` objects."""

    def __init__(self, pre: Net, w, c0: float, then_net: Net, else_net: Net):
        self.pre, self.then_net, self.else_net = pre, then_net, else_net
        self.w = _f64(w)
        self.c0 = float(c0)
        self.d0, self.dT, self.dout = pre.dims[0], pre.dims[-1], then_net.dims[-1]
        assert self.w.shape == (self.dT,)
        assert then_net.dims[0] == self.dT and else_net.dims[0] == self.dT
        assert else_net.dims[-1] == self.dout
        self.c = _Cond(ctypes.pointer(pre.c), _dp(self.w), self.c0, ctypes.pointer(then_net.c),
                       ctypes.pointer(else_net.c))


def _row(net: Cond, x) -> np.ndarray:
    x = _f64(x)
    assert x.shape == (net.d0,)
    return x


def pre(net: Cond, x) -> np.ndarray:
    t = np.empty(net.dT)
    _load().condo_pre(ctypes.byref(net.c), _dp(_row(net, x)), _dp(t))
    return t


def score(net: Cond, x) -> float:
    return float(_load().condo_score(ctypes.byref(net.c), _dp(_row(net, x))))


def branch(net: Cond, x, which: bool) -> np.ndarray:
    """The then (which true) or else branch applied to one example regardless of its condition."""
    r = np.empty(net.dout)
    _load().condo_branch(ctypes.byref(net.c), _dp(_row(net, x)), ctypes.c_int(1 if which else 0), _dp(r))
    return r


def body(net: Cond, x, invariant: int = PER_ITERATION):
    """One iteration: (result [d_out], condition)."""
    r = np.empty(net.dout)
    c = _load().condo_body(ctypes.byref(net.c), _dp(_row(net, x)), ctypes.c_int(int(invariant)), _dp(r))
    return r, bool(c)


def forward(net: Cond, X, invariant: int = PER_ITERATION):
    """pfor over the rows of X: (R [n, d_out], cond [n] int32)."""
    X = _f64(X)
    n = X.shape[0]
    assert X.shape == (n, net.d0)
    R = np.empty((n, net.dout))
    cond = np.empty(n, dtype=np.int32)
    _load().condo_forward(ctypes.byref(net.c), _dp(X), ctypes.c_int64(n), ctypes.c_int(int(invariant)),
                          _dp(R), cond.ctypes.data_as(_c_int32_p))
    return R, cond


def per_example_grads(net: Cond, X, labels, invariant: int = PER_ITERATION):
    """pfor over the rows of X of body = gradients(softmax cross-entropy of the iteration's own
    result).  Returns a dict with, for each of "pre", "then", "else", the lists dW [n, d_{l-1}, d_l]
    and db [n, d_l] (an iteration's gradient for the branch it did not take is zero), plus
    "loss" [n] and "cond" [n] int32."""
    X = _f64(X)
    n = X.shape[0]
    assert X.shape == (n, net.d0)
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (n,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < net.dout
    out, args, keep = {}, [], []
    for name, m in (("pre", net.pre), ("then", net.then_net), ("else", net.else_net)):
        dW = [np.empty((n, m.dims[l], m.dims[l + 1])) for l in range(m.L)]
        db = [np.empty((n, m.dims[l + 1])) for l in range(m.L)]
        out[name] = (dW, db)
        for arrs in (dW, db):
            p = (_c_double_p * m.L)(*[_dp(a) for a in arrs])
            keep.append(p)
            args.append(p)
    loss = np.empty(n)
    cond = np.empty(n, dtype=np.int32)
    _load().condo_per_example_grads(ctypes.byref(net.c), _dp(X), labels.ctypes.data_as(_c_int32_p),
                                    ctypes.c_int64(n), ctypes.c_int(int(invariant)), *args, _dp(loss),
                                    cond.ctypes.data_as(_c_int32_p))
    out["loss"], out["cond"] = loss, cond
    return out
