"""float64 CPU oracle for the unrolled LSTM (test infrastructure, not product code).

The arithmetic lives in ``lstm_oracle.c``; this module builds it with gcc, loads it through ctypes
and marshals numpy arrays (all float64, labels int32).  Only ``tests/``,
``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may import it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import _c_double_p, _c_int32_p, _dp, _f64, compile_source

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lstm_oracle.c")
_LIB = os.path.join(_HERE, "liblstm_oracle.so")


class _Net(ctypes.Structure):
    _fields_ = [("dx", ctypes.c_int32), ("H", ctypes.c_int32), ("dy", ctypes.c_int32),
                ("T", ctypes.c_int32), ("W", _c_double_p), ("b", _c_double_p),
                ("Wout", _c_double_p), ("bout", _c_double_p)]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # PFG_LSTM_ORACLE_LIB: a deliberately broken build, used only by the mutation test
        lib = ctypes.CDLL(os.environ.get("PFG_LSTM_ORACLE_LIB") or build())
        lib.lstmo_loss.restype = ctypes.c_double
        _lib = lib
    return _lib


class Lstm:
    """W [dx + H, 4H] (column blocks i, g, f, o), b [4H] or None, Wout [H, dy], bout [dy] or None,
    unrolled to T steps."""

    def __init__(self, W, b, Wout, bout, T: int):
        self.W, self.Wout = _f64(W), _f64(Wout)
        self.b = None if b is None else _f64(b)
        self.bout = None if bout is None else _f64(bout)
        self.H, self.dy = self.Wout.shape
        self.dx = self.W.shape[0] - self.H
        self.T = int(T)
        assert self.dx >= 1 and self.T >= 1 and self.W.shape == (self.dx + self.H, 4 * self.H)
        assert self.b is None or self.b.shape == (4 * self.H,)
        assert self.bout is None or self.bout.shape == (self.dy,)
        self.c = _Net(self.dx, self.H, self.dy, self.T, _dp(self.W), _dp(self.b), _dp(self.Wout),
                      _dp(self.bout))


def _seq(net: Lstm, x) -> np.ndarray:
    x = _f64(x)
    assert x.shape == (net.T, net.dx)
    return x


def forward(net: Lstm, x) -> np.ndarray:
    y = np.empty(net.dy)
    _load().lstmo_forward(ctypes.byref(net.c), _dp(_seq(net, x)), _dp(y))
    return y


def states(net: Lstm, x):
    """(h [T, H], c [T, H]) after every step."""
    h, c = np.empty((net.T, net.H)), np.empty((net.T, net.H))
    _load().lstmo_states(ctypes.byref(net.c), _dp(_seq(net, x)), _dp(h), _dp(c))
    return h, c


def loss(net: Lstm, x, label: int) -> float:
    assert 0 <= int(label) < net.dy
    return float(_load().lstmo_loss(ctypes.byref(net.c), _dp(_seq(net, x)), ctypes.c_int(int(label))))


def _labels(net: Lstm, labels, B: int) -> np.ndarray:
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (B,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < net.dy
    return labels


def per_example_grads(net: Lstm, X, labels, want_dW: bool = True):
    """(dW [B, dx+H, 4H] or None, db [B, 4H], dWout [B, H, dy], dbout [B, dy], loss [B])."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.T, net.dx)
    labels = _labels(net, labels, B)
    dW = np.empty((B, net.dx + net.H, 4 * net.H)) if want_dW else None
    db = np.empty((B, 4 * net.H))
    dWout = np.empty((B, net.H, net.dy))
    dbout = np.empty((B, net.dy))
    ls = np.empty(B)
    _load().lstmo_per_example_grads(ctypes.byref(net.c), _dp(X), labels.ctypes.data_as(_c_int32_p),
                                    ctypes.c_int64(B), _dp(dW), _dp(db), _dp(dWout), _dp(dbout),
                                    _dp(ls))
    return dW, db, dWout, dbout, ls


def per_example_grad_norms(net: Lstm, X, labels):
    """(sq [B, 4] = squared norms of dW, db, dWout, dbout; norm [B]; loss [B])."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.T, net.dx)
    labels = _labels(net, labels, B)
    sq, norm, ls = np.empty((B, 4)), np.empty(B), np.empty(B)
    _load().lstmo_per_example_grad_norms(ctypes.byref(net.c), _dp(X), labels.ctypes.data_as(_c_int32_p),
                                         ctypes.c_int64(B), _dp(sq), _dp(norm), _dp(ls))
    return sq, norm, ls


def body_per_example_grads(net: Lstm, x, label: int):
    dW = np.empty((net.dx + net.H, 4 * net.H))
    db = np.empty(4 * net.H)
    dWout = np.empty((net.H, net.dy))
    dbout = np.empty(net.dy)
    ls = ctypes.c_double(0.0)
    _load().lstmo_body_per_example_grads(ctypes.byref(net.c), _dp(_seq(net, x)),
                                         ctypes.c_int(int(label)), _dp(dW), _dp(db), _dp(dWout),
                                         _dp(dbout), ctypes.byref(ls))
    return dW, db, dWout, dbout, float(ls.value)


def _seed_args(net: Lstm, B: int, seeds, S: Optional[int]):
    if seeds is None:
        S = net.dy if S is None else S
        assert S == net.dy, "identity seeds need S == dy"
        return None, S, 0
    seeds = _f64(seeds)
    if seeds.ndim == 2:
        assert seeds.shape[1] == net.dy
        return seeds, seeds.shape[0], 0
    assert seeds.ndim == 3 and seeds.shape[0] == B and seeds.shape[2] == net.dy
    return seeds, seeds.shape[1], seeds.shape[1] * net.dy


def jacobian_input(net: Lstm, X, seeds=None, S: Optional[int] = None) -> np.ndarray:
    """J[b, s, t, :] = gradient of <seed row s, y_b> with respect to x_b[t, :], [B, S, T, dx]."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.T, net.dx)
    seeds, S, stride = _seed_args(net, B, seeds, S)
    J = np.empty((B, S, net.T, net.dx))
    _load().lstmo_jacobian_input(ctypes.byref(net.c), _dp(X), ctypes.c_int64(B), _dp(seeds),
                                 ctypes.c_int64(S), ctypes.c_int64(stride), _dp(J))
    return J


def body_jacobian_input_row(net: Lstm, x, seed_row) -> np.ndarray:
    seed_row = _f64(seed_row)
    assert seed_row.shape == (net.dy,)
    row = np.empty((net.T, net.dx))
    _load().lstmo_body_jacobian_input_row(ctypes.byref(net.c), _dp(_seq(net, x)), _dp(seed_row),
                                          _dp(row))
    return row


def varlen_forward(net: Lstm, X, lengths):
    """Every sequence iterated to its own length.  X [sum(lengths), dx] holds the tokens back to
    back.  Returns (h [B, H], y [B, dy]): the last hidden state of each sequence and its readout."""
    lengths = np.asarray(lengths, dtype=np.int64)
    assert lengths.ndim == 1 and (lengths >= 1).all()
    B = lengths.size
    offsets = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    X = _f64(X)
    assert X.shape == (int(offsets[-1]), net.dx)
    h, y = np.empty((B, net.H)), np.empty((B, net.dy))
    _load().lstmo_varlen_forward(ctypes.byref(net.c), _dp(X),
                                 offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                 ctypes.c_int64(B), _dp(h), _dp(y))
    return h, y


def while_forward(net: Lstm, X, lengths, max_steps: int, halt_w=None, halt_c: float = 0.0):
    """Every sequence iterated while it has tokens left, the cap max_steps is not reached and the
    halting score halt_c + <h, halt_w> of its current state is not positive (see lstm_oracle.c).
    lengths may hold zeros.  Returns (h [B, H], y [B, dy], steps [B] int64)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    assert lengths.ndim == 1 and (lengths >= 0).all()
    B = lengths.size
    offsets = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    X = _f64(X).reshape(-1, net.dx)
    assert X.shape == (int(offsets[-1]), net.dx)
    hw = None if halt_w is None else _f64(halt_w)
    assert hw is None or hw.shape == (net.H,)
    h, y = np.empty((B, net.H)), np.empty((B, net.dy))
    steps = np.empty(B, dtype=np.int64)
    _load().lstmo_while_forward(ctypes.byref(net.c), _dp(X),
                                offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                ctypes.c_int64(B), ctypes.c_int64(int(max_steps)), _dp(hw),
                                ctypes.c_double(float(halt_c)), _dp(h), _dp(y),
                                steps.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
    return h, y, steps


def while_per_example_grads(net: Lstm, X, lengths, labels, max_steps: int, halt_w=None, halt_c: float = 0.0):
    """Per-example gradients of -log softmax(y)[label] through the while loop of ``while_forward``
    (see lstm_oracle.c).  Returns dict(dW [B, dx+H, 4H], db [B, 4H], dWout [B, H, dy], dbout [B, dy],
    loss [B], steps [B] int64)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    assert lengths.ndim == 1 and (lengths >= 0).all()
    B = lengths.size
    offsets = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    X = _f64(X).reshape(-1, net.dx)
    assert X.shape == (int(offsets[-1]), net.dx)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    assert labels.shape == (B,) and (labels >= 0).all() and (labels < net.dy).all()
    hw = None if halt_w is None else _f64(halt_w)
    assert hw is None or hw.shape == (net.H,)
    G = 4 * net.H
    out = dict(dW=np.empty((B, net.dx + net.H, G)), db=np.empty((B, G)), dWout=np.empty((B, net.H, net.dy)),
               dbout=np.empty((B, net.dy)), loss=np.empty(B), steps=np.empty(B, dtype=np.int64))
    _load().lstmo_while_per_example_grads(
        ctypes.byref(net.c), _dp(X), offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
        labels.ctypes.data_as(_c_int32_p), ctypes.c_int64(B), ctypes.c_int64(int(max_steps)), _dp(hw),
        ctypes.c_double(float(halt_c)), _dp(out["dW"]), _dp(out["db"]), _dp(out["dWout"]), _dp(out["dbout"]),
        _dp(out["loss"]), out["steps"].ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
    return out


def while_per_example_grad_norms(net: Lstm, X, lengths, labels, max_steps: int, halt_w=None, halt_c: float = 0.0):
    """Norms of the per-example gradients through the while loop (the gradient formed in full, its
    squares added; see lstm_oracle.c).  Returns (sq [B, 4] = squared norms of dW, db, dWout, dbout;
    norm [B]; loss [B]; steps [B] int64)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    assert lengths.ndim == 1 and (lengths >= 0).all()
    B = lengths.size
    offsets = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    X = _f64(X).reshape(-1, net.dx)
    assert X.shape == (int(offsets[-1]), net.dx)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    assert labels.shape == (B,) and (labels >= 0).all() and (labels < net.dy).all()
    hw = None if halt_w is None else _f64(halt_w)
    assert hw is None or hw.shape == (net.H,)
    sq, norm, ls = np.empty((B, 4)), np.empty(B), np.empty(B)
    steps = np.empty(B, dtype=np.int64)
    _load().lstmo_while_per_example_grad_norms(
        ctypes.byref(net.c), _dp(X), offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
        labels.ctypes.data_as(_c_int32_p), ctypes.c_int64(B), ctypes.c_int64(int(max_steps)), _dp(hw),
        ctypes.c_double(float(halt_c)), _dp(sq), _dp(norm), _dp(ls),
        steps.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
    return sq, norm, ls, steps
