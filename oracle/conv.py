"""float64 CPU oracle for the small convolutional network (test infrastructure, not product code).

The arithmetic lives in ``conv_oracle.c``; this module builds it with gcc, loads it through ctypes
and marshals numpy arrays (all float64, labels int32).  Only ``tests/``,
``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may import it.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

from . import _c_double_p, _c_int32_p, _dp, _f64, _ptr_array, compile_source

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")


class _Net(ctypes.Structure):
    _fields_ = [("height", ctypes.c_int32), ("width", ctypes.c_int32), ("channels", ctypes.c_int32),
                ("num_conv", ctypes.c_int32), ("kernel", _c_int32_p), ("filters", _c_int32_p),
                ("Wc", ctypes.POINTER(_c_double_p)), ("bc", ctypes.POINTER(_c_double_p)),
                ("L", ctypes.c_int32), ("dims", _c_int32_p),
                ("W", ctypes.POINTER(_c_double_p)), ("b", ctypes.POINTER(_c_double_p))]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # PFG_CONV_ORACLE_LIB: a deliberately broken build, used only by the mutation test
        lib = ctypes.CDLL(os.environ.get("PFG_CONV_ORACLE_LIB") or build())
        lib.convo_loss.restype = ctypes.c_double
        _lib = lib
    return _lib


class ConvNet:
    """Conv blocks (k x k "same" convolution + bias + ReLU + 2 x 2 max-pooling) followed by dense
    layers (ReLU between them).  Wc[i] is [k, k, c_in, c_out], bc[i] [c_out] or None; Ws[l] is
    [d_l, d_{l+1}], bs[l] [d_{l+1}] or None.  Images are [height, width, channels]."""

    def __init__(self, height: int, width: int, channels: int, Wc: Sequence, bc, Ws: Sequence, bs):
        self.height, self.width, self.channels = int(height), int(width), int(channels)
        self.Wc = [_f64(W) for W in Wc]
        self.nc = len(self.Wc)
        self.bc = [None] * self.nc if bc is None else [None if v is None else _f64(v) for v in bc]
        self.Ws = [_f64(W) for W in Ws]
        self.L = len(self.Ws)
        self.bs = [None] * self.L if bs is None else [None if v is None else _f64(v) for v in bs]
        h, w, c = self.height, self.width, self.channels
        self.kernel, self.filters, self.block_in = [], [], []
        for i, W in enumerate(self.Wc):
            k = W.shape[0]
            assert W.shape[:3] == (k, k, c) and k % 2 == 1 and h % 2 == 0 and w % 2 == 0, W.shape
            assert self.bc[i] is None or self.bc[i].shape == (W.shape[3],)
            self.block_in.append((h, w, c))
            self.kernel.append(k)
            self.filters.append(W.shape[3])
            h, w, c = h // 2, w // 2, W.shape[3]
        self.dims = [self.Ws[0].shape[0]] + [W.shape[1] for W in self.Ws]
        assert self.nc >= 1 and self.L >= 1 and self.dims[0] == h * w * c, (self.dims[0], h, w, c)
        for l, W in enumerate(self.Ws):
            assert W.shape == (self.dims[l], self.dims[l + 1])
            assert self.bs[l] is None or self.bs[l].shape == (self.dims[l + 1],)
        self._kernel = np.asarray(self.kernel, dtype=np.int32)
        self._filters = np.asarray(self.filters, dtype=np.int32)
        self._dims = np.asarray(self.dims, dtype=np.int32)
        self._Wcp = (_c_double_p * self.nc)(*[_dp(W) for W in self.Wc])
        self._bcp = (_c_double_p * self.nc)(*[_dp(v) for v in self.bc])
        self._Wp = (_c_double_p * self.L)(*[_dp(W) for W in self.Ws])
        self._bp = (_c_double_p * self.L)(*[_dp(v) for v in self.bs])
        self.c = _Net(self.height, self.width, self.channels, self.nc,
                      self._kernel.ctypes.data_as(_c_int32_p), self._filters.ctypes.data_as(_c_int32_p),
                      self._Wcp, self._bcp, self.L, self._dims.ctypes.data_as(_c_int32_p), self._Wp,
                      self._bp)


def _img(net: ConvNet, x) -> np.ndarray:
    x = _f64(x)
    assert x.shape == (net.height, net.width, net.channels)
    return x


def forward(net: ConvNet, x) -> np.ndarray:
    y = np.empty(net.dims[-1])
    _load().convo_forward(ctypes.byref(net.c), _dp(_img(net, x)), _dp(y))
    return y


def features(net: ConvNet, x) -> np.ndarray:
    """Flattened output of the last conv block."""
    f = np.empty(net.dims[0])
    _load().convo_features(ctypes.byref(net.c), _dp(_img(net, x)), _dp(f))
    return f


def loss(net: ConvNet, x, label: int) -> float:
    assert 0 <= int(label) < net.dims[-1]
    return float(_load().convo_loss(ctypes.byref(net.c), _dp(_img(net, x)), ctypes.c_int(int(label))))


def per_example_grads(net: ConvNet, X, labels, want_dW: Optional[Sequence[bool]] = None):
    """(dWc list [B, k, k, c_in, c_out], dbc list [B, c_out], dW list [B, d_l, d_{l+1}] or None,
    db list [B, d_{l+1}], loss [B])."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.height, net.width, net.channels)
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (B,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < net.dims[-1]
    want = [True] * net.L if want_dW is None else list(want_dW)
    dWc = [np.empty((B,) + W.shape) for W in net.Wc]
    dbc = [np.empty((B, W.shape[3])) for W in net.Wc]
    dW: List[Optional[np.ndarray]] = [np.empty((B, net.dims[l], net.dims[l + 1])) if want[l] else None
                                      for l in range(net.L)]
    db = [np.empty((B, net.dims[l + 1])) for l in range(net.L)]
    ls = np.empty(B)
    _load().convo_per_example_grads(ctypes.byref(net.c), _dp(X), labels.ctypes.data_as(_c_int32_p),
                                    ctypes.c_int64(B), _ptr_array(dWc), _ptr_array(dbc),
                                    _ptr_array(dW), _ptr_array(db), _dp(ls))
    return dWc, dbc, dW, db, ls


def per_example_grad_norms(net: ConvNet, X, labels):
    """(sq [B, num_conv + L], norm [B], loss [B]): squared norm of every parameter block's
    per-example gradient (a block = a filter or weight matrix together with its bias, when it has
    one; conv blocks first), and the norm of the whole gradient."""
    X = _f64(X)
    B = X.shape[0]
    assert X.shape == (B, net.height, net.width, net.channels)
    labels = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    assert labels.shape == (B,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < net.dims[-1]
    sq = np.empty((B, net.nc + net.L))
    norm = np.empty(B)
    ls = np.empty(B)
    _load().convo_per_example_grad_norms(ctypes.byref(net.c), _dp(X), labels.ctypes.data_as(_c_int32_p),
                                         ctypes.c_int64(B), _dp(sq), _dp(norm), _dp(ls))
    return sq, norm, ls
