"""Python binding of libpfg: per-example gradients and Jacobians of a dense network on MI355X.

This module only marshals arguments: it allocates outputs and workspace as torch tensors on the
GPU, passes raw device pointers and the current HIP stream to the C ABI declared in
``include/pfg.h``, and returns the tensors.  Every step of the computation runs in the library's
HIP kernels.  There is no CPU fallback: if ``libpfg.so`` is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpfg.so")

PFG_OK = 0
PFG_ERR_NULL, PFG_ERR_SHAPE, PFG_ERR_UNSUPPORTED = -1, -2, -3
PFG_ERR_WORKSPACE, PFG_ERR_OVERFLOW, PFG_ERR_DEVICE = -4, -5, -6
ACT = {"identity": 0, "relu": 1, "tanh": 2, "gelu": 3}
DTYPE = {"f32": 0, "bf16": 1}
HEAD = {"logits": 0, "softmax": 1}
OP = {"per_example_grads": 0, "jacobian_input": 1, "jacobian_weights": 2, "grad_norms": 3,
      "hessian_input": 4}

EXPORTS = ["pfg_workspace_bytes", "pfg_per_example_grads", "pfg_per_example_grads_static",
           "pfg_jacobian_input",
           "pfg_jacobian_weights", "pfg_per_example_grad_norms", "pfg_hessian_input",
           "pfg_lstm_workspace_bytes", "pfg_lstm_per_example_grads", "pfg_lstm_jacobian_input",
           "pfg_lstm_per_example_grad_norms",
           "pfg_lstm_varlen_workspace_bytes", "pfg_lstm_varlen_forward",
           "pfg_lstm_while_workspace_bytes", "pfg_lstm_while_forward",
           "pfg_lstm_while_grads_workspace_bytes", "pfg_lstm_while_per_example_grads",
           "pfg_lstm_while_per_example_grad_norms",
           "pfg_convnet_workspace_bytes", "pfg_convnet_per_example_grads",
           "pfg_convnet_grad_norms_workspace_bytes", "pfg_convnet_per_example_grad_norms",
           "pfg_cond_workspace_bytes", "pfg_cond_forward",
           "pfg_cond_grads_workspace_bytes", "pfg_cond_per_example_grads",
           "pfg_last_error", "pfg_timing_enable", "pfg_timing_reset",
           "pfg_timing_query", "pfg_timing_names", "pfg_fill_reference", "pfg_version"]


class PfgError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"pfg status {code}: {message}")
        self.code = code


class pfg_mlp(ctypes.Structure):
    _fields_ = [
        ("num_layers", ctypes.c_int32),
        ("dims", ctypes.POINTER(ctypes.c_int32)),
        ("W", ctypes.POINTER(ctypes.c_void_p)),
        ("b", ctypes.POINTER(ctypes.c_void_p)),
        ("hidden_act", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
    ]


class pfg_lstm(ctypes.Structure):
    _fields_ = [
        ("input_size", ctypes.c_int32),
        ("state_size", ctypes.c_int32),
        ("output_size", ctypes.c_int32),
        ("steps", ctypes.c_int32),
        ("W", ctypes.c_void_p),
        ("b", ctypes.c_void_p),
        ("W_out", ctypes.c_void_p),
        ("b_out", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
    ]


class pfg_convnet(ctypes.Structure):
    _fields_ = [
        ("height", ctypes.c_int32),
        ("width", ctypes.c_int32),
        ("channels", ctypes.c_int32),
        ("num_conv", ctypes.c_int32),
        ("kernel", ctypes.POINTER(ctypes.c_int32)),
        ("filters", ctypes.POINTER(ctypes.c_int32)),
        ("Wc", ctypes.POINTER(ctypes.c_void_p)),
        ("bc", ctypes.POINTER(ctypes.c_void_p)),
        ("dense", pfg_mlp),
    ]


class pfg_cond(ctypes.Structure):
    _fields_ = [
        ("pre", pfg_mlp),
        ("cond_w", ctypes.c_void_p),
        ("cond_c", ctypes.c_float),
        ("then_net", pfg_mlp),
        ("else_net", pfg_mlp),
    ]


LSTM_OP = {"per_example_grads": 0, "jacobian_input": 1, "grad_norms": 2}
PFG_COND_PER_ITERATION = -1

_lib = None


def load_library() -> ctypes.CDLL:
    """Load libpfg.so from the package directory (build it with ``build.py`` first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1903_04243_amd.build` "
                               "(there is no fallback path)")
        # torch first: it brings its own HIP runtime, and the library must bind to that one (a
        # second runtime loaded ahead of torch's would see no device)
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        netp = ctypes.POINTER(pfg_mlp)
        lib.pfg_workspace_bytes.argtypes = [netp, i32, i64, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_per_example_grads.argtypes = [netp, vp, vp, i64, ctypes.POINTER(vp),
                                              ctypes.POINTER(vp), vp, vp, ctypes.c_size_t, vp]
        lib.pfg_per_example_grads_static.argtypes = [netp, vp, vp, i64, ctypes.POINTER(vp),
                                                     ctypes.POINTER(vp), vp, vp]
        lib.pfg_jacobian_input.argtypes = [netp, vp, i64, vp, i64, i64, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_jacobian_weights.argtypes = [netp, vp, i64, i32, vp, i64, i64, ctypes.POINTER(vp),
                                             ctypes.POINTER(vp), vp, ctypes.c_size_t, vp]
        lib.pfg_per_example_grad_norms.argtypes = [netp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_hessian_input.argtypes = [netp, vp, i64, vp, i64, i64, vp, vp, ctypes.c_size_t, vp]
        lstmp = ctypes.POINTER(pfg_lstm)
        lib.pfg_lstm_workspace_bytes.argtypes = [lstmp, i32, i64, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_lstm_per_example_grads.argtypes = [lstmp, vp, vp, i64, vp, vp, vp, vp, vp, vp,
                                                   ctypes.c_size_t, vp]
        lib.pfg_lstm_jacobian_input.argtypes = [lstmp, vp, i64, vp, i64, i64, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_lstm_per_example_grad_norms.argtypes = [lstmp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_lstm_varlen_workspace_bytes.argtypes = [lstmp, i64, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_lstm_varlen_forward.argtypes = [lstmp, vp, ctypes.POINTER(ctypes.c_int32), i64, i64, vp,
                                                vp, vp, ctypes.c_size_t, vp]
        lib.pfg_lstm_while_workspace_bytes.argtypes = [lstmp, i64, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_lstm_while_forward.argtypes = [lstmp, vp, vp, i64, i64, ctypes.c_int32, vp, ctypes.c_float,
                                               vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_lstm_while_grads_workspace_bytes.argtypes = [lstmp, i64, i64, ctypes.c_int32,
                                                             ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_lstm_while_per_example_grads.argtypes = [lstmp, vp, vp, vp, i64, i64, ctypes.c_int32, vp,
                                                         ctypes.c_float, vp, vp, vp, vp, vp, vp, vp,
                                                         ctypes.c_size_t, vp]
        lib.pfg_lstm_while_per_example_grad_norms.argtypes = [lstmp, vp, vp, vp, i64, i64, ctypes.c_int32, vp,
                                                              ctypes.c_float, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        convp = ctypes.POINTER(pfg_convnet)
        lib.pfg_convnet_workspace_bytes.argtypes = [convp, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_convnet_per_example_grads.argtypes = [convp, vp, vp, i64, ctypes.POINTER(vp),
                                                      ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                      ctypes.POINTER(vp), vp, vp, ctypes.c_size_t, vp]
        lib.pfg_convnet_grad_norms_workspace_bytes.argtypes = [convp, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_convnet_per_example_grad_norms.argtypes = [convp, vp, vp, i64, vp, vp, vp, vp,
                                                           ctypes.c_size_t, vp]
        condp = ctypes.POINTER(pfg_cond)
        lib.pfg_cond_workspace_bytes.argtypes = [condp, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_cond_forward.argtypes = [condp, vp, i64, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.pfg_fill_reference.argtypes = [vp, i64, ctypes.c_float, i32, vp]
        pvp = ctypes.POINTER(vp)
        lib.pfg_cond_grads_workspace_bytes.argtypes = [condp, i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.pfg_cond_per_example_grads.argtypes = [condp, vp, vp, i64, i32, pvp, pvp, pvp, pvp, pvp, pvp, vp, vp, vp,
                                                   vp, ctypes.c_size_t, vp]
        lib.pfg_last_error.restype = ctypes.c_char_p
        lib.pfg_timing_enable.argtypes = [i32]
        lib.pfg_timing_query.argtypes = [ctypes.c_char_p, ctypes.POINTER(i64),
                                         ctypes.POINTER(ctypes.c_double)]
        lib.pfg_timing_names.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
        _lib = lib
    return _lib


def _check(rc: int) -> None:
    if rc != PFG_OK:
        raise PfgError(rc, load_library().pfg_last_error().decode())


def pfg_last_error() -> str:
    return load_library().pfg_last_error().decode()


def pfg_version() -> int:
    return int(load_library().pfg_version())


class Mlp:
    """Device-resident network: ``Ws[l]`` is a contiguous [d_l, d_{l+1}] tensor (float32, or
    bfloat16 for dtype "bf16"), ``bs[l]`` a [d_{l+1}] tensor or None."""

    def __init__(self, Ws: Sequence, bs: Optional[Sequence], act: str, dtype: str = "f32"):
        import torch
        want = torch.float32 if dtype == "f32" else torch.bfloat16
        self.Ws = list(Ws)
        self.L = len(self.Ws)
        self.bs = [None] * self.L if bs is None else list(bs)
        for t in self.Ws + [b for b in self.bs if b is not None]:
            if t.dtype != want or not t.is_contiguous() or not t.is_cuda:
                raise ValueError("weights must be contiguous GPU tensors of the network dtype")
        self.dims = [self.Ws[0].shape[0]] + [W.shape[1] for W in self.Ws]
        for l, W in enumerate(self.Ws):
            if tuple(W.shape) != (self.dims[l], self.dims[l + 1]):
                raise ValueError(f"W[{l}] has shape {tuple(W.shape)}")
            if self.bs[l] is not None and tuple(self.bs[l].shape) != (self.dims[l + 1],):
                raise ValueError(f"b[{l}] has shape {tuple(self.bs[l].shape)}")
        self.act, self.dtype = act, dtype
        self.device = self.Ws[0].device
        self._dims = (ctypes.c_int32 * (self.L + 1))(*self.dims)
        self._W = (ctypes.c_void_p * self.L)(*[W.data_ptr() for W in self.Ws])
        self._b = (ctypes.c_void_p * self.L)(*[None if b is None else b.data_ptr()
                                               for b in self.bs])
        self.c = pfg_mlp(self.L, self._dims, self._W, self._b, ACT[act], DTYPE[dtype])

    @staticmethod
    def from_numpy(Ws, bs, act: str, dtype: str = "f32", Ws_bits=None, bs_bits=None,
                   device: str = "cuda:0") -> "Mlp":
        """Upload host arrays.  For bf16 pass the uint16 bit patterns in ``Ws_bits``/``bs_bits``."""
        import torch
        if dtype == "f32":
            tW = [torch.from_numpy(W).to(device) for W in Ws]
            tb = None if bs is None else [None if b is None else torch.from_numpy(b).to(device)
                                          for b in bs]
        else:
            tW = [torch.from_numpy(w.view("int16")).to(device).view(torch.bfloat16) for w in Ws_bits]
            tb = None if bs_bits is None else [
                None if b is None else torch.from_numpy(b.view("int16")).to(device).view(torch.bfloat16)
                for b in bs_bits]
        return Mlp(tW, tb, act, dtype)


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptrs(tensors: Sequence):
    return (ctypes.c_void_p * len(tensors))(*[None if t is None else t.data_ptr() for t in tensors])


def pfg_workspace_bytes(net: Mlp, op: str, B: int, S: int = 1) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_workspace_bytes(ctypes.byref(net.c), OP[op], B, S, ctypes.byref(n)))
    return int(n.value)


def _workspace(net: Mlp, op: str, B: int, S: int, workspace):
    import torch
    need = pfg_workspace_bytes(net, op, B, S)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=net.device)
    return workspace, workspace.numel() * workspace.element_size()


def _check_x(net: Mlp, X):
    import torch
    want = torch.float32 if net.dtype == "f32" else torch.bfloat16
    if X.dtype != want or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.dims[0]:
        raise ValueError("X must be a contiguous [B, d_0] tensor of the network dtype")


def pfg_per_example_grads(net: Mlp, X, labels, want_dW: Optional[Sequence[bool]] = None,
                          want_db: bool = True, want_loss: bool = True, out_dW=None, out_db=None,
                          out_loss=None, workspace=None):
    """Returns (dW list [B, d_{l-1}, d_l] or None per layer, db list [B, d_l] or None, loss [B] or
    None).  ``out_*`` reuse caller tensors instead of allocating."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    want = [True] * net.L if want_dW is None else list(want_dW)
    f32 = dict(dtype=torch.float32, device=net.device)
    dW = out_dW if out_dW is not None else [
        torch.empty((B, net.dims[l], net.dims[l + 1]), **f32) if want[l] else None
        for l in range(net.L)]
    db = out_db if out_db is not None else (
        [torch.empty((B, net.dims[l + 1]), **f32) for l in range(net.L)] if want_db else None)
    loss = out_loss if out_loss is not None else (torch.empty((B,), **f32) if want_loss else None)
    workspace, ws_bytes = _workspace(net, "per_example_grads", B, 1, workspace)
    _check(load_library().pfg_per_example_grads(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, _ptrs(dW),
        _ptrs(db) if db is not None else None, None if loss is None else loss.data_ptr(),
        workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return dW, db, loss


PFG_STATIC_SCRATCH_BYTES = 64 << 20


def pfg_per_example_grads_static(net: Mlp, X, labels, out_dW, out_db=None, out_loss=None):
    """pfg_per_example_grads on the library's built-in scratch buffer: every output is the
    caller's, nothing is allocated here or in the library."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    _check(load_library().pfg_per_example_grads_static(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, _ptrs(out_dW),
        _ptrs(out_db) if out_db is not None else None,
        None if out_loss is None else out_loss.data_ptr(), _stream_ptr()))
    return out_dW, out_db, out_loss


def _seed_args(net: Mlp, B: int, seeds, S: Optional[int]):
    import torch
    dL = net.dims[-1]
    if seeds is None:
        return None, (dL if S is None else S), 0
    if seeds.dtype != torch.float32 or not seeds.is_contiguous() or seeds.shape[-1] != dL:
        raise ValueError("seeds must be a contiguous float32 tensor with last dimension d_L")
    if seeds.dim() == 2:
        return seeds, seeds.shape[0], 0
    if seeds.dim() != 3 or seeds.shape[0] != B:
        raise ValueError("seeds must be [S, d_L] or [B, S, d_L]")
    return seeds, seeds.shape[1], seeds.shape[1] * dL


def pfg_jacobian_input(net: Mlp, X, seeds=None, S: Optional[int] = None, out=None, workspace=None):
    """J[b, s, :] = gradient of <seed row s, y_b> with respect to x_b, shape [B, S, d_0]."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    seeds, S, stride = _seed_args(net, B, seeds, S)
    J = out if out is not None else torch.empty((B, S, net.dims[0]), dtype=torch.float32,
                                                device=net.device)
    workspace, ws_bytes = _workspace(net, "jacobian_input", B, S, workspace)
    _check(load_library().pfg_jacobian_input(
        ctypes.byref(net.c), X.data_ptr(), B, None if seeds is None else seeds.data_ptr(), S,
        stride, J.data_ptr(), workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return J


def pfg_jacobian_weights(net: Mlp, X, head: str = "logits", seeds=None, S: Optional[int] = None,
                         want_JW: Optional[Sequence[bool]] = None, want_Jb: bool = True,
                         out_JW=None, out_Jb=None, workspace=None):
    """Returns (JW list [B, S, d_{l-1}, d_l] or None per layer, Jb list [B, S, d_l] or None)."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    seeds, S, stride = _seed_args(net, B, seeds, S)
    want = [True] * net.L if want_JW is None else list(want_JW)
    f32 = dict(dtype=torch.float32, device=net.device)
    JW = out_JW if out_JW is not None else [
        torch.empty((B, S, net.dims[l], net.dims[l + 1]), **f32) if want[l] else None
        for l in range(net.L)]
    Jb = out_Jb if out_Jb is not None else (
        [torch.empty((B, S, net.dims[l + 1]), **f32) for l in range(net.L)] if want_Jb else None)
    workspace, ws_bytes = _workspace(net, "jacobian_weights", B, S, workspace)
    _check(load_library().pfg_jacobian_weights(
        ctypes.byref(net.c), X.data_ptr(), B, HEAD[head],
        None if seeds is None else seeds.data_ptr(), S, stride, _ptrs(JW),
        _ptrs(Jb) if Jb is not None else None, workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return JW, Jb


def pfg_per_example_grad_norms(net: Mlp, X, labels, want_sq_layers: bool = True, want_norm: bool = True,
                               want_loss: bool = True, out_sq_layers=None, out_norm=None,
                               out_loss=None, workspace=None):
    """Returns (sq_layers [B, L] or None, norm [B] or None, loss [B] or None): squared per-layer
    norms and the overall norm of each example's own gradient, without forming the gradients."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    sq = out_sq_layers if out_sq_layers is not None else (
        torch.empty((B, net.L), **f32) if want_sq_layers else None)
    norm = out_norm if out_norm is not None else (torch.empty((B,), **f32) if want_norm else None)
    loss = out_loss if out_loss is not None else (torch.empty((B,), **f32) if want_loss else None)
    workspace, ws_bytes = _workspace(net, "grad_norms", B, 1, workspace)
    _check(load_library().pfg_per_example_grad_norms(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B,
        None if sq is None else sq.data_ptr(), None if norm is None else norm.data_ptr(),
        None if loss is None else loss.data_ptr(), workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return sq, norm, loss


def pfg_hessian_input(net: Mlp, X, seeds=None, S: Optional[int] = None, out=None, workspace=None):
    """H[b, s, i, j] = second derivative of <seed row s, y_b> with respect to x_b[i], x_b[j],
    shape [B, S, d_0, d_0]."""
    import torch
    _check_x(net, X)
    B = X.shape[0]
    seeds, S, stride = _seed_args(net, B, seeds, S)
    n = net.dims[0]
    H = out if out is not None else torch.empty((B, S, n, n), dtype=torch.float32, device=net.device)
    workspace, ws_bytes = _workspace(net, "hessian_input", B, S, workspace)
    _check(load_library().pfg_hessian_input(
        ctypes.byref(net.c), X.data_ptr(), B, None if seeds is None else seeds.data_ptr(), S,
        stride, H.data_ptr(), workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return H


class Lstm:
    """Device-resident unrolled LSTM: W [dx + H, 4H] (column blocks i, g, f, o), b [4H] or None,
    W_out [H, dy], b_out [dy] or None, all contiguous float32 GPU tensors; T steps."""

    def __init__(self, W, b, W_out, b_out, steps: int):
        import torch
        for t in (W, b, W_out, b_out):
            if t is not None and (t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda):
                raise ValueError("LSTM weights must be contiguous float32 GPU tensors")
        self.H, self.dy = int(W_out.shape[0]), int(W_out.shape[1])
        self.dx = int(W.shape[0]) - self.H
        self.T = int(steps)
        if self.dx < 1 or tuple(W.shape) != (self.dx + self.H, 4 * self.H):
            raise ValueError(f"W has shape {tuple(W.shape)}")
        if b is not None and tuple(b.shape) != (4 * self.H,):
            raise ValueError(f"b has shape {tuple(b.shape)}")
        if b_out is not None and tuple(b_out.shape) != (self.dy,):
            raise ValueError(f"b_out has shape {tuple(b_out.shape)}")
        self.W, self.b, self.W_out, self.b_out = W, b, W_out, b_out
        self.device = W.device
        self.c = pfg_lstm(self.dx, self.H, self.dy, self.T, W.data_ptr(),
                          None if b is None else b.data_ptr(), W_out.data_ptr(),
                          None if b_out is None else b_out.data_ptr(), DTYPE["f32"])

    @staticmethod
    def from_numpy(W, b, W_out, b_out, steps: int, device: str = "cuda:0") -> "Lstm":
        import torch
        up = lambda a: None if a is None else torch.from_numpy(a).to(device)
        return Lstm(up(W), up(b), up(W_out), up(b_out), steps)


def pfg_lstm_workspace_bytes(net: Lstm, op: str, B: int, S: int = 1) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_lstm_workspace_bytes(ctypes.byref(net.c), LSTM_OP[op], B, S,
                                                   ctypes.byref(n)))
    return int(n.value)


def _lstm_workspace(net: Lstm, op: str, B: int, S: int, workspace):
    import torch
    if workspace is None:
        workspace = torch.empty(pfg_lstm_workspace_bytes(net, op, B, S), dtype=torch.uint8,
                                device=net.device)
    return workspace, workspace.numel() * workspace.element_size()


def _check_seq(net: Lstm, X):
    import torch
    if (X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 3 or
            tuple(X.shape[1:]) != (net.T, net.dx)):
        raise ValueError("X must be a contiguous float32 [B, steps, input_size] tensor")


def pfg_lstm_per_example_grads(net: Lstm, X, labels, want_dW: bool = True, want_db: bool = True,
                               want_dWout: bool = True, want_dbout: bool = True,
                               want_loss: bool = True, out=None, workspace=None):
    """Returns (dW [B, dx+H, 4H], db [B, 4H], dWout [B, H, dy], dbout [B, dy], loss [B]), each None
    if not wanted.  ``out`` may hold caller tensors in that order."""
    import torch
    _check_seq(net, X)
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    shapes = [(B, net.dx + net.H, 4 * net.H), (B, 4 * net.H), (B, net.H, net.dy), (B, net.dy), (B,)]
    wants = [want_dW, want_db, want_dWout, want_dbout, want_loss]
    outs = list(out) if out is not None else [torch.empty(sh, **f32) if w else None
                                              for sh, w in zip(shapes, wants)]
    workspace, ws_bytes = _lstm_workspace(net, "per_example_grads", B, 1, workspace)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(load_library().pfg_lstm_per_example_grads(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, ptr(outs[0]), ptr(outs[1]),
        ptr(outs[2]), ptr(outs[3]), ptr(outs[4]), workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return tuple(outs)


def pfg_lstm_per_example_grad_norms(net: Lstm, X, labels, want_sq: bool = True, want_norm: bool = True,
                                    want_loss: bool = True, out=None, workspace=None):
    """Returns (sq [B, 4] = squared norms of dW, db, dWout, dbout; norm [B]; loss [B]); entries that
    are not wanted are None.  ``out`` may hold caller tensors in that structure."""
    import torch
    _check_seq(net, X)
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    if out is not None:
        sq, norm, loss = out
    else:
        sq = torch.empty((B, 4), **f32) if want_sq else None
        norm = torch.empty((B,), **f32) if want_norm else None
        loss = torch.empty((B,), **f32) if want_loss else None
    workspace, ws_bytes = _lstm_workspace(net, "grad_norms", B, 1, workspace)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(load_library().pfg_lstm_per_example_grad_norms(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, ptr(sq), ptr(norm), ptr(loss),
        workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return sq, norm, loss


def pfg_lstm_jacobian_input(net: Lstm, X, seeds=None, S: Optional[int] = None, out=None,
                            workspace=None):
    """J[b, s, t, :] = gradient of <seed row s, y_b> with respect to x_b[t, :], [B, S, T, dx]."""
    import torch
    _check_seq(net, X)
    B = X.shape[0]
    if seeds is None:
        S, stride = (net.dy if S is None else S), 0
    else:
        if seeds.dtype != torch.float32 or not seeds.is_contiguous() or seeds.shape[-1] != net.dy:
            raise ValueError("seeds must be a contiguous float32 tensor with last dimension output_size")
        if seeds.dim() == 2:
            S, stride = seeds.shape[0], 0
        elif seeds.dim() == 3 and seeds.shape[0] == B:
            S, stride = seeds.shape[1], seeds.shape[1] * net.dy
        else:
            raise ValueError("seeds must be [S, dy] or [B, S, dy]")
    J = out if out is not None else torch.empty((B, S, net.T, net.dx), dtype=torch.float32,
                                                device=net.device)
    workspace, ws_bytes = _lstm_workspace(net, "jacobian_input", B, S, workspace)
    _check(load_library().pfg_lstm_jacobian_input(
        ctypes.byref(net.c), X.data_ptr(), B, None if seeds is None else seeds.data_ptr(), S,
        stride, J.data_ptr(), workspace.data_ptr(), ws_bytes, _stream_ptr()))
    return J


def pfg_lstm_varlen_workspace_bytes(net: Lstm, B: int, total_tokens: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_lstm_varlen_workspace_bytes(ctypes.byref(net.c), B, total_tokens,
                                                          ctypes.byref(n)))
    return int(n.value)


def pfg_lstm_varlen_forward(net: Lstm, X, lengths, want_h: bool = True, want_y: bool = True,
                            out_h=None, out_y=None, workspace=None):
    """Sequences of different lengths, tokens back to back in X [sum(lengths), dx]; ``lengths`` is a
    host sequence of ints.  Returns (h [B, H] or None, y [B, dy] or None)."""
    import numpy as np
    import torch
    lengths = np.ascontiguousarray(np.asarray(lengths, dtype=np.int32))
    B, total = int(lengths.size), int(lengths.sum())
    if X.dtype != torch.float32 or not X.is_contiguous() or tuple(X.shape) != (total, net.dx):
        raise ValueError("X must be a contiguous float32 [sum(lengths), input_size] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    h = out_h if out_h is not None else (torch.empty((B, net.H), **f32) if want_h else None)
    y = out_y if out_y is not None else (torch.empty((B, net.dy), **f32) if want_y else None)
    if workspace is None:
        workspace = torch.empty(pfg_lstm_varlen_workspace_bytes(net, B, total), dtype=torch.uint8,
                                device=net.device)
    _check(load_library().pfg_lstm_varlen_forward(
        ctypes.byref(net.c), X.data_ptr(), lengths.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), B,
        total, None if h is None else h.data_ptr(), None if y is None else y.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr()))
    return h, y


def pfg_lstm_while_workspace_bytes(net: Lstm, B: int, total_tokens: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_lstm_while_workspace_bytes(ctypes.byref(net.c), B, total_tokens,
                                                         ctypes.byref(n)))
    return int(n.value)


def pfg_lstm_while_forward(net: Lstm, X, seq_offsets, max_steps: int, halt_w=None, halt_c: float = 0.0,
                           want_h: bool = True, want_y: bool = True, want_steps: bool = True,
                           want_trips: bool = True, out=None, workspace=None):
    """The while loop with a state-dependent condition (see include/pfg.h).  ``X`` [tokens, dx] and
    ``seq_offsets`` (int32 [B + 1]) are GPU tensors.  Returns (h [B, H], y [B, dy], steps [B] int32,
    trips [1] int32), entries that are not wanted are None; ``out`` may hold caller tensors in that
    structure."""
    import torch
    if (seq_offsets.dtype != torch.int32 or not seq_offsets.is_contiguous() or not seq_offsets.is_cuda or
            seq_offsets.dim() != 1 or seq_offsets.numel() < 2):
        raise ValueError("seq_offsets must be a contiguous int32 [B + 1] GPU tensor")
    if X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.dx:
        raise ValueError("X must be a contiguous float32 [total_tokens, input_size] tensor")
    if halt_w is not None and (halt_w.dtype != torch.float32 or not halt_w.is_contiguous() or
                               tuple(halt_w.shape) != (net.H,)):
        raise ValueError("halt_w must be a contiguous float32 [state_size] tensor")
    B, total = seq_offsets.numel() - 1, int(X.shape[0])
    f32 = dict(dtype=torch.float32, device=net.device)
    if out is not None:
        h, y, steps, trips = out
    else:
        h = torch.empty((B, net.H), **f32) if want_h else None
        y = torch.empty((B, net.dy), **f32) if want_y else None
        steps = torch.empty((B,), dtype=torch.int32, device=net.device) if want_steps else None
        trips = torch.empty((1,), dtype=torch.int32, device=net.device) if want_trips else None
    if workspace is None:
        workspace = torch.empty(pfg_lstm_while_workspace_bytes(net, B, total), dtype=torch.uint8,
                                device=net.device)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(load_library().pfg_lstm_while_forward(
        ctypes.byref(net.c), X.data_ptr() if total else None, seq_offsets.data_ptr(), B, total, int(max_steps),
        ptr(halt_w), float(halt_c), ptr(h), ptr(y), ptr(steps), ptr(trips), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr()))
    return h, y, steps, trips


def pfg_lstm_while_grads_workspace_bytes(net: Lstm, B: int, total_tokens: int, max_steps: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_lstm_while_grads_workspace_bytes(ctypes.byref(net.c), B, total_tokens,
                                                               int(max_steps), ctypes.byref(n)))
    return int(n.value)


def pfg_lstm_while_per_example_grads(net: Lstm, X, seq_offsets, labels, max_steps: int, halt_w=None,
                                     halt_c: float = 0.0, want=("dW", "db", "dWout", "dbout", "loss", "steps"),
                                     out=None, workspace=None):
    """Per-example gradients through the while loop (see include/pfg.h).  ``X`` [tokens, dx],
    ``seq_offsets`` (int32 [B + 1]) and ``labels`` (int32 [B]) are GPU tensors.  Returns a dict with the
    entries named in ``want``: dW [B, dx + H, 4H], db [B, 4H], dWout [B, H, dy], dbout [B, dy], loss
    [B], steps [B] int32; ``out`` may hold caller tensors under those names."""
    import torch
    if (seq_offsets.dtype != torch.int32 or not seq_offsets.is_contiguous() or not seq_offsets.is_cuda or
            seq_offsets.dim() != 1 or seq_offsets.numel() < 2):
        raise ValueError("seq_offsets must be a contiguous int32 [B + 1] GPU tensor")
    if X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.dx:
        raise ValueError("X must be a contiguous float32 [total_tokens, input_size] tensor")
    B, total = seq_offsets.numel() - 1, int(X.shape[0])
    if labels.dtype != torch.int32 or not labels.is_contiguous() or tuple(labels.shape) != (B,):
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    if halt_w is not None and (halt_w.dtype != torch.float32 or not halt_w.is_contiguous() or
                               tuple(halt_w.shape) != (net.H,)):
        raise ValueError("halt_w must be a contiguous float32 [state_size] tensor")
    shapes = {"dW": (B, net.dx + net.H, 4 * net.H), "db": (B, 4 * net.H), "dWout": (B, net.H, net.dy),
              "dbout": (B, net.dy), "loss": (B,), "steps": (B,)}
    res = {}
    for name in want:
        if out is not None and name in out:
            res[name] = out[name]
        else:
            res[name] = torch.empty(shapes[name], dtype=torch.int32 if name == "steps" else torch.float32,
                                    device=net.device)
    if workspace is None:
        workspace = torch.empty(pfg_lstm_while_grads_workspace_bytes(net, B, total, max_steps), dtype=torch.uint8,
                                device=net.device)
    ptr = lambda name: res[name].data_ptr() if name in res else None
    _check(load_library().pfg_lstm_while_per_example_grads(
        ctypes.byref(net.c), X.data_ptr() if total else None, seq_offsets.data_ptr(), labels.data_ptr(), B, total,
        int(max_steps), None if halt_w is None else halt_w.data_ptr(), float(halt_c), ptr("dW"), ptr("db"),
        ptr("dWout"), ptr("dbout"), ptr("loss"), ptr("steps"), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr()))
    return res


def pfg_lstm_while_per_example_grad_norms(net: Lstm, X, seq_offsets, labels, max_steps: int, halt_w=None,
                                          halt_c: float = 0.0, want=("sq", "norm", "loss", "steps"), out=None,
                                          workspace=None):
    """Norms of the per-example gradients through the while loop (see include/pfg.h).  Returns a dict
    with the entries named in ``want``: sq [B, 4], norm [B], loss [B], steps [B] int32."""
    import torch
    if (seq_offsets.dtype != torch.int32 or not seq_offsets.is_contiguous() or not seq_offsets.is_cuda or
            seq_offsets.dim() != 1 or seq_offsets.numel() < 2):
        raise ValueError("seq_offsets must be a contiguous int32 [B + 1] GPU tensor")
    if X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.dx:
        raise ValueError("X must be a contiguous float32 [total_tokens, input_size] tensor")
    B, total = seq_offsets.numel() - 1, int(X.shape[0])
    if labels.dtype != torch.int32 or not labels.is_contiguous() or tuple(labels.shape) != (B,):
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    if halt_w is not None and (halt_w.dtype != torch.float32 or not halt_w.is_contiguous() or
                               tuple(halt_w.shape) != (net.H,)):
        raise ValueError("halt_w must be a contiguous float32 [state_size] tensor")
    shapes = {"sq": (B, 4), "norm": (B,), "loss": (B,), "steps": (B,)}
    res = {}
    for name in want:
        if out is not None and name in out:
            res[name] = out[name]
        else:
            res[name] = torch.empty(shapes[name], dtype=torch.int32 if name == "steps" else torch.float32,
                                    device=net.device)
    if workspace is None:
        workspace = torch.empty(pfg_lstm_while_grads_workspace_bytes(net, B, total, max_steps), dtype=torch.uint8,
                                device=net.device)
    ptr = lambda name: res[name].data_ptr() if name in res else None
    _check(load_library().pfg_lstm_while_per_example_grad_norms(
        ctypes.byref(net.c), X.data_ptr() if total else None, seq_offsets.data_ptr(), labels.data_ptr(), B, total,
        int(max_steps), None if halt_w is None else halt_w.data_ptr(), float(halt_c), ptr("sq"), ptr("norm"),
        ptr("loss"), ptr("steps"), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr()))
    return res


class ConvNet:
    """Device-resident convolutional network: conv blocks (Wc[i] [k, k, c_in, c_out], bc[i] [c_out]
    or None; "same" convolution + ReLU + 2 x 2 max-pooling) followed by the dense layers of an
    ``Mlp`` (float32, ReLU) whose input width equals the flattened output of the last block."""

    def __init__(self, height: int, width: int, channels: int, Wc: Sequence, bc: Optional[Sequence],
                 dense: Mlp):
        import torch
        self.height, self.width, self.channels = int(height), int(width), int(channels)
        self.Wc = list(Wc)
        self.nc = len(self.Wc)
        self.bc = [None] * self.nc if bc is None else list(bc)
        for t in self.Wc + [b for b in self.bc if b is not None]:
            if t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
                raise ValueError("conv weights must be contiguous float32 GPU tensors")
        self.kernel = [int(W.shape[0]) for W in self.Wc]
        self.filters = [int(W.shape[3]) for W in self.Wc]
        c = self.channels
        for i, W in enumerate(self.Wc):
            if tuple(W.shape) != (self.kernel[i], self.kernel[i], c, self.filters[i]):
                raise ValueError(f"Wc[{i}] has shape {tuple(W.shape)}")
            if self.bc[i] is not None and tuple(self.bc[i].shape) != (self.filters[i],):
                raise ValueError(f"bc[{i}] has shape {tuple(self.bc[i].shape)}")
            c = self.filters[i]
        self.dense = dense
        self.device = dense.device
        self._kernel = (ctypes.c_int32 * self.nc)(*self.kernel)
        self._filters = (ctypes.c_int32 * self.nc)(*self.filters)
        self._Wc = (ctypes.c_void_p * self.nc)(*[W.data_ptr() for W in self.Wc])
        self._bc = (ctypes.c_void_p * self.nc)(*[None if b is None else b.data_ptr() for b in self.bc])
        self.c = pfg_convnet(self.height, self.width, self.channels, self.nc, self._kernel,
                             self._filters, self._Wc, self._bc, dense.c)

    @staticmethod
    def from_numpy(height, width, channels, Wc, bc, Ws, bs, device: str = "cuda:0") -> "ConvNet":
        import torch
        up = lambda a: None if a is None else torch.from_numpy(a).to(device)
        dense = Mlp.from_numpy(Ws, bs, "relu", "f32", device=device)
        return ConvNet(height, width, channels, [up(W) for W in Wc],
                       None if bc is None else [up(b) for b in bc], dense)


def pfg_convnet_workspace_bytes(net: ConvNet, B: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_convnet_workspace_bytes(ctypes.byref(net.c), B, ctypes.byref(n)))
    return int(n.value)


def pfg_convnet_per_example_grads(net: ConvNet, X, labels, want_dWc: Optional[Sequence[bool]] = None,
                                  want_dbc: bool = True, want_dW: Optional[Sequence[bool]] = None,
                                  want_db: bool = True, want_loss: bool = True, out=None,
                                  workspace=None):
    """Returns (dWc list [B, k, k, c_in, c_out], dbc list [B, c_out], dW list [B, d_l, d_{l+1}],
    db list [B, d_{l+1}], loss [B]); entries / lists that are not wanted are None.  ``out`` may hold
    caller tensors in that structure."""
    import torch
    if (X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 4 or
            tuple(X.shape[1:]) != (net.height, net.width, net.channels)):
        raise ValueError("X must be a contiguous float32 [B, height, width, channels] tensor")
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    dn = net.dense
    if out is not None:
        dWc, dbc, dW, db, loss = out
    else:
        wc = [True] * net.nc if want_dWc is None else list(want_dWc)
        wd = [True] * dn.L if want_dW is None else list(want_dW)
        dWc = [torch.empty((B,) + tuple(net.Wc[i].shape), **f32) if wc[i] else None for i in range(net.nc)]
        dbc = [torch.empty((B, net.filters[i]), **f32) for i in range(net.nc)] if want_dbc else None
        dW = [torch.empty((B, dn.dims[l], dn.dims[l + 1]), **f32) if wd[l] else None for l in range(dn.L)]
        db = [torch.empty((B, dn.dims[l + 1]), **f32) for l in range(dn.L)] if want_db else None
        loss = torch.empty((B,), **f32) if want_loss else None
    if workspace is None:
        workspace = torch.empty(pfg_convnet_workspace_bytes(net, B), dtype=torch.uint8, device=net.device)
    _check(load_library().pfg_convnet_per_example_grads(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, _ptrs(dWc),
        _ptrs(dbc) if dbc is not None else None, _ptrs(dW), _ptrs(db) if db is not None else None,
        None if loss is None else loss.data_ptr(), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr()))
    return dWc, dbc, dW, db, loss


def pfg_convnet_grad_norms_workspace_bytes(net: ConvNet, B: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().pfg_convnet_grad_norms_workspace_bytes(ctypes.byref(net.c), B, ctypes.byref(n)))
    return int(n.value)


def pfg_convnet_per_example_grad_norms(net: ConvNet, X, labels, want_sq: bool = True,
                                       want_norm: bool = True, want_loss: bool = True, out=None,
                                       workspace=None):
    """Returns (sq [B, num_conv + L] = squared gradient norm of every parameter block, conv blocks
    first; norm [B]; loss [B]); entries that are not wanted are None.  ``out`` may hold caller
    tensors in that structure."""
    import torch
    if (X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 4 or
            tuple(X.shape[1:]) != (net.height, net.width, net.channels)):
        raise ValueError("X must be a contiguous float32 [B, height, width, channels] tensor")
    B = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (B,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [B] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    if out is not None:
        sq, norm, loss = out
    else:
        sq = torch.empty((B, net.nc + net.dense.L), **f32) if want_sq else None
        norm = torch.empty((B,), **f32) if want_norm else None
        loss = torch.empty((B,), **f32) if want_loss else None
    if workspace is None:
        workspace = torch.empty(pfg_convnet_grad_norms_workspace_bytes(net, B), dtype=torch.uint8,
                                device=net.device)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(load_library().pfg_convnet_per_example_grad_norms(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), B, ptr(sq), ptr(norm), ptr(loss),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr()))
    return sq, norm, loss


class Cond:
    """Loop body with a conditional: ``t = phi_pre(pre(x))``; ``then_net(t)`` where
    ``t . cond_w + cond_c > 0``, ``else_net(t)`` elsewhere.  The three parts are float32 ``Mlp``
    objects; ``cond_w`` is a float32 [d_T] GPU tensor."""

    def __init__(self, pre: Mlp, cond_w, cond_c: float, then_net: Mlp, else_net: Mlp):
        import torch
        if cond_w is not None and (cond_w.dtype != torch.float32 or not cond_w.is_contiguous() or
                                   not cond_w.is_cuda or tuple(cond_w.shape) != (pre.dims[-1],)):
            raise ValueError("cond_w must be a contiguous float32 [d_T] GPU tensor")
        self.pre, self.then_net, self.else_net = pre, then_net, else_net
        self.cond_w, self.cond_c = cond_w, float(cond_c)
        self.device = pre.device
        self.d0, self.dT, self.dout = pre.dims[0], pre.dims[-1], then_net.dims[-1]
        self.c = pfg_cond(pre.c, None if cond_w is None else cond_w.data_ptr(), self.cond_c, then_net.c,
                          else_net.c)

    @staticmethod
    def from_numpy(pre, cond_w, cond_c, then_net, else_net, act: str, device: str = "cuda:0") -> "Cond":
        """pre, then_net, else_net: (weights, biases) pairs of numpy arrays."""
        import torch
        nets = [Mlp.from_numpy(Ws, bs, act, "f32", device=device) for Ws, bs in (pre, then_net, else_net)]
        return Cond(nets[0], torch.from_numpy(cond_w).to(device), cond_c, nets[1], nets[2])


def pfg_cond_workspace_bytes(net: Cond, n: int) -> int:
    b = ctypes.c_size_t(0)
    _check(load_library().pfg_cond_workspace_bytes(ctypes.byref(net.c), n, ctypes.byref(b)))
    return int(b.value)


def pfg_cond_forward(net: Cond, X, invariant_cond: int = PFG_COND_PER_ITERATION, want_cond: bool = True,
                     want_counts: bool = True, out=None, workspace=None):
    """Returns (R [n, d_out], cond [n] int32 or None, counts [2] int32 or None); ``out`` may hold
    caller tensors in that structure."""
    import torch
    if X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.d0:
        raise ValueError("X must be a contiguous float32 [n, d_0] tensor")
    n = X.shape[0]
    if out is not None:
        R, cond, counts = out
    else:
        R = torch.empty((n, net.dout), dtype=torch.float32, device=net.device)
        cond = torch.empty((n,), dtype=torch.int32, device=net.device) if want_cond else None
        counts = torch.empty((2,), dtype=torch.int32, device=net.device) if want_counts else None
    if workspace is None:
        workspace = torch.empty(pfg_cond_workspace_bytes(net, n), dtype=torch.uint8, device=net.device)
    _check(load_library().pfg_cond_forward(
        ctypes.byref(net.c), X.data_ptr(), n, int(invariant_cond), R.data_ptr(),
        None if cond is None else cond.data_ptr(), None if counts is None else counts.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr()))
    return R, cond, counts


def pfg_cond_grads_workspace_bytes(net: Cond, n: int) -> int:
    b = ctypes.c_size_t(0)
    _check(load_library().pfg_cond_grads_workspace_bytes(ctypes.byref(net.c), n, ctypes.byref(b)))
    return int(b.value)


def pfg_cond_per_example_grads(net: Cond, X, labels, invariant_cond: int = PFG_COND_PER_ITERATION,
                               want_dW: bool = True, want_db: bool = True, out=None, workspace=None):
    """Per-example gradients through the conditional.  Returns a dict: for each of "pre", "then",
    "else" a pair (dW list [n, d_{l-1}, d_l], db list [n, d_l]) -- None when not wanted --, plus
    "loss" [n], "cond" [n] int32 and "counts" [2] int32.  ``out`` may be such a dict of caller tensors."""
    import torch
    if X.dtype != torch.float32 or not X.is_contiguous() or X.dim() != 2 or X.shape[1] != net.d0:
        raise ValueError("X must be a contiguous float32 [n, d_0] tensor")
    n = X.shape[0]
    if labels.dtype != torch.int32 or tuple(labels.shape) != (n,) or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 [n] tensor")
    f32 = dict(dtype=torch.float32, device=net.device)
    if out is None:
        out = {}
        for name, m in (("pre", net.pre), ("then", net.then_net), ("else", net.else_net)):
            dW = [torch.empty((n, m.dims[l], m.dims[l + 1]), **f32) for l in range(m.L)] if want_dW else None
            db = [torch.empty((n, m.dims[l + 1]), **f32) for l in range(m.L)] if want_db else None
            out[name] = (dW, db)
        out["loss"] = torch.empty((n,), **f32)
        out["cond"] = torch.empty((n,), dtype=torch.int32, device=net.device)
        out["counts"] = torch.empty((2,), dtype=torch.int32, device=net.device)
    if workspace is None:
        workspace = torch.empty(pfg_cond_grads_workspace_bytes(net, n), dtype=torch.uint8, device=net.device)
    lists = []
    for name in ("pre", "then", "else"):
        for arrs in out[name]:
            lists.append(None if arrs is None else _ptrs(arrs))
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(load_library().pfg_cond_per_example_grads(
        ctypes.byref(net.c), X.data_ptr(), labels.data_ptr(), n, int(invariant_cond), *lists,
        ptr(out.get("loss")), ptr(out.get("cond")), ptr(out.get("counts")), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr()))
    return out


def pfg_fill_reference(out, value: float = 0.0, stores_per_lane: int = 1) -> None:
    """Fill a contiguous float32 GPU tensor with the library's plain sequential store stream
    (stores_per_lane times 4 KiB per workgroup)."""
    import torch
    if out.dtype != torch.float32 or not out.is_contiguous() or not out.is_cuda:
        raise ValueError("out must be a contiguous float32 GPU tensor")
    _check(load_library().pfg_fill_reference(out.data_ptr(), out.numel(), float(value), int(stores_per_lane),
                                              _stream_ptr()))


def pfg_timing_enable(on: bool) -> None:
    _check(load_library().pfg_timing_enable(1 if on else 0))


def pfg_timing_reset() -> None:
    _check(load_library().pfg_timing_reset())


def pfg_timing_query(name: str):
    """(launches, total milliseconds) of one kernel family since the last reset."""
    n, ms = ctypes.c_int64(0), ctypes.c_double(0.0)
    _check(load_library().pfg_timing_query(name.encode(), ctypes.byref(n), ctypes.byref(ms)))
    return int(n.value), float(ms.value)


def pfg_timing_names() -> List[str]:
    buf = ctypes.create_string_buffer(4096)
    _check(load_library().pfg_timing_names(buf, 4096))
    s = buf.value.decode()
    return s.split("\n") if s else []
