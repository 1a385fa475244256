"""Seeded synthetic inputs for the measured workloads.

This module holds no arithmetic of the method: it only draws random tensors (and rounds them to
bfloat16 where a workload asks for bf16 inputs).  The same host arrays are handed to the GPU
library and to the CPU oracle, so the random number generator is not part of any parity claim.

The paper's own workloads (MNIST images, random 768-vectors, VGG16 inputs; Section 6.1) are not
used; seeded tensors of the same kind of shape stand in for them ("MNIST-shaped" = 784 inputs in
[0, 1), 10 classes).

Draw order for a workload: W_1, b_1, ..., W_L, b_L, X, labels, all from one Philox stream seeded
with ``BASE_SEED + index``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 190304243


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    call: str                      # "per_example_grads" | "jacobian_input" | "jacobian_weights" |
                                   # "grad_norms" | "hessian_input"
    dims: Tuple[int, ...]
    act: str                       # hidden activation
    dtype: str                     # "f32" | "bf16" (dtype of X, W, b; outputs are always f32)
    B: int
    x_dist: str                    # "normal" | "uniform01"
    w_init: str                    # "glorot_uniform" | "normal_fan_in"
    S: int = 1                     # seed rows per example (Jacobians)
    head: str = "logits"           # jacobian_weights only
    layers_out: Optional[Tuple[int, ...]] = None   # 1-based layers whose dW / JW is produced
    also: Tuple[str, ...] = field(default_factory=tuple)   # further calls on the same inputs


WORKLOADS: Dict[str, Workload] = {
    w.name: w for w in [
        Workload("c1_tiny", 0, "per_example_grads", (32, 64, 10), "relu", "f32", 16,
                 "normal", "glorot_uniform", S=10, also=("jacobian_input",)),
        Workload("c2_mnist_mlp_grads", 1, "per_example_grads", (784, 512, 512, 10), "relu", "f32",
                 128, "uniform01", "glorot_uniform"),
        Workload("c3_tanh_jacobian", 2, "jacobian_input", (1024, 2048, 2048, 1024), "tanh", "f32",
                 64, "normal", "normal_fan_in", S=1024),
        Workload("c4_gelu_bf16_grads", 3, "per_example_grads", (4096, 4096, 4096, 10), "gelu",
                 "bf16", 256, "normal", "normal_fan_in"),
        Workload("c5_nested_weight_jacobian", 4, "jacobian_weights", (256, 256, 16), "tanh", "f32",
                 64, "normal", "normal_fan_in", S=16, head="softmax", layers_out=(1,)),
        # the norms of the per-example gradients of c2 and c4 (same inputs), gradients not formed
        Workload("c2_mnist_mlp_grad_norms", 1, "grad_norms", (784, 512, 512, 10), "relu", "f32",
                 128, "uniform01", "glorot_uniform"),
        Workload("c4_gelu_bf16_grad_norms", 3, "grad_norms", (4096, 4096, 4096, 10), "gelu",
                 "bf16", 256, "normal", "normal_fan_in"),
        # Jacobian of the Jacobian: 64 Hessians of 256 x 256 per example
        Workload("c6_tanh_hessian", 5, "hessian_input", (256, 512, 512, 64), "tanh", "f32", 32,
                 "normal", "normal_fan_in", S=64),
    ]
}


def bf16_round(a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Round float32 values to bfloat16 (nearest, ties to even).

    Returns (bits uint16, the rounded values as float32).  Inputs are finite."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    back = (r.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(a32.shape)
    return r.reshape(a32.shape), back


@dataclass
class Inputs:
    """Host arrays of one workload.  ``Ws``/``bs``/``X`` are float32 and, for a bf16 workload,
    already hold bf16-representable values; ``*_bits`` then hold the matching uint16 patterns."""
    workload: Workload
    Ws: List[np.ndarray]
    bs: List[np.ndarray]
    X: np.ndarray
    labels: np.ndarray
    Ws_bits: Optional[List[np.ndarray]] = None
    bs_bits: Optional[List[np.ndarray]] = None
    X_bits: Optional[np.ndarray] = None


def draw_weights(rng: np.random.Generator, dims, w_init: str, bias_scale: float = 0.0):
    Ws, bs = [], []
    for l in range(1, len(dims)):
        fan_in, fan_out = dims[l - 1], dims[l]
        if w_init == "glorot_uniform":
            r = np.sqrt(6.0 / (fan_in + fan_out))
            W = rng.uniform(-r, r, size=(fan_in, fan_out))
        elif w_init == "normal_fan_in":          # variance 1/fan_in
            W = rng.standard_normal(size=(fan_in, fan_out)) / np.sqrt(fan_in)
        else:
            raise ValueError(w_init)
        b = rng.standard_normal(size=(fan_out,)) * bias_scale
        Ws.append(W.astype(np.float32))
        bs.append(b.astype(np.float32))
    return Ws, bs


def make_inputs(w: Workload, B: Optional[int] = None, dims=None, bias_scale: float = 0.0,
                seed: Optional[int] = None) -> Inputs:
    """Draw one workload's tensors.  ``B``/``dims`` override the size (scaled-down parity cases);
    ``bias_scale`` > 0 gives non-zero biases (the measured workloads use zero biases)."""
    B = w.B if B is None else B
    dims = tuple(w.dims if dims is None else dims)
    rng = np.random.Generator(np.random.Philox(BASE_SEED + w.index if seed is None else seed))
    Ws, bs = draw_weights(rng, dims, w.w_init, bias_scale)
    if w.x_dist == "normal":
        X = rng.standard_normal(size=(B, dims[0]))
    elif w.x_dist == "uniform01":
        X = rng.uniform(0.0, 1.0, size=(B, dims[0]))
    else:
        raise ValueError(w.x_dist)
    X = X.astype(np.float32)
    labels = rng.integers(0, dims[-1], size=(B,)).astype(np.int32)
    inp = Inputs(w, Ws, bs, X, labels)
    if w.dtype == "bf16":
        Wr = [bf16_round(W) for W in Ws]
        br = [bf16_round(b) for b in bs]
        Xr = bf16_round(X)
        inp.Ws_bits, inp.Ws = [r[0] for r in Wr], [r[1] for r in Wr]
        inp.bs_bits, inp.bs = [r[0] for r in br], [r[1] for r in br]
        inp.X_bits, inp.X = Xr
    return inp


def output_values(w: Workload, B: Optional[int] = None) -> int:
    """Number of float32 values the workload's call writes (weight and bias gradients, or the
    Jacobian)."""
    B = w.B if B is None else B
    d = w.dims
    if w.call == "per_example_grads":
        return B * sum(d[l - 1] * d[l] + d[l] for l in range(1, len(d)))
    if w.call == "jacobian_input":
        return B * w.S * d[0]
    if w.call == "hessian_input":
        return B * w.S * d[0] * d[0]
    if w.call == "grad_norms":
        return B * (len(d) - 1) + 2 * B
    layers = w.layers_out or tuple(range(1, len(d)))
    return B * w.S * sum(d[l - 1] * d[l] for l in layers)


# --------------------------------------------------------------------------------------------
# Unrolled LSTM workloads (the model of the paper's own per-example-gradient and Jacobian
# benchmarks: sequences of 128-dimensional vectors, state size 256, 10 steps).
# --------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class LstmWorkload:
    name: str
    index: int
    call: str                      # "lstm_per_example_grads" | "lstm_per_example_grad_norms" |
                                   # "lstm_jacobian_input" | "lstm_varlen_forward"
    dx: int
    H: int
    dy: int
    T: int
    B: int
    S: int = 1


LSTM_WORKLOADS: Dict[str, LstmWorkload] = {
    w.name: w for w in [
        LstmWorkload("c7_lstm_grads", 6, "lstm_per_example_grads", 128, 256, 10, 10, 256),
        # the same batch as c7, gradient norms only
        LstmWorkload("c7_lstm_grad_norms", 6, "lstm_per_example_grad_norms", 128, 256, 10, 10, 256),
        LstmWorkload("c8_lstm_jacobian", 7, "lstm_jacobian_input", 128, 256, 128, 10, 64, S=128),
        # sequences of different lengths, each iterated to its own length (T = the longest allowed)
        LstmWorkload("c9_lstm_varlen", 8, "lstm_varlen_forward", 128, 256, 10, 100, 1024),
        # the same sequences under a loop that also stops on a halting score of the hidden state
        LstmWorkload("c12_lstm_while", 8, "lstm_while_forward", 128, 256, 10, 100, 1024),
        # per-example gradients through that loop (the same sequences, condition and labels drawn for them)
        LstmWorkload("c14_lstm_while_grads", 8, "lstm_while_per_example_grads", 128, 256, 10, 100, 1024),
        # the same call with only the norms of the gradients leaving the device
        LstmWorkload("c14_lstm_while_grad_norms", 8, "lstm_while_per_example_grad_norms", 128, 256, 10, 100, 1024),
    ]
}


@dataclass
class LstmInputs:
    workload: LstmWorkload
    W: np.ndarray          # [dx + H, 4H], column blocks i, g, f, o
    b: np.ndarray          # [4H]
    Wout: np.ndarray       # [H, dy]
    bout: np.ndarray       # [dy]
    X: np.ndarray          # [B, T, dx]
    labels: np.ndarray     # [B]


def make_lstm_inputs(w: LstmWorkload, B: Optional[int] = None, dx=None, H=None, dy=None, T=None,
                     bias_scale: float = 0.0, seed: Optional[int] = None) -> LstmInputs:
    """Weights uniform in +-1/sqrt(H) (readout: +-1/sqrt(H)), inputs standard normal, labels
    uniform; draw order W, b, Wout, bout, X, labels from one Philox stream."""
    B = w.B if B is None else B
    dx, H = w.dx if dx is None else dx, w.H if H is None else H
    dy, T = w.dy if dy is None else dy, w.T if T is None else T
    rng = np.random.Generator(np.random.Philox(BASE_SEED + w.index if seed is None else seed))
    r = 1.0 / np.sqrt(H)
    W = rng.uniform(-r, r, size=(dx + H, 4 * H)).astype(np.float32)
    b = (rng.standard_normal(4 * H) * bias_scale).astype(np.float32)
    Wout = rng.uniform(-r, r, size=(H, dy)).astype(np.float32)
    bout = (rng.standard_normal(dy) * bias_scale).astype(np.float32)
    X = rng.standard_normal(size=(B, T, dx)).astype(np.float32)
    labels = rng.integers(0, dy, size=(B,)).astype(np.int32)
    return LstmInputs(w, W, b, Wout, bout, X, labels)


def make_varlen_inputs(w: LstmWorkload, B: Optional[int] = None, dx=None, H=None, dy=None,
                       max_len: Optional[int] = None, bias_scale: float = 0.0,
                       seed: Optional[int] = None):
    """Weights as in make_lstm_inputs; lengths uniform in 1..max_len (inclusive), tokens standard
    normal, stored back to back.  Returns (LstmInputs with X = [sum(lengths), dx], lengths int32)."""
    B = w.B if B is None else B
    max_len = w.T if max_len is None else max_len
    base = make_lstm_inputs(w, B=1, dx=dx, H=H, dy=dy, T=1, bias_scale=bias_scale, seed=seed)
    rng = np.random.Generator(np.random.Philox((BASE_SEED + w.index if seed is None else seed) + 500000))
    lengths = rng.integers(1, max_len + 1, size=(B,)).astype(np.int32)
    X = rng.standard_normal(size=(int(lengths.sum()), base.W.shape[0] - base.Wout.shape[0])).astype(np.float32)
    base.X = X
    base.labels = np.zeros(B, dtype=np.int32)
    return base, lengths


def make_while_inputs(w: LstmWorkload, **kw):
    """make_varlen_inputs plus a halting vector N(0, 4 / H) and the offset -0.5 (on c9's sequences
    29 % of the iterations stop on the score before their tokens run out, 41 148 of 51 957 tokens
    are consumed).  Returns
    (LstmInputs, lengths int32, seq_offsets int32 [B + 1], halt_w float32 [H], halt_c)."""
    inp, lengths = make_varlen_inputs(w, **kw)
    H = inp.Wout.shape[0]
    seed = kw.get("seed")
    rng = np.random.Generator(np.random.Philox((BASE_SEED + w.index if seed is None else seed) + 700000))
    halt_w = (rng.standard_normal(H) * 2.0 / np.sqrt(H)).astype(np.float32)
    offsets = np.zeros(lengths.size + 1, dtype=np.int32)
    np.cumsum(lengths, out=offsets[1:])
    # labels for the gradient workload, from a stream of their own (uniform over the classes)
    lrng = np.random.Generator(np.random.Philox((BASE_SEED + w.index if seed is None else seed) + 800000))
    inp.labels = lrng.integers(0, inp.Wout.shape[1], size=(lengths.size,)).astype(np.int32)
    return inp, lengths, offsets, halt_w, -0.5


# --------------------------------------------------------------------------------------------
# Convolutional workload: the MNIST model of the paper's benchmarks (two conv-relu-maxpool blocks,
# then linear-relu-linear), on seeded MNIST-shaped inputs.
# --------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class ConvWorkload:
    name: str
    index: int
    height: int
    width: int
    channels: int
    blocks: Tuple[Tuple[int, int], ...]     # (kernel size, filters) per conv block
    dense: Tuple[int, ...]                  # widths after the flattened features
    B: int
    call: str = "convnet_per_example_grads"


CONV_WORKLOADS: Dict[str, ConvWorkload] = {
    w.name: w for w in [
        ConvWorkload("c10_mnist_convnet_grads", 9, 28, 28, 1, ((5, 32), (5, 64)), (1024, 10), 128),
        # the same inputs; only the norms of the gradients leave the device
        ConvWorkload("c10_mnist_convnet_grad_norms", 9, 28, 28, 1, ((5, 32), (5, 64)), (1024, 10), 128,
                     "convnet_per_example_grad_norms"),
    ]
}


@dataclass
class ConvInputs:
    workload: ConvWorkload
    Wc: List[np.ndarray]
    bc: List[np.ndarray]
    Ws: List[np.ndarray]
    bs: List[np.ndarray]
    X: np.ndarray            # [B, height, width, channels]
    labels: np.ndarray


def make_conv_inputs(w: ConvWorkload, B: Optional[int] = None, height=None, width=None, channels=None,
                     blocks=None, dense=None, bias_scale: float = 0.0,
                     seed: Optional[int] = None) -> ConvInputs:
    """Weights N(0, 1 / fan_in), images uniform in [0, 1), labels uniform; draw order conv filters
    and biases block by block, dense weights and biases layer by layer, X, labels."""
    B = w.B if B is None else B
    h = w.height if height is None else height
    wd = w.width if width is None else width
    c = w.channels if channels is None else channels
    blocks = w.blocks if blocks is None else blocks
    dense = w.dense if dense is None else dense
    rng = np.random.Generator(np.random.Philox(BASE_SEED + w.index if seed is None else seed))
    Wc, bc = [], []
    hh, ww, cc = h, wd, c
    for k, f in blocks:
        Wc.append((rng.standard_normal((k, k, cc, f)) / np.sqrt(k * k * cc)).astype(np.float32))
        bc.append((rng.standard_normal(f) * bias_scale).astype(np.float32))
        hh, ww, cc = hh // 2, ww // 2, f
    dims = (hh * ww * cc,) + tuple(dense)
    Ws, bs = draw_weights(rng, dims, "normal_fan_in", bias_scale)
    X = rng.uniform(0.0, 1.0, size=(B, h, wd, c)).astype(np.float32)
    labels = rng.integers(0, dims[-1], size=(B,)).astype(np.int32)
    return ConvInputs(w, Wc, bc, Ws, bs, X, labels)


# --------------------------------------------------------------------------------------------
# A loop body with a conditional (Section 3.6): a shared dense part, a per-row condition and two
# dense branches of different cost.
# --------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class CondWorkload:
    name: str
    index: int
    pre: Tuple[int, ...]         # widths d_0 .. d_T of the shared part
    then_dims: Tuple[int, ...]   # widths after d_T of the then branch
    else_dims: Tuple[int, ...]   # widths after d_T of the else branch (same last width)
    act: str
    n: int
    c0: float = 0.0              # offset of the condition
    call: str = "cond_forward"   # or "cond_per_example_grads"


COND_WORKLOADS: Dict[str, CondWorkload] = {
    w.name: w for w in [
        # the offset puts about half of the rows on each side of the condition
        CondWorkload("c11_cond_two_branches", 10, (784, 512), (1024, 1024, 10), (10,), "relu", 8192, -0.55),
        # per-example gradients through the same conditional (8.0 GB of gradients at 1024 rows)
        CondWorkload("c13_cond_grads", 10, (784, 512), (1024, 1024, 10), (10,), "relu", 1024, -0.55,
                     "cond_per_example_grads"),
    ]
}


@dataclass
class CondInputs:
    workload: CondWorkload
    pre: Tuple[List[np.ndarray], List[np.ndarray]]          # (weights, biases)
    then_net: Tuple[List[np.ndarray], List[np.ndarray]]
    else_net: Tuple[List[np.ndarray], List[np.ndarray]]
    w: np.ndarray            # [d_T]
    c0: float
    X: np.ndarray            # [n, d_0]


def make_cond_inputs(w: CondWorkload, n: Optional[int] = None, pre=None, then_dims=None, else_dims=None,
                     bias_scale: float = 0.0, c0: Optional[float] = None,
                     seed: Optional[int] = None) -> CondInputs:
    """Weights N(0, 1 / fan_in), condition vector N(0, 1 / d_T), X standard normal; draw order: shared
    part, then branch, else branch (weights and biases layer by layer), condition vector, X."""
    n = w.n if n is None else n
    pre = tuple(w.pre if pre is None else pre)
    then_dims = tuple(w.then_dims if then_dims is None else then_dims)
    else_dims = tuple(w.else_dims if else_dims is None else else_dims)
    rng = np.random.Generator(np.random.Philox(BASE_SEED + w.index if seed is None else seed))
    nets = [draw_weights(rng, dims, "normal_fan_in", bias_scale)
            for dims in (pre, (pre[-1],) + then_dims, (pre[-1],) + else_dims)]
    wv = (rng.standard_normal(pre[-1]) / np.sqrt(pre[-1])).astype(np.float32)
    X = rng.standard_normal((n, pre[0])).astype(np.float32)
    return CondInputs(w, nets[0], nets[1], nets[2], wv, float(w.c0 if c0 is None else c0), X)


# --------------------------------------------------------------------------------------------
# Integer-valued inputs: every hidden pre-activation is a small integer, exact in bfloat16,
# float32 and float64 alike, so that ReLU kinks (z == 0), pooling ties and condition scores of
# exactly 0 occur often and are decided on identical values by every implementation.
# --------------------------------------------------------------------------------------------
def _sparse_ints(rng: np.random.Generator, shape, density: float, lo: int, hi: int) -> np.ndarray:
    vals = rng.integers(lo, hi + 1, size=shape)
    keep = rng.uniform(size=shape) < density
    return (vals * keep).astype(np.float32)


def draw_integer_weights(rng: np.random.Generator, dims, density: float, last_scale: float,
                         bias: bool = True):
    """Hidden layers: entries in {-1, 0, 1} (non-zero with probability `density`), integer biases in
    {-1, 0, 1}; last layer: the same integers times `last_scale` (a power of two keeps them exact)."""
    Ws, bs = [], []
    L = len(dims) - 1
    for l in range(1, L + 1):
        scale = last_scale if l == L else 1.0
        Ws.append(_sparse_ints(rng, (dims[l - 1], dims[l]), density, -1, 1) * np.float32(scale))
        bs.append((rng.integers(-1, 2, size=(dims[l],)) * scale * (1.0 if bias else 0.0)).astype(np.float32))
    return Ws, bs


def make_integer_inputs(dims, B: int, seed: int, density: float = 0.25, last_scale: float = 1.0 / 16,
                        x_range: int = 2, dtype: str = "f32") -> Inputs:
    """A dense network with integer-valued weights and inputs (X uniform in -x_range..x_range)."""
    dims = tuple(dims)
    rng = np.random.Generator(np.random.Philox(seed))
    Ws, bs = draw_integer_weights(rng, dims, density, last_scale)
    X = rng.integers(-x_range, x_range + 1, size=(B, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], size=(B,)).astype(np.int32)
    w = Workload("integer", 0, "per_example_grads", dims, "relu", dtype, B, "integer", "integer")
    inp = Inputs(w, Ws, bs, X, labels)
    if dtype == "bf16":
        Wr = [bf16_round(W) for W in Ws]
        br = [bf16_round(b) for b in bs]
        Xr = bf16_round(X)
        for (bits, back), orig in zip(Wr + br + [Xr], Ws + bs + [X]):
            assert np.array_equal(back, orig), "integer inputs must be exact in bfloat16"
        inp.Ws_bits, inp.bs_bits, inp.X_bits = [r[0] for r in Wr], [r[0] for r in br], Xr[0]
    return inp


def make_integer_conv_inputs(height: int, width: int, channels: int, blocks, dense, B: int, seed: int,
                             density: float = 0.3, last_scale: float = 1.0 / 16) -> ConvInputs:
    """Integer images in 0..3, filters in {-1, 0, 1}, integer biases: equal entries inside a pooling
    window and pre-activations of exactly 0 are frequent."""
    rng = np.random.Generator(np.random.Philox(seed))
    Wc, bc = [], []
    hh, ww, cc = height, width, channels
    for k, f in blocks:
        Wc.append(_sparse_ints(rng, (k, k, cc, f), density, -1, 1))
        bc.append(rng.integers(-1, 2, size=(f,)).astype(np.float32))
        hh, ww, cc = hh // 2, ww // 2, f
    dims = (hh * ww * cc,) + tuple(dense)
    Ws, bs = draw_integer_weights(rng, dims, density / 4, last_scale)
    X = rng.integers(0, 4, size=(B, height, width, channels)).astype(np.float32)
    labels = rng.integers(0, dims[-1], size=(B,)).astype(np.int32)
    w = ConvWorkload("integer", 0, height, width, channels, tuple(blocks), tuple(dense), B)
    return ConvInputs(w, Wc, bc, Ws, bs, X, labels)


def make_integer_cond_inputs(pre, then_dims, else_dims, n: int, seed: int, density: float = 0.25,
                             c0: float = 0.0, branch_last_scale: float = 1.0) -> CondInputs:
    """Integer-valued shared part, condition vector and branches: many rows have a score of exactly 0.
    branch_last_scale (a power of two) scales the last layer of both branches."""
    pre, then_dims, else_dims = tuple(pre), tuple(then_dims), tuple(else_dims)
    rng = np.random.Generator(np.random.Philox(seed))
    nets = [draw_integer_weights(rng, dims, density, scale)
            for dims, scale in ((pre, 1.0), ((pre[-1],) + then_dims, branch_last_scale),
                                ((pre[-1],) + else_dims, branch_last_scale))]
    wv = _sparse_ints(rng, (pre[-1],), 0.5, -1, 1)
    X = rng.integers(-2, 3, size=(n, pre[0])).astype(np.float32)
    w = CondWorkload("integer", 0, pre, then_dims, else_dims, "relu", n, c0)
    return CondInputs(w, nets[0], nets[1], nets[2], wv, float(c0), X)
