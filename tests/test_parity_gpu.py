"""GPU parity: the HIP library, called through its C ABI, against the float64 CPU oracle on the
same seeded inputs, element by element.  Error measure: for every output tensor and every leading
slice (one example b, or one (b, s) pair) max|gpu - ref| / max|ref| over the slice; the largest
such value must not exceed 1e-4 (float32) or 2e-2 (bf16 inputs, float32 accumulation).  Slices
that are exactly zero in the reference must be exactly zero on the GPU.

ReLU nets: the sign of a hidden pre-activation is a decision taken in float32 on the GPU and in
float64 by the oracle; the inputs are drawn so that every hidden pre-activation is at least 1e-5
away from zero, far beyond float32 round-off, so both sides take the same decision.
"""
import os
import sys

import numpy as np
import pytest

from parity_util import TOL_BF16, TOL_F32, hidden_margin, outer_elem_err, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import NP_ACT, dev, draw, gpu_net, gpu_x, say  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def check_grads(oracle, inp, act, dtype, tol, want_dW=None, tag=""):
    onet = oracle.Net(inp.Ws, inp.bs, act)
    ref_dW, ref_db, ref_loss = oracle.per_example_grads(onet, inp.X, inp.labels, want_dW=want_dW)
    net = gpu_net(inp, act, dtype)
    X = gpu_x(inp, dtype)
    labels = dev(inp.labels)
    B = inp.X.shape[0]
    f32 = dict(dtype=torch.float32, device="cuda:0")
    want = [True] * net.L if want_dW is None else want_dW
    # NaN canaries: every requested output must be overwritten in full
    out_dW = [torch.full((B, net.dims[l], net.dims[l + 1]), float("nan"), **f32) if want[l] else None
              for l in range(net.L)]
    out_db = [torch.full((B, net.dims[l + 1]), float("nan"), **f32) for l in range(net.L)]
    out_loss = torch.full((B,), float("nan"), **f32)
    dW, db, loss = pfg.pfg_per_example_grads(net, X, labels, out_dW=out_dW, out_db=out_db,
                                             out_loss=out_loss)
    torch.cuda.synchronize()
    worst, worst_elem = 0.0, 0.0
    for l in range(net.L):
        if want[l]:
            g = dW[l].cpu().numpy()
            e, ee = slice_rel_err(g, ref_dW[l]), outer_elem_err(g, ref_dW[l])
            say(f"  {tag} dW{l + 1} rel err {e:.3e}, by row and column scale {ee:.3e}")
            worst, worst_elem = max(worst, e), max(worst_elem, ee)
        e = slice_rel_err(db[l].cpu().numpy(), ref_db[l])
        say(f"  {tag} db{l + 1} rel err {e:.3e}")
        worst = max(worst, e)
    e = slice_rel_err(loss.cpu().numpy(), ref_loss, lead=0)
    say(f"  {tag} loss rel err {e:.3e}")
    worst = max(worst, e)
    assert worst <= tol, f"{tag}: max relative error {worst:.3e} > {tol}"
    assert worst_elem <= tol, f"{tag}: max element-wise error (row and column scale) {worst_elem:.3e} > {tol}"
    return worst


# --------------------------------------------------------------------------------------------
# The five workloads.
# --------------------------------------------------------------------------------------------
def test_c1_tiny_grads_and_input_jacobian(oracle):
    w = wl.WORKLOADS["c1_tiny"]
    say("c1_tiny: per_example_grads + jacobian_input, full size")
    inp = draw(w)
    check_grads(oracle, inp, w.act, "f32", TOL_F32, tag="c1")
    onet = oracle.Net(inp.Ws, inp.bs, w.act)
    ref = oracle.jacobian_input(onet, inp.X)
    J = pfg.pfg_jacobian_input(gpu_net(inp, w.act, "f32"), gpu_x(inp, "f32"))
    torch.cuda.synchronize()
    assert tuple(J.shape) == (16, 10, 32)
    e = slice_rel_err(J.cpu().numpy(), ref, lead=2)
    say(f"  c1 J rel err {e:.3e}")
    assert e <= TOL_F32


def test_c2_mnist_mlp_grads_full_size(oracle):
    w = wl.WORKLOADS["c2_mnist_mlp_grads"]
    say("c2_mnist_mlp_grads: full size, every element")
    inp = draw(w)
    check_grads(oracle, inp, w.act, "f32", TOL_F32, tag="c2")


def test_c3_tanh_jacobian_reduced_every_element(oracle):
    w = wl.WORKLOADS["c3_tanh_jacobian"]
    dims, B = (160, 288, 200, 96), 5     # several tiles and ragged tails in every dimension
    say(f"c3 reduced {dims} B={B}: every element")
    inp = draw(w, B=B, dims=dims)
    onet = oracle.Net(inp.Ws, inp.bs, w.act)
    ref = oracle.jacobian_input(onet, inp.X)
    J = pfg.pfg_jacobian_input(gpu_net(inp, w.act, "f32"), gpu_x(inp, "f32"))
    torch.cuda.synchronize()
    e = slice_rel_err(J.cpu().numpy(), ref, lead=2)
    say(f"  c3-reduced J rel err {e:.3e}")
    assert e <= TOL_F32


@pytest.fixture(scope="module")
def c3_full():
    """The full-size Jacobian of c3, computed once for the four groups of examples below."""
    w = wl.WORKLOADS["c3_tanh_jacobian"]
    inp = draw(w)
    net = gpu_net(inp, w.act, "f32")
    out = torch.full((w.B, w.S, w.dims[0]), float("nan"), dtype=torch.float32, device="cuda:0")
    J = pfg.pfg_jacobian_input(net, gpu_x(inp, "f32"), out=out)
    torch.cuda.synchronize()
    assert not torch.isnan(J).any().item(), "the Jacobian was not written in full"
    yield w, inp, J.cpu().numpy()
    del J, out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("group", range(4))
def test_c3_tanh_jacobian_full_size_every_element(oracle, c3_full, group):
    # all 64 examples x 1024 rows x 1024 entries, 16 examples at a time (iterations are independent,
    # so the oracle on a subset of the examples gives those examples' slices)
    w, inp, J = c3_full
    idx = list(range(group * 16, group * 16 + 16))
    say(f"c3_tanh_jacobian: full size, every element of examples {idx[0]}..{idx[-1]}")
    onet = oracle.Net(inp.Ws, inp.bs, w.act)
    ref = oracle.jacobian_input(onet, inp.X[idx])
    e = slice_rel_err(J[idx], ref, lead=2)
    say(f"  c3 J rel err {e:.3e} over {len(idx) * w.S} rows")
    assert e <= TOL_F32


def test_c4_gelu_bf16_reduced_every_element(oracle):
    w = wl.WORKLOADS["c4_gelu_bf16_grads"]
    dims, B = (520, 392, 328, 10), 24
    say(f"c4 reduced {dims} B={B}: bf16 path, every element")
    inp = draw(w, B=B, dims=dims)
    check_grads(oracle, inp, w.act, "bf16", TOL_BF16, tag="c4-reduced-bf16")
    # the float32 path on the same bf16-rounded inputs separates input rounding from kernel error
    say("  same rounded inputs through the float32 path")
    check_grads(oracle, inp, w.act, "f32", TOL_F32, tag="c4-reduced-f32")


@pytest.fixture(scope="module")
def c4_full():
    """The full-size result of c4 (34.4 GB), computed once and kept on the device for the groups of
    examples below."""
    w = wl.WORKLOADS["c4_gelu_bf16_grads"]
    inp = draw(w)
    net = gpu_net(inp, w.act, "bf16")
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out_dW = [torch.full((w.B, net.dims[l], net.dims[l + 1]), float("nan"), **f32) for l in range(net.L)]
    dW, db, loss = pfg.pfg_per_example_grads(net, gpu_x(inp, "bf16"), dev(inp.labels), out_dW=out_dW)
    torch.cuda.synchronize()
    yield w, inp, dW, db, loss
    del dW, db, loss, out_dW
    torch.cuda.empty_cache()


@pytest.mark.parametrize("group", range(8))
def test_c4_gelu_bf16_full_size_every_element(oracle, c4_full, group):
    # all 256 examples, every one of the 8.6e9 values: 32 examples at a time, 16 per oracle call
    # (its float64 result for 16 examples is 8.6 GB), compared on the device
    w, inp, dW, db, loss = c4_full
    onet = oracle.Net(inp.Ws, inp.bs, w.act)
    worst, worst_elem = 0.0, 0.0
    for b0 in range(group * 32, group * 32 + 32, 16):
        idx = slice(b0, b0 + 16)
        rdW, rdb, rloss = oracle.per_example_grads(onet, inp.X[idx], inp.labels[idx])
        for l in range(len(dW)):
            ref = torch.from_numpy(rdW[l]).to("cuda:0")                     # float64 [16, d_in, d_out]
            got = dW[l][idx].double()
            assert torch.isfinite(got).all().item(), f"dW{l + 1} was not written in full"
            diff = (got - ref).abs_()
            den = ref.abs().amax(dim=(1, 2))
            assert (den > 0).all().item()
            worst = max(worst, float((diff.amax(dim=(1, 2)) / den).max().item()))
            # element-wise, as parity_util.outer_elem_err measures it: against the largest entry of
            # the element's row plus that of its column
            ref.abs_()
            diff /= ref.amax(dim=2, keepdim=True) + ref.amax(dim=1, keepdim=True)
            worst_elem = max(worst_elem, float(diff.max().item()))
            del ref, got, diff
            worst = max(worst, slice_rel_err(db[l][idx].cpu().numpy(), rdb[l]))
        worst = max(worst, slice_rel_err(loss[idx].cpu().numpy(), rloss, lead=0))
        del rdW
        say(f"  c4 examples {b0}..{b0 + 15}: every element, running worst rel err {worst:.3e}, "
            f"by row and column scale {worst_elem:.3e}")
    assert worst <= TOL_BF16 and worst_elem <= TOL_BF16


def test_narrow_rows_of_a_large_output_every_element(oracle):
    # layers whose rows are 256 and 512 floats wide and whose gradients fill half a GiB or more leave in
    # launches of their own, one 4 KiB slab (4 or 2 whole rows) per workgroup: 1 GiB + 0.5 GiB here,
    # every element against the oracle, 64 examples at a time, compared on the device
    w = wl.WORKLOADS["c2_mnist_mlp_grads"]
    dims, B = (1024, 256, 512, 10), 1024
    say(f"narrow rows {dims} B={B}: every element")
    act = "tanh"             # (with relu, 800 000 pre-activations cannot all be kept off the kink)
    inp = draw(w, B=B, dims=dims, act=act)
    net = gpu_net(inp, act, "f32")
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out_dW = [torch.full((B, dims[l], dims[l + 1]), float("nan"), **f32) for l in range(3)]
    dW, db, loss = pfg.pfg_per_example_grads(net, gpu_x(inp, "f32"), dev(inp.labels), out_dW=out_dW)
    torch.cuda.synchronize()
    onet = oracle.Net(inp.Ws, inp.bs, act)
    worst = 0.0
    for b0 in range(0, B, 64):
        idx = slice(b0, b0 + 64)
        rdW, rdb, rloss = oracle.per_example_grads(onet, inp.X[idx], inp.labels[idx])
        for l in range(3):
            ref = torch.from_numpy(rdW[l]).to("cuda:0")
            got = dW[l][idx].double()
            assert torch.isfinite(got).all().item(), f"dW{l + 1} was not written in full"
            den = ref.abs().amax(dim=(1, 2))
            err = (got - ref).abs_().amax(dim=(1, 2))
            # an example whose reference slice is identically zero (every unit of a layer off) must be zero
            assert ((den > 0) | (err == 0)).all().item()
            worst = max(worst, float((err / den.clamp_min(1e-300)).max().item()))
            del ref, got
            worst = max(worst, slice_rel_err(db[l][idx].cpu().numpy(), rdb[l]))
        worst = max(worst, slice_rel_err(loss[idx].cpu().numpy(), rloss, lead=0))
    say(f"  worst rel err {worst:.3e}")
    assert worst <= TOL_F32
    del dW, out_dW
    torch.cuda.empty_cache()


def test_c5_nested_weight_jacobian_full_size(oracle):
    w = wl.WORKLOADS["c5_nested_weight_jacobian"]
    say("c5_nested_weight_jacobian: full size, every element")
    inp = draw(w)
    onet = oracle.Net(inp.Ws, inp.bs, w.act)
    ref_JW, ref_Jb = oracle.jacobian_weights(onet, inp.X, head="softmax", want_JW=[True, False])
    net = gpu_net(inp, w.act, "f32")
    out = [torch.full((w.B, w.S, 256, 256), float("nan"), dtype=torch.float32, device="cuda:0"),
           None]
    JW, Jb = pfg.pfg_jacobian_weights(net, gpu_x(inp, "f32"), head="softmax", out_JW=out)
    torch.cuda.synchronize()
    e = max(slice_rel_err(JW[0].cpu().numpy(), ref_JW[0], lead=2), outer_elem_err(JW[0].cpu().numpy(), ref_JW[0]))
    say(f"  c5 JW1 rel err (the larger of per-slice and by row and column scale) {e:.3e}")
    eb = max(slice_rel_err(Jb[l].cpu().numpy(), ref_Jb[l], lead=2) for l in range(2))
    say(f"  c5 Jb rel err {eb:.3e}")
    assert max(e, eb) <= TOL_F32


# --------------------------------------------------------------------------------------------
# Edge cases and odd shapes.
# --------------------------------------------------------------------------------------------
SHAPES = [
    # dims, B, act, bias_scale
    ((7, 5), 1, "relu", 0.3),                 # one layer, one example
    ((3, 1, 2), 3, "tanh", 0.3),              # a hidden layer of width one
    ((33, 65, 129, 10), 9, "gelu", 0.3),      # every size one past a tile edge
    ((64, 128, 64), 128, "relu", 0.0),        # exact tile multiples
    ((130, 6, 4, 260), 17, "identity", 0.3),  # narrow middle, wide ends
    ((1, 1), 1, "tanh", 0.3),                 # the smallest network
    ((20, 300, 12), 70, "tanh", 0.2),
]


@pytest.mark.parametrize("dims,B,act,bias_scale", SHAPES, ids=[f"{s[0]}-B{s[1]}-{s[2]}" for s in SHAPES])
def test_odd_shapes_all_three_calls(oracle, dims, B, act, bias_scale):
    say(f"odd shape {dims} B={B} act={act}")
    w = wl.Workload("odd", 50 + len(dims) + B, "per_example_grads", tuple(dims), act, "f32", B,
                    "normal", "normal_fan_in")
    inp = draw(w, bias_scale=bias_scale, act=act)
    check_grads(oracle, inp, act, "f32", TOL_F32, tag=f"odd{dims}")
    onet = oracle.Net(inp.Ws, inp.bs, act)
    net = gpu_net(inp, act, "f32")
    X = gpu_x(inp, "f32")
    rng = np.random.default_rng(B)
    dL = dims[-1]
    shared = rng.standard_normal((3, dL)).astype(np.float32)
    per_ex = rng.standard_normal((B, 2, dL)).astype(np.float32)
    for name, seeds in (("identity", None), ("shared", shared), ("per-example", per_ex)):
        ref = oracle.jacobian_input(onet, inp.X, seeds=seeds)
        J = pfg.pfg_jacobian_input(net, X, seeds=None if seeds is None else dev(seeds))
        torch.cuda.synchronize()
        e = slice_rel_err(J.cpu().numpy(), ref, lead=2)
        say(f"  J[{name}] rel err {e:.3e}")
        assert e <= TOL_F32
        for head in ("logits", "softmax"):
            rJW, rJb = oracle.jacobian_weights(onet, inp.X, head=head, seeds=seeds)
            JW, Jb = pfg.pfg_jacobian_weights(net, X, head=head,
                                              seeds=None if seeds is None else dev(seeds))
            torch.cuda.synchronize()
            e = max(max(slice_rel_err(JW[l].cpu().numpy(), rJW[l], lead=2),
                        slice_rel_err(Jb[l].cpu().numpy(), rJb[l], lead=2))
                    for l in range(net.L))
            say(f"  JW[{name},{head}] rel err {e:.3e}")
            assert e <= TOL_F32


def test_bf16_odd_shapes(oracle):
    for dims, B, act in (((37, 70, 10), 5, "gelu"), ((64, 64, 64, 16), 33, "tanh"),
                         ((9, 200, 3), 2, "relu")):
        say(f"bf16 odd shape {dims} B={B} act={act}")
        w = wl.Workload("oddbf", 90 + B, "per_example_grads", dims, act, "bf16", B, "normal",
                        "normal_fan_in")
        inp = draw(w, bias_scale=0.25, act=act)
        check_grads(oracle, inp, act, "bf16", TOL_BF16, tag=f"bf16{dims}")
        onet = oracle.Net(inp.Ws, inp.bs, act)
        net = gpu_net(inp, act, "bf16")
        X = gpu_x(inp, "bf16")
        ref = oracle.jacobian_input(onet, inp.X)
        J = pfg.pfg_jacobian_input(net, X)
        rJW, rJb = oracle.jacobian_weights(onet, inp.X, head="softmax")
        JW, Jb = pfg.pfg_jacobian_weights(net, X, head="softmax")
        torch.cuda.synchronize()
        e = slice_rel_err(J.cpu().numpy(), ref, lead=2)
        e2 = max(slice_rel_err(JW[l].cpu().numpy(), rJW[l], lead=2) for l in range(net.L))
        say(f"  bf16 J rel err {e:.3e}, JW rel err {e2:.3e}")
        assert max(e, e2) <= TOL_BF16


def test_skipped_outputs_and_early_stop(oracle):
    w = wl.Workload("skip", 70, "per_example_grads", (24, 40, 36, 8), "tanh", "f32", 6, "normal",
                    "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    check_grads(oracle, inp, "tanh", "f32", TOL_F32, want_dW=[False, True, False], tag="skip")
    onet = oracle.Net(inp.Ws, inp.bs, "tanh")
    net = gpu_net(inp, "tanh", "f32")
    X = gpu_x(inp, "f32")
    # only the top layer's weight gradient, no bias gradients, no loss: the sweep stops early
    dW, db, loss = pfg.pfg_per_example_grads(net, X, dev(inp.labels), want_dW=[False, False, True],
                                             want_db=False, want_loss=False)
    torch.cuda.synchronize()
    assert db is None and loss is None and dW[0] is None and dW[1] is None
    ref_dW, _, _ = oracle.per_example_grads(onet, inp.X, inp.labels)
    assert slice_rel_err(dW[2].cpu().numpy(), ref_dW[2]) <= TOL_F32
    JW, Jb = pfg.pfg_jacobian_weights(net, X, head="softmax", want_JW=[True, False, False],
                                      want_Jb=False)
    torch.cuda.synchronize()
    rJW, _ = oracle.jacobian_weights(onet, inp.X, head="softmax")
    assert Jb is None and JW[1] is None
    assert slice_rel_err(JW[0].cpu().numpy(), rJW[0], lead=2) <= TOL_F32


def test_unaligned_buffers_take_the_scalar_paths(oracle):
    w = wl.Workload("unal", 71, "per_example_grads", (12, 20, 8), "tanh", "f32", 5, "normal",
                    "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    onet = oracle.Net(inp.Ws, inp.bs, "tanh")

    def shifted(a):                        # same values, storage offset by one float (4 bytes)
        flat = torch.empty(a.size + 1, dtype=torch.float32, device="cuda:0")
        flat[1:] = torch.from_numpy(a.reshape(-1)).to("cuda:0")
        return flat[1:].view(*a.shape)

    net = pfg.Mlp([shifted(W) for W in inp.Ws], [shifted(b) for b in inp.bs], "tanh", "f32")
    X = shifted(inp.X)
    B = 5
    out_dW = [shifted(np.full((B, 12, 20), np.nan, np.float32)),
              shifted(np.full((B, 20, 8), np.nan, np.float32))]
    dW, db, loss = pfg.pfg_per_example_grads(net, X, dev(inp.labels), out_dW=out_dW)
    J = pfg.pfg_jacobian_input(net, X, out=shifted(np.full((B, 8, 12), np.nan, np.float32)))
    torch.cuda.synchronize()
    ref_dW, ref_db, _ = oracle.per_example_grads(onet, inp.X, inp.labels)
    for l in range(2):
        assert slice_rel_err(dW[l].cpu().numpy(), ref_dW[l]) <= TOL_F32
        assert slice_rel_err(db[l].cpu().numpy(), ref_db[l]) <= TOL_F32
    assert slice_rel_err(J.cpu().numpy(), oracle.jacobian_input(onet, inp.X), lead=2) <= TOL_F32


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_batch_takes_the_tiled_kernels(oracle, dtype):
    # B = 8200 rows: every product has at least 128 tiles of 64 x 64 and goes through the LDS-tiled
    # kernel (forward [K, N] layout and cotangent [N, K] layout), with a ragged last row tile;
    # dims chosen so that one layer meets the fast-load conditions and one does not
    dims, B, act = (96, 160, 70, 12), 8200, "gelu"
    say(f"tiled kernels: dims {dims} B={B} {dtype}")
    w = wl.Workload("tiled", 60, "per_example_grads", dims, act, dtype, B, "normal", "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    check_grads(oracle, inp, act, dtype, tol, want_dW=[False, False, True], tag=f"tiled-{dtype}")
    # input Jacobian with per-example seeds: M = B * S rows through the cotangent kernels
    Bj, S = 700, 12
    onet = oracle.Net(inp.Ws, inp.bs, act)
    seeds = np.random.default_rng(5).standard_normal((Bj, S, dims[-1])).astype(np.float32)
    ref = oracle.jacobian_input(onet, inp.X[:Bj], seeds=seeds)
    net = gpu_net(inp, act, dtype)
    J = pfg.pfg_jacobian_input(net, gpu_x(inp, dtype)[:Bj].contiguous(), seeds=dev(seeds))
    torch.cuda.synchronize()
    e = slice_rel_err(J.cpu().numpy(), ref, lead=2)
    say(f"  tiled-{dtype} J per-example seeds rel err {e:.3e}")
    assert e <= tol


def test_long_contractions_are_cut_into_pieces(oracle):
    # few rows against wide layers with long contractions: the forward products (K = 2048 and 1024)
    # are computed as 8 and 4 partial products that a second kernel adds; 96 rows leave a ragged
    # row tile
    dims, B, act = (2048, 1024, 1280, 10), 96, "tanh"
    say(f"split contraction: dims {dims} B={B}")
    w = wl.Workload("splitk", 61, "per_example_grads", dims, act, "f32", B, "normal", "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    check_grads(oracle, inp, act, "f32", TOL_F32, want_dW=[False, True, True], tag="splitk")
    onet = oracle.Net(inp.Ws, inp.bs, act)
    net = gpu_net(inp, act, "f32")
    rsq, _ = oracle.per_example_grad_norms(onet, inp.X, inp.labels)
    sq, norm, _ = pfg.pfg_per_example_grad_norms(net, gpu_x(inp, "f32"), dev(inp.labels))
    torch.cuda.synchronize()
    e = float(np.max(np.abs(sq.cpu().numpy() - rsq) / rsq))
    say(f"  splitk norms rel err {e:.3e}")
    assert e <= TOL_F32


def test_float32_product_with_one_workgroup_per_unit_is_cut_in_two(oracle):
    # 800 rows against 1024 x 1024 weights: 208 tiles of 64 x 64, which the tiled kernel would run
    # on 208 of the 256 units; the product is computed as two pieces instead
    dims, B, act = (1024, 1024, 10), 800, "gelu"
    say(f"two-piece product: dims {dims} B={B}")
    w = wl.Workload("split2", 64, "per_example_grads", dims, act, "f32", B, "normal", "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    check_grads(oracle, inp, act, "f32", TOL_F32, want_dW=[False, True], tag="split2")


def test_bf16_few_rows_against_a_long_contraction(oracle):
    # 5 rows, bf16: the first forward product (K = 1024, 512 columns) is cut into 4 pieces although
    # it has less than one full row tile; 150 rows: 3 row tiles, the last one ragged
    for B in (5, 150):
        dims, act = (1024, 512, 10), "tanh"
        say(f"bf16 split contraction: dims {dims} B={B}")
        w = wl.Workload("splitbf", 63, "per_example_grads", dims, act, "bf16", B, "normal", "normal_fan_in")
        inp = draw(w, bias_scale=0.2)
        check_grads(oracle, inp, act, "bf16", TOL_BF16, want_dW=[False, True], tag=f"splitbf-B{B}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_head_with_a_long_contraction_is_cut_into_pieces(oracle, dtype):
    # a 2048-wide last hidden layer and 200 rows: the logits are 32 partial products of 64 columns
    # each, added by the kernel that then does softmax, loss and the cotangent step; the last row
    # tile holds 8 rows, 7 classes leave most of a 32-column tile empty
    dims, B, act = (96, 2048, 7), 200, "gelu"
    say(f"split head: dims {dims} B={B} {dtype}")
    w = wl.Workload("splithead", 62, "per_example_grads", dims, act, dtype, B, "normal", "normal_fan_in")
    inp = draw(w, bias_scale=0.2)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    check_grads(oracle, inp, act, dtype, tol, want_dW=[False, True], tag=f"splithead-{dtype}")
    # only the last layer's weight gradient wanted: no cotangent step rides on the head
    dW, db, loss = pfg.pfg_per_example_grads(gpu_net(inp, act, dtype), gpu_x(inp, dtype), dev(inp.labels),
                                             want_dW=[False, True], want_db=False)
    torch.cuda.synchronize()
    ref_dW, _, ref_loss = oracle.per_example_grads(oracle.Net(inp.Ws, inp.bs, act), inp.X, inp.labels,
                                                   want_dW=[False, True])
    assert slice_rel_err(dW[1].cpu().numpy(), ref_dW[1]) <= tol
    assert slice_rel_err(loss.cpu().numpy(), ref_loss, lead=0) <= tol


def test_deep_network_and_wide_seed_block(oracle):
    # five layers; weight Jacobian with shared seeds S = 40 > d_L, all layers, softmax head
    dims, B, act = (24, 48, 40, 56, 32, 20), 9, "tanh"
    say(f"deep network {dims} B={B}")
    w = wl.Workload("deep", 61, "per_example_grads", dims, act, "f32", B, "normal", "normal_fan_in")
    inp = draw(w, bias_scale=0.3)
    check_grads(oracle, inp, act, "f32", TOL_F32, tag="deep")
    onet = oracle.Net(inp.Ws, inp.bs, act)
    net = gpu_net(inp, act, "f32")
    seeds = np.random.default_rng(6).standard_normal((40, dims[-1])).astype(np.float32)
    rJW, rJb = oracle.jacobian_weights(onet, inp.X, head="softmax", seeds=seeds)
    JW, Jb = pfg.pfg_jacobian_weights(net, gpu_x(inp, "f32"), head="softmax", seeds=dev(seeds))
    J = pfg.pfg_jacobian_input(net, gpu_x(inp, "f32"), seeds=dev(seeds))
    torch.cuda.synchronize()
    e = max(max(slice_rel_err(JW[l].cpu().numpy(), rJW[l], lead=2),
                slice_rel_err(Jb[l].cpu().numpy(), rJb[l], lead=2)) for l in range(net.L))
    say(f"  deep JW/Jb rel err {e:.3e}")
    assert e <= TOL_F32
    e = slice_rel_err(J.cpu().numpy(), oracle.jacobian_input(onet, inp.X, seeds=seeds), lead=2)
    say(f"  deep J rel err {e:.3e}")
    assert e <= TOL_F32


def test_graph_replay_matches_eager(oracle):
    # one call captured into a HIP graph (the library records only kernel launches, no memsets)
    # and replayed several times with eager work and synchronisations in between; every replay
    # must reproduce the eager result bit for bit
    w = wl.WORKLOADS["c2_mnist_mlp_grads"]
    inp = draw(w, B=32)
    net = gpu_net(inp, w.act, "f32")
    X, labels = gpu_x(inp, "f32"), dev(inp.labels)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    B = 32

    def buffers():
        return ([torch.zeros((B, net.dims[l], net.dims[l + 1]), **f32) for l in range(net.L)],
                [torch.zeros((B, net.dims[l + 1]), **f32) for l in range(net.L)],
                torch.zeros((B,), **f32),
                torch.empty(pfg.pfg_workspace_bytes(net, "per_example_grads", B), dtype=torch.uint8,
                            device="cuda:0"))

    dW_e, db_e, loss_e, ws_e = buffers()
    pfg.pfg_per_example_grads(net, X, labels, out_dW=dW_e, out_db=db_e, out_loss=loss_e,
                              workspace=ws_e)
    torch.cuda.synchronize()
    dW_g, db_g, loss_g, ws_g = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pfg.pfg_per_example_grads(net, X, labels, out_dW=dW_g, out_db=db_g, out_loss=loss_g,
                                  workspace=ws_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pfg.pfg_per_example_grads(net, X, labels, out_dW=dW_g, out_db=db_g, out_loss=loss_g,
                                  workspace=ws_g)
    for replay in range(4):
        for t in dW_g + db_g + [loss_g]:
            t.fill_(float("nan"))                      # eager work between the replays
        pfg.pfg_jacobian_input(net, X)                 # an eager call of the library in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(net.L):
            assert torch.equal(dW_g[l], dW_e[l]), f"replay {replay}: dW{l + 1} differs"
            assert torch.equal(db_g[l], db_e[l]), f"replay {replay}: db{l + 1} differs"
        assert torch.equal(loss_g, loss_e)


def test_iterations_are_independent(oracle):
    # permuting the batch permutes the slices bit for bit; a duplicated example gives identical
    # slices (stateless parallel-for, Section 3.4)
    w = wl.WORKLOADS["c1_tiny"]
    inp = draw(w)
    inp.X[5] = inp.X[2]
    inp.labels[5] = inp.labels[2]
    net = gpu_net(inp, w.act, "f32")
    dW, db, loss = pfg.pfg_per_example_grads(net, dev(inp.X), dev(inp.labels))
    perm = np.random.default_rng(0).permutation(16)
    dWp, dbp, lossp = pfg.pfg_per_example_grads(net, dev(inp.X[perm]), dev(inp.labels[perm]))
    torch.cuda.synchronize()
    for l in range(net.L):
        assert torch.equal(dWp[l].cpu(), dW[l].cpu()[perm])
        assert torch.equal(dW[l][5], dW[l][2])
    assert torch.equal(lossp.cpu(), loss.cpu()[perm])


def test_timing_facility_and_error_after_gpu_use(oracle):
    w = wl.WORKLOADS["c1_tiny"]
    inp = draw(w)
    net = gpu_net(inp, w.act, "f32")
    pfg.pfg_timing_reset()
    pfg.pfg_timing_enable(True)
    try:
        for _ in range(3):
            pfg.pfg_per_example_grads(net, dev(inp.X), dev(inp.labels))
    finally:
        pfg.pfg_timing_enable(False)
    # one launch writes the outer products of all layers; with d_L <= 32 the loss head and the
    # cotangent step through the last layer ride on the last forward layer, so this two-layer
    # network needs no separate head or cotangent kernel
    n, ms = pfg.pfg_timing_query("outer_product")
    assert n == 3 and ms > 0.0
    assert set(pfg.pfg_timing_names()) == {"gemm_forward", "outer_product"}
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_jacobian_input(net, dev(inp.X), S=3)
    assert ei.value.code == pfg.PFG_ERR_SHAPE
    pfg.pfg_timing_reset()
