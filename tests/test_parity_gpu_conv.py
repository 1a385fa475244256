"""GPU parity for the convolutional network: per-example gradients from the HIP library, called
through its C ABI, against the float64 CPU oracle (oracle/conv_oracle.c) on the same seeded inputs.
Error measure as in test_parity_gpu.py: per example and per tensor max|gpu - ref| / max|ref|, at
most 1e-4; slices that are exactly zero in the reference must be exactly zero on the GPU.

Decisions taken on floating-point values (the sign of a pre-activation under ReLU, which entry of
a pooling window is largest) are taken in float32 on the GPU and in float64 by the oracle.  With
tens of thousands of units per image some example always has a unit within float32 round-off of
such a boundary, where the two sides may legitimately decide differently.  The test therefore
computes, with a float64 library convolution (not the oracle), each example's distance to the
nearest decision boundary and compares element by element the examples whose distance is at least
2e-6 (round-off of these pre-activations is ~1e-7); it requires that most examples qualify and
that every output of the others is finite.
"""
import numpy as np
import pytest

from parity_util import TOL_F32, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import torch.nn.functional as F  # noqa: E402

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, say  # noqa: E402
from oracle import conv as oconv  # noqa: E402

MARGIN = 2e-6


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def decision_margins(inp):
    """Per example: the smallest distance of any ReLU input from zero and of any pooling window's
    largest entry from its runner-up (float64, library convolution)."""
    a = torch.from_numpy(inp.X.astype(np.float64)).permute(0, 3, 1, 2)
    B = a.shape[0]
    m = torch.full((B,), float("inf"), dtype=torch.float64)
    for W, b in zip(inp.Wc, inp.bc):
        k = W.shape[0]
        z = F.conv2d(a, torch.from_numpy(W.astype(np.float64)).permute(3, 2, 0, 1),
                     torch.from_numpy(b.astype(np.float64)), padding=(k - 1) // 2)
        m = torch.minimum(m, z.abs().flatten(1).min(dim=1).values)
        r = torch.relu(z)
        win = F.unfold(r, 2, stride=2).reshape(B, r.shape[1], 4, -1)          # [B, C, 4, cells]
        top = win.topk(2, dim=2).values
        gap = torch.where(top[:, :, 0] > 0, top[:, :, 0] - top[:, :, 1], torch.full_like(top[:, :, 0], float("inf")))
        m = torch.minimum(m, gap.flatten(1).min(dim=1).values)
        a = F.max_pool2d(r, 2)
    h = a.permute(0, 2, 3, 1).reshape(B, -1)
    for l, (W, b) in enumerate(zip(inp.Ws, inp.bs)):
        h = h @ torch.from_numpy(W.astype(np.float64)) + torch.from_numpy(b.astype(np.float64))
        if l < len(inp.Ws) - 1:
            m = torch.minimum(m, h.abs().min(dim=1).values)
            h = torch.relu(h)
    return m.numpy()


def nan_like(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")


def check_conv(inp, tag, examples=None, min_checked=0.5):
    B, h, w, c = inp.X.shape
    onet = oconv.ConvNet(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    net = pfg.ConvNet.from_numpy(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    dn = net.dense
    out = ([nan_like(B, *W.shape) for W in inp.Wc], [nan_like(B, W.shape[3]) for W in inp.Wc],
           [nan_like(B, dn.dims[l], dn.dims[l + 1]) for l in range(dn.L)],
           [nan_like(B, dn.dims[l + 1]) for l in range(dn.L)], nan_like(B))
    dWc, dbc, dW, db, loss = pfg.pfg_convnet_per_example_grads(net, dev(inp.X), dev(inp.labels), out=out)
    torch.cuda.synchronize()
    got = [t.cpu().numpy() for t in dWc + dbc + dW + db] + [loss.cpu().numpy()]
    names = ([f"dWc{i + 1}" for i in range(net.nc)] + [f"dbc{i + 1}" for i in range(net.nc)] +
             [f"dW{l + 1}" for l in range(dn.L)] + [f"db{l + 1}" for l in range(dn.L)] + ["loss"])
    for n, a in zip(names, got):
        assert np.isfinite(a).all(), f"{n} was not written in full"
    margins = decision_margins(inp)
    idx = [b for b in (range(B) if examples is None else examples) if margins[b] >= MARGIN]
    total = B if examples is None else len(list(examples))
    say(f"  {tag}: {len(idx)} of {total} examples are at least {MARGIN:g} from every decision boundary")
    assert len(idx) >= min_checked * total
    rdWc, rdbc, rdW, rdb, rloss = oconv.per_example_grads(onet, inp.X[idx], inp.labels[idx])
    ref = rdWc + rdbc + rdW + rdb + [rloss]
    worst = 0.0
    for n, a, r in zip(names, got, ref):
        e = slice_rel_err(a[idx], r, lead=0 if n == "loss" else 1)
        say(f"  {tag} {n} rel err {e:.3e}")
        worst = max(worst, e)
    assert worst <= TOL_F32, f"{tag}: max relative error {worst:.3e}"
    return net, (dWc, dbc, dW, db, loss)


CONV_SHAPES = [
    # height, width, channels, blocks, dense, B
    (4, 4, 1, ((3, 2),), (3,), 2),
    (8, 8, 2, ((3, 3), (3, 5)), (6, 4), 3),
    (2, 2, 1, ((1, 1),), (2,), 1),                       # the smallest: a 1 x 1 filter, one window
    (12, 8, 3, ((5, 4), (3, 6)), (9, 40), 5),            # non-square, more than 32 classes
    (16, 16, 1, ((5, 8), (5, 16), (3, 8)), (10,), 4),    # three blocks
    (20, 12, 2, ((7, 5),), (33, 7), 70),                 # a 7 x 7 filter; enough rows for the tiled kernels
    (8, 12, 4, ((3, 12), (3, 8)), (11, 6), 140),         # filter gradients read the patches transposed
    (8, 8, 8, ((3, 64),), (9,), 70),                     # the same with a wide filter bank
    (10, 6, 8, ((5, 16),), (12,), 300),                  # products that gather their patches from the image (c % 4 == 0, many rows)
    (12, 20, 3, ((3, 4), (1, 8)), (5,), 37),             # few taps per output: both blocks go from image to pooled output in one kernel
    (28, 6, 1, ((7, 8),), (6,), 600),                    # the same with one workgroup per example (14 pooled rows in a band)
    (20, 8, 1, ((5, 12),), (7,), 90),                    # bands of 2 pooled rows and a ragged last one (5 rows)
    # blocks with many channels on a small map, enough examples for the matrix-core kernels that read the
    # image from LDS (the library takes them from about half a chip of workgroups on)
    (16, 16, 4, ((3, 32), (3, 64)), (12,), 120),         # 8 x 8 x 32 -> 64, 3 x 3: two position tiles, one per workgroup in the reverse kernel
    (28, 28, 1, ((5, 32), (5, 64)), (16, 10), 66),       # the MNIST model's second block: 7 tiles dealt 3 + 3 + 1 in the reverse kernel
    (8, 8, 8, ((3, 64), (3, 32)), (7,), 130),            # 64 -> 32 channels: two channel tiles in the reverse kernels
    (24, 24, 2, ((3, 32), (5, 32)), (8,), 230),          # 12 x 12 positions: five tiles in one workgroup
    (16, 16, 4, ((3, 32), (3, 64)), (12,), 5),           # the same blocks with few examples: the tiled products
]


@pytest.mark.parametrize("h,w,c,blocks,dense,B", CONV_SHAPES,
                         ids=[f"{s[0]}x{s[1]}x{s[2]}-{len(s[3])}blocks-B{s[5]}" for s in CONV_SHAPES])
def test_convnet_odd_shapes(h, w, c, blocks, dense, B):
    say(f"convnet {h}x{w}x{c} blocks={blocks} dense={dense} B={B}")
    wk = wl.ConvWorkload("oddc", 500 + h + w + B, h, w, c, blocks, dense, B)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    check_conv(inp, "conv-odd")


def test_convnet_skipped_outputs_and_batch_order():
    wk = wl.ConvWorkload("skipc", 540, 8, 8, 2, ((3, 4), (3, 6)), (8, 5), 6)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    net, full = check_conv(inp, "conv-skip")
    X, labels = dev(inp.X), dev(inp.labels)
    # only the dense gradients: the reverse pass through the conv blocks is skipped
    dWc, dbc, dW, db, loss = pfg.pfg_convnet_per_example_grads(net, X, labels, want_dWc=[False, False],
                                                               want_dbc=False)
    torch.cuda.synchronize()
    assert dbc is None and dWc == [None, None]
    assert all(torch.equal(a, b) for a, b in zip(dW + db + [loss], full[2] + full[3] + [full[4]]))
    # only the top conv block's filter gradient: the sweep stops above the first block
    dWc, dbc, dW, db, loss = pfg.pfg_convnet_per_example_grads(net, X, labels, want_dWc=[False, True],
                                                               want_dbc=False, want_dW=[False, False],
                                                               want_db=False, want_loss=False)
    torch.cuda.synchronize()
    assert dWc[0] is None and torch.equal(dWc[1], full[0][1])
    # iteration independence: a permuted batch gives the permuted results, bit for bit
    perm = np.random.default_rng(54).permutation(6)
    outp = pfg.pfg_convnet_per_example_grads(net, dev(inp.X[perm]), dev(inp.labels[perm]))
    torch.cuda.synchronize()
    tperm = torch.from_numpy(perm).to("cuda:0")
    assert torch.equal(outp[0][0], full[0][0][tperm]) and torch.equal(outp[0][1], full[0][1][tperm])
    assert torch.equal(outp[2][0], full[2][0][tperm]) and torch.equal(outp[4], full[4][tperm])


def test_c10_mnist_convnet_full_size():
    wk = wl.CONV_WORKLOADS["c10_mnist_convnet_grads"]
    say("c10_mnist_convnet_grads: full size (128 images, 28 x 28), sampled examples element by element")
    inp = wl.make_conv_inputs(wk)
    picks = sorted(set([0, wk.B - 1] + np.random.default_rng(10).integers(0, wk.B, size=24).tolist()))
    net, out = check_conv(inp, "c10", examples=picks)
    # a property that holds for every example: the first dense layer's gradient is the outer
    # product of the conv features and that layer's bias gradient, so its rows are multiples of db1
    dW1, db1 = out[2][0], out[3][0]
    j = db1.abs().argmax(dim=1)
    rows = torch.arange(wk.B, device="cuda:0")
    feat = dW1[rows, :, j] / db1[rows, j].unsqueeze(1)
    recon = feat.unsqueeze(2) * db1.unsqueeze(1)
    dev_rel = ((recon - dW1).abs().amax(dim=(1, 2)) / dW1.abs().amax(dim=(1, 2)).clamp_min(1e-30)).max().item()
    say(f"  c10 dW1 rank-one consistency {dev_rel:.3e}")
    assert dev_rel < 1e-4


def check_conv_norms(inp, tag, examples=None, min_checked=0.5, drop_bias=()):
    """Gradient norms without the gradients against the oracle's (the gradient formed, its
    squares summed); drop_bias names parameter blocks (conv blocks first) that lose their bias."""
    B, h, w, c = inp.X.shape
    nc = len(inp.Wc)
    bc = [None if i in drop_bias else v for i, v in enumerate(inp.bc)]
    bs = [None if nc + l in drop_bias else v for l, v in enumerate(inp.bs)]
    onet = oconv.ConvNet(h, w, c, inp.Wc, bc, inp.Ws, bs)
    net = pfg.ConvNet.from_numpy(h, w, c, inp.Wc, bc, inp.Ws, bs)
    cols = nc + net.dense.L
    out = (nan_like(B, cols), nan_like(B), nan_like(B))
    sq, norm, loss = pfg.pfg_convnet_per_example_grad_norms(net, dev(inp.X), dev(inp.labels), out=out)
    torch.cuda.synchronize()
    got = [t.cpu().numpy() for t in (sq, norm, loss)]
    for n, a in zip(("sq", "norm", "loss"), got):
        assert np.isfinite(a).all(), f"{n} was not written in full"
    biased = type(inp)(inp.workload, inp.Wc, [np.zeros_like(v) if b is None else b for v, b in zip(inp.bc, bc)],
                       inp.Ws, [np.zeros_like(v) if b is None else b for v, b in zip(inp.bs, bs)], inp.X, inp.labels)
    margins = decision_margins(biased)
    idx = [b for b in (range(B) if examples is None else examples) if margins[b] >= MARGIN]
    total = B if examples is None else len(list(examples))
    say(f"  {tag}: {len(idx)} of {total} examples are at least {MARGIN:g} from every decision boundary")
    assert len(idx) >= min_checked * total
    rsq, rnorm, rloss = oconv.per_example_grad_norms(onet, inp.X[idx], inp.labels[idx])
    worst = 0.0
    for j in range(cols):                       # every column against its own scale
        e = float(np.max(np.abs(got[0][idx, j] - rsq[:, j]) / np.maximum(np.abs(rsq[:, j]), 1e-300)))
        say(f"  {tag} sq[:, {j}] rel err {e:.3e}")
        worst = max(worst, e)
    e = float(np.max(np.abs(got[1][idx] - rnorm) / rnorm))
    say(f"  {tag} norm rel err {e:.3e}")
    worst = max(worst, e, slice_rel_err(got[2][idx], rloss, lead=0))
    assert worst <= TOL_F32, f"{tag}: max relative error {worst:.3e}"
    return net, (sq, norm, loss)


NORM_SHAPES = [
    # height, width, channels, blocks, dense, B, parameter blocks without a bias
    (4, 4, 1, ((3, 2),), (3,), 2, ()),
    (8, 8, 2, ((3, 3), (3, 5)), (6, 4), 3, (0, 3)),
    (2, 2, 1, ((1, 1),), (2,), 1, ()),
    (12, 8, 3, ((5, 4), (3, 6)), (9, 40), 5, (1,)),
    (16, 16, 1, ((5, 8), (5, 16), (3, 8)), (10,), 4, ()),
    (20, 12, 2, ((7, 5),), (33, 7), 70, (0, 1, 2)),
    (8, 12, 4, ((3, 12), (3, 8)), (11, 6), 140, ()),
    (8, 8, 8, ((3, 64),), (9,), 70, ()),
    (10, 6, 8, ((5, 16),), (12,), 300, (0,)),
    (12, 20, 3, ((3, 4), (1, 8)), (5,), 37, (1,)),       # image-to-pooled-output kernel, one block without a bias
    (16, 16, 4, ((3, 32), (3, 64)), (12,), 120, (1,)),   # matrix-core kernels on the LDS image, a block without a bias
    (24, 24, 2, ((3, 32), (5, 32)), (8,), 230, ()),
]


@pytest.mark.parametrize("h,w,c,blocks,dense,B,drop", NORM_SHAPES,
                         ids=[f"{s[0]}x{s[1]}x{s[2]}-{len(s[3])}blocks-B{s[5]}" for s in NORM_SHAPES])
def test_convnet_grad_norms_odd_shapes(h, w, c, blocks, dense, B, drop):
    say(f"convnet norms {h}x{w}x{c} blocks={blocks} dense={dense} B={B} without bias: {drop}")
    wk = wl.ConvWorkload("oddn", 600 + h + w + B, h, w, c, blocks, dense, B)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    check_conv_norms(inp, "conv-norms-odd", drop_bias=drop)


def test_convnet_grad_norms_agree_with_the_gradients_and_skip_outputs():
    wk = wl.ConvWorkload("normc", 560, 8, 8, 2, ((3, 4), (3, 6)), (8, 5), 9)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    net, (sq, norm, loss) = check_conv_norms(inp, "conv-norms")
    X, labels = dev(inp.X), dev(inp.labels)
    # the same sweep produced the gradients: their squared sums agree to rounding for EVERY example
    dWc, dbc, dW, db, loss_g = pfg.pfg_convnet_per_example_grads(net, X, labels)
    torch.cuda.synchronize()
    want = torch.stack([(a.double() ** 2).flatten(1).sum(1) + (b.double() ** 2).sum(1)
                        for a, b in zip(dWc + dW, dbc + db)], dim=1)
    assert ((sq.double() - want).abs() / want).max().item() < 1e-5
    assert torch.equal(loss, loss_g)
    # either output alone
    only_norm = pfg.pfg_convnet_per_example_grad_norms(net, X, labels, want_sq=False, want_loss=False)
    only_sq = pfg.pfg_convnet_per_example_grad_norms(net, X, labels, want_norm=False)
    torch.cuda.synchronize()
    assert only_norm[0] is None and only_norm[2] is None and torch.equal(only_norm[1], norm)
    assert only_sq[1] is None and torch.equal(only_sq[0], sq)
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_convnet_per_example_grad_norms(net, X, labels, want_sq=False, want_norm=False)
    assert ei.value.code == pfg.PFG_ERR_NULL
    # the gradients' workspace is too small for the norms
    small = torch.empty(pfg.pfg_convnet_workspace_bytes(net, wk.B), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_convnet_per_example_grad_norms(net, X, labels, workspace=small)
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE


def test_convnet_grad_norms_with_more_blocks_than_one_launch_takes():
    # 2 conv blocks + 17 dense layers = 19 parameter blocks: the norm kernel takes 16 per launch, the
    # whole-gradient norm then comes from a finishing kernel (from the workspace when no per-block
    # output is asked for)
    wk = wl.ConvWorkload("deepn", 561, 8, 8, 1, ((3, 2), (3, 3)), (6,) * 16 + (4,), 5)
    inp = wl.make_conv_inputs(wk, bias_scale=0.3)
    net, (sq, norm, loss) = check_conv_norms(inp, "conv-norms-deep", min_checked=0.2)
    assert sq.shape == (5, 19)
    only_norm = pfg.pfg_convnet_per_example_grad_norms(net, dev(inp.X), dev(inp.labels), want_sq=False)
    torch.cuda.synchronize()
    assert only_norm[0] is None and torch.equal(only_norm[1], norm)


def test_c10_mnist_convnet_grad_norms_full_size():
    wk = wl.CONV_WORKLOADS["c10_mnist_convnet_grad_norms"]
    say("c10_mnist_convnet_grad_norms: full size (128 images, 28 x 28), sampled examples")
    inp = wl.make_conv_inputs(wk)
    picks = sorted(set([0, wk.B - 1] + np.random.default_rng(11).integers(0, wk.B, size=24).tolist()))
    net, (sq, norm, loss) = check_conv_norms(inp, "c10-norms", examples=picks)
    # properties that hold for every example
    assert torch.isfinite(sq).all() and (sq >= 0).all()
    assert ((norm.double() ** 2 - sq.double().sum(1)).abs() / sq.double().sum(1)).max().item() < 1e-5
    # the last layer's block from the softmax alone: (|a|^2 + 1) |p - onehot|^2 >= |p - onehot|^2
    p_label = torch.exp(-loss.double())
    assert (sq[:, -1].double() >= (1.0 - p_label) ** 2 * (1 - 1e-5)).all()


GRAPH_SHAPES = [
    # the products that gather their patches from the image, the fused unpool + bias kernel and the
    # split filter products
    (12, 12, 4, ((3, 8), (3, 16)), (24, 7), 96),
    # the matrix-core kernels that read the image from LDS (more than 64 KB of it, dynamically sized),
    # and the norms call that keeps only sums of squares of the filter gradients
    (16, 16, 4, ((3, 32), (3, 64)), (12,), 120),
]


@pytest.mark.parametrize("h,w,c,blocks,dense,B", GRAPH_SHAPES, ids=["gathered", "lds-image"])
def test_convnet_calls_replay_from_a_graph(h, w, c, blocks, dense, B):
    # gradients and gradient norms of one network captured into one HIP graph (the library records
    # kernel launches only) and replayed with eager work and synchronisations in between: every
    # replay reproduces the eager results bit for bit.
    wk = wl.ConvWorkload("graphc", 560, h, w, c, blocks, dense, B)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    B, h, w, c = inp.X.shape
    net = pfg.ConvNet.from_numpy(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    X, labels = dev(inp.X), dev(inp.labels)
    eager = pfg.pfg_convnet_per_example_grads(net, X, labels)
    eager_n = pfg.pfg_convnet_per_example_grad_norms(net, X, labels)
    torch.cuda.synchronize()
    flat = lambda o: list(o[0]) + list(o[1]) + list(o[2]) + list(o[3]) + [o[4]]
    out = tuple([torch.empty_like(t) for t in part] if isinstance(part, list) else torch.empty_like(part)
                for part in eager)
    out_n = tuple(torch.empty_like(t) for t in eager_n)
    ws = torch.empty(pfg.pfg_convnet_workspace_bytes(net, B), dtype=torch.uint8, device="cuda:0")
    ws_n = torch.empty(pfg.pfg_convnet_grad_norms_workspace_bytes(net, B), dtype=torch.uint8,
                       device="cuda:0")
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        pfg.pfg_convnet_per_example_grads(net, X, labels, out=out, workspace=ws)
        pfg.pfg_convnet_per_example_grad_norms(net, X, labels, out=out_n, workspace=ws_n)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        pfg.pfg_convnet_per_example_grads(net, X, labels, out=out, workspace=ws)
        pfg.pfg_convnet_per_example_grad_norms(net, X, labels, out=out_n, workspace=ws_n)
    for rep in range(3):
        for t in flat(out) + list(out_n):
            t.fill_(float("nan"))
        pfg.pfg_convnet_per_example_grad_norms(net, X, labels)     # an eager call in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(flat(out), flat(eager))), f"replay {rep}: gradients"
        assert all(torch.equal(a, b) for a, b in zip(out_n, eager_n)), f"replay {rep}: norms"


def test_convnet_rejects_bad_arguments():
    wk = wl.ConvWorkload("badc", 541, 6, 6, 1, ((3, 2),), (4,), 2)      # 6 -> 3: fine for one block
    inp = wl.make_conv_inputs(wk)
    net = pfg.ConvNet.from_numpy(6, 6, 1, inp.Wc, inp.bc, inp.Ws, inp.bs)
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_convnet_per_example_grads(net, dev(inp.X), dev(inp.labels), workspace=small)
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
    # a dense input width that does not match the conv output
    bad = pfg.ConvNet.from_numpy(6, 6, 1, inp.Wc, inp.bc, [np.zeros((7, 4), np.float32)], None)
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_convnet_workspace_bytes(bad, 2)
    assert ei.value.code == pfg.PFG_ERR_SHAPE
