"""GPU parity at the points where a convention decides the result, at sizes that reach every
kernel family: ReLU pre-activations of exactly 0 (derivative 0), pooling windows whose largest
value occurs twice (first in scan order wins), condition scores of exactly 0 (else branch).

The networks are integer-valued (paper_1903_04243_amd.workloads.make_integer_*): every hidden
pre-activation is a small integer, computed exactly by float32 and bfloat16 products as by the
float64 oracle, whatever the order of summation.  Both sides therefore decide on identical values,
thousands of units sit exactly on a boundary, and a kernel that read `z >= 0`, broke a tie the other
way or tested `score >= 0` would disagree with the oracle on whole rows.  Where the whole
computation is exact (Jacobians of the logits, forward results of the conditional) the comparison
is bit for bit.
"""
import numpy as np
import pytest

from parity_util import TOL_BF16, TOL_F32, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, gpu_net, gpu_x, say  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def hidden_preactivations(inp):
    """Integer [B, d_l] per hidden layer: the pre-activations, by integer arithmetic in numpy (index
    logic of the test, not a reference result)."""
    a = inp.X.astype(np.int64)
    out = []
    for l in range(len(inp.Ws) - 1):
        z = a @ inp.Ws[l].astype(np.int64) + inp.bs[l].astype(np.int64)
        out.append(z)
        a = np.maximum(z, 0)
    return out


def kink_units(inp):
    return [z == 0 for z in hidden_preactivations(inp)]


DENSE = [
    # dims, B, density, last_scale, dtype, what the shape reaches
    ((33, 65, 129, 10), 9, 0.25, 1 / 32, "f32"),            # 16 x 16 small-problem kernel
    ((784, 512, 512, 10), 128, 0.25, 1 / 512, "f32"),       # c2's shape: 32 x 32 kernel, fused head
    ((96, 160, 70, 12), 8200, 0.25, 1 / 32, "f32"),         # LDS-tiled kernels, mask in the epilogue
    ((2048, 1024, 1280, 10), 96, 0.25, 1 / 8192, "f32"),    # forward products cut along the contraction
    ((96, 2048, 7), 200, 0.25, 1 / 128, "f32"),             # head from partial logits
    ((64, 48, 32, 10), 300, 0.2, 1 / 8, "bf16"),
    ((520, 392, 328, 10), 24, 0.08, 1 / 64, "bf16"),        # c4's reduced shape
    ((96, 160, 70, 12), 8200, 0.1, 1 / 16, "bf16"),         # bf16 on the LDS-tiled kernels
]


@pytest.mark.parametrize("dims,B,density,last_scale,dtype", DENSE,
                         ids=[f"{d[0]}-B{d[1]}-{d[4]}" for d in DENSE])
def test_relu_kinks_dense(oracle, dims, B, density, last_scale, dtype):
    say(f"integer ReLU network {dims} B={B} {dtype}")
    inp = wl.make_integer_inputs(dims, B, 4243 + B, density=density, last_scale=last_scale, dtype=dtype)
    zs = hidden_preactivations(inp)
    kinks = [z == 0 for z in zs]
    for l, k in enumerate(kinks):
        say(f"  hidden layer {l + 1}: {int(k.sum())} of {k.size} units sit exactly on the kink")
        assert k.sum() >= 5
    net = gpu_net(inp, "relu", dtype)
    X, labels = gpu_x(inp, dtype), dev(inp.labels)
    big = B * dims[0] * dims[1] > (1 << 26)
    want = [not big] + [True] * (len(dims) - 2)
    dW, db, loss = pfg.pfg_per_example_grads(net, X, labels, want_dW=want)
    sq, norm, _ = pfg.pfg_per_example_grad_norms(net, X, labels)
    torch.cuda.synchronize()
    onet = oracle.Net(inp.Ws, inp.bs, "relu")
    rdW, rdb, rloss = oracle.per_example_grads(onet, inp.X, inp.labels, want_dW=want)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    worst = 0.0
    for l in range(net.L):
        if want[l]:
            worst = max(worst, slice_rel_err(dW[l].cpu().numpy(), rdW[l]))
        worst = max(worst, slice_rel_err(db[l].cpu().numpy(), rdb[l]))
    worst = max(worst, slice_rel_err(loss.cpu().numpy(), rloss, lead=0))
    say(f"  gradients: rel err vs oracle {worst:.3e}")
    assert worst <= tol
    # the convention itself: a unit on the kink passes no cotangent, on either side, and the unit's
    # column of the weight gradient is exactly 0
    live = 0
    for l, k in enumerate(kinks):
        g = db[l].cpu().numpy()
        assert (g[k] == 0.0).all(), f"hidden layer {l + 1}: a unit with z == 0 passed a cotangent"
        assert (rdb[l][k] == 0.0).all()
        if want[l]:
            col = dW[l].cpu().numpy().transpose(0, 2, 1)[k]          # [units on the kink, d_{l-1}]
            assert (col == 0.0).all()
        # units below the kink are off, units above it are on wherever the oracle's cotangent is not
        # itself zero to within the tolerance (cotangents that cancel, or that bf16 rounding of the
        # operands makes equal, may legitimately come out as 0)
        z = zs[l]
        assert (g[z < 0] == 0.0).all(), f"hidden layer {l + 1}: a unit with z < 0 passed a cotangent"
        on = (z > 0) & (np.abs(rdb[l]) > tol * np.abs(rdb[l]).max())
        assert (g[on] != 0.0).all(), f"hidden layer {l + 1}: a unit with z > 0 passed nothing"
        live += int((g != 0.0).sum())
    assert live > 0
    rsq, rnorm = oracle.per_example_grad_norms(onet, inp.X, inp.labels)
    e = float(np.max(np.abs(norm.cpu().numpy() - rnorm) / rnorm))
    say(f"  norms: rel err vs oracle {e:.3e}")
    assert e <= tol


JAC = [
    ((33, 65, 129, 10), 9),
    ((96, 160, 70, 12), 700),         # 8400 cotangent rows: tiled kernels, mask applied while staging A
    ((200, 136, 72, 40), 64),
]


@pytest.mark.parametrize("dims,B", JAC, ids=[f"{d[0]}-B{d[1]}" for d in JAC])
def test_relu_kinks_jacobians_are_exact(oracle, dims, B):
    # seeds e_s, weights in {-1, 0, 1} (last layer / 32): every cotangent is a small multiple of 1/32
    # and every sum is exact in float32, so the Jacobians must equal the oracle's bit for bit
    say(f"integer ReLU network {dims} B={B}: Jacobians, bit for bit")
    inp = wl.make_integer_inputs(dims, B, 977 + B, density=0.25, last_scale=1 / 32)
    assert all(k.sum() >= 5 for k in kink_units(inp))
    net = gpu_net(inp, "relu", "f32")
    X = gpu_x(inp, "f32")
    onet = oracle.Net(inp.Ws, inp.bs, "relu")
    J = pfg.pfg_jacobian_input(net, X)
    torch.cuda.synchronize()
    ref = oracle.jacobian_input(onet, inp.X)
    assert np.array_equal(ref, ref.astype(np.float32).astype(np.float64)), "not exactly representable"
    assert np.array_equal(J.cpu().numpy().astype(np.float64), ref), "input Jacobian differs"
    shared = np.random.default_rng(3).integers(-2, 3, size=(5, dims[-1])).astype(np.float32)
    J = pfg.pfg_jacobian_input(net, X, seeds=dev(shared))
    torch.cuda.synchronize()
    assert np.array_equal(J.cpu().numpy().astype(np.float64), oracle.jacobian_input(onet, inp.X, seeds=shared))
    Bw = min(B, 40)
    JW, Jb = pfg.pfg_jacobian_weights(net, X[:Bw].contiguous(), head="logits")
    torch.cuda.synchronize()
    rJW, rJb = oracle.jacobian_weights(onet, inp.X[:Bw], head="logits")
    for l in range(net.L):
        assert np.array_equal(JW[l].cpu().numpy().astype(np.float64), rJW[l]), f"JW{l + 1} differs"
        assert np.array_equal(Jb[l].cpu().numpy().astype(np.float64), rJb[l]), f"Jb{l + 1} differs"


CONV = [
    # height, width, channels, blocks, dense, B, last_scale
    (12, 12, 1, ((3, 8), (3, 8)), (32, 10), 50, 1 / 16),
    (28, 28, 1, ((5, 32), (5, 64)), (1024, 10), 40, 1 / 4096),     # c10's network
    (8, 12, 4, ((3, 12), (3, 8)), (11, 6), 140, 1 / 8),
    (10, 6, 8, ((5, 16),), (12,), 300, 1 / 32),
    (12, 20, 3, ((3, 4), (1, 8)), (5,), 37, 1 / 16),
    (12, 12, 1, ((3, 8), (3, 8)), (32, 10), 7, 1 / 16),            # fewer than 32 examples: the other unpooling route
    # enough examples and channels for the matrix-core kernels on the LDS image (their own pooling decision)
    (28, 28, 1, ((5, 32), (5, 64)), (64, 10), 130, 1 / 256),
    (8, 8, 8, ((3, 32), (3, 32)), (6,), 230, 1 / 16),
]


@pytest.mark.parametrize("h,w,c,blocks,dense,B,last_scale", CONV,
                         ids=[f"{s[0]}x{s[1]}x{s[2]}-B{s[5]}" for s in CONV])
def test_pooling_ties_and_relu_kinks_conv(h, w, c, blocks, dense, B, last_scale):
    from oracle import conv as oconv
    say(f"integer convnet {h}x{w}x{c} blocks={blocks} dense={dense} B={B}")
    inp = wl.make_integer_conv_inputs(h, w, c, blocks, dense, B, 31 + h + B, last_scale=last_scale)
    onet = oconv.ConvNet(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    net = pfg.ConvNet.from_numpy(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    # how many pooling windows of the first block hold their (positive) maximum twice, and how many
    # pre-activations are exactly 0: integer arithmetic in numpy, index logic of the test
    k = blocks[0][0]
    p = (k - 1) // 2
    Xp = np.pad(inp.X.astype(np.int64), ((0, 0), (p, p), (p, p), (0, 0)))
    z = np.zeros((B, h, w, blocks[0][1]), dtype=np.int64) + inp.bc[0].astype(np.int64)
    for ky in range(k):
        for kx in range(k):
            z += Xp[:, ky:ky + h, kx:kx + w, :] @ inp.Wc[0][ky, kx].astype(np.int64)
    r = np.maximum(z, 0).reshape(B, h // 2, 2, w // 2, 2, -1).transpose(0, 1, 3, 5, 2, 4).reshape(B, h // 2, w // 2, -1, 4)
    top = np.sort(r, axis=-1)
    ties = int(((top[..., 3] == top[..., 2]) & (top[..., 3] > 0)).sum())
    say(f"  first block: {ties} windows with a tied positive maximum, {int((z == 0).sum())} pre-activations of exactly 0")
    assert ties >= 20 and (z == 0).sum() >= 20
    # EVERY example is compared: no example has to be set aside for sitting near a boundary
    dWc, dbc, dW, db, loss = pfg.pfg_convnet_per_example_grads(net, dev(inp.X), dev(inp.labels))
    sq, norm, _ = pfg.pfg_convnet_per_example_grad_norms(net, dev(inp.X), dev(inp.labels))
    torch.cuda.synchronize()
    rdWc, rdbc, rdW, rdb, rloss = oconv.per_example_grads(onet, inp.X, inp.labels)
    worst = 0.0
    for got, ref in zip(dWc + dbc + dW + db, rdWc + rdbc + rdW + rdb):
        worst = max(worst, slice_rel_err(got.cpu().numpy(), ref))
    worst = max(worst, slice_rel_err(loss.cpu().numpy(), rloss, lead=0))
    say(f"  gradients of all {B} examples: rel err vs oracle {worst:.3e}")
    assert worst <= TOL_F32
    rsq, rnorm, _ = oconv.per_example_grad_norms(onet, inp.X, inp.labels)
    e = float(np.max(np.abs(norm.cpu().numpy() - rnorm) / rnorm))
    say(f"  norms: rel err vs oracle {e:.3e}")
    assert e <= TOL_F32


COND = [
    # pre, then, else, n
    ((12, 16), (24, 5), (5,), 200),
    ((40, 64), (96, 10), (10,), 9000),           # LDS-tiled branch products
    ((8, 8), (8, 3), (3,), 70000),               # beyond 64 Ki rows: block counts ahead of the placing step
]


@pytest.mark.parametrize("pre,then_dims,else_dims,n", COND, ids=[f"n{c[3]}" for c in COND])
def test_condition_scores_of_exactly_zero(oracle, pre, then_dims, else_dims, n):
    from oracle import cond as ocond
    say(f"integer conditional pre={pre} then={then_dims} else={else_dims} n={n}")
    ci = wl.make_integer_cond_inputs(pre, then_dims, else_dims, n, 555 + n)
    mk = lambda pair: oracle.Net(pair[0], pair[1], "relu")
    onet = ocond.Cond(mk(ci.pre), ci.w, ci.c0, mk(ci.then_net), mk(ci.else_net))
    rR, rflags = ocond.forward(onet, ci.X)
    # rows whose score is exactly 0 (integer arithmetic in numpy; index logic of the test)
    t = np.maximum(ci.X.astype(np.int64) @ ci.pre[0][0].astype(np.int64) + ci.pre[1][0].astype(np.int64), 0)
    zero = (t @ ci.w.astype(np.int64)) == 0
    say(f"  {int(zero.sum())} of {n} rows have a score of exactly 0; {int(rflags.sum())} rows take the then branch")
    assert zero.sum() >= 20 and 0 < rflags.sum() < n
    assert not rflags[zero].any(), "the oracle sends a score of 0 to the else branch"
    cnet = pfg.Cond.from_numpy(ci.pre, ci.w, ci.c0, ci.then_net, ci.else_net, "relu")
    R, flags, counts = pfg.pfg_cond_forward(cnet, dev(ci.X))
    torch.cuda.synchronize()
    assert np.array_equal(flags.cpu().numpy(), rflags), "the index sets differ from the oracle's"
    assert counts.tolist() == [int(rflags.sum()), n - int(rflags.sum())]
    assert np.array_equal(R.cpu().numpy().astype(np.float64), rR), "results differ (all values are exact integers)"
