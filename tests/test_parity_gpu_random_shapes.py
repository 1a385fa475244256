"""GPU parity on seeded random shapes.

The kernel a product runs on is chosen from its shape (tile counts, contraction length, batch
entries, channel counts): the cases below draw widths, batch sizes, step counts and image sizes
from sets that straddle those rules and compare every output with the float64 oracles, as the
fixed-shape parity tests do.  Same error measure and tolerances.  Activations are smooth here (the
fixed-shape tests cover ReLU with inputs drawn away from its kink); conv nets are compared on the
examples that are clear of every ReLU / pooling decision boundary.
"""
import numpy as np
import pytest

from parity_util import TOL_BF16, TOL_F32, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

import gpu_helpers as gh  # noqa: E402
from gpu_helpers import dev, say  # noqa: E402
import oracle  # noqa: E402
from oracle import conv as oconv, lstm as olstm  # noqa: E402
from test_parity_gpu_conv import MARGIN, decision_margins  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    oracle.build()
    yield


def dense_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        L = int(rng.integers(2, 4))
        dims = tuple(int(rng.choice([64, 200, 256, 512, 1024, 1536, 2048])) for _ in range(L)) + \
            (int(rng.choice([3, 10, 32, 40, 300])),)
        B = int(rng.choice([5, 40, 64, 100, 130, 200, 260, 520, 800, 1100]))
        if sum(dims[l] * dims[l + 1] for l in range(L)) * B <= 4e8:
            out.append((dims, B, str(rng.choice(["tanh", "gelu"]))))
    return out


@pytest.mark.parametrize("dims,B,act", dense_cases(2024, 14), ids=lambda v: str(v).replace(" ", ""))
def test_dense_grads_and_norms_random_shapes(dims, B, act):
    say(f"random dense {dims} B={B} {act}")
    L = len(dims) - 1
    w = wl.Workload("rnd", 900 + B + L, "per_example_grads", dims, act, "f32", B, "normal", "normal_fan_in")
    inp = wl.make_inputs(w, bias_scale=0.2)
    onet = oracle.Net(inp.Ws, inp.bs, act)
    net = pfg.Mlp.from_numpy(inp.Ws, inp.bs, act, "f32")
    X, labels = dev(inp.X), dev(inp.labels)
    want = [False] * (L - 1) + [True]
    rsq, _ = oracle.per_example_grad_norms(onet, inp.X, inp.labels)
    rdW, rdb, rloss = oracle.per_example_grads(onet, inp.X, inp.labels, want_dW=want)
    sq, _, loss = pfg.pfg_per_example_grad_norms(net, X, labels)
    dW, db, loss2 = pfg.pfg_per_example_grads(net, X, labels, want_dW=want)
    torch.cuda.synchronize()
    e = float(np.max(np.abs(sq.cpu().numpy() - rsq) / np.maximum(rsq, 1e-300)))
    e = max(e, slice_rel_err(loss.cpu().numpy(), rloss, lead=0), slice_rel_err(loss2.cpu().numpy(), rloss, lead=0),
            slice_rel_err(dW[-1].cpu().numpy(), rdW[-1]))
    e = max([e] + [slice_rel_err(db[l].cpu().numpy(), rdb[l]) for l in range(L)])
    say(f"  rel err {e:.3e}")
    assert e <= TOL_F32


def bf16_cases(seed, count):
    rng = np.random.default_rng(seed)
    return [((int(rng.choice([256, 1024, 2048])), int(rng.choice([512, 1024, 2048])), int(rng.choice([10, 40]))),
             int(rng.choice([5, 64, 150, 300])), str(rng.choice(["tanh", "gelu"]))) for _ in range(count)]


@pytest.mark.parametrize("dims,B,act", bf16_cases(78, 5), ids=lambda v: str(v).replace(" ", ""))
def test_bf16_grads_random_shapes(dims, B, act):
    say(f"random bf16 {dims} B={B} {act}")
    w = wl.Workload("rndb", 1100 + B, "per_example_grads", dims, act, "bf16", B, "normal", "normal_fan_in")
    inp = gh.draw(w, bias_scale=0.2)
    onet = oracle.Net(inp.Ws, inp.bs, act)
    rdW, rdb, rloss = oracle.per_example_grads(onet, inp.X, inp.labels, want_dW=[False, True])
    dW, db, loss = pfg.pfg_per_example_grads(gh.gpu_net(inp, act, "bf16"), gh.gpu_x(inp, "bf16"), dev(inp.labels),
                                             want_dW=[False, True])
    torch.cuda.synchronize()
    e = max(slice_rel_err(dW[1].cpu().numpy(), rdW[1]), slice_rel_err(db[0].cpu().numpy(), rdb[0]),
            slice_rel_err(db[1].cpu().numpy(), rdb[1]), slice_rel_err(loss.cpu().numpy(), rloss, lead=0))
    say(f"  rel err {e:.3e}")
    assert e <= TOL_BF16


def jacobian_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        L = int(rng.integers(1, 4))
        dims = tuple(int(rng.choice([20, 64, 128, 200, 256, 512])) for _ in range(L)) + (int(rng.choice([4, 16, 48])),)
        B = int(rng.choice([2, 16, 70, 200]))
        if B * dims[-1] * max(dims) <= 3e6:
            out.append((dims, B, str(rng.choice(["tanh", "gelu"]))))
    return out


@pytest.mark.parametrize("dims,B,act", jacobian_cases(99, 8), ids=lambda v: str(v).replace(" ", ""))
def test_jacobians_and_hessian_random_shapes(dims, B, act):
    say(f"random jacobian {dims} B={B} {act}")
    L, S = len(dims) - 1, dims[-1]
    w = wl.Workload("rndj", 1200 + B + L, "jacobian_input", dims, act, "f32", B, "normal", "normal_fan_in")
    inp = wl.make_inputs(w, bias_scale=0.2)
    onet = oracle.Net(inp.Ws, inp.bs, act)
    net = pfg.Mlp.from_numpy(inp.Ws, inp.bs, act, "f32")
    X = dev(inp.X)
    J = pfg.pfg_jacobian_input(net, X)
    torch.cuda.synchronize()
    e = slice_rel_err(J.cpu().numpy(), oracle.jacobian_input(onet, inp.X), lead=2)
    if B * S * sum(dims[l] * dims[l + 1] for l in range(L)) < 3e7:
        JW, Jb = pfg.pfg_jacobian_weights(net, X, head="softmax")
        torch.cuda.synchronize()
        rJW, rJb = oracle.jacobian_weights(onet, inp.X, head="softmax")
        e = max([e] + [slice_rel_err(JW[l].cpu().numpy(), rJW[l], lead=2) for l in range(L)] +
                [slice_rel_err(Jb[l].cpu().numpy(), rJb[l], lead=2) for l in range(L)])
    if L >= 2 and B * S * dims[0] * dims[0] < 2e7:
        H = pfg.pfg_hessian_input(net, X)
        torch.cuda.synchronize()
        e = max(e, slice_rel_err(H.cpu().numpy(), oracle.hessian_input(onet, inp.X), lead=2))
    say(f"  rel err {e:.3e}")
    assert e <= TOL_F32


def lstm_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        dx, H, dy = int(rng.choice([4, 16, 33])), int(rng.choice([8, 30, 64, 128])), int(rng.choice([3, 10, 40]))
        T, B = int(rng.choice([1, 3, 17, 40])), int(rng.choice([3, 70, 600, 900, 1300]))
        if B * (dx + H) * 4 * H <= 1.2e8:
            out.append((dx, H, dy, T, B))
    return out


@pytest.mark.parametrize("dx,H,dy,T,B", lstm_cases(2025, 7), ids=lambda v: str(v))
def test_lstm_grads_random_shapes(dx, H, dy, T, B):
    say(f"random LSTM dx={dx} H={H} dy={dy} T={T} B={B}")
    w = wl.LstmWorkload("rndl", 950 + H + T, "lstm_per_example_grads", dx, H, dy, T, B)
    inp = wl.make_lstm_inputs(w, bias_scale=0.3)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, T)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, T)
    ref = olstm.per_example_grads(onet, inp.X, inp.labels)
    got = pfg.pfg_lstm_per_example_grads(net, dev(inp.X), dev(inp.labels))
    torch.cuda.synchronize()
    e = max(slice_rel_err(g.cpu().numpy(), r, lead=0 if r.ndim == 1 else 1) for g, r in zip(got, ref))
    say(f"  rel err {e:.3e}")
    assert e <= TOL_F32


def conv_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        nb = int(rng.integers(1, 3))
        h, w = int(rng.choice([4, 8, 12, 16, 20])), int(rng.choice([4, 8, 12, 16]))
        if nb == 2:
            h, w = h - h % 4, w - w % 4
        c = int(rng.choice([1, 2, 4, 8, 12]))
        blocks = tuple((int(rng.choice([1, 3, 5])), int(rng.choice([4, 6, 16, 32, 64]))) for _ in range(nb))
        dense = (int(rng.choice([7, 32, 100])), int(rng.choice([3, 10])))
        B = int(rng.choice([3, 40, 130, 300, 700]))
        hh, ww, cc, tot = h, w, c, 0
        for k, f in blocks:
            tot += hh * ww * k * k * cc
            hh, ww, cc = hh // 2, ww // 2, f
        if hh >= 1 and ww >= 1 and tot * B <= 3e7:
            out.append((h, w, c, blocks, dense, B))
    return out


@pytest.mark.parametrize("h,w,c,blocks,dense,B", conv_cases(77, 10), ids=lambda v: str(v).replace(" ", ""))
def test_convnet_grads_and_norms_random_shapes(h, w, c, blocks, dense, B):
    say(f"random convnet {h}x{w}x{c} {blocks} {dense} B={B}")
    wk = wl.ConvWorkload("rndc", 1000 + h + w + B, h, w, c, blocks, dense, B)
    inp = wl.make_conv_inputs(wk, bias_scale=0.2)
    onet = oconv.ConvNet(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    net = pfg.ConvNet.from_numpy(h, w, c, inp.Wc, inp.bc, inp.Ws, inp.bs)
    X, labels = dev(inp.X), dev(inp.labels)
    margins = decision_margins(inp)
    idx = [b for b in range(B) if margins[b] >= MARGIN]
    assert len(idx) >= B // 2
    got = pfg.pfg_convnet_per_example_grads(net, X, labels)
    sq, norm, loss = pfg.pfg_convnet_per_example_grad_norms(net, X, labels)
    torch.cuda.synchronize()
    for t in [t for group in got[:4] for t in group] + [got[4], sq, norm, loss]:
        assert torch.isfinite(t).all()
    ref = oconv.per_example_grads(onet, inp.X[idx], inp.labels[idx])
    rsq, rnorm, rloss = oconv.per_example_grad_norms(onet, inp.X[idx], inp.labels[idx])
    e = max(slice_rel_err(gt.cpu().numpy()[idx], rt) for gl, rl in zip(got[:4], ref[:4]) for gt, rt in zip(gl, rl))
    e = max(e, slice_rel_err(got[4].cpu().numpy()[idx], ref[4], lead=0),
            slice_rel_err(loss.cpu().numpy()[idx], rloss, lead=0),
            float(np.max(np.abs(norm.cpu().numpy()[idx] - rnorm) / rnorm)))
    say(f"  rel err {e:.3e} on {len(idx)} of {B} examples")
    assert e <= TOL_F32


def cond_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        pre = tuple(int(rng.choice([6, 24, 64, 200])) for _ in range(int(rng.integers(2, 4))))
        dout = int(rng.choice([3, 8, 40]))
        then_dims = tuple(int(rng.choice([16, 96, 512])) for _ in range(int(rng.integers(0, 3)))) + (dout,)
        else_dims = tuple(int(rng.choice([12, 64])) for _ in range(int(rng.integers(0, 2)))) + (dout,)
        out.append((pre, then_dims, else_dims, str(rng.choice(["tanh", "gelu"])), int(rng.choice([5, 90, 1500, 9000]))))
    return out


@pytest.mark.parametrize("pre,then_dims,else_dims,act,n", cond_cases(31, 6), ids=lambda v: str(v).replace(" ", ""))
def test_cond_random_shapes(pre, then_dims, else_dims, act, n):
    from test_parity_gpu_cond import check_cond
    say(f"random cond pre={pre} then={then_dims} else={else_dims} {act} n={n}")
    wk = wl.CondWorkload("rndq", 1300 + n, pre, then_dims, else_dims, act, n)
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    check_cond(inp, act, "cond-rnd", expect_split=n >= 64)


@pytest.mark.parametrize("dx,H,dy,max_len,B", [(7, 20, 3, 25, 300), (32, 128, 10, 6, 1000), (4, 8, 2, 60, 17)],
                         ids=lambda v: str(v))
def test_varlen_random_shapes(dx, H, dy, max_len, B):
    from test_parity_gpu_lstm import check_varlen
    say(f"random varlen dx={dx} H={H} dy={dy} L<={max_len} B={B}")
    w = wl.LstmWorkload("rndv", 1400 + H + B, "lstm_varlen_forward", dx, H, dy, max_len, B)
    inp, lengths = wl.make_varlen_inputs(w, bias_scale=0.3)
    check_varlen(inp, lengths, f"varlen-rnd dx={dx} H={H} L<={max_len}")
