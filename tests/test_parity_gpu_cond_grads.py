"""GPU parity for the per-example gradients through the conditional (Section 3.6 under Section 5.3):
the HIP library, called through its C ABI, against the float64 oracle's literal loop with an `if`.

The condition is a float32 decision on the GPU and a float64 one in the oracle.  Rows whose float64
score is at least 1e-4 from zero must take the oracle's branch and are compared element by element
(relative error per example and tensor at most 1e-4; the slices of the branch an iteration did not
take must be exactly zero).  The integer-valued cases have exact scores, so there every row is
compared, rows with a score of exactly 0 included.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from parity_util import TOL_F32, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, say  # noqa: E402
import oracle  # noqa: E402
from oracle import cond as ocond  # noqa: E402

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MARGIN = 1e-4


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def nan_outputs(net, n):
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out = {}
    for name, m in (("pre", net.pre), ("then", net.then_net), ("else", net.else_net)):
        out[name] = ([torch.full((n, m.dims[l], m.dims[l + 1]), float("nan"), **f32) for l in range(m.L)],
                     [torch.full((n, m.dims[l + 1]), float("nan"), **f32) for l in range(m.L)])
    out["loss"] = torch.full((n,), float("nan"), **f32)
    out["cond"] = torch.full((n,), -7, dtype=torch.int32, device="cuda:0")
    out["counts"] = torch.full((2,), -7, dtype=torch.int32, device="cuda:0")
    return out


def check_cond_grads(ci, labels, act, tag, invariant=-1, exact_scores=False):
    mk = lambda pair: oracle.Net(pair[0], pair[1], act)
    onet = ocond.Cond(mk(ci.pre), ci.w, ci.c0, mk(ci.then_net), mk(ci.else_net))
    net = pfg.Cond.from_numpy(ci.pre, ci.w, ci.c0, ci.then_net, ci.else_net, act)
    n = ci.X.shape[0]
    out = pfg.pfg_cond_per_example_grads(net, dev(ci.X), dev(labels), invariant_cond=invariant, out=nan_outputs(net, n))
    torch.cuda.synchronize()
    ref = ocond.per_example_grads(onet, ci.X, labels, invariant=invariant)
    flags = out["cond"].cpu().numpy()
    if invariant >= 0 or exact_scores:
        sure = np.ones(n, dtype=bool)
    else:
        scores = np.array([ocond.score(onet, x) for x in ci.X])
        sure = np.abs(scores) >= MARGIN
    say(f"  {tag}: {int(sure.sum())} of {n} rows compared, {int(ref['cond'].sum())} take the then branch")
    assert sure.mean() > 0.95
    assert np.array_equal(flags[sure], ref["cond"][sure]), "rows took another branch than in the oracle"
    assert out["counts"].tolist() == [int(flags.sum()), n - int(flags.sum())]
    worst = 0.0
    for name in ("pre", "then", "else"):
        for kind in (0, 1):
            for l, (g, r) in enumerate(zip(out[name][kind], ref[name][kind])):
                gh = g.cpu().numpy()
                assert np.isfinite(gh).all(), f"{name} {'dW' if kind == 0 else 'db'}{l + 1} was not written in full"
                e = slice_rel_err(gh[sure], r[sure])
                worst = max(worst, e)
                if name != "pre":
                    # an iteration outside this branch's set: exact zeros (whatever branch the GPU chose)
                    outside = flags == (0 if name == "then" else 1)
                    assert not gh[outside].any(), f"{name}: non-zero gradient for an iteration of the other set"
    e = slice_rel_err(out["loss"].cpu().numpy()[sure], ref["loss"][sure], lead=0)
    worst = max(worst, e)
    say(f"  {tag}: max rel err {worst:.3e}")
    assert worst <= TOL_F32
    return net, out


def test_gradient_fixture_through_the_c_abi():
    g = json.load(open(os.path.join(GOLD, "cond_grad_2_2.json")))
    units = {"q": 1.0 / (1.0 + math.exp(1.0)), "u": 1.0 - 1.0 / (1.0 + math.exp(2.0)), "h": 0.5}
    f32 = lambda a: np.ascontiguousarray(np.asarray(a, dtype=np.float32))
    mk = lambda Ws, bs: ([f32(W) for W in Ws], [f32(b) for b in bs])
    net = pfg.Cond.from_numpy(mk([g["W_pre"]], [g["b_pre"]]), f32(g["w"]), g["c0"], mk(g["then_W"], g["then_b"]),
                              mk(g["else_W"], g["else_b"]), "relu")

    def want(entry, shape):
        if not entry:
            return np.zeros(shape)
        (name, mult), = entry.items()
        return units[name] * np.array(mult, dtype=float)

    for copies in (1, 40, 3000):             # 4 to 12 000 rows: the small-problem and the tiled kernels
        X = dev(np.tile(f32(g["X"]), (copies, 1)))
        labels = dev(np.tile(np.array(g["labels"], np.int32), copies))
        out = pfg.pfg_cond_per_example_grads(net, X, labels)
        torch.cuda.synchronize()
        assert out["cond"].cpu().numpy().tolist() == g["cond"] * copies
        for i in range(4):
            for b in {i, 4 * (copies - 1) + i}:
                for name in ("pre", "then", "else"):
                    for kind, key, shape in ((0, f"dW_{name}", (2, 2)), (1, f"db_{name}", (2,))):
                        w = want(g[key][i], shape)
                        got = out[name][kind][0][b].cpu().numpy().astype(np.float64)
                        zero = w == 0.0
                        assert (got[zero] == 0.0).all(), f"{key}[{b}]: entries that must be exactly 0 are {got[zero]}"
                        if (~zero).any():
                            assert np.max(np.abs(got - w)[~zero] / np.abs(w[~zero])) <= 2e-6, (key, b, got, w)
                lw = eval(g["loss_formulas"][i], {"log": math.log, "exp": math.exp})
                assert abs(float(out["loss"][b]) - lw) <= 2e-6 * max(1.0, abs(lw))
        say(f"  cond_grad_2_2 x {copies}: every entry equals the hand-worked value")


SHAPES = [
    # pre, then, else, act, n
    ((12, 16), (24, 5), (5,), "tanh", 200),
    ((7, 9, 6), (11, 4), (5, 8, 4), "gelu", 70),                 # two layers in front, a deeper else branch
    ((33, 65), (129, 10), (10,), "relu", 150),                   # one past the tile edges
    ((40, 64), (96, 10), (10,), "tanh", 9000),                   # LDS-tiled products in both directions
    ((20, 24), (3,), (16, 3), "relu", 2500),                     # a one-layer then branch
]


@pytest.mark.parametrize("pre,then_dims,else_dims,act,n", SHAPES, ids=[f"{s[0]}-{s[3]}-n{s[4]}" for s in SHAPES])
def test_cond_grads_shapes(pre, then_dims, else_dims, act, n):
    say(f"conditional gradients pre={pre} then={then_dims} else={else_dims} act={act} n={n}")
    w = wl.CondWorkload("cg", 800 + n % 97 + len(pre), pre, then_dims, else_dims, act, n)
    ci = wl.make_cond_inputs(w, bias_scale=0.2)
    # an offset that splits the rows roughly in half (index logic of the test: the median score)
    phi = {"tanh": np.tanh, "relu": lambda z: np.maximum(z, 0.0),
           "gelu": lambda z: z * 0.5 * (1.0 + scipy.special.erf(z / math.sqrt(2.0)))}[act]
    t = ci.X.astype(np.float64)
    for W, b in zip(*ci.pre):
        t = phi(t @ W + b)
    ci.c0 = -float(np.median(t @ ci.w))
    labels = np.random.default_rng(n).integers(0, then_dims[-1], size=n).astype(np.int32)
    net, out = check_cond_grads(ci, labels, act, f"cond-grads n={n}")
    flags = out["cond"].cpu().numpy()
    assert 0 < flags.sum() < n


def test_cond_grads_with_a_loop_invariant_condition():
    w = wl.CondWorkload("cgi", 830, (10, 14), (18, 6), (6,), "tanh", 300)
    ci = wl.make_cond_inputs(w, bias_scale=0.2)
    labels = np.random.default_rng(3).integers(0, 6, size=300).astype(np.int32)
    for flag in (1, 0):
        check_cond_grads(ci, labels, "tanh", f"invariant {flag}", invariant=flag)


@pytest.mark.parametrize("n", [300, 9000, 70000])
def test_cond_grads_integer_network_every_row(n):
    # integer-valued network: scores are exact, many are exactly 0 (else branch), many units of the
    # shared part and of the then branch sit exactly on the ReLU kink
    pre, then_dims, else_dims = ((8, 8), (8, 3), (3,)) if n > 20000 else ((24, 32), (40, 6), (6,))
    ci = wl.make_integer_cond_inputs(pre, then_dims, else_dims, n, 900 + n, branch_last_scale=1 / 16)
    labels = np.random.default_rng(n).integers(0, then_dims[-1], size=n).astype(np.int32)
    t = np.maximum(ci.X.astype(np.int64) @ ci.pre[0][0].astype(np.int64) + ci.pre[1][0].astype(np.int64), 0)
    zero = (t @ ci.w.astype(np.int64)) == 0
    say(f"integer conditional n={n}: {int(zero.sum())} rows have a score of exactly 0")
    assert zero.sum() >= 10
    net, out = check_cond_grads(ci, labels, "relu", f"integer n={n}", exact_scores=True)
    assert not out["cond"].cpu().numpy()[zero].any()


def test_cond_grads_skipped_outputs_and_errors():
    w = wl.CondWorkload("cgs", 840, (6, 8), (10, 4), (4,), "tanh", 50)
    ci = wl.make_cond_inputs(w, bias_scale=0.2)
    labels = np.random.default_rng(4).integers(0, 4, size=50).astype(np.int32)
    net, full = check_cond_grads(ci, labels, "tanh", "skip-reference")
    X, lab = dev(ci.X), dev(labels)
    only_db = pfg.pfg_cond_per_example_grads(net, X, lab, want_dW=False)
    only_dW = pfg.pfg_cond_per_example_grads(net, X, lab, want_db=False)
    torch.cuda.synchronize()
    for name in ("pre", "then", "else"):
        assert only_db[name][0] is None and only_dW[name][1] is None
        assert all(torch.equal(a, b) for a, b in zip(only_db[name][1], full[name][1]))
        assert all(torch.equal(a, b) for a, b in zip(only_dW[name][0], full[name][0]))
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_cond_per_example_grads(net, X, lab, workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_cond_per_example_grads(net, X, lab, invariant_cond=2)
    assert ei.value.code == pfg.PFG_ERR_UNSUPPORTED


def test_c13_full_size_in_the_benchmark_configuration():
    """c13 as `bench.py` times it (1024 rows, 8.15 GB of gradients; the two large layers of the then
    branch leave through the list-driven wide writer): 40 rows spread over the batch against the oracle,
    element by element; every row: exact zeros in the slices of the branch it did not take, and
    agreement with the library's own result on chunks of 16 rows (small launches through the general
    writer, which the tests above hold against the oracle)."""
    w = wl.COND_WORKLOADS["c13_cond_grads"]
    ci = wl.make_cond_inputs(w)
    n = w.n
    labels = np.random.Generator(np.random.Philox(wl.BASE_SEED + w.index + 900000)).integers(
        0, w.then_dims[-1], size=n).astype(np.int32)
    mk = lambda pair: oracle.Net(pair[0], pair[1], w.act)
    onet = ocond.Cond(mk(ci.pre), ci.w, ci.c0, mk(ci.then_net), mk(ci.else_net))
    net = pfg.Cond.from_numpy(ci.pre, ci.w, ci.c0, ci.then_net, ci.else_net, w.act)
    X, lab = dev(ci.X), dev(labels)
    say(f"c13 full size: n={n}")
    out = pfg.pfg_cond_per_example_grads(net, X, lab, out=nan_outputs(net, n))
    torch.cuda.synchronize()
    flags = out["cond"].cpu().numpy()
    scores = np.array([ocond.score(onet, x) for x in ci.X])
    sure = np.abs(scores) >= MARGIN
    assert sure.mean() > 0.95
    assert np.array_equal(flags[sure], (scores > 0)[sure].astype(flags.dtype))
    assert out["counts"].tolist() == [int(flags.sum()), n - int(flags.sum())]
    assert 0.3 * n < flags.sum() < 0.7 * n
    # (1) sampled rows against the oracle
    rows = np.unique(np.concatenate([np.arange(8), np.arange(n - 8, n), np.linspace(8, n - 9, 24).astype(int)]))
    rows = rows[sure[rows]]
    ref = ocond.per_example_grads(onet, ci.X[rows], labels[rows])
    worst = 0.0
    for name in ("pre", "then", "else"):
        for kind in (0, 1):
            for g, r in zip(out[name][kind], ref[name][kind]):
                worst = max(worst, slice_rel_err(g[torch.from_numpy(rows).to(g.device)].cpu().numpy(), r))
    worst = max(worst, slice_rel_err(out["loss"].cpu().numpy()[rows], ref["loss"], lead=0))
    say(f"  {len(rows)} rows against the oracle: max rel err {worst:.3e}")
    assert worst <= TOL_F32
    # (2) every row: written in full, zeros outside its branch
    ft = torch.from_numpy(flags).to("cuda:0")
    for name in ("pre", "then", "else"):
        for kind in (0, 1):
            for g in out[name][kind]:
                assert bool(torch.isfinite(g).all()), f"{name}: not written in full"
                if name != "pre":
                    outside = ft == (0 if name == "then" else 1)
                    assert not bool(g[outside].any()), f"{name}: non-zero gradient for an iteration of the other set"
    # (3) every row against the library's own result on 16 rows at a time
    worst = 0.0
    for lo in range(0, n, 16):
        part = pfg.pfg_cond_per_example_grads(net, X[lo:lo + 16], lab[lo:lo + 16])
        for name in ("pre", "then", "else"):
            for kind in (0, 1):
                for g, q in zip(out[name][kind], part[name][kind]):
                    a, b = g[lo:lo + 16].reshape(16, -1), q.reshape(16, -1)
                    scale = b.abs().amax(dim=1).clamp_min(1e-30)
                    worst = max(worst, float(((a - b).abs().amax(dim=1) / scale).max()))
        assert torch.equal(part["cond"], out["cond"][lo:lo + 16])
    torch.cuda.synchronize()
    say(f"  all rows against calls of 16 rows: max rel err {worst:.3e}")
    assert worst <= TOL_F32
