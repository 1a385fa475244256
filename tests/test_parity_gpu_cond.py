"""GPU parity for the conditional inside a parallel-for (Section 3.6): the HIP library, called
through its C ABI, against the float64 CPU oracle (oracle/cond_oracle.c, a loop with an `if`) on the
same seeded inputs.

What is compared.  The condition is a comparison of a floating-point score with zero; the GPU
takes it in float32, the oracle in float64.  For rows whose float64 score (numpy, not the oracle)
is at least MARGIN away from zero the two must agree exactly; for the few rows closer than that
either decision is legitimate.  Every row, near the boundary or not, must hold the output of the
branch that the GPU says it took (the oracle's `branch` applies one branch regardless of the
condition): per row max|gpu - ref| <= 1e-4 * max(max|ref row|, 0.05 * max|ref|).  The index work
is integer: the returned set sizes must equal the counts of the returned flags, and every row of
the NaN-filled output must have been written.
"""
import numpy as np
import pytest

from parity_util import TOL_F32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, say  # noqa: E402
from oracle import cond as ocond  # noqa: E402

MARGIN = 1e-4     # scores are O(1); float32 round-off of a score is ~1e-6


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def oracle_net(inp, act):
    return ocond.Cond(oracle.Net(*inp.pre, act), inp.w, inp.c0, oracle.Net(*inp.then_net, act),
                      oracle.Net(*inp.else_net, act))


def gpu_net(inp, act):
    return pfg.Cond.from_numpy(inp.pre, inp.w, inp.c0, inp.then_net, inp.else_net, act)


def np_scores(inp, act):
    """float64 scores with numpy's matrix products (for the margin only)."""
    f = {"relu": lambda z: np.maximum(z, 0.0), "tanh": np.tanh, "identity": lambda z: z}[act]
    a = inp.X.astype(np.float64)
    for W, b in zip(*inp.pre):
        a = f(a @ W.astype(np.float64) + b.astype(np.float64))
    return a @ inp.w.astype(np.float64) + inp.c0


def row_err(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    scale = np.maximum(np.abs(ref).max(axis=1), 0.05 * np.abs(ref).max())
    return float((np.abs(got - ref).max(axis=1) / scale).max()) if len(ref) else 0.0


def check_cond(inp, act, tag, invariant=-1, rows=None, expect_split=True):
    n = inp.X.shape[0]
    onet, net = oracle_net(inp, act), gpu_net(inp, act)
    R = torch.full((n, net.dout), float("nan"), dtype=torch.float32, device="cuda:0")
    cond = torch.full((n,), -7, dtype=torch.int32, device="cuda:0")
    counts = torch.full((2,), -7, dtype=torch.int32, device="cuda:0")
    pfg.pfg_cond_forward(net, dev(inp.X), invariant, out=(R, cond, counts))
    torch.cuda.synchronize()
    R, cond, counts = R.cpu().numpy(), cond.cpu().numpy(), counts.cpu().numpy()
    assert np.isfinite(R).all(), f"{tag}: some row of R was not written"
    assert set(np.unique(cond).tolist()) <= {0, 1}
    assert counts.tolist() == [int(cond.sum()), n - int(cond.sum())]
    if invariant >= 0:
        assert (cond == invariant).all()
    else:
        s = np_scores(inp, act) if act != "gelu" else np.array([ocond.score(onet, x) for x in inp.X])
        clear = np.abs(s) >= MARGIN
        assert np.array_equal(cond[clear], (s[clear] > 0).astype(np.int32)), f"{tag}: wrong branch taken"
        say(f"  {tag}: {int(cond.sum())} then / {n - int(cond.sum())} else rows, "
            f"{int((~clear).sum())} within {MARGIN:g} of the boundary")
        if expect_split:
            assert 0 < cond.sum() < n
    pick = range(n) if rows is None else rows
    ref = np.stack([ocond.branch(onet, inp.X[j], bool(cond[j])) for j in pick]) if len(pick) else np.zeros((0, net.dout))
    if invariant < 0 and rows is None:
        # the oracle's own loop agrees with its per-branch function wherever the decision is clear
        Rloop, cloop = ocond.forward(onet, inp.X)
        same = cloop == cond
        assert np.array_equal(Rloop[same], ref[same])
    e = row_err(R[list(pick)], ref)
    say(f"  {tag}: R rel err {e:.3e} over {len(pick)} rows")
    assert e <= TOL_F32, f"{tag}: max relative error {e:.3e}"
    return net, R, cond


COND_SHAPES = [
    # pre widths, then widths, else widths, act, n
    ((3, 4), (2,), (2,), "relu", 3),
    ((5, 7, 6), (9, 4), (4,), "tanh", 70),                    # nothing a multiple of 4: scalar loads
    ((16, 32), (48, 24, 8), (40, 8), "relu", 2500),           # three placing workgroups
    ((33, 20), (17, 10), (10,), "gelu", 257),
    ((64, 128), (256, 16), (16,), "tanh", 1),                 # a single iteration
    ((24, 512), (512,), (96, 512), "relu", 1100),             # wide enough for the LDS-tiled kernel
    ((12, 16), (8,), (8,), "identity", 1025),
    ((6, 8), (12, 5), (5,), "tanh", 70001),                   # many rows: block counts in the placing step
]


@pytest.mark.parametrize("pre,then_dims,else_dims,act,n", COND_SHAPES,
                         ids=[f"{'-'.join(map(str, s[0]))}_n{s[4]}_{s[3]}" for s in COND_SHAPES])
def test_cond_shapes(pre, then_dims, else_dims, act, n):
    say(f"cond pre={pre} then={then_dims} else={else_dims} act={act} n={n}")
    wk = wl.CondWorkload("oddq", 700 + n, pre, then_dims, else_dims, act, n)
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    check_cond(inp, act, "cond-odd", expect_split=n >= 64)


def test_cond_one_sided_and_invariant():
    wk = wl.CondWorkload("oneq", 720, (20, 24), (30, 6), (6,), "tanh", 300)
    # every row takes the same branch: the other branch's index set is empty and its products
    # have no live rows
    for c0, flag in ((1e6, 1), (-1e6, 0)):
        inp = wl.make_cond_inputs(wk, bias_scale=0.2, c0=c0)
        net, R, cond = check_cond(inp, "tanh", f"cond-all-{flag}", expect_split=False)
        assert (cond == flag).all()
        # a loop-invariant condition of that value gives the same rows, without index sets
        net2, R2, _ = check_cond(inp, "tanh", f"cond-invariant-{flag}", invariant=flag)
        assert np.array_equal(R, R2)
    # invariant condition with no condition vector at all
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    nets = [pfg.Mlp.from_numpy(Ws, bs, "tanh", "f32") for Ws, bs in (inp.pre, inp.then_net, inp.else_net)]
    bare = pfg.Cond(nets[0], None, 0.0, nets[1], nets[2])
    R, cond, counts = pfg.pfg_cond_forward(bare, dev(inp.X), 1)
    torch.cuda.synchronize()
    _, Rref, _ = check_cond(inp, "tanh", "cond-invariant-bare", invariant=1)
    assert np.array_equal(R.cpu().numpy(), Rref) and counts.tolist() == [300, 0]
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_cond_forward(bare, dev(inp.X), pfg.PFG_COND_PER_ITERATION)
    assert ei.value.code == pfg.PFG_ERR_NULL


def test_cond_row_on_the_boundary_takes_a_valid_branch():
    """An offset that puts one row's float64 score at ~1e-9: float32 may decide either way, and the
    row must then hold that branch's output."""
    wk = wl.CondWorkload("edgeq", 730, (10, 12), (14, 5), (5,), "tanh", 64)
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    s = np_scores(inp, "tanh")
    j = int(np.argsort(np.abs(s))[len(s) // 2])
    inp.c0 = float(inp.c0 - s[j] + 1e-9)
    net, R, cond = check_cond(inp, "tanh", "cond-edge")
    assert abs(np_scores(inp, "tanh")[j]) < 1e-8


def test_cond_skipped_outputs_and_row_order():
    wk = wl.CondWorkload("permq", 740, (18, 40), (64, 12), (28, 12), "relu", 700)
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    net, R, cond = check_cond(inp, "relu", "cond-perm")
    X = dev(inp.X)
    R2, c2, k2 = pfg.pfg_cond_forward(net, X, want_cond=False, want_counts=False)
    torch.cuda.synchronize()
    assert c2 is None and k2 is None and np.array_equal(R2.cpu().numpy(), R)
    # iteration independence: permuted rows give the permuted result bit for bit, although every
    # row then sits at another place of its index set
    perm = np.random.default_rng(74).permutation(700)
    Rp, cp, _ = pfg.pfg_cond_forward(net, dev(inp.X[perm]))
    torch.cuda.synchronize()
    assert np.array_equal(cp.cpu().numpy(), cond[perm]) and np.array_equal(Rp.cpu().numpy(), R[perm])
    # a second call into the same workspace with fewer rows
    ws = torch.empty(pfg.pfg_cond_workspace_bytes(net, 700), dtype=torch.uint8, device="cuda:0")
    pfg.pfg_cond_forward(net, X, workspace=ws)
    Rs, cs, ks = pfg.pfg_cond_forward(net, dev(inp.X[:45]), workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(Rs.cpu().numpy(), R[:45]) and ks.tolist() == [int(cond[:45].sum()), 45 - int(cond[:45].sum())]


def test_cond_replays_from_a_graph_with_other_data():
    """The launch sequence does not depend on the data: a call captured once into a HIP graph is
    replayed on other inputs (other index sets, other set sizes, one replay with an empty set) and
    must reproduce the eager results bit for bit every time."""
    wk = wl.CondWorkload("graphq", 760, (20, 48), (96, 7), (7,), "tanh", 900)
    inp = wl.make_cond_inputs(wk, bias_scale=0.2)
    net = gpu_net(inp, "tanh")
    rng = np.random.default_rng(76)
    batches = [inp.X, rng.standard_normal(inp.X.shape).astype(np.float32),
               (inp.X + 2.0 * np.sign(inp.w[:1])).astype(np.float32),
               np.repeat(inp.X[:1], 900, axis=0)]                    # all rows equal: one set is empty
    eager = []
    for Xb in batches:
        R, c, k = pfg.pfg_cond_forward(net, dev(Xb))
        torch.cuda.synchronize()
        eager.append((R.clone(), c.clone(), k.clone()))
    assert len({tuple(e[2].tolist()) for e in eager}) >= 3            # the set sizes really differ
    assert 0 in eager[3][2].tolist()
    Xs = dev(batches[0]).clone()
    out = (torch.empty_like(eager[0][0]), torch.empty_like(eager[0][1]), torch.empty_like(eager[0][2]))
    ws = torch.empty(pfg.pfg_cond_workspace_bytes(net, 900), dtype=torch.uint8, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pfg.pfg_cond_forward(net, Xs, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pfg.pfg_cond_forward(net, Xs, out=out, workspace=ws)
    for replay in (0, 1, 2, 3, 1, 0):
        Xs.copy_(dev(batches[replay]))
        out[0].fill_(float("nan"))                                    # eager work between the replays
        pfg.pfg_cond_forward(net, dev(batches[(replay + 1) % 4]))     # an eager call in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want, name in zip(out, eager[replay], ("R", "cond", "counts")):
            assert torch.equal(got, want), f"replay of batch {replay}: {name} differs"


def test_c11_cond_full_size():
    wk = wl.COND_WORKLOADS["c11_cond_two_branches"]
    say(f"{wk.name}: full size ({wk.n} rows), sampled rows element by element")
    inp = wl.make_cond_inputs(wk)
    picks = sorted(set([0, wk.n - 1] + np.random.default_rng(11).integers(0, wk.n, size=200).tolist()))
    net, R, cond = check_cond(inp, wk.act, "c11", rows=picks)
    # every row: against a float32 library computation of BOTH branches on the GPU, selected by the
    # returned flags (a looser bound: both sides are float32)
    X = dev(inp.X)
    f = torch.relu
    T = f(X @ dev(inp.pre[0][0]) + dev(inp.pre[1][0]))
    def mlp(A, Ws, bs):
        for l, (W, b) in enumerate(zip(Ws, bs)):
            A = A @ dev(W) + dev(b)
            if l < len(Ws) - 1:
                A = f(A)
        return A
    both = torch.where(dev(cond).bool().unsqueeze(1), mlp(T, *inp.then_net), mlp(T, *inp.else_net)).cpu().numpy()
    e = row_err(R, both)
    say(f"  c11: all {wk.n} rows against a float32 library select of both branches: {e:.3e}")
    assert e <= 5 * TOL_F32


def test_cond_rejects_bad_arguments():
    wk = wl.CondWorkload("badq", 750, (6, 8), (5,), (5,), "relu", 10)
    inp = wl.make_cond_inputs(wk)
    net = gpu_net(inp, "relu")
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_cond_forward(net, dev(inp.X), workspace=small)
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_cond_forward(net, dev(inp.X), 5)
    assert ei.value.code == pfg.PFG_ERR_UNSUPPORTED
