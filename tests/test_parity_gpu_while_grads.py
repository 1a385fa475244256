"""GPU parity for the per-example gradients through the while loop (Section 3.7 under Section 5.3):
the library runs the reverse trips on the lists of active iterations its forward loop kept on the
device; the float64 oracle (oracle/lstm_oracle.c) runs a literal `while` per sequence and then its
trips in reverse.

The halting decision compares a float32 score with zero on the GPU and a float64 one in the oracle.
As in the forward tests the oracle's trip counts are taken with the offset moved by -1e-4, 0 and
+1e-4: a sequence whose trip count is the same in all three runs is at least 1e-4 away from every
decision, must make the oracle's number of trips on the GPU and is compared element by element
(relative error per example and tensor at most 1e-4); the others must stop between the two shifted
runs.
"""
import numpy as np
import pytest

from parity_util import TOL_F32, slice_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, say  # noqa: E402
from oracle import lstm as olstm  # noqa: E402

MARGIN = 1e-4
NAMES = ("dW", "db", "dWout", "dbout", "loss")


@pytest.fixture(scope="module", autouse=True)
def gpu_ready():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    pfg.load_library()
    yield


def offsets_of(lengths):
    off = np.zeros(len(lengths) + 1, dtype=np.int32)
    np.cumsum(lengths, out=off[1:])
    return off


def draw(dx, H, dy, max_len, B, seed, min_len=0):
    w = wl.LstmWorkload("whileg", seed, "lstm_varlen_forward", dx, H, dy, max_len, B)
    inp, _ = wl.make_varlen_inputs(w, bias_scale=0.3)
    rng = np.random.default_rng(seed)
    lengths = rng.integers(min_len, max_len + 1, size=B).astype(np.int32)
    inp.X = rng.standard_normal((int(lengths.sum()), dx)).astype(np.float32)
    halt_w = (rng.standard_normal(H) * 2.0 / np.sqrt(H)).astype(np.float32)
    labels = rng.integers(0, dy, size=B).astype(np.int32)
    return inp, lengths, halt_w, labels


def poisoned(net, B):
    f32 = dict(dtype=torch.float32, device="cuda:0")
    nan = float("nan")
    return {"dW": torch.full((B, net.dx + net.H, 4 * net.H), nan, **f32), "db": torch.full((B, 4 * net.H), nan, **f32),
            "dWout": torch.full((B, net.H, net.dy), nan, **f32), "dbout": torch.full((B, net.dy), nan, **f32),
            "loss": torch.full((B,), nan, **f32), "steps": torch.full((B,), -7, dtype=torch.int32, device="cuda:0")}


def run_gpu(net, X, lengths, labels, max_steps, halt_w, halt_c, **kw):
    B = len(lengths)
    res = pfg.pfg_lstm_while_per_example_grads(
        net, dev(np.ascontiguousarray(X).reshape(-1, net.dx)), dev(offsets_of(lengths)), dev(labels), max_steps,
        halt_w=None if halt_w is None else dev(halt_w), halt_c=halt_c, out=poisoned(net, B), **kw)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items()}


def check(inp, lengths, labels, max_steps, halt_w, halt_c, tag, min_robust=0.9):
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    got = run_gpu(net, inp.X, lengths, labels, max_steps, halt_w, halt_c)
    ref = olstm.while_per_example_grads(onet, inp.X, lengths, labels, max_steps, halt_w, halt_c)
    if halt_w is None:
        lo = hi = ref["steps"]
    else:
        _, _, hi = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c - MARGIN)
        _, _, lo = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c + MARGIN)
    robust = lo == hi
    steps = got["steps"]
    say(f"  {tag}: {int(robust.sum())} of {len(lengths)} sequences compared; trip counts {ref['steps'].min()}"
        f"..{ref['steps'].max()}, {int((ref['steps'] == 0).sum())} make no trip")
    assert robust.mean() >= min_robust
    assert (steps[robust] == ref["steps"][robust]).all(), "trip counts differ from the oracle's"
    assert ((lo <= steps) & (steps <= hi)).all()
    worst = 0.0
    for name in NAMES:
        assert np.isfinite(got[name]).all(), f"{name} was not written in full"
        e = slice_rel_err(got[name][robust], ref[name][robust]) if name != "loss" else float(
            np.abs(got[name][robust] - ref[name][robust]).max() / max(1e-30, np.abs(ref[name][robust]).max()))
        say(f"  {tag}: {name} rel err {e:.3e}")
        worst = max(worst, e)
    assert worst <= TOL_F32
    return net, got, ref, robust


SHAPES = [
    # dx, H, dy, max_len, B, max_steps, halt_c
    (3, 4, 2, 6, 7, 10, -0.05),
    (1, 1, 1, 3, 2, 5, -0.01),
    (7, 20, 3, 25, 37, 30, -0.1),              # more trips than one run of the summing kernel
    (33, 65, 10, 12, 40, 8, -0.05),            # one past the tile edges, ragged column tail; the cap cuts
    (16, 32, 40, 30, 100, 40, -0.1),           # a head wider than 32
    (16, 64, 5, 12, 600, 12, -0.08),           # many row tiles
    (10, 300, 4, 5, 20, 5, -0.2),              # more than 1024 gate columns: two column chunks
    # widths that are multiples of 4 take the LDS-staged summing kernel: two row groups with a ragged
    # second one and a ragged last column chunk, trip counts around its chunk of 16 (15 .. 18, 31 .. 34)
    (100, 60, 3, 34, 48, 34, -3.0),
    (4, 4, 2, 40, 9, 33, -0.5),                # the smallest such widths: one piece per operand row
    (132, 128, 6, 20, 30, 17, -0.2),           # three row groups, the x rows end inside the second
]


@pytest.mark.parametrize("dx,H,dy,max_len,B,max_steps,halt_c", SHAPES,
                         ids=[f"dx{s[0]}-H{s[1]}-L{s[3]}-B{s[4]}" for s in SHAPES])
def test_while_grads_shapes(dx, H, dy, max_len, B, max_steps, halt_c):
    inp, lengths, halt_w, labels = draw(dx, H, dy, max_len, B, 900 + dx + H + B)
    if max_len >= 34:
        lengths_fixed = np.array([15, 16, 17, 18, 31, 32, 33, 34], dtype=np.int32)[:min(8, B)]
        lengths[:len(lengths_fixed)] = lengths_fixed
        inp.X = np.random.default_rng(B).standard_normal((int(lengths.sum()), dx)).astype(np.float32)
    say(f"while-loop gradients dx={dx} H={H} dy={dy} B={B} lengths 0..{max_len} cap {max_steps}")
    check(inp, lengths, labels, max_steps, halt_w, halt_c, "grads")


def test_while_grads_special_cases():
    inp, lengths, halt_w, labels = draw(6, 12, 4, 9, 11, 960, min_len=1)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    # only the lengths stop the loop: the gradients of an LSTM unrolled to each sequence's own length
    net, got, ref, _ = check(inp, lengths, labels, 20, None, 0.0, "lengths only")
    assert got["steps"].tolist() == lengths.tolist()
    # sequences of one common length reduce to the unrolled model's per-example gradients
    T = 5
    Xc = np.random.default_rng(3).standard_normal((11, T, 6)).astype(np.float32)
    g5 = run_gpu(net, Xc, np.full(11, T, np.int32), labels, T, None, 0.0)
    r5 = olstm.per_example_grads(olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, T), Xc, labels)
    for name, r in zip(("dW", "db", "dWout", "dbout", "loss"), r5):
        assert slice_rel_err(g5[name].reshape(11, -1), np.asarray(r).reshape(11, -1)) <= TOL_F32, name
    # the smallest positive score stops every iteration before its first trip: the state stays zero
    z = run_gpu(net, inp.X, lengths, labels, 20, np.zeros(12, np.float32), 1e-30)
    assert z["steps"].tolist() == [0] * 11
    assert not z["dW"].any() and not z["db"].any() and not z["dWout"].any()
    p = np.exp(inp.bout - inp.bout.max()); p /= p.sum()
    onehot = np.eye(4)[labels]
    assert np.abs(z["dbout"] - (p[None, :] - onehot)).max() <= 1e-6
    assert np.abs(z["loss"] + np.log(p[labels])).max() <= 1e-5
    # no trips enqueued at all
    z0 = run_gpu(net, inp.X, lengths, labels, 0, halt_w, -0.1)
    assert z0["steps"].tolist() == [0] * 11 and not z0["dW"].any() and np.array_equal(z0["dbout"], z["dbout"])
    # the cap
    check(inp, lengths, labels, 3, None, -1.0, "cap 3")
    # sequences without tokens among the others, and a batch without any token
    l2 = lengths.copy()
    l2[[0, 5, 10]] = 0
    off = offsets_of(lengths)
    X2 = np.concatenate([inp.X[off[b]:off[b + 1]] for b in range(11) if l2[b]])
    inp2 = type(inp)(inp.workload, inp.W, inp.b, inp.Wout, inp.bout, X2, inp.labels)
    _, g2, _, _ = check(inp2, l2, labels, 20, halt_w, -0.1, "some empty", min_robust=0.8)
    assert not g2["dW"][[0, 5, 10]].any()
    e = pfg.pfg_lstm_while_per_example_grads(net, dev(np.zeros((0, 6), np.float32)), dev(np.zeros(4, np.int32)),
                                             dev(labels[:3]), 5, halt_w=dev(halt_w), halt_c=-0.1, out=poisoned(net, 3))
    torch.cuda.synchronize()
    assert e["steps"].tolist() == [0] * 3 and not e["dW"].cpu().numpy().any()
    assert np.array_equal(e["dbout"].cpu().numpy(), z["dbout"][:3])
    # iterations are independent: another order of the same sequences gives the same slices, bit for bit
    order = np.array([4, 0, 8, 2, 6, 1, 3, 7, 5, 10, 9])
    Xp = np.concatenate([inp.X[off[b]:off[b + 1]] for b in order])
    ga = run_gpu(net, inp.X, lengths, labels, 20, halt_w, -0.1)
    gb = run_gpu(net, Xp, lengths[order], labels[order], 20, halt_w, -0.1)
    for name in NAMES + ("steps",):
        assert np.array_equal(gb[name], ga[name][order]), name
    # a subset of the outputs: the loss alone (no reverse sweep), the cell's weight gradient alone
    only = pfg.pfg_lstm_while_per_example_grads(net, dev(inp.X), dev(off), dev(labels), 20, halt_w=dev(halt_w),
                                                halt_c=-0.1, want=("loss",))
    torch.cuda.synchronize()
    assert list(only) == ["loss"] and np.array_equal(only["loss"].cpu().numpy(), ga["loss"])
    only = pfg.pfg_lstm_while_per_example_grads(net, dev(inp.X), dev(off), dev(labels), 20, halt_w=dev(halt_w),
                                                halt_c=-0.1, want=("dW",))
    torch.cuda.synchronize()
    assert np.array_equal(only["dW"].cpu().numpy(), ga["dW"])
    only = pfg.pfg_lstm_while_per_example_grads(net, dev(inp.X), dev(off), dev(labels), 20, halt_w=dev(halt_w),
                                                halt_c=-0.1, want=("db", "dbout"))
    torch.cuda.synchronize()
    assert np.array_equal(only["db"].cpu().numpy(), ga["db"]) and np.array_equal(only["dbout"].cpu().numpy(), ga["dbout"])


def test_while_grads_sum_to_the_batch_gradient_and_agree_with_the_forward_call():
    # the per-example gradients of iterations that share W add up to the gradient of the summed loss,
    # which autograd gives for a padded loop over the trip counts the library reported; and the trip
    # counts are those of the forward entry point
    inp, lengths, halt_w, labels = draw(5, 16, 3, 8, 24, 970)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    got = run_gpu(net, inp.X, lengths, labels, 8, halt_w, -0.1)
    _, _, steps_f, _ = pfg.pfg_lstm_while_forward(net, dev(inp.X), dev(offsets_of(lengths)), 8, halt_w=dev(halt_w),
                                                  halt_c=-0.1)
    torch.cuda.synchronize()
    assert np.array_equal(steps_f.cpu().numpy(), got["steps"])
    W = torch.tensor(inp.W, dtype=torch.float64, requires_grad=True)
    b = torch.tensor(inp.b, dtype=torch.float64, requires_grad=True)
    Wo = torch.tensor(inp.Wout, dtype=torch.float64)
    bo = torch.tensor(inp.bout, dtype=torch.float64)
    off = offsets_of(lengths)
    total = 0.0
    H = 16
    for i in range(24):
        h = torch.zeros(H, dtype=torch.float64)
        c = torch.zeros(H, dtype=torch.float64)
        for t in range(int(got["steps"][i])):
            z = torch.cat([torch.tensor(inp.X[off[i] + t], dtype=torch.float64), h]) @ W + b
            c = torch.sigmoid(z[2 * H:3 * H]) * c + torch.sigmoid(z[:H]) * torch.tanh(z[H:2 * H])
            h = torch.sigmoid(z[3 * H:]) * torch.tanh(c)
        total = total - torch.log_softmax(h @ Wo + bo, dim=0)[int(labels[i])]
    total.backward()
    assert slice_rel_err(got["dW"].astype(np.float64).sum(axis=0), W.grad.numpy(), lead=0) <= TOL_F32
    assert slice_rel_err(got["db"].astype(np.float64).sum(axis=0), b.grad.numpy(), lead=0) <= TOL_F32


def test_while_grads_replay_from_a_graph_on_other_inputs():
    inp, lengths, halt_w, labels = draw(8, 16, 3, 10, 50, 980)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    B, cap, tokens = 50, 10, 500
    X = torch.zeros((tokens, 8), dtype=torch.float32, device="cuda:0")
    off = torch.zeros((B + 1,), dtype=torch.int32, device="cuda:0")
    lab = torch.zeros((B,), dtype=torch.int32, device="cuda:0")
    hw = torch.zeros((16,), dtype=torch.float32, device="cuda:0")
    out = poisoned(net, B)
    ws = torch.empty(pfg.pfg_lstm_while_grads_workspace_bytes(net, B, tokens, cap), dtype=torch.uint8, device="cuda:0")

    def load(seed):
        rng = np.random.default_rng(seed)
        l = rng.integers(0, 11, size=B).astype(np.int32)
        x = np.zeros((tokens, 8), np.float32)
        x[:int(l.sum())] = rng.standard_normal((int(l.sum()), 8))
        X.copy_(torch.from_numpy(x))
        off.copy_(torch.from_numpy(offsets_of(l)))
        lab.copy_(torch.from_numpy(rng.integers(0, 3, size=B).astype(np.int32)))
        hw.copy_(torch.from_numpy((rng.standard_normal(16) * 0.5).astype(np.float32)))

    call = lambda: pfg.pfg_lstm_while_per_example_grads(net, X, off, lab, cap, halt_w=hw, halt_c=-0.1, out=out,
                                                        workspace=ws)
    load(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for seed in (2, 3, 1, 4):
        load(seed)
        call()
        torch.cuda.synchronize()
        eager = {k: t.clone() for k, t in out.items()}
        for t in out.values():
            t.fill_(-3)                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], eager[k]), f"replay on inputs {seed} differs from the eager call in {k}"


def test_c14_lstm_while_grads_full_size():
    # all 1024 sequences on the GPU in the launch configuration the benchmark times, and every one of
    # them that is at least 1e-4 from each of its decisions against the oracle, element by element
    # (iterations are independent, so the oracle takes them 128 at a time to bound the host memory)
    w = wl.LSTM_WORKLOADS["c14_lstm_while_grads"]
    inp, lengths, offsets, halt_w, halt_c = wl.make_while_inputs(w)
    labels = inp.labels.astype(np.int32)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    B = w.B
    res = pfg.pfg_lstm_while_per_example_grads(net, dev(inp.X), dev(offsets), dev(labels), w.T, halt_w=dev(halt_w),
                                               halt_c=halt_c, out=poisoned(net, B))
    torch.cuda.synchronize()
    steps = res["steps"].cpu().numpy()
    _, _, rsteps = olstm.while_forward(onet, inp.X, lengths, w.T, halt_w, halt_c)
    _, _, hi = olstm.while_forward(onet, inp.X, lengths, w.T, halt_w, halt_c - MARGIN)
    _, _, lo = olstm.while_forward(onet, inp.X, lengths, w.T, halt_w, halt_c + MARGIN)
    robust = lo == hi
    say(f"c14_lstm_while_grads: {int(robust.sum())} of {B} sequences at least {MARGIN:g} from every decision, "
        f"{int(steps.sum())} trips in all")
    assert robust.mean() >= 0.95 and (steps[robust] == rsteps[robust]).all() and ((lo <= steps) & (steps <= hi)).all()
    for name in NAMES:
        assert bool(torch.isfinite(res[name]).all()), f"{name} was not written in full"
    cand = np.flatnonzero(robust)
    worst = dict.fromkeys(NAMES, 0.0)
    for c0 in range(0, len(cand), 128):
        pick = cand[c0:c0 + 128]
        Xs = np.concatenate([inp.X[offsets[b]:offsets[b + 1]] for b in pick])
        ref = olstm.while_per_example_grads(onet, Xs, lengths[pick], labels[pick], w.T, halt_w, halt_c)
        assert np.array_equal(ref["steps"], rsteps[pick])
        idx = torch.from_numpy(pick).to("cuda:0")
        for name in NAMES:
            g = res[name][idx].cpu().numpy()
            worst[name] = max(worst[name], slice_rel_err(g.reshape(len(pick), -1), ref[name].reshape(len(pick), -1)))
        del ref
    for name in NAMES:
        say(f"  c14: {name} rel err {worst[name]:.3e} over {len(cand)} sequences, every element")
    assert max(worst.values()) <= TOL_F32
    # every sequence that made no trip has exact zeros in the gradients of the cell and of W_out
    none = torch.from_numpy(np.flatnonzero(steps == 0)).to("cuda:0")
    if none.numel():
        assert not bool(res["dW"][none].any()) and not bool(res["dWout"][none].any())


# --------------------------------------------------------------------------------------------
# Norms of those gradients without the gradients (two Gram matrices per iteration).
# --------------------------------------------------------------------------------------------
def check_norms(inp, lengths, labels, max_steps, halt_w, halt_c, tag, min_robust=0.9):
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    B = len(lengths)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    out = {"sq": torch.full((B, 4), float("nan"), **f32), "norm": torch.full((B,), float("nan"), **f32),
           "loss": torch.full((B,), float("nan"), **f32), "steps": torch.full((B,), -7, dtype=torch.int32, device="cuda:0")}
    got = pfg.pfg_lstm_while_per_example_grad_norms(
        net, dev(np.ascontiguousarray(inp.X).reshape(-1, net.dx)), dev(offsets_of(lengths)), dev(labels), max_steps,
        halt_w=None if halt_w is None else dev(halt_w), halt_c=halt_c, out=out)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in got.items()}
    rsq, rnorm, rloss, rsteps = olstm.while_per_example_grad_norms(onet, inp.X, lengths, labels, max_steps, halt_w, halt_c)
    if halt_w is None:
        lo = hi = rsteps
    else:
        _, _, hi = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c - MARGIN)
        _, _, lo = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c + MARGIN)
    robust = lo == hi
    assert robust.mean() >= min_robust
    assert (got["steps"][robust] == rsteps[robust]).all() and ((lo <= got["steps"]) & (got["steps"] <= hi)).all()
    for name in ("sq", "norm", "loss"):
        assert np.isfinite(got[name]).all(), f"{name} was not written in full"
    # each squared norm against its own value (a sum of squares has no cancellation to excuse)
    e_sq = float(np.max(np.abs(got["sq"][robust] - rsq[robust]) / np.maximum(rsq[robust], 1e-30), initial=0.0))
    e_norm = float(np.max(np.abs(got["norm"][robust] - rnorm[robust]) / np.maximum(rnorm[robust], 1e-30), initial=0.0))
    e_loss = float(np.max(np.abs(got["loss"][robust] - rloss[robust]), initial=0.0) / max(1e-30, np.abs(rloss[robust]).max()))
    say(f"  {tag}: {int(robust.sum())} of {B} sequences compared, trip counts {rsteps.min()}..{rsteps.max()}; "
        f"rel err sq {e_sq:.3e}, norm {e_norm:.3e}, loss {e_loss:.3e}")
    zero = robust & (rsteps == 0)
    assert not got["sq"][zero][:, :3].any(), "an iteration without a trip has non-zero norms"
    assert max(e_sq, e_norm, e_loss) <= TOL_F32
    return net, got


NORM_SHAPES = [
    (3, 4, 2, 6, 7, 10, -0.05),
    (1, 1, 1, 3, 2, 5, -0.01),
    (7, 20, 3, 25, 37, 30, -0.1),              # widths that are no multiples of 4: element-wise staging
    (33, 65, 10, 12, 40, 8, -0.05),
    (16, 32, 40, 30, 100, 40, -0.1),           # two row tiles of trips: three Gram tiles
    (100, 60, 3, 34, 48, 34, -3.0),            # trip counts on both sides of 32
    (8, 12, 4, 128, 12, 128, -3.0),            # up to 128 trips: all ten tiles, three per wave
    (128, 256, 10, 20, 64, 20, -0.5),          # c14's widths
]


@pytest.mark.parametrize("dx,H,dy,max_len,B,max_steps,halt_c", NORM_SHAPES,
                         ids=[f"dx{s[0]}-H{s[1]}-L{s[3]}-B{s[4]}" for s in NORM_SHAPES])
def test_while_grad_norms_shapes(dx, H, dy, max_len, B, max_steps, halt_c):
    inp, lengths, halt_w, labels = draw(dx, H, dy, max_len, B, 1300 + dx + H + B)
    if max_len >= 34:
        fixed = np.array([31, 32, 33, 34, 63, 64, 65, 96, 97, 127, 128, 1], dtype=np.int32)
        fixed = fixed[fixed <= max_len][:B]
        lengths[:len(fixed)] = fixed
        inp.X = np.random.default_rng(B).standard_normal((int(lengths.sum()), dx)).astype(np.float32)
    say(f"norms of while-loop gradients dx={dx} H={H} dy={dy} B={B} lengths 0..{max_len} cap {max_steps}")
    check_norms(inp, lengths, labels, max_steps, halt_w, halt_c, "norms")


def test_while_grad_norms_agree_with_the_gradient_call_and_special_cases():
    inp, lengths, halt_w, labels = draw(6, 12, 4, 9, 11, 1360, min_len=1)
    net, got = check_norms(inp, lengths, labels, 20, halt_w, -0.1, "norms")
    # the squares of the gradients the other entry point writes
    g = run_gpu(net, inp.X, lengths, labels, 20, halt_w, -0.1)
    assert np.array_equal(g["steps"], got["steps"]) and np.array_equal(g["loss"], got["loss"])
    for k, name in enumerate(("dW", "db", "dWout", "dbout")):
        want = (g[name].astype(np.float64) ** 2).reshape(11, -1).sum(axis=1)
        assert np.max(np.abs(got["sq"][:, k] - want) / np.maximum(want, 1e-30)) <= 1e-5, name
    # no trip at all: only the readout bias has a gradient
    z = pfg.pfg_lstm_while_per_example_grad_norms(net, dev(inp.X), dev(offsets_of(lengths)), dev(labels), 20,
                                                  halt_w=dev(np.zeros(12, np.float32)), halt_c=1e-30)
    torch.cuda.synchronize()
    sq = z["sq"].cpu().numpy()
    assert z["steps"].tolist() == [0] * 11 and not sq[:, :3].any() and (sq[:, 3] > 0).all()
    assert np.allclose(z["norm"].cpu().numpy(), np.sqrt(sq[:, 3]), rtol=1e-6)
    # one output alone, the cap, lengths only
    only = pfg.pfg_lstm_while_per_example_grad_norms(net, dev(inp.X), dev(offsets_of(lengths)), dev(labels), 20,
                                                     halt_w=dev(halt_w), halt_c=-0.1, want=("norm",))
    torch.cuda.synchronize()
    assert list(only) == ["norm"] and np.array_equal(only["norm"].cpu().numpy(), got["norm"])
    check_norms(inp, lengths, labels, 3, None, -1.0, "cap 3")
    check_norms(inp, lengths, labels, 20, None, 0.0, "lengths only")
    # rejected: more trips than the Gram tiles of a workgroup cover, no output
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_per_example_grad_norms(net, dev(inp.X), dev(offsets_of(lengths)), dev(labels), 129)
    assert ei.value.code == pfg.PFG_ERR_UNSUPPORTED
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_per_example_grad_norms(net, dev(inp.X), dev(offsets_of(lengths)), dev(labels), 20,
                                                  want=("loss",))
    assert ei.value.code == pfg.PFG_ERR_NULL


def test_c14_lstm_while_grad_norms_full_size():
    w = wl.LSTM_WORKLOADS["c14_lstm_while_grad_norms"]
    inp, lengths, offsets, halt_w, halt_c = wl.make_while_inputs(w)
    say(f"c14_lstm_while_grad_norms: {w.B} sequences, every one against the oracle")
    check_norms(inp, lengths, inp.labels.astype(np.int32), w.T, halt_w, halt_c, "c14 norms", min_robust=0.95)


def test_while_grads_reject_bad_arguments():
    inp, lengths, halt_w, labels = draw(4, 6, 3, 5, 4, 991)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    X, off, lab = dev(inp.X), dev(offsets_of(lengths)), dev(labels)
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_per_example_grads(net, X, off, lab, -1)
    assert ei.value.code == pfg.PFG_ERR_SHAPE
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_per_example_grads(net, X, off, lab, 5, want=("steps",))
    assert ei.value.code == pfg.PFG_ERR_NULL
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_per_example_grads(net, X, off, lab, 5,
                                             workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
