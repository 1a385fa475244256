"""GPU parity for the while loop with a state-dependent condition (Section 3.7): the library keeps
the list of active iterations on the device and evaluates the condition every trip; the float64
oracle (oracle/lstm_oracle.c) runs a literal `while` per sequence.

The halting decision compares a float32 score with zero on the GPU and a float64 one in the oracle.
The oracle is therefore run three times, with the offset moved by -1e-4, 0 and +1e-4: a sequence
whose trip count is the same in all three runs is at least 1e-4 away from every decision along its
way, and for those (nearly all) the GPU must give the oracle's trip count and, within 1e-4, its
state; for the others the GPU's trip count must lie between the two shifted runs.
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
    w = wl.LstmWorkload("while", seed, "lstm_varlen_forward", dx, H, dy, max_len, B)
    inp, _ = wl.make_varlen_inputs(w, bias_scale=0.3)
    rng = np.random.default_rng(seed)
    lengths = rng.integers(min_len, max_len + 1, size=B).astype(np.int32)
    inp.X = rng.standard_normal((int(lengths.sum()), dx)).astype(np.float32)
    halt_w = (rng.standard_normal(H) * 2.0 / np.sqrt(H)).astype(np.float32)
    return inp, lengths, halt_w


def run_gpu(net, X, lengths, max_steps, halt_w, halt_c, **kw):
    B = len(lengths)
    out = (torch.full((B, net.H), float("nan"), dtype=torch.float32, device="cuda:0"),
           torch.full((B, net.dy), float("nan"), dtype=torch.float32, device="cuda:0"),
           torch.full((B,), -7, dtype=torch.int32, device="cuda:0"),
           torch.full((1,), -7, dtype=torch.int32, device="cuda:0"))
    h, y, steps, trips = pfg.pfg_lstm_while_forward(
        net, dev(X.reshape(-1, net.dx)), dev(offsets_of(lengths)), max_steps,
        halt_w=None if halt_w is None else dev(halt_w), halt_c=halt_c, out=out, **kw)
    torch.cuda.synchronize()
    return h.cpu().numpy(), y.cpu().numpy(), steps.cpu().numpy(), int(trips.item())


def check_while(inp, lengths, max_steps, halt_w, halt_c, tag, min_robust=0.9):
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    h, y, steps, trips = run_gpu(net, inp.X, lengths, max_steps, halt_w, halt_c)
    rh, ry, rsteps = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c)
    if halt_w is None:
        lo = hi = rsteps
    else:
        _, _, hi = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c - MARGIN)   # stops later
        _, _, lo = olstm.while_forward(onet, inp.X, lengths, max_steps, halt_w, halt_c + MARGIN)   # stops earlier
    assert (lo <= rsteps).all() and (rsteps <= hi).all()
    robust = lo == hi
    say(f"  {tag}: {int(robust.sum())} of {len(lengths)} sequences are at least {MARGIN:g} from every decision; "
        f"trip counts from {rsteps.min()} to {rsteps.max()}, {trips} trips of the vectorised loop")
    assert robust.mean() >= min_robust
    assert (steps[robust] == rsteps[robust]).all(), "trip counts differ from the oracle's"
    assert ((lo <= steps) & (steps <= hi)).all()
    assert trips == int(steps.max(initial=0))
    assert np.isfinite(h).all() and np.isfinite(y).all()
    eh = slice_rel_err(h[robust], rh[robust])
    ey = slice_rel_err(y[robust], ry[robust])
    say(f"  {tag}: h rel err {eh:.3e}, y rel err {ey:.3e}")
    assert max(eh, ey) <= TOL_F32
    return net, h, y, steps


SHAPES = [
    # dx, H, dy, max_len, B, max_steps, halt_c
    (3, 4, 2, 6, 7, 10, -0.05),
    (1, 1, 1, 3, 1, 5, -0.01),
    (7, 20, 3, 25, 37, 30, -0.1),
    (33, 65, 10, 12, 40, 8, -0.05),          # one past the tile edges; the cap cuts long sequences
    (16, 32, 40, 30, 100, 40, -0.1),
    (16, 64, 5, 12, 900, 12, -0.08),         # many row tiles
    (4, 8, 2, 6, 70000, 6, -0.03),           # beyond 64 Ki rows: block counts ahead of the placing step
]


@pytest.mark.parametrize("dx,H,dy,max_len,B,max_steps,halt_c", SHAPES,
                         ids=[f"dx{s[0]}-H{s[1]}-L{s[3]}-B{s[4]}" for s in SHAPES])
def test_while_forward_shapes(dx, H, dy, max_len, B, max_steps, halt_c):
    inp, lengths, halt_w = draw(dx, H, dy, max_len, B, 700 + dx + H + B % 1000)
    say(f"while loop dx={dx} H={H} B={B} lengths 0..{max_len} cap {max_steps}")
    check_while(inp, lengths, max_steps, halt_w, halt_c, "while")


def test_while_forward_special_cases():
    inp, lengths, halt_w = draw(6, 12, 4, 9, 11, 760, min_len=1)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    # only the lengths stop the loop: no halting vector, a non-positive offset
    net, h, y, steps = check_while(inp, lengths, 20, None, 0.0, "lengths only")
    assert steps.tolist() == lengths.tolist()
    rh, ry = olstm.varlen_forward(onet, inp.X, lengths)
    assert slice_rel_err(h, rh) <= TOL_F32
    # a score of exactly 0 lets the loop go on ...
    h0, y0, s0, trips = run_gpu(net, inp.X, lengths, 20, np.zeros(12, np.float32), 0.0)
    assert s0.tolist() == lengths.tolist() and np.array_equal(h0, h) and trips == int(lengths.max())
    # ... the smallest positive one stops every iteration before its first trip
    h1, y1, s1, trips = run_gpu(net, inp.X, lengths, 20, np.zeros(12, np.float32), 1e-30)
    assert s1.tolist() == [0] * 11 and not h1.any() and trips == 0
    assert np.array_equal(y1, np.tile(inp.bout, (11, 1)))
    # the cap: 3 trips at most, none at all
    _, _, s3, trips = run_gpu(net, inp.X, lengths, 3, None, -1.0)
    assert s3.tolist() == np.minimum(lengths, 3).tolist() and trips == 3
    hz, yz, sz, trips = run_gpu(net, inp.X, lengths, 0, halt_w, -0.1)
    assert sz.tolist() == [0] * 11 and not hz.any() and trips == 0
    # sequences without tokens, and a batch in which no sequence has any
    l2 = lengths.copy()
    l2[[0, 5, 10]] = 0
    X2 = np.concatenate([inp.X[offsets_of(lengths)[b]:offsets_of(lengths)[b + 1]] for b in range(11) if l2[b]])
    inp2 = type(inp)(inp.workload, inp.W, inp.b, inp.Wout, inp.bout, X2, inp.labels)
    check_while(inp2, l2, 20, halt_w, -0.1, "some empty", min_robust=0.8)
    hE, yE, sE, trips = run_gpu(net, np.zeros((0, 6), np.float32), np.zeros(4, np.int32), 5, halt_w, -0.1)
    assert sE.tolist() == [0] * 4 and not hE.any() and trips == 0
    # iterations are independent: the same sequences in another order give the same rows, bit for bit
    order = np.array([4, 0, 8, 2, 6, 1, 3, 7, 5, 10, 9])
    off = offsets_of(lengths)
    Xp = np.concatenate([inp.X[off[b]:off[b + 1]] for b in order])
    ha, ya, sa, _ = run_gpu(net, inp.X, lengths, 20, halt_w, -0.1)
    hb, yb, sb, _ = run_gpu(net, Xp, lengths[order], 20, halt_w, -0.1)
    assert np.array_equal(hb, ha[order]) and np.array_equal(sb, sa[order]) and np.array_equal(yb, ya[order])
    # only one output wanted
    hh, none_y, none_s, none_t = pfg.pfg_lstm_while_forward(net, dev(inp.X), dev(off), 20, halt_w=dev(halt_w),
                                                            halt_c=-0.1, want_y=False, want_steps=False,
                                                            want_trips=False)
    torch.cuda.synchronize()
    assert none_y is None and none_s is None and none_t is None and np.array_equal(hh.cpu().numpy(), ha)


def test_while_forward_cuts_token_ranges_to_the_token_array():
    # seq_offsets lives on the device and is not checked by the host: a range that leaves X is cut to
    # it (here the last two sequences claim 9 and 6 rows beyond the 40 that exist)
    inp, lengths, halt_w = draw(5, 9, 3, 8, 10, 770, min_len=2)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    total = 40
    X = inp.X[:total] if inp.X.shape[0] >= total else np.concatenate([inp.X, np.zeros((total - inp.X.shape[0], 5), np.float32)])
    off = np.array([0, 5, 9, 14, 20, 26, 31, 35, 38, 49, 55], dtype=np.int32)
    h, y, steps, trips = pfg.pfg_lstm_while_forward(net, dev(X), dev(off), 20)
    torch.cuda.synchronize()
    eff = np.array([5, 4, 5, 6, 6, 5, 4, 3, 2, 0], dtype=np.int64)        # the last starts beyond the array
    assert steps.cpu().numpy().tolist() == eff.tolist()
    packed = np.concatenate([X[off[b]:off[b] + eff[b]] for b in range(10)])
    rh, _, _ = olstm.while_forward(onet, packed, eff, 20, None, 0.0)
    assert slice_rel_err(h.cpu().numpy()[:9], rh[:9]) <= TOL_F32 and not h.cpu().numpy()[9].any()


def test_c12_lstm_while_full_size():
    w = wl.LSTM_WORKLOADS["c12_lstm_while"]
    inp, lengths, offsets, halt_w, halt_c = wl.make_while_inputs(w)
    say(f"c12_lstm_while: c9's {w.B} sequences of 1..{w.T} tokens under a loop that also stops on a halting score")
    net, h, y, steps = check_while(inp, lengths, w.T, halt_w, halt_c, "c12", min_robust=0.95)
    assert (steps < lengths).sum() > 50 and (steps == lengths).sum() > 50      # both ways of stopping occur


def test_while_forward_replays_from_a_graph_on_other_inputs():
    # the launch sequence does not depend on the data: a captured call replayed after the token
    # ranges, the tokens and the halting vector have been overwritten reproduces the eager results
    inp, lengths, halt_w = draw(8, 16, 3, 10, 50, 780)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    B, cap = 50, 10
    tokens = 50 * 10
    X = torch.zeros((tokens, 8), dtype=torch.float32, device="cuda:0")
    off = torch.zeros((B + 1,), dtype=torch.int32, device="cuda:0")
    hw = torch.zeros((16,), dtype=torch.float32, device="cuda:0")
    out = (torch.zeros((B, 16), device="cuda:0"), torch.zeros((B, 3), device="cuda:0"),
           torch.zeros((B,), dtype=torch.int32, device="cuda:0"), torch.zeros((1,), dtype=torch.int32, device="cuda:0"))
    ws = torch.empty(pfg.pfg_lstm_while_workspace_bytes(net, B, tokens), dtype=torch.uint8, device="cuda:0")

    def load(seed):
        rng = np.random.default_rng(seed)
        l = rng.integers(0, 11, size=B).astype(np.int32)
        x = np.zeros((tokens, 8), np.float32)
        x[:int(l.sum())] = rng.standard_normal((int(l.sum()), 8))
        X.copy_(torch.from_numpy(x))
        off.copy_(torch.from_numpy(offsets_of(l)))
        hw.copy_(torch.from_numpy((rng.standard_normal(16) * 0.5).astype(np.float32)))

    call = lambda: pfg.pfg_lstm_while_forward(net, X, off, cap, halt_w=hw, halt_c=-0.1, out=out, workspace=ws)
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
        eager = [t.clone() for t in out]
        for t in out:
            t.fill_(-3)                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(out, eager):
            assert torch.equal(a, b), f"replay on inputs {seed} differs from the eager call"


def test_varlen_calls_back_to_back_without_synchronising():
    # the host-lengths entry point stages its index arrays in a host buffer that an asynchronous copy
    # reads; a second call must not overwrite that buffer before the first call's copy has read it
    w = wl.LstmWorkload("b2b", 790, "lstm_varlen_forward", 6, 12, 4, 9, 300)
    inp, lengths = wl.make_varlen_inputs(w, bias_scale=0.2)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    onet = olstm.Lstm(inp.W, inp.b, inp.Wout, inp.bout, 1)
    rng = np.random.default_rng(5)
    cases = []
    for _ in range(6):
        l = rng.integers(1, 10, size=300).astype(np.int32)
        x = rng.standard_normal((int(l.sum()), 6)).astype(np.float32)
        cases.append((l, x, dev(x)))
    torch.cuda.synchronize()
    results = [pfg.pfg_lstm_varlen_forward(net, xd, l, want_y=False)[0] for l, x, xd in cases]   # no sync in between
    torch.cuda.synchronize()
    for (l, x, _), h in zip(cases, results):
        rh, _ = olstm.varlen_forward(onet, x, l)
        assert slice_rel_err(h.cpu().numpy(), rh) <= TOL_F32


def test_while_forward_rejects_bad_arguments():
    inp, lengths, halt_w = draw(4, 6, 3, 5, 4, 791)
    net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
    X, off = dev(inp.X), dev(offsets_of(lengths))
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_forward(net, X, off, -1)
    assert ei.value.code == pfg.PFG_ERR_SHAPE
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_forward(net, X, off, 5, want_h=False, want_y=False, want_steps=False)
    assert ei.value.code == pfg.PFG_ERR_NULL
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_lstm_while_forward(net, X, off, 5, workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
