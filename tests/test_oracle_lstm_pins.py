"""Pins for the float64 LSTM oracle (oracle/lstm_oracle.c), against things other than itself: a
hand-worked scalar fixture, the library LSTM cell of torch (float64), autograd through that cell,
central finite differences, closed forms for one step, and invariants.

CPU only.  Nothing here touches the HIP library.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import lstm

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_lstm(rng, dx, H, dy, T, bias=True, scale=1.0):
    W = rng.standard_normal((dx + H, 4 * H)) * scale / math.sqrt(dx + H)
    b = rng.standard_normal(4 * H) * 0.3 if bias else None
    Wout = rng.standard_normal((H, dy)) / math.sqrt(H)
    bout = rng.standard_normal(dy) * 0.3 if bias else None
    return lstm.Lstm(W, b, Wout, bout, T)


def torch_cell(net, requires_grad=False):
    """torch.nn.LSTMCell (gate order i, f, g, o; weights [4H, in]) holding the oracle's weights
    (column blocks i, g, f, o of a [dx + H, 4H] matrix), plus the readout as tensors."""
    H, dx = net.H, net.dx
    blocks = [0, 2, 1, 3]                                   # torch block k is our block blocks[k]
    cols = np.concatenate([np.arange(k * H, (k + 1) * H) for k in blocks])
    cell = torch.nn.LSTMCell(dx, H, bias=True, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(net.W[:dx][:, cols].T.copy()))
        cell.weight_hh.copy_(torch.from_numpy(net.W[dx:][:, cols].T.copy()))
        cell.bias_ih.copy_(torch.from_numpy((net.b if net.b is not None else np.zeros(4 * H))[cols]))
        cell.bias_hh.zero_()
    Wout = torch.from_numpy(net.Wout).clone().requires_grad_(requires_grad)
    bout = torch.from_numpy(net.bout if net.bout is not None else np.zeros(net.dy)).clone()
    bout.requires_grad_(requires_grad)
    return cell, Wout, bout, cols


def torch_run(net, cell, Wout, bout, x):
    h = torch.zeros(1, net.H, dtype=torch.float64)
    c = torch.zeros(1, net.H, dtype=torch.float64)
    hs, cs = [], []
    for t in range(net.T):
        h, c = cell(x[t:t + 1], (h, c))
        hs.append(h[0])
        cs.append(c[0])
    return h[0] @ Wout + bout, hs, cs


def test_hand_fixture_two_steps():
    g = json.load(open(os.path.join(GOLD, "lstm_1_1_2_T2.json")))
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    i1, g1, o1 = sig(0.5), math.tanh(-1.0), sig(2.0)
    c1 = i1 * g1
    h1 = o1 * math.tanh(c1)
    i2, g2, f2, o2 = sig(-0.5 + h1), math.tanh(1.0 + 0.5 * h1), sig(0.75 - 0.5 * h1), sig(-2.0 - h1)
    c2 = f2 * c1 + i2 * g2
    h2 = o2 * math.tanh(c2)
    net = lstm.Lstm(np.array(g["W"], float), np.array(g["b"], float), np.array(g["Wout"], float),
                    np.array(g["bout"], float), g["T"])
    x = np.array(g["x"], float)
    h, c = lstm.states(net, x)
    np.testing.assert_allclose(h[:, 0], [h1, h2], rtol=1e-14)
    np.testing.assert_allclose(c[:, 0], [c1, c2], rtol=1e-14)
    np.testing.assert_allclose(lstm.forward(net, x), [2 * h2 + 0.5, -3 * h2], rtol=1e-14)


@pytest.mark.parametrize("bias", [True, False])
def test_states_match_the_library_cell(bias):
    rng = np.random.default_rng(61)
    net = rand_lstm(rng, 5, 7, 3, 6, bias=bias)
    x = rng.standard_normal((6, 5))
    cell, Wout, bout, _ = torch_cell(net)
    with torch.no_grad():
        y, hs, cs = torch_run(net, cell, Wout, bout, torch.from_numpy(x))
    h, c = lstm.states(net, x)
    np.testing.assert_allclose(h, torch.stack(hs).numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(c, torch.stack(cs).numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lstm.forward(net, x), y.numpy(), rtol=1e-12, atol=1e-14)
    p = scipy.special.softmax(y.numpy())
    assert lstm.loss(net, x, 1) == pytest.approx(-math.log(p[1]), rel=1e-12)


def test_one_step_closed_form():
    # T = 1 from a zero state: c = i g, h = o tanh(c); the forget gate multiplies c_0 = 0
    rng = np.random.default_rng(62)
    net = rand_lstm(rng, 4, 3, 2, 1)
    x = rng.standard_normal((1, 4))
    z = x[0] @ net.W[:4] + net.b
    i, g, o = scipy.special.expit(z[0:3]), np.tanh(z[3:6]), scipy.special.expit(z[9:12])
    h = o * np.tanh(i * g)
    np.testing.assert_allclose(lstm.forward(net, x), h @ net.Wout + net.bout, rtol=1e-13)
    # gradient with respect to the forget-gate columns and the recurrent rows is exactly zero
    dW, db, _, _, _ = lstm.body_per_example_grads(net, x, 0)
    assert not dW[:, 6:9].any() and not db[6:9].any() and not dW[4:].any()


def test_per_example_grads_against_autograd_through_the_library_cell():
    rng = np.random.default_rng(63)
    net = rand_lstm(rng, 4, 6, 5, 7)
    B = 3
    X = rng.standard_normal((B, 7, 4))
    labels = rng.integers(0, 5, size=B)
    dW, db, dWout, dbout, loss = lstm.per_example_grads(net, X, labels)
    for b in range(B):
        cell, Wout, bout, cols = torch_cell(net, requires_grad=True)
        y, _, _ = torch_run(net, cell, Wout, bout, torch.from_numpy(X[b]))
        ell = -torch.log_softmax(y, dim=0)[int(labels[b])]
        g_ih, g_hh, g_b, g_Wout, g_bout = torch.autograd.grad(
            ell, [cell.weight_ih, cell.weight_hh, cell.bias_ih, Wout, bout])
        want_W = np.empty_like(net.W)
        want_W[:4][:, cols] = g_ih.numpy().T
        want_W[4:][:, cols] = g_hh.numpy().T
        want_b = np.empty(24)
        want_b[cols] = g_b.numpy()
        np.testing.assert_allclose(dW[b], want_W, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(db[b], want_b, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(dWout[b], g_Wout.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(dbout[b], g_bout.numpy(), rtol=1e-10, atol=1e-13)
        assert loss[b] == pytest.approx(float(ell.detach()), rel=1e-12)


def test_grad_norms_against_autograd_and_the_gram_identity():
    """The norm of an example's gradient, (a) from autograd through the library cell, tensor by
    tensor, and (b) without any gradient tensor: the weight gradient is sum_t u_t^T dz_t, so its
    squared norm is sum_{t,t'} (u_t . u_t') (dz_t . dz_t'), with u_t = [x_t, h_{t-1}] from the library
    cell and dz_t recovered from autograd's gradient with respect to the step's pre-activations."""
    rng = np.random.default_rng(64)
    net = rand_lstm(rng, 3, 5, 4, 6)
    B = 4
    X = rng.standard_normal((B, 6, 3))
    labels = rng.integers(0, 4, size=B)
    sq, norm, loss = lstm.per_example_grad_norms(net, X, labels)
    for b in range(B):
        cell, Wout, bout, cols = torch_cell(net, requires_grad=True)
        y, hs, _ = torch_run(net, cell, Wout, bout, torch.from_numpy(X[b]))
        ell = -torch.log_softmax(y, dim=0)[int(labels[b])]
        g_ih, g_hh, g_b, g_Wout, g_bout = torch.autograd.grad(
            ell, [cell.weight_ih, cell.weight_hh, cell.bias_ih, Wout, bout])
        want = [float((g_ih ** 2).sum() + (g_hh ** 2).sum()), float((g_b ** 2).sum()),
                float((g_Wout ** 2).sum()), float((g_bout ** 2).sum())]
        np.testing.assert_allclose(sq[b], want, rtol=1e-10)
        assert norm[b] == pytest.approx(math.sqrt(sum(want)), rel=1e-12)
        assert loss[b] == pytest.approx(float(ell.detach()), rel=1e-12)
        # (b) the Gram form: dz_t as the gradient with respect to a zero offset added to step t's
        # pre-activations (an extra bias used at that step only)
        cell2, Wout2, bout2, _ = torch_cell(net)
        offs = [torch.zeros(4 * net.H, dtype=torch.float64, requires_grad=True) for _ in range(net.T)]
        h = torch.zeros(net.H, dtype=torch.float64)
        c = torch.zeros(net.H, dtype=torch.float64)
        us = []
        xb = torch.from_numpy(X[b])
        for t in range(net.T):
            us.append(torch.cat([xb[t], h]).detach().numpy())
            z = cell2.weight_ih @ xb[t] + cell2.weight_hh @ h + cell2.bias_ih + offs[t]
            i, f, g, o = z.split(net.H)                    # torch's gate order
            c = torch.sigmoid(f) * c + torch.sigmoid(i) * torch.tanh(g)
            h = torch.sigmoid(o) * torch.tanh(c)
        ell2 = -torch.log_softmax(h @ Wout2 + bout2, dim=0)[int(labels[b])]
        dzs = [d.numpy() for d in torch.autograd.grad(ell2, offs)]
        gram = sum(float(us[t] @ us[u]) * float(dzs[t] @ dzs[u]) for t in range(net.T) for u in range(net.T))
        assert sq[b, 0] == pytest.approx(gram, rel=1e-10)
        assert sq[b, 1] == pytest.approx(float(np.sum(np.sum(dzs, axis=0) ** 2)), rel=1e-10)


def test_per_example_grads_by_central_finite_differences():
    rng = np.random.default_rng(64)
    net = rand_lstm(rng, 3, 4, 3, 5)
    x = rng.standard_normal((5, 3))
    label = int(np.argmin(lstm.forward(net, x)))           # least likely class: a large gradient
    dW, db, dWout, dbout, _ = lstm.body_per_example_grads(net, x, label)
    h = 1e-6

    def fd(arr, idx):
        keep = arr[idx]
        arr[idx] = keep + h
        up = lstm.loss(lstm.Lstm(net.W, net.b, net.Wout, net.bout, net.T), x, label)
        arr[idx] = keep - h
        dn = lstm.loss(lstm.Lstm(net.W, net.b, net.Wout, net.bout, net.T), x, label)
        arr[idx] = keep
        return (up - dn) / (2 * h)

    for idx in [(0, 0), (2, 5), (3, 9), (6, 15), (5, 2), (1, 12)]:     # input rows and recurrent rows
        assert dW[idx] == pytest.approx(fd(net.W, idx), rel=1e-6, abs=1e-9)
    for k in (0, 5, 10, 15):
        assert db[k] == pytest.approx(fd(net.b, k), rel=1e-6, abs=1e-9)
    assert dWout[2, 1] == pytest.approx(fd(net.Wout, (2, 1)), rel=1e-6, abs=1e-9)
    assert dbout[0] == pytest.approx(fd(net.bout, 0), rel=1e-6, abs=1e-9)


def test_readout_gradients_closed_form_and_weight_sharing_over_steps():
    rng = np.random.default_rng(65)
    net = rand_lstm(rng, 3, 5, 4, 6)
    X = rng.standard_normal((4, 6, 3))
    labels = rng.integers(0, 4, size=4)
    dW, db, dWout, dbout, loss = lstm.per_example_grads(net, X, labels)
    for b in range(4):
        h, _ = lstm.states(net, X[b])
        p = scipy.special.softmax(lstm.forward(net, X[b]))
        assert loss[b] == pytest.approx(-math.log(p[labels[b]]), rel=1e-12)
        p[labels[b]] -= 1.0
        np.testing.assert_allclose(dbout[b], p, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(dWout[b], np.outer(h[-1], p), rtol=1e-12, atol=1e-15)
        # the bias gradient is the sum over steps of the same rows that multiply u_t in dW: the
        # input rows of dW are sum_t x_t dz_t; with x_t = e_0 for every t they equal db
    ones = np.zeros((1, 6, 3))
    ones[:, :, 0] = 1.0
    dW1, db1, _, _, _ = lstm.per_example_grads(net, ones, [0])
    np.testing.assert_allclose(dW1[0, 0], db1[0], rtol=1e-12, atol=1e-15)
    assert not dW1[0, 1:3].any()


def test_pfor_driver_equals_body_and_permutes_with_the_batch():
    rng = np.random.default_rng(66)
    net = rand_lstm(rng, 3, 4, 3, 4)
    X = rng.standard_normal((5, 4, 3))
    labels = rng.integers(0, 3, size=5)
    outs = lstm.per_example_grads(net, X, labels)
    for b in range(5):
        body = lstm.body_per_example_grads(net, X[b], int(labels[b]))
        for got, want in zip(outs, body):
            np.testing.assert_array_equal(got[b], want)
    perm = rng.permutation(5)
    outs_p = lstm.per_example_grads(net, X[perm], labels[perm])
    for got, want in zip(outs_p, outs):
        np.testing.assert_array_equal(got, want[perm])


def test_input_jacobian_against_autograd_and_finite_differences():
    rng = np.random.default_rng(67)
    net = rand_lstm(rng, 3, 5, 4, 6)
    X = rng.standard_normal((2, 6, 3))
    J = lstm.jacobian_input(net, X)
    assert J.shape == (2, 4, 6, 3)
    cell, Wout, bout, _ = torch_cell(net)
    for b in range(2):
        f = lambda x: torch_run(net, cell, Wout, bout, x)[0]
        want = torch.autograd.functional.jacobian(f, torch.from_numpy(X[b])).numpy()
        np.testing.assert_allclose(J[b], want, rtol=1e-10, atol=1e-13)
    h = 1e-6
    for (t, r) in [(0, 0), (3, 2), (5, 1)]:
        xp, xm = X[0].copy(), X[0].copy()
        xp[t, r] += h
        xm[t, r] -= h
        fd = (lstm.forward(net, xp) - lstm.forward(net, xm)) / (2 * h)
        np.testing.assert_allclose(J[0, :, t, r], fd, rtol=1e-6, atol=1e-9)


def test_jacobian_seed_forms_and_rows():
    rng = np.random.default_rng(68)
    net = rand_lstm(rng, 2, 4, 3, 5)
    X = rng.standard_normal((3, 5, 2))
    J = lstm.jacobian_input(net, X)
    shared = rng.standard_normal((2, 3))
    Js = lstm.jacobian_input(net, X, seeds=shared)
    np.testing.assert_allclose(Js, np.einsum("so,botr->bstr", shared, J), rtol=1e-12, atol=1e-15)
    tiled = np.broadcast_to(shared, (3, 2, 3)).copy()
    np.testing.assert_array_equal(lstm.jacobian_input(net, X, seeds=tiled), Js)
    per = rng.standard_normal((3, 2, 3))
    Jp = lstm.jacobian_input(net, X, seeds=per)
    np.testing.assert_allclose(Jp, np.einsum("bso,botr->bstr", per, J), rtol=1e-12, atol=1e-15)
    np.testing.assert_array_equal(lstm.body_jacobian_input_row(net, X[2], per[2, 1]), Jp[2, 1])
    # the last step's block of the Jacobian does not involve the recurrent weights:
    # d y / d x_T = Wout^T diag-chain through the last cell only; check it against one-step FD
    zero_out = lstm.Lstm(net.W, net.b, np.zeros_like(net.Wout), net.bout, net.T)
    assert not lstm.jacobian_input(zero_out, X).any()


# --------------------------------------------------------------------------------------------
# Sequences of different lengths (the while loop inside the parallel-for, Section 3.7).
# --------------------------------------------------------------------------------------------
def test_varlen_forward_matches_the_library_cell_sequence_by_sequence():
    rng = np.random.default_rng(71)
    net = rand_lstm(rng, 4, 6, 3, 1)
    lengths = np.array([3, 1, 7, 2, 7, 5])
    X = rng.standard_normal((int(lengths.sum()), 4))
    h, y = lstm.varlen_forward(net, X, lengths)
    cell, Wout, bout, _ = torch_cell(net)
    start = 0
    for b, n in enumerate(lengths):
        hb = torch.zeros(1, 6, dtype=torch.float64)
        cb = torch.zeros(1, 6, dtype=torch.float64)
        with torch.no_grad():
            for t in range(n):
                hb, cb = cell(torch.from_numpy(X[start + t:start + t + 1]), (hb, cb))
            want_y = hb[0] @ Wout + bout
        np.testing.assert_allclose(h[b], hb[0].numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(y[b], want_y.numpy(), rtol=1e-12, atol=1e-14)
        start += n


def test_varlen_forward_reduces_to_the_fixed_length_model_and_ignores_the_batch_order():
    rng = np.random.default_rng(72)
    T = 5
    net = rand_lstm(rng, 3, 4, 2, T)
    X = rng.standard_normal((4, T, 3))
    h, y = lstm.varlen_forward(net, X.reshape(4 * T, 3), [T] * 4)
    for b in range(4):
        hs, _ = lstm.states(net, X[b])
        np.testing.assert_array_equal(h[b], hs[-1])
        np.testing.assert_array_equal(y[b], lstm.forward(net, X[b]))
    # a sequence's result depends on its own tokens only: truncating it to n tokens gives the
    # state after n steps, whatever the other sequences in the batch are
    lengths = [2, 5, 1, 4]
    packed = np.concatenate([X[b, :n] for b, n in enumerate(lengths)])
    hv, _ = lstm.varlen_forward(net, packed, lengths)
    for b, n in enumerate(lengths):
        hs, _ = lstm.states(net, X[b])
        np.testing.assert_array_equal(hv[b], hs[n - 1])
    order = [2, 0, 3, 1]
    packed_p = np.concatenate([X[b, :lengths[b]] for b in order])
    hp, _ = lstm.varlen_forward(net, packed_p, [lengths[b] for b in order])
    np.testing.assert_array_equal(hp, hv[order])


# --------------------------------------------------------------------------------------------
# A while loop whose condition depends on the state (Section 3.7): t < len, t < max_steps and a
# halting score of the current hidden state that is not positive.
# --------------------------------------------------------------------------------------------
def packed(X, lengths):
    return np.concatenate([X[b, :n] for b, n in enumerate(lengths)] + [np.zeros((0, X.shape[2]))])


def test_while_forward_matches_the_library_cell_under_a_python_while():
    rng = np.random.default_rng(91)
    net = rand_lstm(rng, 4, 6, 3, 1)
    lengths = np.array([3, 0, 9, 2, 9, 5, 1, 7])
    X = rng.standard_normal((len(lengths), 9, 4))
    w = rng.standard_normal(6)
    c0 = -0.15
    h, y, steps = lstm.while_forward(net, packed(X, lengths), lengths, 6, w, c0)
    cell, Wout, bout, _ = torch_cell(net)
    seen = set()
    for b, n in enumerate(lengths):
        hb = torch.zeros(1, 6, dtype=torch.float64)
        cb = torch.zeros(1, 6, dtype=torch.float64)
        t = 0
        with torch.no_grad():
            while True:
                score = c0 + float(hb[0].numpy() @ w)
                assert abs(score) > 1e-9                  # the decision is not a matter of round-off
                if not (t < n and t < 6 and score <= 0.0):
                    break
                hb, cb = cell(torch.from_numpy(X[b, t:t + 1]), (hb, cb))
                t += 1
            want_y = hb[0] @ Wout + bout
        assert steps[b] == t
        np.testing.assert_allclose(h[b], hb[0].numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(y[b], want_y.numpy(), rtol=1e-12, atol=1e-14)
        seen.add("cap" if t == 6 else "len" if t == n else "halt")
    assert seen == {"cap", "len", "halt"}, seen            # every way of leaving the loop occurs


def test_while_forward_stops_at_the_first_positive_score():
    # an independent definition from the pinned state history: with h_0 = 0 and h_1 .. h_T the states
    # of the fixed-length model, steps = the first t with score(h_t) > 0, capped by len and max_steps
    rng = np.random.default_rng(92)
    T = 8
    net = rand_lstm(rng, 3, 5, 2, T)
    B = 12
    X = rng.standard_normal((B, T, 3))
    lengths = rng.integers(0, T + 1, size=B)
    w = rng.standard_normal(5) * 2.0
    c0 = -0.2
    for cap in (T + 3, 4):
        h, y, steps = lstm.while_forward(net, packed(X, lengths), lengths, cap, w, c0)
        for b in range(B):
            hs, _ = lstm.states(net, X[b])
            hist = np.concatenate([np.zeros((1, 5)), hs])              # hist[t] = state after t steps
            scores = c0 + hist @ w
            first = next((t for t in range(T + 1) if scores[t] > 0.0), T + 1)
            want = min(first, int(lengths[b]), cap)
            assert steps[b] == want
            np.testing.assert_array_equal(h[b], hist[want])
            np.testing.assert_allclose(y[b], hist[want] @ net.Wout + net.bout, rtol=1e-13, atol=1e-15)
    assert len(set(steps.tolist())) >= 3


def test_while_forward_special_cases():
    rng = np.random.default_rng(93)
    T = 6
    net = rand_lstm(rng, 3, 4, 2, T)
    X = rng.standard_normal((5, T, 3))
    lengths = [2, 6, 1, 4, 6]
    P = packed(X, lengths)
    hv, yv = lstm.varlen_forward(net, P, lengths)
    # no halting vector and a non-positive offset: only the lengths stop the loop
    h, y, steps = lstm.while_forward(net, P, lengths, 100, None, 0.0)
    np.testing.assert_array_equal(h, hv)
    np.testing.assert_array_equal(y, yv)
    assert steps.tolist() == lengths
    # a score of exactly 0 does not stop the loop (the loop runs while the score is <= 0) ...
    h, y, steps = lstm.while_forward(net, P, lengths, 100, np.zeros(4), 0.0)
    np.testing.assert_array_equal(h, hv)
    assert steps.tolist() == lengths
    # ... the smallest positive score does, before the first trip: the state stays zero
    h, y, steps = lstm.while_forward(net, P, lengths, 100, np.zeros(4), 5e-324)
    assert steps.tolist() == [0] * 5 and not h.any()
    np.testing.assert_array_equal(y, np.tile(net.bout, (5, 1)))
    # the cap on the trip count
    h, y, steps = lstm.while_forward(net, P, lengths, 3, None, -1.0)
    assert steps.tolist() == [2, 3, 1, 3, 3]
    for b in range(5):
        hs, _ = lstm.states(net, X[b])
        np.testing.assert_array_equal(h[b], hs[steps[b] - 1])
    assert lstm.while_forward(net, P, lengths, 0, None, -1.0)[2].tolist() == [0] * 5
    # the score is affine in the offset and reads the hidden state, not the cell state: with
    # w = e_k the loop stops at the first t with h_t[k] > -c0
    w = np.zeros(4)
    w[2] = 1.0
    h, y, steps = lstm.while_forward(net, P, lengths, 100, w, 0.05)
    for b in range(5):
        hs, _ = lstm.states(net, X[b])
        hist = np.concatenate([np.zeros((1, 4)), hs])
        first = next((t for t in range(T + 1) if hist[t, 2] + 0.05 > 0.0), T + 1)
        assert steps[b] == min(first, lengths[b])
    # iterations are independent: a permuted batch gives the permuted results
    order = [3, 0, 4, 2, 1]
    Pp = np.concatenate([X[b, :lengths[b]] for b in order])
    wv = rng.standard_normal(4)
    h1, y1, s1 = lstm.while_forward(net, P, lengths, 100, wv, -0.1)
    h2, y2, s2 = lstm.while_forward(net, Pp, [lengths[b] for b in order], 100, wv, -0.1)
    np.testing.assert_array_equal(h2, h1[order])
    np.testing.assert_array_equal(s2, s1[order])


# --------------------------------------------------------------------------------------------
# Per-example gradients through the while loop (Section 3.7 under Section 5.3).
# --------------------------------------------------------------------------------------------
def test_while_grads_against_autograd_through_the_library_cell_under_a_python_while():
    rng = np.random.default_rng(102)
    dx, H, dy, cap = 4, 6, 5, 6
    net = rand_lstm(rng, dx, H, dy, 1)
    lengths = np.array([3, 0, 9, 2, 9, 5, 1, 7])
    B = len(lengths)
    X = rng.standard_normal((B, 9, dx))
    labels = rng.integers(0, dy, size=B)
    w = rng.standard_normal(H)
    c0 = -0.15
    got = lstm.while_per_example_grads(net, packed(X, lengths), lengths, labels, cap, w, c0)
    seen = set()
    for b, n in enumerate(lengths):
        cell, Wout, bout, cols = torch_cell(net, requires_grad=True)
        hb = torch.zeros(1, H, dtype=torch.float64)
        cb = torch.zeros(1, H, dtype=torch.float64)
        t = 0
        while True:
            score = c0 + float(hb[0].detach().numpy() @ w)
            assert abs(score) > 1e-9
            if not (t < n and t < cap and score <= 0.0):
                break
            hb, cb = cell(torch.from_numpy(X[b, t:t + 1]), (hb, cb))
            t += 1
        assert got["steps"][b] == t
        seen.add("none" if t == 0 else "cap" if t == cap else "len" if t == n else "halt")
        ell = -torch.log_softmax(hb[0] @ Wout + bout, dim=0)[int(labels[b])]
        g_ih, g_hh, g_b, g_Wout, g_bout = torch.autograd.grad(
            ell, [cell.weight_ih, cell.weight_hh, cell.bias_ih, Wout, bout], allow_unused=True)
        zero = lambda g, like: torch.zeros_like(like) if g is None else g       # no trip: the cell is unused
        g_ih, g_hh, g_b = zero(g_ih, cell.weight_ih), zero(g_hh, cell.weight_hh), zero(g_b, cell.bias_ih)
        want_W = np.empty_like(net.W)
        want_W[:dx][:, cols] = g_ih.numpy().T
        want_W[dx:][:, cols] = g_hh.numpy().T
        want_b = np.empty(4 * H)
        want_b[cols] = g_b.numpy()
        np.testing.assert_allclose(got["dW"][b], want_W, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(got["db"][b], want_b, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(got["dWout"][b], g_Wout.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(got["dbout"][b], g_bout.numpy(), rtol=1e-10, atol=1e-13)
        assert got["loss"][b] == pytest.approx(float(ell.detach()), rel=1e-12)
    assert seen == {"none", "cap", "len", "halt"}, seen


def test_while_grads_by_central_differences_of_the_pinned_forward_loop():
    """The loss recomputed from the readout of `while_forward` (pinned above) at parameters moved by
    +-1e-6: the trip counts do not change (every score is at least 1e-3 from the threshold), so the
    difference quotient is the derivative of the loop's result."""
    rng = np.random.default_rng(102)
    dx, H, dy = 3, 4, 3
    net = rand_lstm(rng, dx, H, dy, 1)
    lengths = np.array([5, 2, 7, 4])
    X = rng.standard_normal((4, 7, dx))
    P = packed(X, lengths)
    labels = np.array([0, 2, 1, 1])
    w = rng.standard_normal(H) * 1.5
    c0 = -0.12
    got = lstm.while_per_example_grads(net, P, lengths, labels, 6, w, c0)
    assert len(set(got["steps"].tolist())) >= 3
    # margins of every decision taken
    for b in range(4):
        full = lstm.Lstm(net.W, net.b, net.Wout, net.bout, 7)
        hs, _ = lstm.states(full, X[b])
        hist = np.concatenate([np.zeros((1, H)), hs])
        for t in range(int(got["steps"][b]) + 1):
            assert abs(c0 + hist[t] @ w) > 1e-3
    eps = 1e-6

    def losses():
        n2 = lstm.Lstm(net.W, net.b, net.Wout, net.bout, 1)
        _, y, steps = lstm.while_forward(n2, P, lengths, 6, w, c0)
        assert np.array_equal(steps, got["steps"])
        return np.array([-(y[b, labels[b]] - scipy.special.logsumexp(y[b])) for b in range(4)])

    def fd(arr, idx):
        keep = arr[idx]
        arr[idx] = keep + eps
        up = losses()
        arr[idx] = keep - eps
        dn = losses()
        arr[idx] = keep
        return (up - dn) / (2 * eps)

    for idx in [(0, 0), (2, 5), (1, 9), (4, 15), (6, 2), (3, 12), (5, 7)]:     # input rows and recurrent rows
        np.testing.assert_allclose(got["dW"][(slice(None),) + idx], fd(net.W, idx), rtol=2e-6, atol=1e-9)
    for k in (0, 5, 10, 15):
        np.testing.assert_allclose(got["db"][:, k], fd(net.b, k), rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(got["dWout"][:, 2, 1], fd(net.Wout, (2, 1)), rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(got["dbout"][:, 0], fd(net.bout, 0), rtol=2e-6, atol=1e-9)


def test_while_grads_reduce_to_the_fixed_length_gradients_and_special_cases():
    rng = np.random.default_rng(103)
    T, dx, H, dy = 5, 3, 4, 3
    net = rand_lstm(rng, dx, H, dy, T)
    B = 6
    X = rng.standard_normal((B, T, dx))
    labels = rng.integers(0, dy, size=B)
    # only the lengths stop the loop and every sequence is T long: the unrolled model's gradients
    dW, db, dWout, dbout, loss = lstm.per_example_grads(net, X, labels)
    got = lstm.while_per_example_grads(net, X.reshape(B * T, dx), [T] * B, labels, 100, None, 0.0)
    assert got["steps"].tolist() == [T] * B
    for a, b in ((got["dW"], dW), (got["db"], db), (got["dWout"], dWout), (got["dbout"], dbout), (got["loss"], loss)):
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-16)
    # a cap of n trips: the gradients of the model unrolled to n steps on the first n tokens
    for n in (1, 3):
        short = lstm.Lstm(net.W, net.b, net.Wout, net.bout, n)
        sW, sb, sWo, sbo, sl = lstm.per_example_grads(short, X[:, :n], labels)
        g = lstm.while_per_example_grads(net, X.reshape(B * T, dx), [T] * B, labels, n, None, -1.0)
        assert g["steps"].tolist() == [n] * B
        np.testing.assert_allclose(g["dW"], sW, rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(g["db"], sb, rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(g["dWout"], sWo, rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(g["loss"], sl, rtol=1e-13)
    # no trip at all (a positive score before the first one, or no tokens): the state is zero, so the
    # cell's parameters and the readout weights get a zero gradient, the readout bias softmax - onehot
    for lens, c0 in (([T] * B, 1e-300), ([0] * B, -1.0)):
        Xp = X.reshape(B * T, dx) if lens[0] else np.zeros((0, dx))
        g = lstm.while_per_example_grads(net, Xp, lens, labels, 100, np.zeros(H), c0)
        assert g["steps"].tolist() == [0] * B
        assert not g["dW"].any() and not g["db"].any() and not g["dWout"].any()
        p = scipy.special.softmax(net.bout)
        for b in range(B):
            want = p.copy()
            want[labels[b]] -= 1.0
            np.testing.assert_allclose(g["dbout"][b], want, rtol=1e-13)
            assert g["loss"][b] == pytest.approx(-math.log(p[labels[b]]), rel=1e-13)
    # iterations are independent (permutation), and rows of dbout sum to zero
    lengths = [2, 5, 0, 4, 1, 3]
    P = packed(X, lengths)
    wv = rng.standard_normal(H)
    g1 = lstm.while_per_example_grads(net, P, lengths, labels, 100, wv, -0.1)
    order = [3, 0, 4, 2, 5, 1]
    Pp = np.concatenate([X[b, :lengths[b]] for b in order])
    g2 = lstm.while_per_example_grads(net, Pp, [lengths[b] for b in order], labels[order], 100, wv, -0.1)
    for k in g1:
        np.testing.assert_array_equal(g2[k], g1[k][order])
    np.testing.assert_allclose(g1["dbout"].sum(axis=1), 0.0, atol=1e-15)
    # the forward results agree with the pinned forward loop
    _, _, steps = lstm.while_forward(net, P, lengths, 100, wv, -0.1)
    assert np.array_equal(steps, g1["steps"])


# --------------------------------------------------------------------------------------------
# Norms of the per-example gradients through the while loop.
# --------------------------------------------------------------------------------------------
def test_while_grad_norms_against_autograd_through_the_library_cell_under_a_python_while():
    rng = np.random.default_rng(102)
    dx, H, dy, cap = 4, 6, 5, 6
    net = rand_lstm(rng, dx, H, dy, 1)
    lengths = np.array([3, 0, 9, 2, 9, 5, 1, 7])
    B = len(lengths)
    X = rng.standard_normal((B, 9, dx))
    labels = rng.integers(0, dy, size=B)
    w = rng.standard_normal(H)
    c0 = -0.15
    sq, norm, loss, steps = lstm.while_per_example_grad_norms(net, packed(X, lengths), lengths, labels, cap, w, c0)
    seen = set()
    for b, n in enumerate(lengths):
        cell, Wout, bout, _ = torch_cell(net, requires_grad=True)
        hb = torch.zeros(1, H, dtype=torch.float64)
        cb = torch.zeros(1, H, dtype=torch.float64)
        t = 0
        while True:
            score = c0 + float(hb[0].detach().numpy() @ w)
            if not (t < n and t < cap and score <= 0.0):
                break
            hb, cb = cell(torch.from_numpy(X[b, t:t + 1]), (hb, cb))
            t += 1
        assert steps[b] == t
        seen.add("none" if t == 0 else "cap" if t == cap else "len" if t == n else "halt")
        ell = -torch.log_softmax(hb[0] @ Wout + bout, dim=0)[int(labels[b])]
        g = torch.autograd.grad(ell, [cell.weight_ih, cell.weight_hh, cell.bias_ih, Wout, bout], allow_unused=True)
        ss = [0.0 if t_ is None else float((t_ ** 2).sum()) for t_ in g]
        want = np.array([ss[0] + ss[1], ss[2], ss[3], ss[4]])
        np.testing.assert_allclose(sq[b], want, rtol=1e-10, atol=1e-300)
        assert norm[b] == pytest.approx(math.sqrt(want.sum()), rel=1e-10)
        assert loss[b] == pytest.approx(float(ell.detach()), rel=1e-12)
    assert seen == {"none", "cap", "len", "halt"}, seen


def test_while_grad_norms_closed_forms_and_special_cases():
    rng = np.random.default_rng(113)
    T, dx, H, dy = 5, 3, 4, 3
    net = rand_lstm(rng, dx, H, dy, T)
    B = 6
    X = rng.standard_normal((B, T, dx))
    labels = rng.integers(0, dy, size=B)
    # only the lengths stop the loop and every sequence is T long: the norms of the unrolled model
    usq, unorm, uloss = lstm.per_example_grad_norms(net, X, labels)
    sq, norm, loss, steps = lstm.while_per_example_grad_norms(net, X.reshape(B * T, dx), [T] * B, labels, 100, None, 0.0)
    assert steps.tolist() == [T] * B
    np.testing.assert_allclose(sq, usq, rtol=1e-13)
    np.testing.assert_allclose(norm, unorm, rtol=1e-13)
    np.testing.assert_allclose(loss, uloss, rtol=1e-13)
    # the readout's gradient is the outer product of the last state and softmax - onehot, both known
    # from the pinned forward loop: |dbout|^2 = |p - e|^2, |dWout|^2 = |h|^2 |p - e|^2
    lengths = [2, 5, 0, 4, 1, 3]
    P = packed(X, lengths)
    wv = rng.standard_normal(H)
    sq, norm, loss, steps = lstm.while_per_example_grad_norms(net, P, lengths, labels, 100, wv, -0.1)
    h, y, fsteps = lstm.while_forward(net, P, lengths, 100, wv, -0.1)
    assert np.array_equal(steps, fsteps)
    for b in range(B):
        d = scipy.special.softmax(y[b])
        assert loss[b] == pytest.approx(-math.log(d[labels[b]]), rel=1e-13)
        d[labels[b]] -= 1.0
        assert sq[b, 3] == pytest.approx(float(d @ d), rel=1e-13)
        assert sq[b, 2] == pytest.approx(float(h[b] @ h[b]) * float(d @ d), rel=1e-13, abs=1e-300)
        assert norm[b] == pytest.approx(math.sqrt(sq[b].sum()), rel=1e-14)
    # no trip: only the readout bias has a gradient
    assert steps[2] == 0 and sq[2, 0] == 0.0 and sq[2, 1] == 0.0 and sq[2, 2] == 0.0 and sq[2, 3] > 0.0
    # the squares are those of the pinned gradients (cell weights and bias)
    g = lstm.while_per_example_grads(net, P, lengths, labels, 100, wv, -0.1)
    np.testing.assert_allclose(sq[:, 0], (g["dW"] ** 2).sum(axis=(1, 2)), rtol=1e-13)
    np.testing.assert_allclose(sq[:, 1], (g["db"] ** 2).sum(axis=1), rtol=1e-13)
    # iterations are independent
    order = [3, 0, 4, 2, 5, 1]
    Pp = np.concatenate([X[b, :lengths[b]] for b in order])
    sq2, norm2, loss2, steps2 = lstm.while_per_example_grad_norms(net, Pp, [lengths[b] for b in order], labels[order],
                                                                  100, wv, -0.1)
    np.testing.assert_array_equal(sq2, sq[order])
    np.testing.assert_array_equal(norm2, norm[order])
    np.testing.assert_array_equal(steps2, steps[order])
    # the cap
    short = lstm.Lstm(net.W, net.b, net.Wout, net.bout, 2)
    ssq, snorm, sloss = lstm.per_example_grad_norms(short, X[:, :2], labels)
    sq3, norm3, loss3, steps3 = lstm.while_per_example_grad_norms(net, X.reshape(B * T, dx), [T] * B, labels, 2, None, -1.0)
    assert steps3.tolist() == [2] * B
    np.testing.assert_allclose(sq3, ssq, rtol=1e-13)
