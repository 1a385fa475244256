"""Pins for the float64 oracle of a loop body with a conditional (oracle/cond_oracle.c), against
things other than itself: a hand-worked fixture, numpy's matrix products with a `where` select over
both branches evaluated for every row, the already pinned dense-network oracle, and invariants.

CPU only.  Nothing here touches the HIP library.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle import cond

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def np_act(name, z):
    if name == "relu":
        return np.maximum(z, 0.0)
    if name == "tanh":
        return np.tanh(z)
    if name == "gelu":
        return z * scipy.special.ndtr(z)
    return z


def np_mlp(net, A, last_act=False):
    for l in range(net.L):
        A = A @ net.Ws[l]
        if net.bs[l] is not None:
            A = A + net.bs[l]
        if l < net.L - 1 or last_act:
            A = np_act(net.act, A)
    return A


def rand_net(rng, dims, act, bias=True):
    Ws = [rng.standard_normal((dims[l], dims[l + 1])) / np.sqrt(dims[l]) for l in range(len(dims) - 1)]
    bs = [rng.standard_normal(dims[l + 1]) * 0.3 if bias else None for l in range(len(dims) - 1)]
    return oracle.Net(Ws, bs, act)


def rand_cond(rng, pre, then_dims, else_dims, act="tanh", act_branch=None, c0=0.1, bias=True):
    p = rand_net(rng, pre, act, bias)
    t = rand_net(rng, (pre[-1],) + tuple(then_dims), act_branch or act, bias)
    e = rand_net(rng, (pre[-1],) + tuple(else_dims), act_branch or act, bias)
    return cond.Cond(p, rng.standard_normal(pre[-1]), c0, t, e)


def test_hand_fixture():
    g = json.load(open(os.path.join(GOLD, "cond_2_2.json")))
    pre = oracle.Net([np.array(g["W_pre"], float)], [np.array(g["b_pre"], float)], "relu")
    then_net = oracle.Net([np.array(W, float) for W in g["then_W"]], [np.array(b, float) for b in g["then_b"]], "relu")
    else_net = oracle.Net([np.array(W, float) for W in g["else_W"]], [np.array(b, float) for b in g["else_b"]], "relu")
    net = cond.Cond(pre, g["w"], g["c0"], then_net, else_net)
    X = np.array(g["X"], float)
    for i, x in enumerate(X):
        assert np.array_equal(cond.pre(net, x), np.array(g["t"][i], float))
        assert cond.score(net, x) == g["score"][i]
        r, c = cond.body(net, x)
        assert c == bool(g["cond"][i]) and np.array_equal(r, np.array(g["R"][i], float))
    R, c = cond.forward(net, X)
    assert np.array_equal(R, np.array(g["R"], float)) and c.tolist() == g["cond"]
    R1, c1 = cond.forward(net, X, invariant=1)
    assert np.array_equal(R1, np.array(g["R_invariant_true"], float)) and c1.tolist() == [1, 1, 1]
    R0, c0 = cond.forward(net, X, invariant=0)
    assert np.array_equal(R0, np.array(g["R_invariant_false"], float)) and c0.tolist() == [0, 0, 0]


@pytest.mark.parametrize("act", ["relu", "tanh", "gelu", "identity"])
def test_matches_both_branches_selected_by_where(act):
    """Both branches for every row with library matrix products, then a select: what the loop with
    an `if` must equal (the branches have no side effects)."""
    rng = np.random.default_rng(5)
    net = rand_cond(rng, (7, 9, 6), (11, 4), (5, 8, 4), act=act, c0=0.0)
    X = rng.standard_normal((40, 7))
    T = np_mlp(net.pre, X, last_act=True)
    # an offset that splits the rows roughly in half
    net = cond.Cond(net.pre, net.w, -float(np.median(T @ net.w)) + 1e-3, net.then_net, net.else_net)
    s = T @ net.w + net.c0
    want = np.where((s > 0)[:, None], np_mlp(net.then_net, T), np_mlp(net.else_net, T))
    R, c = cond.forward(net, X)
    assert 5 < int((s > 0).sum()) < 35                      # both branches are exercised
    assert np.array_equal(c, (s > 0).astype(np.int32))
    np.testing.assert_allclose(R, want, rtol=1e-12, atol=1e-13)
    for i in (0, 17, 39):
        np.testing.assert_allclose(cond.pre(net, X[i]), T[i], rtol=1e-13, atol=1e-14)
        assert abs(cond.score(net, X[i]) - s[i]) < 1e-12
        np.testing.assert_allclose(cond.branch(net, X[i], True), np_mlp(net.then_net, T[i:i + 1])[0],
                                   rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(cond.branch(net, X[i], False), np_mlp(net.else_net, T[i:i + 1])[0],
                                   rtol=1e-12, atol=1e-13)


def test_invariant_condition_is_one_dense_network():
    """With a loop-invariant condition the body is the shared part followed by one branch: a single
    dense network, for which the dense oracle (pinned on its own) gives the output."""
    rng = np.random.default_rng(6)
    net = rand_cond(rng, (6, 8), (10, 3), (3,), act="tanh")
    X = rng.standard_normal((9, 6))
    for flag, br in ((1, net.then_net), (0, net.else_net)):
        whole = oracle.Net(net.pre.Ws + br.Ws, net.pre.bs + br.bs, "tanh")
        R, c = cond.forward(net, X, invariant=flag)
        assert c.tolist() == [flag] * 9
        for i in range(9):
            np.testing.assert_allclose(R[i], oracle.forward(whole, X[i]), rtol=1e-12, atol=1e-13)


def test_rows_are_independent_and_extreme_conditions():
    rng = np.random.default_rng(7)
    net = rand_cond(rng, (5, 6), (4, 2), (7, 2), act="relu")
    X = rng.standard_normal((25, 5))
    R, c = cond.forward(net, X)
    perm = rng.permutation(25)
    Rp, cp = cond.forward(net, X[perm])
    assert np.array_equal(Rp, R[perm]) and np.array_equal(cp, c[perm])
    # a large positive / negative offset sends every row down one branch: the per-iteration
    # condition then agrees with the loop-invariant one
    for c0, flag in ((1e6, 1), (-1e6, 0)):
        far = cond.Cond(net.pre, net.w, c0, net.then_net, net.else_net)
        Ra, ca = cond.forward(far, X)
        Rb, _ = cond.forward(far, X, invariant=flag)
        assert ca.tolist() == [flag] * 25 and np.array_equal(Ra, Rb)
    # no rows at all
    R0, c0_ = cond.forward(net, np.zeros((0, 5)))
    assert R0.shape == (0, 2) and c0_.shape == (0,)


def test_condition_uses_offset_and_every_component():
    """The score is affine in c0 and in w: score(c0 + d) = score + d, and moving one component of
    w by d moves the score by d * t[k]."""
    rng = np.random.default_rng(8)
    net = rand_cond(rng, (4, 5), (3,), (3,), act="tanh", c0=0.25)
    x = rng.standard_normal(4)
    t = cond.pre(net, x)
    base = cond.score(net, x)
    assert abs(base - (float(t @ net.w) + 0.25)) < 1e-13
    shifted = cond.Cond(net.pre, net.w, 1.25, net.then_net, net.else_net)
    assert abs(cond.score(shifted, x) - (base + 1.0)) < 1e-13
    for k in range(5):
        w2 = net.w.copy()
        w2[k] += 0.5
        assert abs(cond.score(cond.Cond(net.pre, w2, 0.25, net.then_net, net.else_net), x) -
                   (base + 0.5 * t[k])) < 1e-13


# --------------------------------------------------------------------------------------------
# Per-example gradients through the conditional (Section 3.6 under Section 5.3).
# --------------------------------------------------------------------------------------------
def fixture_value(entry, shape):
    """An entry of cond_grad_2_2.json: {} is an exact zero, {"unit": multiples} a multiple of a unit."""
    units = {"q": 1.0 / (1.0 + math.exp(1.0)), "u": 1.0 - 1.0 / (1.0 + math.exp(2.0)), "h": 0.5}
    if not entry:
        return np.zeros(shape)
    (name, mult), = entry.items()
    return units[name] * np.array(mult, dtype=float)


def test_gradient_hand_fixture():
    g = json.load(open(os.path.join(GOLD, "cond_grad_2_2.json")))
    mk = lambda Ws, bs: oracle.Net([np.array(W, float) for W in Ws], [np.array(b, float) for b in bs], "relu")
    net = cond.Cond(mk([g["W_pre"]], [g["b_pre"]]), g["w"], g["c0"], mk(g["then_W"], g["then_b"]),
                    mk(g["else_W"], g["else_b"]))
    out = cond.per_example_grads(net, np.array(g["X"], float), g["labels"])
    assert out["cond"].tolist() == g["cond"]
    for i in range(4):
        for name in ("pre", "then", "else"):
            want_W = fixture_value(g[f"dW_{name}"][i], (2, 2))
            want_b = fixture_value(g[f"db_{name}"][i], (2,))
            np.testing.assert_allclose(out[name][0][0][i], want_W, rtol=1e-13, atol=0)
            np.testing.assert_allclose(out[name][1][0][i], want_b, rtol=1e-13, atol=0)
        assert out["loss"][i] == pytest.approx(eval(g["loss_formulas"][i], {"log": math.log, "exp": math.exp}),
                                               rel=1e-13)


def torch_net(m, x, last_act, params):
    act = {"relu": torch.relu, "tanh": torch.tanh, "identity": lambda v: v,
           "gelu": lambda v: torch.nn.functional.gelu(v)}[m.act]
    h = x
    for l in range(m.L):
        W = torch.from_numpy(m.Ws[l]).clone().requires_grad_(True)
        b = torch.from_numpy(m.bs[l] if m.bs[l] is not None else np.zeros(m.dims[l + 1])).clone().requires_grad_(True)
        params.append((W, b))
        h = h @ W + b
        if l < m.L - 1 or last_act:
            h = act(h)
    return h


@pytest.mark.parametrize("act", ["relu", "tanh", "gelu"])
def test_gradients_match_autograd_through_the_taken_branch(act):
    rng = np.random.default_rng(21)
    net = rand_cond(rng, (6, 8, 5), (7, 4), (9, 6, 4), act=act, c0=0.0)
    n = 14
    X = rng.standard_normal((n, 6))
    labels = rng.integers(0, 4, size=n)
    T = np_mlp(net.pre, X, last_act=True)
    net = cond.Cond(net.pre, net.w, -float(np.median(T @ net.w)) + 1e-3, net.then_net, net.else_net)
    out = cond.per_example_grads(net, X, labels)
    s = T @ net.w + net.c0
    assert 3 < int((s > 0).sum()) < 11 and np.array_equal(out["cond"], (s > 0).astype(np.int32))
    for i in range(n):
        pp, pb = [], []
        t = torch_net(net.pre, torch.from_numpy(X[i]), True, pp)
        taken, other = (("then", "else") if s[i] > 0 else ("else", "then"))
        r = torch_net(net.then_net if s[i] > 0 else net.else_net, t, False, pb)
        loss = -torch.log_softmax(r, dim=0)[int(labels[i])]
        loss.backward()
        assert out["loss"][i] == pytest.approx(float(loss.detach()), rel=1e-12)
        for l, (W, b) in enumerate(pp):
            np.testing.assert_allclose(out["pre"][0][l][i], W.grad.numpy(), rtol=1e-10, atol=1e-14)
            np.testing.assert_allclose(out["pre"][1][l][i], b.grad.numpy(), rtol=1e-10, atol=1e-14)
        for l, (W, b) in enumerate(pb):
            np.testing.assert_allclose(out[taken][0][l][i], W.grad.numpy(), rtol=1e-10, atol=1e-14)
            np.testing.assert_allclose(out[taken][1][l][i], b.grad.numpy(), rtol=1e-10, atol=1e-14)
        for arrs in out[other]:
            for a in arrs:
                assert not a[i].any(), "the branch that was not taken has a non-zero gradient"


def test_gradients_with_an_invariant_condition_are_those_of_the_concatenated_network():
    # loop-invariant condition: every row takes the same branch, so pre followed by that branch is one
    # dense network (same activation throughout) and the pinned dense oracle gives its gradients
    rng = np.random.default_rng(22)
    net = rand_cond(rng, (5, 7), (6, 3), (3,), act="tanh")
    X = rng.standard_normal((9, 5))
    labels = rng.integers(0, 3, size=9)
    for flag, name, br in ((1, "then", net.then_net), (0, "else", net.else_net)):
        out = cond.per_example_grads(net, X, labels, invariant=flag)
        assert out["cond"].tolist() == [flag] * 9
        whole = oracle.Net(net.pre.Ws + br.Ws, net.pre.bs + br.bs, "tanh")
        dW, db, loss = oracle.per_example_grads(whole, X, labels)
        got_W, got_b = out["pre"][0] + out[name][0], out["pre"][1] + out[name][1]
        for l in range(whole.L):
            np.testing.assert_allclose(got_W[l], dW[l], rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(got_b[l], db[l], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(out["loss"], loss, rtol=1e-12)
        other = "else" if flag else "then"
        assert not any(a.any() for arrs in out[other] for a in arrs)


def test_gradients_match_central_differences_of_the_pinned_forward_pass():
    rng = np.random.default_rng(23)
    net = rand_cond(rng, (4, 5), (6, 3), (3,), act="tanh", c0=0.05)
    X = rng.standard_normal((6, 4))
    labels = rng.integers(0, 3, size=6)
    out = cond.per_example_grads(net, X, labels)
    assert 0 < out["cond"].sum() < 6
    scores = np.array([cond.score(net, x) for x in X])
    assert np.abs(scores).min() > 1e-3                     # no row changes branch under the perturbation

    def losses():
        R, _ = cond.forward(net, X)
        R = R - R.max(axis=1, keepdims=True)
        return -(R[np.arange(6), labels] - np.log(np.exp(R).sum(axis=1)))

    h = 1e-6
    for name, m, which in (("pre", net.pre, 0), ("then", net.then_net, 1), ("else", net.else_net, 0)):
        for (i, j) in ((0, 1), (m.dims[which] - 1, m.dims[which + 1] - 1)):
            W = m.Ws[which]
            keep = W[i, j]
            W[i, j] = keep + h
            up = losses()
            W[i, j] = keep - h
            dn = losses()
            W[i, j] = keep
            np.testing.assert_allclose(out[name][0][which][:, i, j], (up - dn) / (2 * h), rtol=1e-6, atol=1e-9)


def test_gradients_permute_with_the_rows():
    rng = np.random.default_rng(24)
    net = rand_cond(rng, (5, 6), (4, 3), (3,), act="relu", c0=0.0)
    X = rng.standard_normal((10, 5))
    labels = rng.integers(0, 3, size=10)
    a = cond.per_example_grads(net, X, labels)
    perm = rng.permutation(10)
    b = cond.per_example_grads(net, X[perm], labels[perm])
    for name in ("pre", "then", "else"):
        for x, y in zip(a[name][0] + a[name][1], b[name][0] + b[name][1]):
            np.testing.assert_array_equal(y, x[perm])
    np.testing.assert_array_equal(b["loss"], a["loss"][perm])
