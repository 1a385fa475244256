"""Pins for the float64 oracle of a loop body with a conditional (oracle/cond_oracle.c), against
things other than itself: a hand-worked fixture, numpy's matrix products with a `where` select over
both branches evaluated for every row, the already pinned dense-network oracle, and invariants.

CPU only.  Nothing here touches the HIP library.
"""
import json
import os

import numpy as np
import pytest
import scipy.special

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
