"""Pins for the float64 CPU oracle: what the paper and the mathematics fix, checked against
something other than the oracle itself (hand-worked fixtures, closed forms, invariants, central
finite differences, an independent autograd library, library softmax / normal CDF).

CPU only.  Nothing here touches the HIP library.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ACTS = ["identity", "relu", "tanh", "gelu"]


def rand_net(oracle, rng, dims, act, bias=True, scale=1.0):
    Ws = [rng.standard_normal((dims[l], dims[l + 1])) * scale / math.sqrt(dims[l])
          for l in range(len(dims) - 1)]
    bs = [rng.standard_normal(dims[l + 1]) * 0.3 for l in range(len(dims) - 1)] if bias else None
    return oracle.Net(Ws, bs, act)


def np_forward(net, X, act_fn):
    """Matrix-form forward with numpy matmul (library routine); returns activations list."""
    a = [np.asarray(X, dtype=np.float64)]
    zs = []
    for l in range(net.L):
        z = a[-1] @ net.Ws[l] + (0.0 if net.bs[l] is None else net.bs[l])
        zs.append(z)
        a.append(act_fn(z) if l < net.L - 1 else z)
    return a, zs


NP_ACT = {
    "identity": lambda z: z,
    "relu": lambda z: np.maximum(z, 0.0),
    "tanh": np.tanh,
    "gelu": lambda z: z * scipy.stats.norm.cdf(z),
}


def torch_net_forward(net, x, act):
    a = x
    for l in range(net.L):
        z = a @ torch.from_numpy(net.Ws[l])
        if net.bs[l] is not None:
            z = z + torch.from_numpy(net.bs[l])
        if l < net.L - 1:
            if act == "relu":
                a = torch.relu(z)
            elif act == "tanh":
                a = torch.tanh(z)
            elif act == "gelu":
                a = torch.nn.functional.gelu(z)      # exact erf form
            else:
                a = z
        else:
            a = z
    return a


# --------------------------------------------------------------------------------------------
# Stacking convention: Section 4's worked example.
# --------------------------------------------------------------------------------------------
def test_pfor_worked_example_section4(oracle):
    rng = np.random.default_rng(1)
    a = rng.uniform(size=(10, 20))
    b = rng.uniform(size=(10, 20))
    s, d = oracle.pfor_add_sub(a, b)
    assert s.shape == (10, 20) and d.shape == (10, 20)
    np.testing.assert_array_equal(s, a + b)
    np.testing.assert_array_equal(d, a - b)


# --------------------------------------------------------------------------------------------
# Forward pass.
# --------------------------------------------------------------------------------------------
def test_forward_hand_fixture(oracle):
    g = json.load(open(os.path.join(GOLD, "forward_2x3.json")))
    net = oracle.Net([np.array(g["W"], dtype=float)], [np.array(g["b"], dtype=float)], "identity")
    np.testing.assert_array_equal(oracle.forward(net, g["x"]), np.array(g["y"]))


@pytest.mark.parametrize("act", ["relu", "tanh", "gelu"])
def test_forward_zero_input_zero_bias_is_zero(oracle, act):
    rng = np.random.default_rng(2)
    net = rand_net(oracle, rng, (5, 7, 4, 3), act, bias=False)
    np.testing.assert_array_equal(oracle.forward(net, np.zeros(5)), np.zeros(3))


@pytest.mark.parametrize("act", ACTS)
def test_forward_matches_numpy_matmul(oracle, act):
    rng = np.random.default_rng(3)
    net = rand_net(oracle, rng, (6, 9, 5, 4), act)
    X = rng.standard_normal((7, 6))
    a, _ = np_forward(net, X, NP_ACT[act])
    for b in range(7):
        np.testing.assert_allclose(oracle.forward(net, X[b]), a[-1][b], rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------------------------
# Activations and their derivatives.
# --------------------------------------------------------------------------------------------
def test_activation_special_values(oracle):
    assert oracle.act_deriv("gelu", 0.0) == 0.5
    assert oracle.act_deriv("tanh", 0.0) == 1.0
    assert oracle.act_deriv("relu", 0.0) == 0.0            # convention: relu'(0) = 0
    assert oracle.act_deriv("relu", 1e-300) == 1.0
    assert oracle.act_deriv("relu", -1e-300) == 0.0
    assert oracle.act("relu", -2.0) == 0.0 and oracle.act("relu", 2.5) == 2.5
    assert oracle.act_deriv("identity", 3.0) == 1.0 and oracle.act("identity", -3.0) == -3.0
    # GELU(z) = z * Phi(z), Phi from a library
    for z in (-3.0, -0.7, 0.2, 1.0, 4.0):
        assert oracle.act("gelu", z) == pytest.approx(z * scipy.stats.norm.cdf(z), rel=1e-13)
        assert oracle.act("tanh", z) == pytest.approx(math.tanh(z), rel=1e-15)


@pytest.mark.parametrize("act", ["tanh", "gelu", "identity"])
def test_activation_derivative_by_finite_differences(oracle, act):
    h = 1e-6
    for z in np.linspace(-4.0, 4.0, 41):
        fd = (oracle.act(act, z + h) - oracle.act(act, z - h)) / (2 * h)
        assert oracle.act_deriv(act, z) == pytest.approx(fd, rel=1e-7, abs=1e-9)


# --------------------------------------------------------------------------------------------
# Loss head.
# --------------------------------------------------------------------------------------------
def test_softmax_matches_library_and_is_shift_invariant(oracle):
    rng = np.random.default_rng(4)
    y = rng.standard_normal(11) * 5
    np.testing.assert_allclose(oracle.softmax(y), scipy.special.softmax(y), rtol=1e-13)
    np.testing.assert_allclose(oracle.softmax(y + 700.0), scipy.special.softmax(y), rtol=1e-12)
    assert abs(oracle.softmax(y).sum() - 1.0) < 1e-15


def test_uniform_logits_head(oracle):
    # W = 0 and equal biases give uniform logits: loss = log d_L, delta = 1/d_L - onehot
    dL = 10
    net = oracle.Net([np.zeros((4, dL))], [np.full(dL, 0.37)], "relu")
    X = np.random.default_rng(5).standard_normal((3, 4))
    labels = np.array([0, 9, 4])
    dW, db, loss = oracle.per_example_grads(net, X, labels)
    np.testing.assert_allclose(loss, math.log(dL), rtol=1e-14)
    expect = np.full((3, dL), 1.0 / dL)
    expect[np.arange(3), labels] -= 1.0
    np.testing.assert_allclose(db[0], expect, rtol=1e-14)
    assert np.abs(db[0].sum(axis=1)).max() < 1e-15


# --------------------------------------------------------------------------------------------
# Per-example gradients.
# --------------------------------------------------------------------------------------------
def test_hand_worked_relu_net_fixture(oracle):
    g = json.load(open(os.path.join(GOLD, "relu_2_2_2.json")))
    p1 = 1.0 / (1.0 + math.exp(3.0))
    net = oracle.Net([np.array(g["W1"], float), np.array(g["W2"], float)],
                     [np.array(g["b1"], float), np.array(g["b2"], float)], g["act"])
    dW, db, loss = oracle.per_example_grads(net, np.array([g["x"]], float), [g["label"]])
    np.testing.assert_allclose(dW[1][0], p1 * np.array(g["dW2_in_units_of_p1"]), rtol=1e-13)
    np.testing.assert_allclose(db[1][0], p1 * np.array(g["db2_in_units_of_p1"]), rtol=1e-13)
    np.testing.assert_allclose(dW[0][0], p1 * np.array(g["dW1_in_units_of_p1"]), rtol=1e-13)
    np.testing.assert_allclose(db[0][0], p1 * np.array(g["db1_in_units_of_p1"]), rtol=1e-13)
    assert loss[0] == pytest.approx(-math.log(1.0 - p1), rel=1e-13)


def test_single_linear_layer_gradient_is_outer_product(oracle):
    # closed form: dW[b] = x_b^T (softmax(x_b W + b) - onehot)
    rng = np.random.default_rng(6)
    net = rand_net(oracle, rng, (7, 5), "relu")
    X = rng.standard_normal((6, 7))
    labels = rng.integers(0, 5, 6)
    dW, db, loss = oracle.per_example_grads(net, X, labels)
    P = scipy.special.softmax(X @ net.Ws[0] + net.bs[0], axis=1)
    D = P.copy()
    D[np.arange(6), labels] -= 1.0
    np.testing.assert_allclose(db[0], D, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dW[0], X[:, :, None] * D[:, None, :], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(loss, -np.log(P[np.arange(6), labels]), rtol=1e-12)


@pytest.mark.parametrize("act", ACTS)
def test_weight_gradient_structure(oracle, act):
    # every dW_l[b] is the outer product of the layer input and db_l[b] (rank one), and the
    # last layer's rows sum to zero because softmax - onehot sums to zero
    rng = np.random.default_rng(7)
    net = rand_net(oracle, rng, (5, 8, 6, 4), act)
    X = rng.standard_normal((4, 5))
    labels = rng.integers(0, 4, 4)
    dW, db, _ = oracle.per_example_grads(net, X, labels)
    a, _ = np_forward(net, X, NP_ACT[act])
    for l in range(net.L):
        np.testing.assert_allclose(dW[l], a[l][:, :, None] * db[l][:, None, :], rtol=1e-12,
                                   atol=1e-15)
    assert np.abs(dW[-1].sum(axis=2)).max() < 1e-14


@pytest.mark.parametrize("act", ACTS)
def test_per_example_grads_against_autograd_library(oracle, act):
    # independent implementation: torch autograd in float64, one example at a time, plus the
    # batch gradient of the SUMMED loss (Section 5.3: per-example contributions, not summed)
    rng = np.random.default_rng(8)
    net = rand_net(oracle, rng, (6, 9, 7, 5), act)
    B = 5
    X = rng.standard_normal((B, 6))
    labels = rng.integers(0, 5, B)
    dW, db, loss = oracle.per_example_grads(net, X, labels)

    tW = [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Ws]
    tb = [torch.from_numpy(b).clone().requires_grad_(True) for b in net.bs]

    def tforward(x):
        a = x
        for l in range(net.L):
            z = a @ tW[l] + tb[l]
            a = z if l == net.L - 1 else {"relu": torch.relu, "tanh": torch.tanh,
                                          "gelu": torch.nn.functional.gelu,
                                          "identity": lambda t: t}[act](z)
        return a

    tX = torch.from_numpy(X)
    tl = torch.from_numpy(labels.astype(np.int64))
    for b in range(B):
        lb = torch.nn.functional.cross_entropy(tforward(tX[b:b + 1]), tl[b:b + 1], reduction="sum")
        grads = torch.autograd.grad(lb, tW + tb)
        assert loss[b] == pytest.approx(lb.item(), rel=1e-12)
        for l in range(net.L):
            np.testing.assert_allclose(dW[l][b], grads[l].numpy(), rtol=1e-10, atol=1e-14)
            np.testing.assert_allclose(db[l][b], grads[net.L + l].numpy(), rtol=1e-10, atol=1e-14)
    total = torch.nn.functional.cross_entropy(tforward(tX), tl, reduction="sum")
    grads = torch.autograd.grad(total, tW + tb)
    for l in range(net.L):
        np.testing.assert_allclose(dW[l].sum(axis=0), grads[l].numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(db[l].sum(axis=0), grads[net.L + l].numpy(), rtol=1e-10,
                                   atol=1e-13)


def _fd_grad(f, arr, h):
    """Central differences of scalar f() with respect to every entry of arr (modified in place)."""
    g = np.empty_like(arr)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = arr[idx]
        arr[idx] = old + h
        fp = f()
        arr[idx] = old - h
        fm = f()
        arr[idx] = old
        g[idx] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("act", ["tanh", "gelu", "relu"])
def test_per_example_grads_by_central_finite_differences(oracle, act):
    rng = np.random.default_rng(9)
    dims = (4, 6, 5, 3)
    net = rand_net(oracle, rng, dims, act)
    h = 1e-6
    for trial in range(3):
        x = rng.standard_normal(4)
        # the least likely class: the gradient is then O(1), well above the round-off of the
        # difference quotient (about 1e-16 * |loss| / h = 1e-10)
        label = int(np.argmin(oracle.forward(net, x)))
        if act == "relu":      # stay away from the kink: every hidden pre-activation >> h
            _, zs = np_forward(net, x[None, :], NP_ACT[act])
            assert min(np.abs(z).min() for z in zs[:-1]) > 1e-3
        dW, db, _ = oracle.body_per_example_grads(net, x, label)
        for l in range(net.L):
            gW = _fd_grad(lambda: oracle.loss(net, x, label), net.Ws[l], h)
            gb = _fd_grad(lambda: oracle.loss(net, x, label), net.bs[l], h)
            scale = np.abs(gW).max()
            assert np.abs(dW[l] - gW).max() <= 1e-6 * scale
            assert np.abs(db[l] - gb).max() <= 1e-6 * np.abs(gb).max()


def test_pfor_driver_equals_body_and_is_order_independent(oracle):
    # stacked result == running the body per example; permuting the batch permutes the slices;
    # a duplicated example gives a duplicated slice (stateless iterations, Section 3.4)
    rng = np.random.default_rng(10)
    net = rand_net(oracle, rng, (5, 7, 4), "tanh")
    X = rng.standard_normal((6, 5))
    X[4] = X[1]
    labels = rng.integers(0, 4, 6)
    labels[4] = labels[1]
    dW, db, loss = oracle.per_example_grads(net, X, labels)
    for b in range(6):
        dWb, dbb, lb = oracle.body_per_example_grads(net, X[b], labels[b])
        for l in range(net.L):
            np.testing.assert_array_equal(dW[l][b], dWb[l])
            np.testing.assert_array_equal(db[l][b], dbb[l])
        assert loss[b] == lb
    perm = rng.permutation(6)
    dWp, dbp, lossp = oracle.per_example_grads(net, X[perm], labels[perm])
    for l in range(net.L):
        np.testing.assert_array_equal(dWp[l], dW[l][perm])
        np.testing.assert_array_equal(dW[l][4], dW[l][1])
    np.testing.assert_array_equal(lossp, loss[perm])


# --------------------------------------------------------------------------------------------
# Input Jacobian (Section 5.1).
# --------------------------------------------------------------------------------------------
def test_input_jacobian_of_linear_net_is_weight_product(oracle):
    rng = np.random.default_rng(11)
    net = rand_net(oracle, rng, (5, 7, 6, 4), "identity")
    X = rng.standard_normal((3, 5))
    J = oracle.jacobian_input(net, X)
    prod = (net.Ws[0] @ net.Ws[1] @ net.Ws[2]).T          # [d_L, d_0]
    assert J.shape == (3, 4, 5)
    for b in range(3):
        np.testing.assert_allclose(J[b], prod, rtol=1e-12, atol=1e-15)


def test_input_jacobian_of_tanh_net_at_origin(oracle):
    # tanh'(0) = 1, so at x = 0 with zero biases the Jacobian is again the weight product
    rng = np.random.default_rng(12)
    net = rand_net(oracle, rng, (4, 6, 3), "tanh", bias=False)
    J = oracle.jacobian_input(net, np.zeros((2, 4)))
    np.testing.assert_allclose(J[0], (net.Ws[0] @ net.Ws[1]).T, rtol=1e-13, atol=1e-16)
    np.testing.assert_array_equal(J[0], J[1])


def test_input_jacobian_scalar_chain_rule(oracle):
    # 1 -> 1 -> 1 tanh net: y = w2 tanh(w1 x + b1) + b2, dy/dx = w2 (1 - tanh^2(w1 x + b1)) w1
    w1, b1, w2, b2, x = 2.0, -0.3, 3.0, 0.25, 0.5
    net = oracle.Net([np.array([[w1]]), np.array([[w2]])], [np.array([b1]), np.array([b2])],
                     "tanh")
    J = oracle.jacobian_input(net, np.array([[x]]))
    expect = w2 * (1.0 - math.tanh(w1 * x + b1) ** 2) * w1
    assert J.shape == (1, 1, 1) and J[0, 0, 0] == pytest.approx(expect, rel=1e-14)


@pytest.mark.parametrize("act", ACTS)
def test_input_jacobian_against_autograd_library(oracle, act):
    rng = np.random.default_rng(13)
    net = rand_net(oracle, rng, (5, 8, 6, 4), act)
    X = rng.standard_normal((3, 5))
    J = oracle.jacobian_input(net, X)
    for b in range(3):
        Jt = torch.autograd.functional.jacobian(lambda x: torch_net_forward(net, x, act),
                                                torch.from_numpy(X[b]))
        np.testing.assert_allclose(J[b], Jt.numpy(), rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("act", ["tanh", "gelu"])
def test_input_jacobian_by_finite_differences(oracle, act):
    rng = np.random.default_rng(14)
    net = rand_net(oracle, rng, (5, 7, 6, 4), act)
    x = rng.standard_normal(5)
    J = oracle.jacobian_input(net, x[None, :])[0]           # [d_L, d_0]
    h = 1e-6
    for i in range(5):
        e = np.zeros(5)
        e[i] = h
        col = (oracle.forward(net, x + e) - oracle.forward(net, x - e)) / (2 * h)
        assert np.abs(J[:, i] - col).max() <= 1e-6 * np.abs(J).max()
    v = rng.standard_normal(5)
    jv = (oracle.forward(net, x + h * v) - oracle.forward(net, x - h * v)) / (2 * h)
    np.testing.assert_allclose(J @ v, jv, rtol=1e-6, atol=1e-8)


def test_jacobian_rows_are_gradients_of_single_outputs(oracle):
    # "each iteration computes the gradient of one scalar value in the output" (Section 5.1)
    rng = np.random.default_rng(15)
    net = rand_net(oracle, rng, (5, 6, 4), "gelu")
    X = rng.standard_normal((2, 5))
    J = oracle.jacobian_input(net, X)
    for b in range(2):
        for s in range(4):
            e = np.zeros(4)
            e[s] = 1.0
            np.testing.assert_array_equal(J[b, s], oracle.body_jacobian_input_row(net, X[b], e))


def test_shared_seeds_equal_tiled_seeds(oracle):
    # a loop-invariant operand gives the same answer as if it were tiled n times (Section 3.4)
    rng = np.random.default_rng(16)
    net = rand_net(oracle, rng, (5, 6, 4), "tanh")
    X = rng.standard_normal((3, 5))
    seeds = rng.standard_normal((7, 4))
    J_shared = oracle.jacobian_input(net, X, seeds=seeds)
    J_tiled = oracle.jacobian_input(net, X, seeds=np.tile(seeds[None], (3, 1, 1)))
    np.testing.assert_array_equal(J_shared, J_tiled)
    J_id = oracle.jacobian_input(net, X)
    np.testing.assert_array_equal(J_id, oracle.jacobian_input(net, X, seeds=np.eye(4)))
    # general seeds are linear combinations of Jacobian rows
    np.testing.assert_allclose(J_shared, np.einsum("sk,bki->bsi", seeds, J_id), rtol=1e-12,
                               atol=1e-15)
    per_ex = rng.standard_normal((3, 2, 4))
    np.testing.assert_allclose(oracle.jacobian_input(net, X, seeds=per_ex),
                               np.einsum("bsk,bki->bsi", per_ex, J_id), rtol=1e-12, atol=1e-15)


# --------------------------------------------------------------------------------------------
# Weight Jacobian (nested parallel-for, Section 3.7).
# --------------------------------------------------------------------------------------------
def test_softmax_jacobian_row_closed_form(oracle):
    y = np.array([0.3, -1.2, 2.0, 0.0])
    p = scipy.special.softmax(y)
    for k in range(4):
        np.testing.assert_allclose(oracle.softmax_jacobian_row(y, k),
                                   p[k] * (np.eye(4)[k] - p), rtol=1e-13)
    h = 1e-6
    for j in range(4):
        e = np.zeros(4)
        e[j] = h
        col = (scipy.special.softmax(y + e) - scipy.special.softmax(y - e)) / (2 * h)
        for k in range(4):
            assert oracle.softmax_jacobian_row(y, k)[j] == pytest.approx(col[k], rel=1e-6,
                                                                         abs=1e-10)


@pytest.mark.parametrize("act", ["tanh", "relu", "gelu"])
def test_weight_jacobian_invariants_and_cross_pin(oracle, act):
    rng = np.random.default_rng(17)
    net = rand_net(oracle, rng, (5, 7, 6, 4), act)
    B = 3
    X = rng.standard_normal((B, 5))
    labels = rng.integers(0, 4, B)
    JW, Jb = oracle.jacobian_weights(net, X, head="softmax")
    dW, db, _ = oracle.per_example_grads(net, X, labels)
    a, _ = np_forward(net, X, NP_ACT[act])
    P = scipy.special.softmax(a[-1], axis=1)
    for l in range(net.L):
        assert JW[l].shape == (B, 4) + net.Ws[l].shape
        # softmax outputs sum to one, so their gradients sum to zero over k
        assert np.abs(JW[l].sum(axis=1)).max() < 1e-14
        assert np.abs(Jb[l].sum(axis=1)).max() < 1e-14
        # cross-entropy gradient from the softmax Jacobian: d(-log p_c) = -d p_c / p_c
        for b in range(B):
            c = labels[b]
            np.testing.assert_allclose(dW[l][b], -JW[l][b, c] / P[b, c], rtol=1e-11, atol=1e-15)
            np.testing.assert_allclose(db[l][b], -Jb[l][b, c] / P[b, c], rtol=1e-11, atol=1e-15)
        # each slice is the outer product of the layer input and its bias row
        np.testing.assert_allclose(JW[l], a[l][:, None, :, None] * Jb[l][:, :, None, :],
                                   rtol=1e-12, atol=1e-16)
    # logits head with identity seeds, contracted with (p - onehot), is the CE gradient again
    JWl, Jbl = oracle.jacobian_weights(net, X, head="logits")
    D = P.copy()
    D[np.arange(B), labels] -= 1.0
    for l in range(net.L):
        np.testing.assert_allclose(np.einsum("bk,bkij->bij", D, JWl[l]), dW[l], rtol=1e-11,
                                   atol=1e-15)
        np.testing.assert_allclose(np.einsum("bk,bkj->bj", D, Jbl[l]), db[l], rtol=1e-11,
                                   atol=1e-15)


@pytest.mark.parametrize("head", ["logits", "softmax"])
def test_weight_jacobian_by_finite_differences(oracle, head):
    rng = np.random.default_rng(18)
    net = rand_net(oracle, rng, (3, 4, 3), "tanh")
    x = rng.standard_normal(3)
    JW, Jb = oracle.jacobian_weights(net, x[None, :], head=head)
    h = 1e-6

    def out():
        y = oracle.forward(net, x)
        return scipy.special.softmax(y) if head == "softmax" else y

    for l in range(net.L):
        for arr, Jarr in ((net.Ws[l], JW[l][0]), (net.bs[l], Jb[l][0])):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arr[idx]
                arr[idx] = old + h
                fp = out()
                arr[idx] = old - h
                fm = out()
                arr[idx] = old
                fd = (fp - fm) / (2 * h)
                got = np.array([Jarr[(k,) + idx] for k in range(3)])
                assert np.abs(got - fd).max() <= 1e-6 * max(np.abs(Jarr).max(), 1e-3)


def test_weight_jacobian_against_autograd_library_and_seed_forms(oracle):
    rng = np.random.default_rng(19)
    net = rand_net(oracle, rng, (4, 5, 3), "gelu")
    B = 2
    X = rng.standard_normal((B, 4))
    JW, Jb = oracle.jacobian_weights(net, X, head="softmax")
    tW = [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Ws]
    tb = [torch.from_numpy(b).clone().requires_grad_(True) for b in net.bs]
    for b in range(B):
        a = torch.from_numpy(X[b])
        z = torch.nn.functional.gelu(a @ tW[0] + tb[0]) @ tW[1] + tb[1]
        p = torch.softmax(z, dim=0)
        for k in range(3):
            grads = torch.autograd.grad(p[k], tW + tb, retain_graph=True)
            for l in range(2):
                np.testing.assert_allclose(JW[l][b, k], grads[l].numpy(), rtol=1e-10, atol=1e-15)
                np.testing.assert_allclose(Jb[l][b, k], grads[2 + l].numpy(), rtol=1e-10,
                                           atol=1e-15)
    # explicit seeds: shared == tiled, identity == None, general = linear combination
    seeds = rng.standard_normal((5, 3))
    for head in ("logits", "softmax"):
        JW_id, _ = oracle.jacobian_weights(net, X, head=head)
        JW_eye, _ = oracle.jacobian_weights(net, X, head=head, seeds=np.eye(3))
        JW_sh, Jb_sh = oracle.jacobian_weights(net, X, head=head, seeds=seeds)
        JW_ti, Jb_ti = oracle.jacobian_weights(net, X, head=head,
                                               seeds=np.tile(seeds[None], (B, 1, 1)))
        for l in range(2):
            np.testing.assert_allclose(JW_id[l], JW_eye[l], rtol=1e-13, atol=1e-17)
            np.testing.assert_array_equal(JW_sh[l], JW_ti[l])
            np.testing.assert_array_equal(Jb_sh[l], Jb_ti[l])
            np.testing.assert_allclose(JW_sh[l], np.einsum("sk,bkij->bsij", seeds, JW_id[l]),
                                       rtol=1e-11, atol=1e-15)


def test_skipped_outputs_do_not_change_the_rest(oracle):
    rng = np.random.default_rng(20)
    net = rand_net(oracle, rng, (4, 5, 3), "tanh")
    X = rng.standard_normal((3, 4))
    labels = rng.integers(0, 3, 3)
    dW, db, _ = oracle.per_example_grads(net, X, labels)
    dW2, db2, _ = oracle.per_example_grads(net, X, labels, want_dW=[False, True])
    assert dW2[0] is None
    np.testing.assert_array_equal(dW2[1], dW[1])
    np.testing.assert_array_equal(db2[0], db[0])
    JW, Jb = oracle.jacobian_weights(net, X, head="softmax", want_JW=[True, False])
    JWf, _ = oracle.jacobian_weights(net, X, head="softmax")
    assert JW[1] is None
    np.testing.assert_array_equal(JW[0], JWf[0])


# --------------------------------------------------------------------------------------------
# Per-example gradient norms.
# --------------------------------------------------------------------------------------------
def test_grad_norm_hand_fixture(oracle):
    g = json.load(open(os.path.join(GOLD, "relu_2_2_2.json")))
    p1 = 1.0 / (1.0 + math.exp(3.0))
    net = oracle.Net([np.array(g["W1"], float), np.array(g["W2"], float)],
                     [np.array(g["b1"], float), np.array(g["b2"], float)], g["act"])
    sq, norm = oracle.per_example_grad_norms(net, np.array([g["x"]], float), [g["label"]])
    np.testing.assert_allclose(sq[0], p1 * p1 * np.array(g["sq_layers_in_units_of_p1_squared"]),
                               rtol=1e-13)
    assert norm[0] == pytest.approx(p1 * math.sqrt(g["norm_squared_in_units_of_p1_squared"]),
                                    rel=1e-13)


@pytest.mark.parametrize("bias", [True, False])
def test_grad_norm_single_linear_layer_closed_form(oracle, bias):
    # ell = -log softmax(x W + b)[y]: d/dW = outer(x, p - e_y), d/db = p - e_y, so the squared
    # norm is (|x|^2 + 1) |p - e_y|^2 with a bias and |x|^2 |p - e_y|^2 without
    rng = np.random.default_rng(41)
    net = rand_net(oracle, rng, (7, 5), "relu", bias=bias)
    X = rng.standard_normal((6, 7))
    labels = rng.integers(0, 5, size=6)
    sq, norm = oracle.per_example_grad_norms(net, X, labels)
    z = X @ net.Ws[0] + (net.bs[0] if bias else 0.0)
    p = scipy.special.softmax(z, axis=1)
    p[np.arange(6), labels] -= 1.0
    want = ((X * X).sum(1) + (1.0 if bias else 0.0)) * (p * p).sum(1)
    np.testing.assert_allclose(sq[:, 0], want, rtol=1e-12)
    np.testing.assert_allclose(norm, np.sqrt(want), rtol=1e-12)


@pytest.mark.parametrize("act", ACTS)
def test_grad_norm_against_autograd_library(oracle, act):
    rng = np.random.default_rng(42)
    net = rand_net(oracle, rng, (6, 9, 7, 4), act)
    net_nb = oracle.Net(net.Ws, [net.bs[0], None, net.bs[2]], act)   # middle layer without a bias
    X = rng.standard_normal((5, 6))
    labels = rng.integers(0, 4, size=5)
    for n in (net, net_nb):
        sq, norm = oracle.per_example_grad_norms(n, X, labels)
        for b in range(5):
            Ws = [torch.from_numpy(W).clone().requires_grad_(True) for W in n.Ws]
            bs = [None if v is None else torch.from_numpy(v).clone().requires_grad_(True)
                  for v in n.bs]
            a = torch.from_numpy(X[b])
            for l in range(n.L):
                z = a @ Ws[l]
                if bs[l] is not None:
                    z = z + bs[l]
                a = z if l == n.L - 1 else {"identity": lambda t: t, "relu": torch.relu,
                                            "tanh": torch.tanh,
                                            "gelu": torch.nn.functional.gelu}[act](z)
            ell = -torch.log_softmax(a, dim=0)[int(labels[b])]
            params = Ws + [v for v in bs if v is not None]
            grads = torch.autograd.grad(ell, params)
            per_layer = []
            k = n.L
            for l in range(n.L):
                s = float((grads[l] ** 2).sum())
                if bs[l] is not None:
                    s += float((grads[k] ** 2).sum())
                    k += 1
                per_layer.append(s)
            np.testing.assert_allclose(sq[b], per_layer, rtol=1e-11)
            assert norm[b] == pytest.approx(math.sqrt(sum(per_layer)), rel=1e-11)


def test_grad_norm_is_rank_one_product_and_permutes_with_the_batch(oracle):
    # the gradient of a layer is the outer product of its input and its cotangent, whose squared
    # Frobenius norm factorises; the cotangent is the bias gradient the (pinned) gradient call gives
    rng = np.random.default_rng(43)
    net = rand_net(oracle, rng, (5, 8, 6, 3), "tanh")
    X = rng.standard_normal((7, 5))
    labels = rng.integers(0, 3, size=7)
    sq, norm = oracle.per_example_grad_norms(net, X, labels)
    _, db, _ = oracle.per_example_grads(net, X, labels)
    a, _ = np_forward(net, X, NP_ACT["tanh"])
    for l in range(net.L):
        want = ((a[l] * a[l]).sum(1) + 1.0) * (db[l] * db[l]).sum(1)
        np.testing.assert_allclose(sq[:, l], want, rtol=1e-12)
    perm = rng.permutation(7)
    sq_p, norm_p = oracle.per_example_grad_norms(net, X[perm], labels[perm])
    np.testing.assert_array_equal(sq_p, sq[perm])
    np.testing.assert_array_equal(norm_p, norm[perm])


# --------------------------------------------------------------------------------------------
# Hessians (Jacobian of the Jacobian, Section 5.1).
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("act", ACTS)
def test_activation_second_derivative_by_finite_differences(oracle, act):
    for z in (-2.3, -0.7, -0.1, 0.4, 1.1, 2.9):
        h = 1e-5
        fd = (oracle.act_deriv(act, z + h) - oracle.act_deriv(act, z - h)) / (2 * h)
        assert oracle.act_deriv2(act, z) == pytest.approx(fd, abs=1e-8)
    assert oracle.act_deriv2("relu", 0.0) == 0.0
    assert oracle.act_deriv2("tanh", 0.0) == 0.0
    assert oracle.act_deriv2("gelu", 0.0) == pytest.approx(2.0 / math.sqrt(2.0 * math.pi), rel=1e-14)


def test_hessian_hand_fixture(oracle):
    g = json.load(open(os.path.join(GOLD, "hessian_tanh_2_1_2.json")))
    t = math.tanh(0.5)
    c = -2.0 * t * (1.0 - t * t)
    net = oracle.Net([np.array(g["W1"], float), np.array(g["W2"], float)],
                     [np.array(g["b1"], float), np.array(g["b2"], float)], g["act"])
    H = oracle.hessian_input(net, np.array([g["x"]], float))
    assert H.shape == (1, 2, 2, 2)
    np.testing.assert_allclose(H[0], c * np.array(g["H_in_units_of_c"], float), rtol=1e-13)


@pytest.mark.parametrize("act", ["tanh", "gelu"])
def test_hessian_one_hidden_layer_closed_form(oracle, act):
    # y_o = sum_k W2[k, o] phi(z_k) + b2[o], z = x W1 + b1:
    # H_o = W1 diag(W2[:, o] phi''(z)) W1^T, with phi'' from library routines
    rng = np.random.default_rng(51)
    net = rand_net(oracle, rng, (4, 6, 3), act)
    X = rng.standard_normal((3, 4))
    H = oracle.hessian_input(net, X)
    z = X @ net.Ws[0] + net.bs[0]
    if act == "tanh":
        d2 = -2.0 * np.tanh(z) / np.cosh(z) ** 2
    else:
        d2 = scipy.stats.norm.pdf(z) * (2.0 - z * z)
    want = np.einsum("ik,bk,ko,jk->boij", net.Ws[0], d2, net.Ws[1], net.Ws[0])
    np.testing.assert_allclose(H, want, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("act", ["identity", "relu"])
def test_hessian_of_piecewise_linear_net_is_zero(oracle, act):
    rng = np.random.default_rng(52)
    net = rand_net(oracle, rng, (4, 5, 5, 3), act)
    H = oracle.hessian_input(net, rng.standard_normal((3, 4)))
    assert np.all(H == 0.0)


@pytest.mark.parametrize("act", ["tanh", "gelu"])
def test_hessian_by_finite_differences_of_the_jacobian(oracle, act):
    # the inner Jacobian is pinned on its own; difference it along every input direction
    rng = np.random.default_rng(53)
    net = rand_net(oracle, rng, (5, 7, 6, 4), act)
    X = rng.standard_normal((2, 5))
    seeds = rng.standard_normal((2, 3, 4))
    H = oracle.hessian_input(net, X, seeds=seeds)
    h = 1e-5
    for j in range(5):
        Xp, Xm = X.copy(), X.copy()
        Xp[:, j] += h
        Xm[:, j] -= h
        fd = (oracle.jacobian_input(net, Xp, seeds=seeds) -
              oracle.jacobian_input(net, Xm, seeds=seeds)) / (2 * h)
        np.testing.assert_allclose(H[:, :, :, j], fd, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("act", ["tanh", "gelu"])
def test_hessian_against_autograd_library(oracle, act):
    rng = np.random.default_rng(54)
    net = rand_net(oracle, rng, (4, 6, 5, 3), act)
    X = rng.standard_normal((2, 4))
    H = oracle.hessian_input(net, X)
    for b in range(2):
        for o in range(3):
            f = lambda x: torch_net_forward(net, x, act)[o]
            want = torch.autograd.functional.hessian(f, torch.from_numpy(X[b])).numpy()
            np.testing.assert_allclose(H[b, o], want, rtol=1e-10, atol=1e-13)


def test_hessian_symmetry_seed_linearity_and_seed_forms(oracle):
    rng = np.random.default_rng(55)
    net = rand_net(oracle, rng, (4, 5, 3), "tanh")
    X = rng.standard_normal((3, 4))
    H = oracle.hessian_input(net, X)                      # identity seeds: one per output
    np.testing.assert_allclose(H, H.transpose(0, 1, 3, 2), rtol=1e-12, atol=1e-15)
    shared = rng.standard_normal((2, 3))
    Hs = oracle.hessian_input(net, X, seeds=shared)
    np.testing.assert_allclose(Hs, np.einsum("so,boij->bsij", shared, H), rtol=1e-12, atol=1e-15)
    tiled = np.broadcast_to(shared, (3, 2, 3)).copy()
    np.testing.assert_array_equal(oracle.hessian_input(net, X, seeds=tiled), Hs)
    per = rng.standard_normal((3, 2, 3))
    Hp = oracle.hessian_input(net, X, seeds=per)
    np.testing.assert_allclose(Hp, np.einsum("bso,boij->bsij", per, H), rtol=1e-12, atol=1e-15)
    # one iteration of the parfor is one column of one example's Hessian
    col = oracle.body_hessian_input_dir(net, X[1], per[1, 0], 2)
    np.testing.assert_array_equal(col, Hp[1, 0, :, 2])
