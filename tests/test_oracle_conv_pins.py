"""Pins for the float64 convolutional-network oracle (oracle/conv_oracle.c), against things other
than itself: a hand-worked fixture, torch's conv2d / max_pool2d in float64, autograd through them,
central finite differences, closed forms and invariants.

CPU only.  Nothing here touches the HIP library.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import torch
import torch.nn.functional as F

from oracle import conv

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_net(rng, h, w, c, blocks, dense, bias=True):
    """blocks: [(k, filters), ...]; dense: widths after the flattened features."""
    Wc, bc = [], []
    cin, hh, ww = c, h, w
    for k, f in blocks:
        Wc.append(rng.standard_normal((k, k, cin, f)) / math.sqrt(k * k * cin))
        bc.append(rng.standard_normal(f) * 0.2 if bias else None)
        cin, hh, ww = f, hh // 2, ww // 2
    dims = [hh * ww * cin] + list(dense)
    Ws = [rng.standard_normal((dims[l], dims[l + 1])) / math.sqrt(dims[l]) for l in range(len(dense))]
    bs = [rng.standard_normal(dims[l + 1]) * 0.2 if bias else None for l in range(len(dense))]
    return conv.ConvNet(h, w, c, Wc, bc, Ws, bs)


def torch_forward(net, x, params=None):
    """x: [H, W, C] float64 tensor.  Library convolution and pooling (NCHW inside)."""
    Wc = [torch.from_numpy(W) for W in net.Wc] if params is None else params["Wc"]
    bc = [None if v is None else torch.from_numpy(v) for v in net.bc] if params is None else params["bc"]
    Ws = [torch.from_numpy(W) for W in net.Ws] if params is None else params["Ws"]
    bs = [None if v is None else torch.from_numpy(v) for v in net.bs] if params is None else params["bs"]
    a = x.permute(2, 0, 1).unsqueeze(0)                      # [1, C, H, W]
    for i in range(net.nc):
        k = net.kernel[i]
        a = F.conv2d(a, Wc[i].permute(3, 2, 0, 1), bc[i], padding=(k - 1) // 2)
        a = F.max_pool2d(torch.relu(a), 2)
    feat = a[0].permute(1, 2, 0).reshape(-1)                 # (y, x, c) order
    h = feat
    for l in range(net.L):
        h = h @ Ws[l]
        if bs[l] is not None:
            h = h + bs[l]
        if l < net.L - 1:
            h = torch.relu(h)
    return h, feat


def test_hand_fixture_forward_and_filter_gradient():
    g = json.load(open(os.path.join(GOLD, "conv_4x4_k3.json")))
    Wc = np.array(g["filter"], float).reshape(3, 3, 1, 1)
    net = conv.ConvNet(4, 4, 1, [Wc], [np.array([g["bias"]], float)], [np.array(g["dense"], float)], None)
    x = np.array(g["image"], float).reshape(4, 4, 1)
    np.testing.assert_array_equal(conv.features(net, x), g["features"])
    np.testing.assert_array_equal(conv.forward(net, x), g["logits"])
    q = 1.0 / (1.0 + math.exp(-3.0))
    dWc, dbc, dW, db, loss = conv.per_example_grads(net, x[None], [0])
    np.testing.assert_allclose(dWc[0][0, :, :, 0, 0], q * np.array(g["filter_gradient_in_units_of_q"]),
                               rtol=1e-13)
    assert abs(dbc[0][0, 0]) < 1e-15
    np.testing.assert_allclose(db[0][0], [-q, q], rtol=1e-13)
    np.testing.assert_allclose(dW[0][0], np.outer(g["features"], [-q, q]), rtol=1e-13)
    assert loss[0] == pytest.approx(math.log(1.0 + math.exp(3.0)), rel=1e-13)


@pytest.mark.parametrize("bias", [True, False])
def test_forward_matches_library_convolution_and_pooling(bias):
    rng = np.random.default_rng(81)
    net = rand_net(rng, 8, 12, 2, [(3, 4), (5, 3)], [7, 4], bias=bias)
    for _ in range(3):
        x = rng.standard_normal((8, 12, 2))
        with torch.no_grad():
            y, feat = torch_forward(net, torch.from_numpy(x))
        np.testing.assert_allclose(conv.features(net, x), feat.numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(conv.forward(net, x), y.numpy(), rtol=1e-12, atol=1e-14)
        p = scipy.special.softmax(y.numpy())
        assert conv.loss(net, x, 2) == pytest.approx(-math.log(p[2]), rel=1e-12)


def test_per_example_grads_against_autograd_through_the_library_ops():
    rng = np.random.default_rng(82)
    net = rand_net(rng, 8, 8, 2, [(3, 3), (3, 5)], [6, 4])
    B = 3
    X = rng.standard_normal((B, 8, 8, 2))
    labels = rng.integers(0, 4, size=B)
    dWc, dbc, dW, db, loss = conv.per_example_grads(net, X, labels)
    for b in range(B):
        params = {
            "Wc": [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Wc],
            "bc": [torch.from_numpy(v).clone().requires_grad_(True) for v in net.bc],
            "Ws": [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Ws],
            "bs": [torch.from_numpy(v).clone().requires_grad_(True) for v in net.bs],
        }
        y, _ = torch_forward(net, torch.from_numpy(X[b]), params)
        ell = -torch.log_softmax(y, dim=0)[int(labels[b])]
        flat = params["Wc"] + params["bc"] + params["Ws"] + params["bs"]
        grads = torch.autograd.grad(ell, flat)
        got = [t[b] for t in dWc] + [t[b] for t in dbc] + [t[b] for t in dW] + [t[b] for t in db]
        for g_got, g_want in zip(got, grads):
            np.testing.assert_allclose(g_got, g_want.numpy(), rtol=1e-10, atol=1e-13)
        assert loss[b] == pytest.approx(float(ell.detach()), rel=1e-12)


def test_per_example_grads_by_central_finite_differences():
    rng = np.random.default_rng(83)
    net = rand_net(rng, 8, 8, 1, [(3, 2), (3, 3)], [4, 3])
    x = rng.standard_normal((8, 8, 1))
    label = int(np.argmin(conv.forward(net, x)))
    dWc, dbc, dW, db, _ = conv.per_example_grads(net, x[None], [label])
    h = 1e-6

    def fd(arr, idx):
        keep = arr[idx]
        arr[idx] = keep + h
        up = conv.loss(conv.ConvNet(8, 8, 1, net.Wc, net.bc, net.Ws, net.bs), x, label)
        arr[idx] = keep - h
        dn = conv.loss(conv.ConvNet(8, 8, 1, net.Wc, net.bc, net.Ws, net.bs), x, label)
        arr[idx] = keep
        return (up - dn) / (2 * h)

    for idx in [(0, 0, 0, 0), (1, 1, 0, 1), (2, 0, 0, 1), (0, 2, 0, 0)]:
        assert dWc[0][0][idx] == pytest.approx(fd(net.Wc[0], idx), rel=1e-5, abs=1e-9)
    for idx in [(0, 0, 0, 0), (1, 2, 1, 2), (2, 1, 0, 1)]:
        assert dWc[1][0][idx] == pytest.approx(fd(net.Wc[1], idx), rel=1e-5, abs=1e-9)
    assert dbc[0][0][1] == pytest.approx(fd(net.bc[0], 1), rel=1e-5, abs=1e-9)
    assert dbc[1][0][2] == pytest.approx(fd(net.bc[1], 2), rel=1e-5, abs=1e-9)
    assert dW[0][0][2, 1] == pytest.approx(fd(net.Ws[0], (2, 1)), rel=1e-5, abs=1e-9)
    assert db[1][0][0] == pytest.approx(fd(net.bs[1], 0), rel=1e-5, abs=1e-9)


def test_dense_part_closed_forms_and_driver_properties():
    rng = np.random.default_rng(84)
    net = rand_net(rng, 4, 4, 2, [(3, 3)], [5, 3])
    X = rng.standard_normal((5, 4, 4, 2))
    labels = rng.integers(0, 3, size=5)
    dWc, dbc, dW, db, loss = conv.per_example_grads(net, X, labels)
    for b in range(5):
        feat = conv.features(net, X[b])
        p = scipy.special.softmax(conv.forward(net, X[b]))
        assert loss[b] == pytest.approx(-math.log(p[labels[b]]), rel=1e-12)
        p[labels[b]] -= 1.0
        np.testing.assert_allclose(db[1][b], p, rtol=1e-12, atol=1e-15)
        # rank-one structure of the first dense layer's gradient in terms of the conv features
        np.testing.assert_allclose(dW[0][b], np.outer(feat, db[0][b]), rtol=1e-12, atol=1e-15)
    # one example at a time gives the same slices; a permuted batch gives permuted results
    for b in range(5):
        one = conv.per_example_grads(net, X[b:b + 1], labels[b:b + 1])
        np.testing.assert_array_equal(one[0][0][0], dWc[0][b])
        np.testing.assert_array_equal(one[2][1][0], dW[1][b])
    perm = rng.permutation(5)
    outs = conv.per_example_grads(net, X[perm], labels[perm])
    np.testing.assert_array_equal(outs[0][0], dWc[0][perm])
    np.testing.assert_array_equal(outs[1][0], dbc[0][perm])
    np.testing.assert_array_equal(outs[4], loss[perm])


def test_a_centre_tap_filter_is_the_identity_and_a_dead_block_has_no_gradient():
    rng = np.random.default_rng(85)
    Wc = np.zeros((3, 3, 1, 1))
    Wc[1, 1, 0, 0] = 1.0
    dense = rng.standard_normal((4, 3))
    net = conv.ConvNet(4, 4, 1, [Wc], None, [dense], None)
    x = rng.uniform(0.1, 1.0, size=(4, 4, 1))             # positive: relu is the identity
    want = x[:, :, 0].reshape(2, 2, 2, 2).max(axis=(1, 3)).reshape(-1)
    np.testing.assert_allclose(conv.features(net, x), want, rtol=1e-15)
    # a bias that switches every unit off: no gradient reaches the conv parameters
    dead = conv.ConvNet(4, 4, 1, [Wc], [np.array([-5.0])], [dense], None)
    dWc, dbc, _, _, _ = conv.per_example_grads(dead, x[None], [1])
    assert not dWc[0].any() and not dbc[0].any()


def autograd_block_sqnorms(net, x, label):
    """Squared gradient norm of every parameter block (conv blocks first) from autograd through
    the library convolution and pooling; a block without a bias counts its weights only."""
    params = {
        "Wc": [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Wc],
        "bc": [None if v is None else torch.from_numpy(v).clone().requires_grad_(True) for v in net.bc],
        "Ws": [torch.from_numpy(W).clone().requires_grad_(True) for W in net.Ws],
        "bs": [None if v is None else torch.from_numpy(v).clone().requires_grad_(True) for v in net.bs],
    }
    y, _ = torch_forward(net, torch.from_numpy(x), params)
    ell = -torch.log_softmax(y, dim=0)[int(label)]
    ell.backward()
    out = []
    for W, v in list(zip(params["Wc"], params["bc"])) + list(zip(params["Ws"], params["bs"])):
        s = float((W.grad ** 2).sum())
        if v is not None:
            s += float((v.grad ** 2).sum())
        out.append(s)
    return out, float(ell.detach())


@pytest.mark.parametrize("bias", ["all", "none", "mixed"])
def test_grad_norms_against_autograd_through_the_library_ops(bias):
    rng = np.random.default_rng(86)
    net = rand_net(rng, 8, 8, 2, [(3, 3), (3, 5)], [6, 4], bias=(bias != "none"))
    if bias == "mixed":      # first conv block and last dense layer lose their bias
        net = conv.ConvNet(8, 8, 2, net.Wc, [None, net.bc[1]], net.Ws, [net.bs[0], None])
    B = 4
    X = rng.standard_normal((B, 8, 8, 2))
    labels = rng.integers(0, 4, size=B)
    sq, norm, loss = conv.per_example_grad_norms(net, X, labels)
    assert sq.shape == (B, 4)
    for b in range(B):
        want, ell = autograd_block_sqnorms(net, X[b], labels[b])
        np.testing.assert_allclose(sq[b], want, rtol=1e-10)
        assert norm[b] == pytest.approx(math.sqrt(sum(want)), rel=1e-10)
        assert loss[b] == pytest.approx(ell, rel=1e-12)
    # every column differs from the others: a misplaced column cannot pass by symmetry
    assert len(set(np.round(sq[0] / sq[0].max(), 6))) == 4


def test_grad_norms_dense_factorisation_and_stacking():
    rng = np.random.default_rng(87)
    net = rand_net(rng, 4, 4, 2, [(3, 3)], [5, 3])
    B = 6
    X = rng.standard_normal((B, 4, 4, 2))
    labels = rng.integers(0, 3, size=B)
    sq, norm, loss = conv.per_example_grad_norms(net, X, labels)
    for b in range(B):
        feat = conv.features(net, X[b])
        p = scipy.special.softmax(conv.forward(net, X[b]))
        p[labels[b]] -= 1.0                                   # cotangent of the logits
        # last dense layer: (|a|^2 + 1) |delta|^2 with a = relu of the first dense layer
        a1 = np.maximum(feat @ net.Ws[0] + net.bs[0], 0.0)
        assert sq[b, 2] == pytest.approx((a1 @ a1 + 1.0) * (p @ p), rel=1e-12)
        d1 = (net.Ws[1] @ p) * (a1 > 0)
        assert sq[b, 1] == pytest.approx((feat @ feat + 1.0) * (d1 @ d1), rel=1e-12)
    np.testing.assert_allclose(norm, np.sqrt(sq.sum(axis=1)), rtol=1e-14)
    perm = rng.permutation(B)
    sq2, norm2, loss2 = conv.per_example_grad_norms(net, X[perm], labels[perm])
    np.testing.assert_array_equal(sq2, sq[perm])
    np.testing.assert_array_equal(norm2, norm[perm])
    np.testing.assert_array_equal(loss2, loss[perm])
    assert len(set(norm.tolist())) == B
