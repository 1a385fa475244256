"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/pfg.h declares, sizes workspaces as documented and rejects bad arguments before anything
is enqueued (no kernel is launched by any test in this file)."""
import ctypes
import os
import re

import pytest

import paper_1903_04243_amd as pfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pfg.LIB_PATH):
        from paper_1903_04243_amd import build
        build.build()
    return pfg.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pfg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pfg_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(pfg.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.pfg_version() == 104


FAKE = 0x1000  # a non-NULL, 256-aligned value; never dereferenced because validation fails first


def make_net(dims, act=1, dtype=0, W_null_at=None, with_W=True):
    L = len(dims) - 1
    d = (ctypes.c_int32 * (L + 1))(*dims)
    W = (ctypes.c_void_p * L)(*[None if W_null_at == l else FAKE for l in range(L)])
    net = pfg.pfg_mlp(L, d, W if with_W else None, None, act, dtype)
    net._keep = (d, W)
    return net


def ws_bytes(lib, net, op, B, S):
    n = ctypes.c_size_t(0)
    rc = lib.pfg_workspace_bytes(ctypes.byref(net), op, B, S, ctypes.byref(n))
    return rc, n.value


def up(x):
    return (x + 255) // 256 * 256


def test_workspace_sizes(lib):
    net = make_net([784, 512, 512, 10])
    B = 128
    rc, n = ws_bytes(lib, net, 0, B, 1)
    assert rc == 0
    expect = 4 * up(4 * B * 512) + up(4 * B * 10) + 2 * up(4 * B * 512) + up(4 * B * 10)
    assert n == expect
    # per-example gradients ignore S
    assert ws_bytes(lib, net, 0, B, 77) == (0, expect)
    # few rows, a wide layer and a long contraction: room for the 8 partial results [8, B, 1024] of
    # the first forward product, which is cut along its contraction
    wide = make_net([3136, 1024, 10])
    assert ws_bytes(lib, wide, 0, B, 1) == (0, 2 * up(4 * B * 1024) + up(4 * B * 10) + up(4 * B * 1024) +
                                            up(4 * B * 10) + up(4 * 8 * B * 1024))
    # bf16, 256 rows against 4096-wide layers: 32 partial logits [32, B, 10] of the head, whose
    # contraction is cut, and the 2 partial results [2, B, 4096] of a forward product
    big = make_net([4096, 4096, 4096, 10], act=3, dtype=1)
    Bb = 256
    assert ws_bytes(lib, big, 0, Bb, 1) == (0, 4 * up(4 * Bb * 4096) + up(4 * Bb * 10) + 2 * up(4 * Bb * 4096) +
                                            up(4 * Bb * 10) + up(4 * 32 * Bb * 10) + up(4 * 2 * Bb * 4096))
    net3 = make_net([1024, 2048, 2048, 1024], act=2)
    rc, n = ws_bytes(lib, net3, 1, 64, 1024)
    assert rc == 0
    assert n == 4 * up(4 * 64 * 2048) + up(4 * 1024 * 2048) + 2 * up(4 * 64 * 1024 * 2048)
    net5 = make_net([256, 256, 16], act=2)
    rc, n = ws_bytes(lib, net5, 2, 64, 16)
    assert rc == 0
    assert n == 2 * up(4 * 64 * 256) + up(4 * 64 * 16) + up(4 * 1024 * 256) + up(4 * 1024 * 16)
    assert ws_bytes(lib, make_net([3, 2]), 1, 1, 2)[1] % 256 == 0


def test_workspace_bytes_rejects_bad_arguments(lib):
    net = make_net([4, 3, 2])
    n = ctypes.c_size_t(0)
    assert lib.pfg_workspace_bytes(None, 0, 1, 1, ctypes.byref(n)) == pfg.PFG_ERR_NULL
    assert lib.pfg_workspace_bytes(ctypes.byref(net), 0, 1, 1, None) == pfg.PFG_ERR_NULL
    assert ws_bytes(lib, net, 5, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert ws_bytes(lib, net, -1, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert ws_bytes(lib, net, 0, 0, 1)[0] == pfg.PFG_ERR_SHAPE
    assert ws_bytes(lib, net, 1, 1, 0)[0] == pfg.PFG_ERR_SHAPE
    assert ws_bytes(lib, net, 1, 1 << 20, 1 << 20)[0] == pfg.PFG_ERR_OVERFLOW
    assert ws_bytes(lib, make_net([4, 0, 2]), 0, 1, 1)[0] == pfg.PFG_ERR_SHAPE
    assert ws_bytes(lib, make_net([4, 3, 2], act=9), 0, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert ws_bytes(lib, make_net([4, 3, 2], dtype=5), 0, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    big = make_net([1 << 24, 1 << 24])
    assert ws_bytes(lib, big, 0, 1 << 20, 1)[0] == pfg.PFG_ERR_OVERFLOW
    bad = pfg.pfg_mlp(0, None, None, None, 0, 0)
    assert ws_bytes(lib, bad, 0, 1, 1)[0] == pfg.PFG_ERR_SHAPE
    nodims = pfg.pfg_mlp(2, None, None, None, 0, 0)
    assert ws_bytes(lib, nodims, 0, 1, 1)[0] == pfg.PFG_ERR_NULL
    assert "dims" in lib.pfg_last_error().decode()


def call_grads(lib, net, X=FAKE, labels=FAKE, B=4, ws=FAKE, ws_bytes_=1 << 30):
    L = net.num_layers
    outs = (ctypes.c_void_p * L)(*[FAKE] * L)
    return lib.pfg_per_example_grads(ctypes.byref(net), X, labels, B, outs, outs, None, ws,
                                     ws_bytes_, None)


def test_per_example_grads_rejects_before_launch(lib):
    net = make_net([4, 3, 2])
    assert call_grads(lib, net, X=None) == pfg.PFG_ERR_NULL
    assert call_grads(lib, net, labels=None) == pfg.PFG_ERR_NULL
    assert call_grads(lib, net, B=0) == pfg.PFG_ERR_SHAPE
    assert call_grads(lib, net, ws=None) == pfg.PFG_ERR_WORKSPACE
    assert call_grads(lib, net, ws=FAKE + 8) == pfg.PFG_ERR_WORKSPACE
    assert call_grads(lib, net, ws_bytes_=16) == pfg.PFG_ERR_WORKSPACE
    assert "needed" in lib.pfg_last_error().decode()
    assert call_grads(lib, make_net([4, 3, 2], W_null_at=1)) == pfg.PFG_ERR_NULL
    assert call_grads(lib, make_net([4, 3, 2], with_W=False)) == pfg.PFG_ERR_NULL
    assert call_grads(lib, make_net([4, 3, 2], act=-1)) == pfg.PFG_ERR_UNSUPPORTED
    assert lib.pfg_per_example_grads(None, FAKE, FAKE, 1, None, None, None, FAKE, 1 << 20,
                                     None) == pfg.PFG_ERR_NULL


def test_jacobians_reject_before_launch(lib):
    net = make_net([4, 3, 2], act=2)
    ji = lib.pfg_jacobian_input
    big = 1 << 30
    assert ji(ctypes.byref(net), None, 2, None, 2, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert ji(ctypes.byref(net), FAKE, 2, None, 2, 0, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    # identity seeds need S == d_L
    assert ji(ctypes.byref(net), FAKE, 2, None, 3, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert "identity" in lib.pfg_last_error().decode()
    # explicit seeds: stride must be 0 or >= S * d_L
    assert ji(ctypes.byref(net), FAKE, 2, FAKE, 3, 5, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert ji(ctypes.byref(net), FAKE, 2, FAKE, 0, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert ji(ctypes.byref(net), FAKE, 2, None, 2, 0, FAKE, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert ji(ctypes.byref(net), FAKE, 2, None, 2, 0, FAKE, FAKE, 8, None) == pfg.PFG_ERR_WORKSPACE
    jw = lib.pfg_jacobian_weights
    outs = (ctypes.c_void_p * 2)(FAKE, FAKE)
    assert jw(ctypes.byref(net), FAKE, 2, 7, None, 2, 0, outs, outs, FAKE, big,
              None) == pfg.PFG_ERR_UNSUPPORTED
    assert jw(ctypes.byref(net), None, 2, 1, None, 2, 0, outs, outs, FAKE, big,
              None) == pfg.PFG_ERR_NULL
    assert jw(ctypes.byref(net), FAKE, 2, 1, None, 5, 0, outs, outs, FAKE, big,
              None) == pfg.PFG_ERR_SHAPE
    assert jw(ctypes.byref(net), FAKE, 2, 1, None, 2, 0, outs, outs, FAKE, 0,
              None) == pfg.PFG_ERR_WORKSPACE


def test_grad_norms_workspace_and_rejections(lib):
    net = make_net([784, 512, 512, 10])
    B = 128
    grads = ws_bytes(lib, net, 0, B, 1)[1]
    # the gradient call's blocks plus [B, L] squared norms; S is ignored
    assert ws_bytes(lib, net, 3, B, 1) == (0, grads + up(4 * B * 3))
    assert ws_bytes(lib, net, 3, B, 55) == (0, grads + up(4 * B * 3))
    fn = lib.pfg_per_example_grad_norms
    big = 1 << 30
    small = make_net([4, 3, 2])
    r = ctypes.byref(small)
    assert fn(r, None, FAKE, 2, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, None, 2, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, FAKE, 2, None, None, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert "both NULL" in lib.pfg_last_error().decode()
    assert fn(r, FAKE, FAKE, 0, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(r, FAKE, FAKE, 2, FAKE, FAKE, None, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, FAKE, 2, FAKE, FAKE, None, FAKE, 16, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(None, FAKE, FAKE, 2, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL


def test_hessian_workspace_and_rejections(lib):
    net = make_net([256, 512, 512, 64], act=2)
    B, S, n, ktot = 32, 64, 256, 1024
    rc, nbytes = ws_bytes(lib, net, 4, B, S)
    assert rc == 0
    expect = (6 * up(4 * B * 512)                    # a_l, phi'(z_l), phi''(z_l) for two hidden layers
              + up(4 * B * n * ktot)                 # tangents
              + up(4 * B * S * ktot)                 # curvature weights
              + up(4 * S * 512)                      # loop-invariant seed block
              + 2 * up(4 * B * S * 512))             # two cotangent blocks
    assert nbytes == expect
    # a one-layer network has no hidden layer: nothing but the minimum
    assert ws_bytes(lib, make_net([7, 3], act=2), 4, 5, 3) == (0, 256)
    assert ws_bytes(lib, make_net([4, 3, 2], act=2, dtype=1), 4, 1, 2) == ws_bytes(lib, make_net([4, 3, 2], act=2), 4, 1, 2)
    assert ws_bytes(lib, make_net([1 << 16, 3, 2], act=2), 4, 1, 2)[0] == pfg.PFG_ERR_OVERFLOW
    fn = lib.pfg_hessian_input
    big = 1 << 30
    small = make_net([4, 3, 2], act=2)
    r = ctypes.byref(small)
    assert fn(r, None, 2, None, 2, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, 2, None, 2, 0, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, 2, None, 3, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE      # identity seeds
    assert fn(r, FAKE, 2, FAKE, 3, 5, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE      # stride < S * d_L
    assert fn(r, FAKE, 0, None, 2, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(r, FAKE, 2, None, 2, 0, FAKE, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, 2, None, 2, 0, FAKE, FAKE, 8, None) == pfg.PFG_ERR_WORKSPACE
    bf = make_net([4, 3, 2], act=2, dtype=1)                      # bfloat16 networks pass the same checks
    assert fn(ctypes.byref(bf), FAKE, 2, None, 3, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(ctypes.byref(bf), FAKE, 2, None, 2, 0, FAKE, FAKE, 8, None) == pfg.PFG_ERR_WORKSPACE


def make_lstm(dx=128, H=256, dy=10, T=10, dtype=0, W=FAKE, W_out=FAKE):
    return pfg.pfg_lstm(dx, H, dy, T, W, None, W_out, None, dtype)


def lstm_ws(lib, net, op, B, S):
    n = ctypes.c_size_t(0)
    rc = lib.pfg_lstm_workspace_bytes(ctypes.byref(net), op, B, S, ctypes.byref(n))
    return rc, n.value


def test_lstm_workspace_and_rejections(lib):
    net = make_lstm()
    B, T, H, dy = 256, 10, 256, 10
    fwd = 2 * up(4 * B * T * 4 * H) + up(4 * B * 4 * H) + 2 * up(4 * B * T * H)
    grads = fwd + 2 * up(4 * B * dy) + 2 * up(4 * B * H) + up(4 * B * T * 4 * H)
    assert lstm_ws(lib, net, 0, B, 1) == (0, grads)
    assert lstm_ws(lib, net, 0, B, 99) == (0, grads)          # S is ignored
    jac_net = make_lstm(dy=128)
    B, S = 64, 128
    fwd = 2 * up(4 * B * T * 4 * H) + up(4 * B * 4 * H) + 2 * up(4 * B * T * H)
    assert lstm_ws(lib, jac_net, 1, B, S) == (0, fwd + up(4 * S * H) + 2 * up(4 * B * S * H) +
                                              2 * up(4 * B * S * 4 * H))
    assert lstm_ws(lib, net, 2, 256, 1) == (0, grads)         # gradient norms: the same sweep, no outputs
    assert lstm_ws(lib, net, 3, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert lstm_ws(lib, net, 0, 0, 1)[0] == pfg.PFG_ERR_SHAPE
    assert lstm_ws(lib, net, 1, 1, 0)[0] == pfg.PFG_ERR_SHAPE
    assert lstm_ws(lib, net, 1, 1 << 20, 1 << 20)[0] == pfg.PFG_ERR_OVERFLOW
    assert lstm_ws(lib, make_lstm(H=0), 0, 1, 1)[0] == pfg.PFG_ERR_SHAPE
    assert lstm_ws(lib, make_lstm(T=0), 0, 1, 1)[0] == pfg.PFG_ERR_SHAPE
    assert lstm_ws(lib, make_lstm(dtype=1), 0, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert lstm_ws(lib, make_lstm(W=None), 0, 1, 1)[0] == pfg.PFG_ERR_NULL
    assert lstm_ws(lib, make_lstm(W_out=None), 0, 1, 1)[0] == pfg.PFG_ERR_NULL
    n = ctypes.c_size_t(0)
    assert lib.pfg_lstm_workspace_bytes(None, 0, 1, 1, ctypes.byref(n)) == pfg.PFG_ERR_NULL
    assert lib.pfg_lstm_workspace_bytes(ctypes.byref(net), 0, 1, 1, None) == pfg.PFG_ERR_NULL

    big = 1 << 40
    r = ctypes.byref(net)
    gr = lib.pfg_lstm_per_example_grads
    assert gr(r, None, FAKE, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert gr(r, FAKE, None, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert gr(r, FAKE, FAKE, 0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert gr(r, FAKE, FAKE, 2, FAKE, FAKE, FAKE, FAKE, FAKE, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert gr(r, FAKE, FAKE, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 4, big, None) == pfg.PFG_ERR_WORKSPACE
    assert gr(r, FAKE, FAKE, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE
    nr = lib.pfg_lstm_per_example_grad_norms
    assert nr(r, None, FAKE, 2, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert nr(r, FAKE, FAKE, 2, None, None, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert "both NULL" in lib.pfg_last_error().decode()
    assert nr(ctypes.byref(make_lstm(T=65)), FAKE, FAKE, 2, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_UNSUPPORTED
    assert nr(r, FAKE, FAKE, 2, FAKE, None, None, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE
    ja = lib.pfg_lstm_jacobian_input
    assert ja(r, None, 2, None, 10, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert ja(r, FAKE, 2, None, 10, 0, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert ja(r, FAKE, 2, None, 7, 0, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE       # identity seeds
    assert "identity" in lib.pfg_last_error().decode()
    assert ja(r, FAKE, 2, FAKE, 3, 5, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE       # stride < S * dy
    assert ja(r, FAKE, 2, None, 10, 0, FAKE, FAKE, 8, None) == pfg.PFG_ERR_WORKSPACE


def test_lstm_varlen_workspace_and_rejections(lib):
    net = make_lstm()
    B, tokens, H = 1024, 51957, 256
    n = ctypes.c_size_t(0)
    r = ctypes.byref(net)
    assert lib.pfg_lstm_varlen_workspace_bytes(r, B, tokens, ctypes.byref(n)) == 0
    assert n.value == up(4 * tokens * 4 * H) + up(4 * 3 * B * H) + up(4 * B * H) + up(4 * 3 * B)
    assert lib.pfg_lstm_varlen_workspace_bytes(r, 0, 5, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_lstm_varlen_workspace_bytes(r, 8, 7, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE   # a length < 1
    assert lib.pfg_lstm_varlen_workspace_bytes(r, 8, 1 << 40, ctypes.byref(n)) == pfg.PFG_ERR_OVERFLOW
    assert lib.pfg_lstm_varlen_workspace_bytes(r, 8, 9, None) == pfg.PFG_ERR_NULL
    fn = lib.pfg_lstm_varlen_forward
    big = 1 << 40
    lens = (ctypes.c_int32 * 3)(2, 1, 4)
    assert fn(r, None, lens, 3, 7, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, None, 3, 7, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, lens, 3, 7, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, lens, 3, 8, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE       # sum mismatch
    assert "add up" in lib.pfg_last_error().decode()
    zero = (ctypes.c_int32 * 3)(2, 0, 5)
    assert fn(r, FAKE, zero, 3, 7, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(r, FAKE, lens, 3, 7, FAKE, FAKE, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, lens, 3, 7, FAKE, FAKE, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE


def test_lstm_while_workspace_and_rejections(lib):
    net = make_lstm()
    B, tokens, H = 1024, 51957, 256
    n = ctypes.c_size_t(0)
    r = ctypes.byref(net)
    assert lib.pfg_lstm_while_workspace_bytes(r, B, tokens, ctypes.byref(n)) == 0
    groups = (B + 31) // 32 + (B + 1023) // 1024
    pieces = up(4 * B * ((H + 7) // 8))          # halting score in pieces: lists of at most 1024 rows only
    assert n.value == (up(4 * tokens * 4 * H) + up(4 * 3 * B * H) + pieces + up(4 * B * H) + up(4 * 2 * B) + up(16) +
                       up(4 * B) + up(4 * groups) + up(4 * B))
    assert lib.pfg_lstm_while_workspace_bytes(r, 2 * B, tokens, ctypes.byref(n)) == 0
    groups2 = (2 * B + 31) // 32 + (2 * B + 1023) // 1024
    assert n.value == (up(4 * tokens * 4 * H) + up(4 * 3 * 2 * B * H) + up(4 * 2 * B * H) + up(4 * 2 * 2 * B) + up(16) +
                       up(4 * 2 * B) + up(4 * groups2) + up(4 * 2 * B))
    assert lib.pfg_lstm_while_workspace_bytes(r, 4, 0, ctypes.byref(n)) == 0          # no tokens at all is allowed
    assert lib.pfg_lstm_while_workspace_bytes(r, 0, 5, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_lstm_while_workspace_bytes(r, 8, -1, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_lstm_while_workspace_bytes(r, 8, 1 << 40, ctypes.byref(n)) == pfg.PFG_ERR_OVERFLOW
    assert lib.pfg_lstm_while_workspace_bytes(r, 1 << 25, 9, ctypes.byref(n)) == pfg.PFG_ERR_OVERFLOW
    assert lib.pfg_lstm_while_workspace_bytes(r, 8, 9, None) == pfg.PFG_ERR_NULL
    fn = lib.pfg_lstm_while_forward
    fn.argtypes = [ctypes.POINTER(pfg.pfg_lstm), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                   ctypes.c_int32, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    big = 1 << 40
    assert fn(r, None, FAKE, 3, 7, 5, None, 0.0, FAKE, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, None, 3, 7, 5, None, 0.0, FAKE, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, FAKE, 3, 7, 5, None, 0.0, None, None, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, FAKE, 3, 7, -1, None, 0.0, FAKE, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert "max_steps" in lib.pfg_last_error().decode()
    assert fn(r, FAKE, FAKE, 3, 7, 5, None, 0.0, FAKE, FAKE, FAKE, None, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, FAKE, 3, 7, 5, None, 0.0, FAKE, FAKE, FAKE, None, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE


def test_lstm_while_grads_workspace_and_rejections(lib):
    net = make_lstm()
    B, tokens, H, dy, cap = 1024, 51957, 256, net.output_size, 100
    n = ctypes.c_size_t(0)
    r = ctypes.byref(net)
    wsfn = lib.pfg_lstm_while_grads_workspace_bytes
    wsfn.argtypes = [ctypes.POINTER(pfg.pfg_lstm), ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                     ctypes.POINTER(ctypes.c_size_t)]
    assert wsfn(r, B, tokens, cap, ctypes.byref(n)) == 0
    groups = (B + 31) // 32 + (B + 1023) // 1024
    forward = (up(4 * tokens * 4 * H) + up(4 * 3 * B * H) + up(4 * B * ((H + 7) // 8)) + up(4 * B * H) +
               up(4 * (cap + 1) * B) + up(8 * (cap + 1)) + up(4 * B) + up(4 * groups) + up(4 * B))
    history = up(4 * tokens * 4 * H) + 2 * up(4 * tokens * H) + up(4 * tokens * 4 * H)     # gates, c, h, dz by token
    sweep = up(4 * B * H) + up(4 * (B * H + 2 * B * 4 * H)) + 2 * up(4 * B * dy)
    assert n.value == forward + history + sweep
    assert wsfn(r, B, tokens, -1, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert wsfn(r, B, tokens, (1 << 16) + 1, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert wsfn(r, 65536, tokens, cap, ctypes.byref(n)) == pfg.PFG_ERR_UNSUPPORTED
    assert "65535" in lib.pfg_last_error().decode()
    assert wsfn(r, 0, tokens, cap, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert wsfn(r, B, tokens, cap, None) == pfg.PFG_ERR_NULL
    fn = lib.pfg_lstm_while_per_example_grads
    vp = ctypes.c_void_p
    fn.argtypes = [ctypes.POINTER(pfg.pfg_lstm), vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, vp,
                   ctypes.c_float, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    big = 1 << 40
    ok = (FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    assert fn(r, None, FAKE, FAKE, 3, 7, 5, None, 0.0, *ok, FAKE, big, None) == pfg.PFG_ERR_NULL      # X
    assert fn(r, FAKE, None, FAKE, 3, 7, 5, None, 0.0, *ok, FAKE, big, None) == pfg.PFG_ERR_NULL      # seq_offsets
    assert fn(r, FAKE, FAKE, None, 3, 7, 5, None, 0.0, *ok, FAKE, big, None) == pfg.PFG_ERR_NULL      # labels
    assert "labels" in lib.pfg_last_error().decode()
    none = (None, None, None, None, None, FAKE)                                                       # trip counts alone
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, *none, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, -1, None, 0.0, *ok, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, *ok, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, *ok, FAKE + 8, big, None) == pfg.PFG_ERR_WORKSPACE
    assert "aligned" in lib.pfg_last_error().decode()
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, *ok, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE


def test_lstm_while_grad_norms_rejections(lib):
    net = make_lstm()
    r = ctypes.byref(net)
    fn = lib.pfg_lstm_while_per_example_grad_norms
    vp = ctypes.c_void_p
    fn.argtypes = [ctypes.POINTER(pfg.pfg_lstm), vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, vp,
                   ctypes.c_float, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    big = 1 << 40
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, None, None, FAKE, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert "sq_out and norm_out" in lib.pfg_last_error().decode()
    assert fn(r, FAKE, FAKE, None, 3, 7, 5, None, 0.0, FAKE, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 129, None, 0.0, FAKE, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_UNSUPPORTED
    assert "128" in lib.pfg_last_error().decode()
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, -1, None, 0.0, FAKE, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_SHAPE
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, FAKE, None, None, None, FAKE, 64, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r, FAKE, FAKE, FAKE, 3, 7, 5, None, 0.0, None, FAKE, None, None, None, big, None) == pfg.PFG_ERR_WORKSPACE


def make_convnet(h=28, w=28, c=1, kernel=(5, 5), filters=(32, 64), dense=(3136, 1024, 10), Wc_null=None,
                 dtype=0):
    nc = len(kernel)
    k = (ctypes.c_int32 * nc)(*kernel)
    f = (ctypes.c_int32 * nc)(*filters)
    Wc = (ctypes.c_void_p * nc)(*[None if Wc_null == i else FAKE for i in range(nc)])
    dn = make_net(list(dense), act=1, dtype=dtype)
    net = pfg.pfg_convnet(h, w, c, nc, k, f, Wc, None, dn)
    net._keep = (k, f, Wc, dn)
    return net


def test_convnet_workspace_and_rejections(lib):
    net = make_convnet()
    B = 128
    n = ctypes.c_size_t(0)
    assert lib.pfg_convnet_workspace_bytes(ctypes.byref(net), B, ctypes.byref(n)) == 0
    dense = ws_bytes(lib, net.dense, 0, B, 1)[1]
    blk1 = (2 * up(4 * B * 784 * 25) + 2 * up(4 * B * 784 * 32) + up(4 * B * 196 * 32) + up(B * 196 * 32))
    blk2 = (2 * up(4 * B * 196 * 800) + 2 * up(4 * B * 196 * 64) + up(4 * B * 49 * 64) + up(B * 49 * 64))
    assert n.value == blk1 + blk2 + 2 * up(4 * B * 196 * 32) + up(4 * B * 8 * 64) + dense
    r = lambda net_: ctypes.byref(net_)
    assert lib.pfg_convnet_workspace_bytes(None, B, ctypes.byref(n)) == pfg.PFG_ERR_NULL
    assert lib.pfg_convnet_workspace_bytes(r(net), B, None) == pfg.PFG_ERR_NULL
    assert lib.pfg_convnet_workspace_bytes(r(net), 0, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_convnet_workspace_bytes(r(make_convnet(kernel=(4, 5))), B, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert "odd" in lib.pfg_last_error().decode()
    assert lib.pfg_convnet_workspace_bytes(r(make_convnet(h=30)), B, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE    # 30 -> 15, odd
    assert lib.pfg_convnet_workspace_bytes(r(make_convnet(dense=(3000, 10))), B, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert "features" in lib.pfg_last_error().decode()
    assert lib.pfg_convnet_workspace_bytes(r(make_convnet(dtype=1)), B, ctypes.byref(n)) == pfg.PFG_ERR_UNSUPPORTED
    fn = lib.pfg_convnet_per_example_grads
    big = 1 << 40
    o2 = (ctypes.c_void_p * 2)(FAKE, FAKE)
    assert fn(r(net), None, FAKE, 4, o2, o2, o2, o2, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, None, 4, o2, o2, o2, o2, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(make_convnet(Wc_null=1)), FAKE, FAKE, 4, o2, o2, o2, o2, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, FAKE, 4, o2, o2, o2, o2, None, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, FAKE, 4, o2, o2, o2, o2, None, FAKE, 1024, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, FAKE, 1 << 20, o2, o2, o2, o2, None, FAKE, big, None) == pfg.PFG_ERR_SHAPE


def test_convnet_grad_norms_workspace_and_rejections(lib):
    net = make_convnet()
    B = 128
    n, n0 = ctypes.c_size_t(0), ctypes.c_size_t(0)
    r = lambda net_: ctypes.byref(net_)
    assert lib.pfg_convnet_workspace_bytes(r(net), B, ctypes.byref(n0)) == 0
    assert lib.pfg_convnet_grad_norms_workspace_bytes(r(net), B, ctypes.byref(n)) == 0
    # the gradients' workspace plus every block's filter and bias gradients and the [B, 2 + 2] sums
    extra = up(4 * B * 25 * 32) + up(4 * B * 32) + up(4 * B * 800 * 64) + up(4 * B * 64) + up(4 * B * 4)
    assert n.value == n0.value + extra
    assert lib.pfg_convnet_grad_norms_workspace_bytes(None, B, ctypes.byref(n)) == pfg.PFG_ERR_NULL
    assert lib.pfg_convnet_grad_norms_workspace_bytes(r(net), B, None) == pfg.PFG_ERR_NULL
    assert lib.pfg_convnet_grad_norms_workspace_bytes(r(net), 0, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_convnet_grad_norms_workspace_bytes(r(make_convnet(kernel=(5, 6))), B, ctypes.byref(n)) == pfg.PFG_ERR_SHAPE
    fn = lib.pfg_convnet_per_example_grad_norms
    big = 1 << 40
    assert fn(r(net), None, FAKE, 4, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, None, 4, FAKE, FAKE, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, FAKE, 4, None, None, FAKE, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert "both NULL" in lib.pfg_last_error().decode()
    assert fn(r(make_convnet(Wc_null=0)), FAKE, FAKE, 4, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, FAKE, 4, FAKE, None, None, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, FAKE, 4, FAKE, None, None, FAKE, n0.value // 32, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, FAKE, 4, FAKE, None, None, FAKE + 8, big, None) == pfg.PFG_ERR_WORKSPACE
    assert "aligned" in lib.pfg_last_error().decode()


def make_cond(pre=(784, 512), then_dims=(1024, 10), else_dims=(10,), dtype=0, w=FAKE, W_null_at=None):
    parts = [make_net(pre, dtype=dtype), make_net((pre[-1],) + tuple(then_dims), W_null_at=W_null_at),
             make_net((pre[-1],) + tuple(else_dims))]
    net = pfg.pfg_cond(parts[0], w, 0.0, parts[1], parts[2])
    net._keep = parts
    return net


def test_cond_workspace_and_rejections(lib):
    net = make_cond()
    n = 1000
    b = ctypes.c_size_t(0)
    assert lib.pfg_cond_workspace_bytes(ctypes.byref(net), n, ctypes.byref(b)) == 0
    # shared-part output, two hidden buffers of the widest hidden layer, flags, group and block counts, index
    # sets, the two {count, offset} descriptors
    assert b.value == (up(4 * n * 512) + 2 * up(4 * n * 1024) + up(4 * n) + up(4 * ((n + 31) // 32 + (n + 1023) // 1024)) +
                       up(4 * n) + up(16))
    r = lambda net_: ctypes.byref(net_)
    assert lib.pfg_cond_workspace_bytes(None, n, ctypes.byref(b)) == pfg.PFG_ERR_NULL
    assert lib.pfg_cond_workspace_bytes(r(net), n, None) == pfg.PFG_ERR_NULL
    assert lib.pfg_cond_workspace_bytes(r(net), 0, ctypes.byref(b)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_cond_workspace_bytes(r(net), (1 << 24) + 1, ctypes.byref(b)) == pfg.PFG_ERR_OVERFLOW
    assert lib.pfg_cond_workspace_bytes(r(make_cond(dtype=1)), n, ctypes.byref(b)) == pfg.PFG_ERR_UNSUPPORTED
    assert lib.pfg_cond_workspace_bytes(r(make_cond(else_dims=(11,))), n, ctypes.byref(b)) == pfg.PFG_ERR_SHAPE
    assert "same output width" in lib.pfg_last_error().decode()
    bad = make_cond()
    bad.then_net = make_net((500, 10))
    assert lib.pfg_cond_workspace_bytes(r(bad), n, ctypes.byref(b)) == pfg.PFG_ERR_SHAPE
    assert "outputs of pre" in lib.pfg_last_error().decode()
    fn = lib.pfg_cond_forward
    big = 1 << 40
    assert fn(r(net), None, n, -1, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, n, -1, None, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(make_cond(w=None)), FAKE, n, -1, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert "cond_w" in lib.pfg_last_error().decode()
    assert fn(r(make_cond(W_null_at=1)), FAKE, n, -1, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_NULL
    assert fn(r(net), FAKE, n, 2, FAKE, None, None, FAKE, big, None) == pfg.PFG_ERR_UNSUPPORTED
    assert fn(r(net), FAKE, n, -1, FAKE, None, None, None, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, n, -1, FAKE, None, None, FAKE + 16, big, None) == pfg.PFG_ERR_WORKSPACE
    assert fn(r(net), FAKE, n, -1, FAKE, None, None, FAKE, 4096, None) == pfg.PFG_ERR_WORKSPACE


def test_last_error_is_cleared_by_a_good_call(lib):
    net = make_net([4, 3, 2])
    assert ws_bytes(lib, net, 9, 1, 1)[0] == pfg.PFG_ERR_UNSUPPORTED
    assert lib.pfg_last_error().decode() != ""
    assert ws_bytes(lib, net, 0, 1, 1)[0] == 0
    assert lib.pfg_last_error().decode() == ""


def test_timing_query_without_launches(lib):
    assert lib.pfg_timing_reset() == 0
    n, ms = ctypes.c_int64(0), ctypes.c_double(0)
    assert lib.pfg_timing_query(b"outer_product", ctypes.byref(n), ctypes.byref(ms)) == pfg.PFG_ERR_SHAPE
    assert lib.pfg_timing_query(None, ctypes.byref(n), ctypes.byref(ms)) == pfg.PFG_ERR_NULL
    buf = ctypes.create_string_buffer(64)
    assert lib.pfg_timing_names(buf, 64) == 0 and buf.value == b""


def test_bf16_rounding_of_inputs():
    import numpy as np
    from paper_1903_04243_amd.workloads import bf16_round
    import torch
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-3, 65504.0, 0.0, -0.0,
                  1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8], dtype=np.float32)
    bits, back = bf16_round(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(back, t.to(torch.float32).numpy())
    np.testing.assert_array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))
    rng = np.random.default_rng(0)
    y = rng.standard_normal(10000).astype(np.float32)
    bits, back = bf16_round(y)
    t = torch.from_numpy(y).to(torch.bfloat16)
    np.testing.assert_array_equal(back, t.to(torch.float32).numpy())


def test_static_scratch_entry_point_rejects_before_any_device_call(lib):
    # argument checks and the size limit are host logic: nothing below reaches the GPU runtime
    lib.pfg_per_example_grads_static.restype = ctypes.c_int
    big = make_net([64, 8192, 8192, 10])
    rc, need = ws_bytes(lib, big, 0, 1024, 1)
    assert rc == 0 and need > pfg.PFG_STATIC_SCRATCH_BYTES
    rc = lib.pfg_per_example_grads_static(ctypes.byref(big), FAKE, FAKE, 1024, None, None, None, None)
    assert rc == pfg.PFG_ERR_WORKSPACE
    assert b"built-in buffer" in lib.pfg_last_error()
    assert lib.pfg_per_example_grads_static(ctypes.byref(big), None, FAKE, 8, None, None, None, None) == pfg.PFG_ERR_NULL
    assert lib.pfg_per_example_grads_static(ctypes.byref(big), FAKE, FAKE, 0, None, None, None, None) == pfg.PFG_ERR_SHAPE
    header = open(os.path.join(ROOT, "include", "pfg.h")).read()
    m = re.search(r"#define PFG_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == pfg.PFG_STATIC_SCRATCH_BYTES
