"""The entry point that allocates nothing (pfg_per_example_grads_static), called through the C ABI:
its results must equal those of pfg_per_example_grads bit for bit (same kernels, same order), on two
calls in a row that share the library's built-in scratch buffer, the second on a smaller input."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_1903_04243_amd as pfg  # noqa: E402
from paper_1903_04243_amd import workloads as wl  # noqa: E402

from gpu_helpers import dev, draw, gpu_net, gpu_x, say  # noqa: E402
from parity_util import TOL_F32, slice_rel_err  # noqa: E402


def outputs(net, B, fill):
    f32 = dict(dtype=torch.float32, device="cuda:0")
    return ([torch.full((B, net.dims[l], net.dims[l + 1]), fill, **f32) for l in range(net.L)],
            [torch.full((B, net.dims[l + 1]), fill, **f32) for l in range(net.L)],
            torch.full((B,), fill, **f32))


def test_static_scratch_entry_point_matches_the_workspace_entry_point(oracle):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    pfg.load_library()
    w = wl.WORKLOADS["c2_mnist_mlp_grads"]
    # first call: the full batch of 128; second call: 37 examples of a narrower network, so the
    # second call finds the first call's contents in the shared buffer
    cases = [(draw(w), w.dims, w.B, "relu"),
             (draw(w, B=37, dims=(200, 136, 72, 10), bias_scale=0.2), (200, 136, 72, 10), 37, "relu")]
    for call, (inp, dims, B, act) in enumerate(cases):
        say(f"static scratch call {call}: dims {dims} B={B}")
        net = gpu_net(inp, act, "f32")
        X, labels = gpu_x(inp, "f32"), dev(inp.labels)
        ref_dW, ref_db, ref_loss = outputs(net, B, float("nan"))
        pfg.pfg_per_example_grads(net, X, labels, out_dW=ref_dW, out_db=ref_db, out_loss=ref_loss)
        torch.cuda.synchronize()
        dW, db, loss = outputs(net, B, float("nan"))
        # torch's running count of allocations (frees, e.g. by a garbage collection of earlier tests'
        # tensors in between, do not change it)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        pfg.pfg_per_example_grads_static(net, X, labels, dW, db, loss)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        for l in range(net.L):
            assert torch.equal(dW[l], ref_dW[l]), f"call {call}: dW{l + 1} differs"
            assert torch.equal(db[l], ref_db[l]), f"call {call}: db{l + 1} differs"
        assert torch.equal(loss, ref_loss), f"call {call}: loss differs"
        # and both agree with the oracle
        onet = oracle.Net(inp.Ws, inp.bs, act)
        o_dW, o_db, o_loss = oracle.per_example_grads(onet, inp.X, inp.labels)
        worst = max([slice_rel_err(dW[l].cpu().numpy(), o_dW[l]) for l in range(net.L)] +
                    [slice_rel_err(db[l].cpu().numpy(), o_db[l]) for l in range(net.L)] +
                    [slice_rel_err(loss.cpu().numpy(), o_loss, lead=0)])
        say(f"  call {call}: rel err vs oracle {worst:.3e}")
        assert worst <= TOL_F32


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    pfg.load_library()
    dims = (64, 4096, 4096, 10)
    Ws = [torch.zeros((dims[l], dims[l + 1]), dtype=torch.float32, device="cuda:0") for l in range(3)]
    net = pfg.Mlp(Ws, None, "relu", "f32")
    B = 2048                      # 2 hidden layers x (a, phi') + cotangents: over 100 MB
    assert pfg.pfg_workspace_bytes(net, "per_example_grads", B) > pfg.PFG_STATIC_SCRATCH_BYTES
    X = torch.zeros((B, 64), dtype=torch.float32, device="cuda:0")
    labels = torch.zeros((B,), dtype=torch.int32, device="cuda:0")
    with pytest.raises(pfg.PfgError) as ei:
        pfg.pfg_per_example_grads_static(net, X, labels, [None, None, None])
    assert ei.value.code == pfg.PFG_ERR_WORKSPACE
    assert "built-in buffer" in str(ei.value)
