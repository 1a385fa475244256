"""Plumbing shared by the GPU parity tests: uploads, input draws, progress lines.  No arithmetic
of the method."""
import sys

import numpy as np
import torch

import paper_1903_04243_amd as pfg
from paper_1903_04243_amd import workloads as wl
from parity_util import hidden_margin

NP_ACT = {"identity": lambda z: z, "relu": lambda z: np.maximum(z, 0.0), "tanh": np.tanh,
          "gelu": None}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t if dtype is None else t.to(dtype)


def gpu_net(inp, act, dtype):
    return pfg.Mlp.from_numpy(inp.Ws, inp.bs, act, dtype, inp.Ws_bits, inp.bs_bits)


def gpu_x(inp, dtype):
    if dtype == "bf16":
        return torch.from_numpy(inp.X_bits.view(np.int16)).to("cuda:0").view(torch.bfloat16)
    return dev(inp.X)


def draw(w, B=None, dims=None, bias_scale=0.0, act=None):
    """Inputs of a workload; for ReLU re-draw (next seed) until no hidden unit sits on the kink."""
    act = act or w.act
    seed = wl.BASE_SEED + w.index
    for attempt in range(20):
        inp = wl.make_inputs(w, B=B, dims=dims, bias_scale=bias_scale, seed=seed + 1000 * attempt)
        if act != "relu" or hidden_margin(inp.Ws, inp.bs, inp.X, NP_ACT["relu"]) > 1e-5:
            return inp
    raise AssertionError("could not draw inputs away from the ReLU kink")
