#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only-primary] [--no-cpu-baseline]

A step is one call of the library on one batch of seeded synthetic input that is already
resident in HBM.  The last line of stdout is the headline record: the largest per-example-gradient
workload that fits one GPU (4096 -> 4096 -> 4096 -> 10, GELU, bf16 inputs and weights, float32
accumulation and output, batch 256: 34.4 GB written per step), with its roofline and the CPU
baseline; the other dense workloads appear in it as short entries.  The full records of every
workload go to the file named by --detail-file and, a workload a line, to stderr.  Per-kernel
durations come from HIP events the library records on the call's stream in a second, instrumented pass over the same steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--only-primary", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="do not also time a HIP-graph replay")
    ap.add_argument("--copy-reference", action="store_true",
                    help="run a plain elementwise copy of known size (scale for HBM counters)")
    ap.add_argument("--fill-reference", action="store_true",
                    help="measure plain sequential fills of several sizes (the practical HBM write ceiling)")
    ap.add_argument("--launch-floor", action="store_true",
                    help="measure the cost per launch of a chain of dependent near-empty kernels")
    ap.add_argument("--detail-file", default=os.path.join("gpurun_out", "bench_detail.json"),
                    help="where the full per-workload records go (relative to the repository root)")
    ap.add_argument("--workload", default=None,
                    help="measure only this workload and print its record (for profiling runs)")
    ap.add_argument("--batch", type=int, default=None,
                    help="with --workload: the same workload at another batch size (rows for the conditional)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this library has no multi-GPU path (parallel-for "
                 "iterations are independent; a batch would simply be split across devices). "
                 "Run with --gpus 1.")

    import numpy as np
    import torch

    import paper_1903_04243_amd as pfg
    from paper_1903_04243_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if not os.path.exists(pfg.LIB_PATH):
        from paper_1903_04243_amd import build as pfg_build
        pfg_build.build()
    pfg.load_library()
    dev = "cuda:0"

    def pick(table, name):
        """The named workload, at the batch size of --batch if that was given."""
        import dataclasses
        w = table[name]
        if args.batch is None or not args.workload:
            return w
        return dataclasses.replace(w, **{"n" if hasattr(w, "n") else "B": args.batch})
    torch.cuda.set_device(0)
    def upload(w):
        inp = wl.make_inputs(w)
        net = pfg.Mlp.from_numpy(inp.Ws, inp.bs, w.act, w.dtype, inp.Ws_bits, inp.bs_bits)
        if w.dtype == "bf16":
            X = torch.from_numpy(inp.X_bits.view(np.int16)).to(dev).view(torch.bfloat16)
        else:
            X = torch.from_numpy(inp.X).to(dev)
        labels = torch.from_numpy(inp.labels).to(dev)
        return inp, net, X, labels

    def make_step(w, net, X, labels):
        """Allocate outputs and workspace once; return the step function."""
        f32 = dict(dtype=torch.float32, device=dev)
        L, d, B, S = net.L, net.dims, w.B, w.S
        if w.call == "per_example_grads":
            dW = [torch.empty((B, d[l], d[l + 1]), **f32) for l in range(L)]
            db = [torch.empty((B, d[l + 1]), **f32) for l in range(L)]
            loss = torch.empty((B,), **f32)
            ws = torch.empty(pfg.pfg_workspace_bytes(net, w.call, B), dtype=torch.uint8, device=dev)
            return lambda: pfg.pfg_per_example_grads(net, X, labels, out_dW=dW, out_db=db,
                                                     out_loss=loss, workspace=ws)
        if w.call == "grad_norms":
            sq = torch.empty((B, L), **f32)
            norm = torch.empty((B,), **f32)
            loss = torch.empty((B,), **f32)
            ws = torch.empty(pfg.pfg_workspace_bytes(net, w.call, B), dtype=torch.uint8, device=dev)
            return lambda: pfg.pfg_per_example_grad_norms(net, X, labels, out_sq_layers=sq,
                                                          out_norm=norm, out_loss=loss, workspace=ws)
        if w.call == "hessian_input":
            H = torch.empty((B, S, d[0], d[0]), **f32)
            ws = torch.empty(pfg.pfg_workspace_bytes(net, w.call, B, S), dtype=torch.uint8,
                             device=dev)
            return lambda: pfg.pfg_hessian_input(net, X, out=H, workspace=ws)
        if w.call == "jacobian_input":
            J = torch.empty((B, S, d[0]), **f32)
            ws = torch.empty(pfg.pfg_workspace_bytes(net, w.call, B, S), dtype=torch.uint8,
                             device=dev)
            return lambda: pfg.pfg_jacobian_input(net, X, out=J, workspace=ws)
        layers = w.layers_out or tuple(range(1, L + 1))
        JW = [torch.empty((B, S, d[l], d[l + 1]), **f32) if (l + 1) in layers else None
              for l in range(L)]
        Jb = [torch.empty((B, S, d[l + 1]), **f32) for l in range(L)]
        ws = torch.empty(pfg.pfg_workspace_bytes(net, w.call, B, S), dtype=torch.uint8, device=dev)
        return lambda: pfg.pfg_jacobian_weights(net, X, head=w.head, out_JW=JW, out_Jb=Jb,
                                                workspace=ws)

    # Passes of K steps a workload is timed for; the fastest counts.  The headline workload is timed
    # once, exactly K steps.  The others get two passes in the default run: on a machine that has just
    # come up, one launch-bound workload per run (the first after the large buffers were released) has
    # been seen at a third of its launch rate for about 0.1 s, kernel times unchanged.
    timing_passes = {"n": 1}

    def timed(step, steps, warmup):
        best = None
        for _ in range(timing_passes["n"]):
            for _ in range(warmup):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / steps
            best = sec if best is None else min(best, sec)
        return best

    def timed_graph(step, steps, warmup):
        """The same step captured once into a HIP graph and replayed."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def kernel_times(step, steps):
        """Average duration per launch of every kernel family, from the library's HIP events."""
        pfg.pfg_timing_reset()
        pfg.pfg_timing_enable(True)
        try:
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
        finally:
            pfg.pfg_timing_enable(False)
        out = {}
        for name in pfg.pfg_timing_names():
            n, ms = pfg.pfg_timing_query(name)
            out[name] = {"launches_per_step": n / steps, "ms_per_step": ms / steps}
        pfg.pfg_timing_reset()
        return out

    def is_wide(M, d_in, d_out):
        # rows of 1024 floats or more from 128 MiB on; rows of 256 or 512 floats from 512 MiB on
        if d_out in (256, 512) and M <= 65535 and 4 * M * d_in * d_out >= (512 << 20):
            return True
        return (d_out % 4 == 0 and d_out >= 1024 and M <= 65535 and d_in <= 65535 and
                4 * M * d_in * d_out >= (128 << 20))

    def algorithmic(w):
        """Algorithmic work of the dominant kernels of one step."""
        d, B, S = w.dims, w.B, w.S
        if w.call == "per_example_grads":
            # large outputs with wide rows leave in a kernel of their own (the library's rule, restated;
            # the roofline below fails loudly if the launches disagree with it)
            wide = [l for l in range(1, len(d)) if is_wide(B, d[l - 1], d[l])]
            if wide:
                return {"outer_product_wide": {"bytes": 4 * B * sum(d[l - 1] * d[l] for l in wide),
                                               "launches": len(wide)}}
            return {"outer_product": {"bytes": 4 * B * sum(d[l - 1] * d[l] for l in range(1, len(d)))}}
        if w.call == "grad_norms":
            # no large output: the forward products dominate; each reads its weights once, reads
            # its input rows and writes a_l and phi'(z_l)
            elem = 2 if w.dtype == "bf16" else 4
            L = len(d) - 1
            return {"gemm_forward": {"bytes": sum(
                elem * d[l - 1] * d[l] + (elem if l == 1 else 4) * B * d[l - 1] +
                (8 if l < L else 4) * B * d[l] for l in range(1, L + 1))}}
        if w.call == "hessian_input":
            # each H[b, s] is symmetric: with 128 x 128 tiles only the T (T + 1) / 2 tiles on and above
            # the diagonal of its T x T tiles are computed (the rest are mirrored), so these are the
            # flops the kernel executes, not 2 B S d_0^2 K
            full = 2 * B * S * d[0] * d[0] * sum(d[1:-1])
            T = d[0] // 128
            return {"gemm_hessian": {"flops": full * (T + 1) // (2 * T) if d[0] % 128 == 0 else full}}
        if w.call == "jacobian_input":
            rows = B * S
            cot = sum(2 * rows * d[l] * d[l - 1] for l in range(2, len(d) - 1))
            return {"gemm_cotangent": {"flops": cot},
                    "gemm_jacobian": {"flops": 2 * rows * d[1] * d[0]}}
        layers = w.layers_out or tuple(range(1, len(d)))
        return {"outer_product": {"bytes": 4 * B * S * sum(d[l - 1] * d[l] for l in layers)}}

    def measured_traffic(name):
        """HBM bytes per launch of the outer-product kernel from the committed counter runs, or
        None if that kernel's source has changed since they were taken."""
        import hashlib
        try:
            rec = json.load(open(os.path.join(ROOT, "profiles", "outer_product_hbm_traffic.txt")))
            src = os.path.join(ROOT, "paper_1903_04243_amd", "csrc", "writer.hip")
            if hashlib.sha256(open(src, "rb").read()).hexdigest() != rec["writer_hip_sha256"]:
                return None
            return rec["workloads"][name]["hbm_bytes_per_launch"]
        except (OSError, KeyError, ValueError):
            return None

    def roofline(w, kt):
        alg = algorithmic(w)
        fam = next(iter(alg))
        if "bytes" in alg[fam]:
            k = kt[fam]
            if "launches" in alg[fam] and round(k["launches_per_step"]) != alg[fam]["launches"]:
                raise RuntimeError(f"{alg[fam]['launches']} launches of {fam} expected per step, "
                                   f"{k['launches_per_step']} recorded")
            per_launch_bytes = alg[fam]["bytes"] / k["launches_per_step"]
            per_launch_ms = k["ms_per_step"] / k["launches_per_step"]
            gbs = per_launch_bytes / (per_launch_ms * 1e-3) / 1e9
            return {"kernel": fam, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                    "traffic": measured_traffic(w.name) if (fam.startswith("outer_product") and args.batch is None) else None,
                    "bytes_per_launch": per_launch_bytes, "ms_per_launch": per_launch_ms,
                    "launches_per_step": k["launches_per_step"]}
        flops = sum(v["flops"] for v in alg.values())
        ms = sum(kt[name]["ms_per_step"] for name in alg)
        launches = sum(kt[name]["launches_per_step"] for name in alg)
        tf = flops / (ms * 1e-3) / 1e12
        peak = MFMA_PEAK_TFLOPS[w.dtype]
        return {"kernel": "+".join(alg), "bound": "mfma", "achieved": tf, "peak": peak,
                "unit": "TFLOP/s", "frac": tf / peak, "traffic": None,
                "flops_per_launch": flops / launches, "ms_per_launch": ms / launches,
                "launches_per_step": launches}

    def measure(name, steps, warmup):
        w = pick(wl.WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp, net, X, labels = upload(w)
        step = make_step(w, net, X, labels)
        step()
        torch.cuda.synchronize()
        log(f"[bench] {name}: timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:  # graph capture is optional; eager timing stands
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        # one isolated call at a time (synchronised before and after), median of 15
        singles = []
        for _ in range(15):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            step()
            torch.cuda.synchronize()
            singles.append(time.perf_counter() - t0)
        single_ms = sorted(singles)[len(singles) // 2] * 1e3
        # the small products (M = B rows): flops and weight bytes against both peaks
        d, B, S = w.dims, w.B, w.S
        elem = 2 if w.dtype == "bf16" else 4
        last = len(d) - 1
        fwd_layers = range(1, last) if w.call in ("jacobian_input", "hessian_input") else range(1, last + 1)
        fwd_flops = sum(2 * B * d[l - 1] * d[l] for l in fwd_layers)
        fwd_bytes = sum(elem * d[l - 1] * d[l] for l in fwd_layers)
        gemm_report = {}
        for fam, flops, nbytes in (("gemm_forward", fwd_flops, fwd_bytes),):
            if fam in kt and kt[fam]["ms_per_step"] > 0:
                sec_f = kt[fam]["ms_per_step"] * 1e-3
                tf, gbs = flops / sec_f / 1e12, nbytes / sec_f / 1e9
                gemm_report[fam] = {
                    "flops_per_step": flops, "TFLOP/s": tf,
                    "mfma_frac": tf / MFMA_PEAK_TFLOPS[w.dtype], "weight_bytes_per_step": nbytes,
                    "GB/s": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
                    "bound": "launch and memory latency (M = B rows: neither roofline is near)"
                    if max(tf / MFMA_PEAK_TFLOPS[w.dtype], gbs / HBM_PEAK_GBS) < 0.25 else "see fractions"}
        values = wl.output_values(w)
        rec = {
            "workload": name, "call": w.call, "dims": list(w.dims), "act": w.act, "dtype": w.dtype,
            "B": w.B, "S": w.S, "steps": steps, "ms_per_step": sec * 1e3,
            "ms_single_call": single_ms, "small_products": gemm_report,
            "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
            "output_values": values, "output_GB": values * 4 / 1e9,
            "kernels": kt, "roofline": roofline(w, kt),
        }
        if w.call == "per_example_grads":
            rec["per_example_grads_per_sec"] = w.B / sec
        elif w.call == "grad_norms":
            rec["per_example_grad_norms_per_sec"] = w.B / sec
        elif w.call == "hessian_input":
            rec["hessian_entries_per_sec"] = values / sec
            rec["hessians_per_sec"] = w.B * w.S / sec
        else:
            rec["jacobian_entries_per_sec"] = values / sec
            rec["jacobian_rows_per_sec"] = w.B * w.S / sec
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, roofline frac "
            f"{rec['roofline']['frac']:.3f}")
        return rec, inp

    def measure_varlen(name, steps, warmup):
        w = pick(wl.LSTM_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp, lengths = wl.make_varlen_inputs(w)
        net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
        X = torch.from_numpy(inp.X).to(dev)
        B, H, dx, dy = w.B, w.H, w.dx, w.dy
        tokens = int(lengths.sum())
        f32 = dict(dtype=torch.float32, device=dev)
        h, y = torch.empty((B, H), **f32), torch.empty((B, dy), **f32)
        ws = torch.empty(pfg.pfg_lstm_varlen_workspace_bytes(net, B, tokens), dtype=torch.uint8,
                         device=dev)
        step = lambda: pfg.pfg_lstm_varlen_forward(net, X, lengths, out_h=h, out_y=y, workspace=ws)
        step()
        torch.cuda.synchronize()
        log(f"[bench] {name}: timing {steps} steps")
        sec = timed(step, steps, warmup)
        kt = kernel_times(step, steps)
        # every token passes the recurrent product once: 2 * H * 4H flops, plus its input projection
        flops = tokens * (2 * H * 4 * H)
        fam = "lstm_step"
        tf = flops / kt[fam]["ms_per_step"] / 1e9
        roof = {"kernel": fam, "bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["f32"],
                "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                "flops_per_launch": flops / kt[fam]["launches_per_step"],
                "ms_per_launch": kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"],
                "launches_per_step": kt[fam]["launches_per_step"],
                "note": "a chain of max(length) dependent launches on a shrinking batch: bound by "
                        "launch and memory latency, not by either roofline"}
        rec = {"workload": name, "call": w.call, "input_size": dx, "state_size": H, "output_size": dy,
               "dtype": "f32", "B": B, "tokens": tokens, "longest": int(lengths.max()), "steps": steps,
               "ms_per_step": sec * 1e3, "ms_per_step_graph_replay": None,
               "tokens_per_sec": tokens / sec, "sequences_per_sec": B / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()),
               "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, {rec['tokens_per_sec'] / 1e6:.1f} M tokens/s, "
            f"roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_while(name, steps, warmup):
        w = pick(wl.LSTM_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp, lengths, offsets, halt_w, halt_c = wl.make_while_inputs(w)
        net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
        X, off, hw = torch.from_numpy(inp.X).to(dev), torch.from_numpy(offsets).to(dev), torch.from_numpy(halt_w).to(dev)
        B, H, dx, dy = w.B, w.H, w.dx, w.dy
        tokens = int(lengths.sum())
        out = (torch.empty((B, H), dtype=torch.float32, device=dev), torch.empty((B, dy), dtype=torch.float32, device=dev),
               torch.empty((B,), dtype=torch.int32, device=dev), torch.empty((1,), dtype=torch.int32, device=dev))
        ws = torch.empty(pfg.pfg_lstm_while_workspace_bytes(net, B, tokens), dtype=torch.uint8, device=dev)
        step = lambda: pfg.pfg_lstm_while_forward(net, X, off, w.T, halt_w=hw, halt_c=halt_c, out=out, workspace=ws)
        step()
        torch.cuda.synchronize()
        used = int(out[2].sum().item())
        trips = int(out[3].item())
        log(f"[bench] {name}: {used} of {tokens} tokens consumed, {trips} trips; timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        flops = used * (2 * H * 4 * H)
        fam = "lstm_step"
        tf = flops / kt[fam]["ms_per_step"] / 1e9
        roof = {"kernel": fam, "bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["f32"],
                "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                "flops_per_launch": flops / kt[fam]["launches_per_step"],
                "ms_per_launch": kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"],
                "launches_per_step": kt[fam]["launches_per_step"],
                "note": "a chain of dependent launches (condition, then body, per trip) on a shrinking list: "
                        "bound by launch and memory latency, not by either roofline"}
        rec = {"workload": name, "call": w.call, "input_size": dx, "state_size": H, "output_size": dy,
               "dtype": "f32", "B": B, "tokens": tokens, "tokens_consumed": used, "trips": trips,
               "max_steps": w.T, "steps": steps, "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "tokens_per_sec": used / sec, "sequences_per_sec": B / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()), "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, {rec['tokens_per_sec'] / 1e6:.1f} M tokens/s, "
            f"roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_while_grads(name, steps, warmup):
        w = pick(wl.LSTM_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp, lengths, offsets, halt_w, halt_c = wl.make_while_inputs(w)
        net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, 1)
        X, off, hw = torch.from_numpy(inp.X).to(dev), torch.from_numpy(offsets).to(dev), torch.from_numpy(halt_w).to(dev)
        labels = torch.from_numpy(inp.labels).to(dev)
        B, H, dx, dy = w.B, w.H, w.dx, w.dy
        tokens = int(lengths.sum())
        f32 = dict(dtype=torch.float32, device=dev)
        norms = (w.call == "lstm_while_per_example_grad_norms")
        ws = torch.empty(pfg.pfg_lstm_while_grads_workspace_bytes(net, B, tokens, w.T), dtype=torch.uint8, device=dev)
        if norms:
            out = {"sq": torch.empty((B, 4), **f32), "norm": torch.empty((B,), **f32), "loss": torch.empty((B,), **f32),
                   "steps": torch.empty((B,), dtype=torch.int32, device=dev)}
            step = lambda: pfg.pfg_lstm_while_per_example_grad_norms(net, X, off, labels, w.T, halt_w=hw,
                                                                     halt_c=halt_c, out=out, workspace=ws)
        else:
            out = {"dW": torch.empty((B, dx + H, 4 * H), **f32), "db": torch.empty((B, 4 * H), **f32),
                   "dWout": torch.empty((B, H, dy), **f32), "dbout": torch.empty((B, dy), **f32),
                   "loss": torch.empty((B,), **f32), "steps": torch.empty((B,), dtype=torch.int32, device=dev)}
            step = lambda: pfg.pfg_lstm_while_per_example_grads(net, X, off, labels, w.T, halt_w=hw, halt_c=halt_c,
                                                                out=out, workspace=ws)
        step()
        torch.cuda.synchronize()
        used = int(out["steps"].sum().item())
        log(f"[bench] {name}: {used} of {tokens} tokens consumed; timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        if norms:
            # no large output: the Gram kernel reads x, h and dz of every consumed token once and multiplies the
            # rows of every iteration with each other on the matrix cores; priced by the flops of the tiles it runs
            fam = "while_grad_sqnorms"
            tl = np.minimum(out["steps"].cpu().numpy(), 128)
            tiles = (((tl + 31) // 32) * ((tl + 31) // 32 + 1) // 2).sum()
            flops = float(tiles) * 2 * 32 * 32 * (4 * H + dx + H)
            tf = flops / kt[fam]["ms_per_step"] / 1e9
            roof = {"kernel": fam, "bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["f32"],
                    "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                    "flops_per_launch": flops, "ms_per_launch": kt[fam]["ms_per_step"],
                    "launches_per_step": kt[fam]["launches_per_step"],
                    "note": "the step itself is the two chains of dependent launches, one per forward and reverse trip"}
        else:
            # the one large output is the stacked weight gradient: 4 bytes per value of dW and db
            fam = "outer_sum_ragged"
            nbytes = 4 * B * (dx + H + 1) * 4 * H
            gbs = nbytes / kt[fam]["ms_per_step"] / 1e6
            roof = {"kernel": fam, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": None,
                    "bytes_per_launch": nbytes / kt[fam]["launches_per_step"],
                    "ms_per_launch": kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"],
                    "launches_per_step": kt[fam]["launches_per_step"],
                    "note": "the writer forms an iteration's product over its trips (2 * tokens_consumed * (dx + H) * 4H "
                            "flops on the matrix cores) before it stores; the rest of the step is two chains of "
                            "dependent launches, one per forward and reverse trip"}
        rec = {"workload": name, "call": w.call, "input_size": dx, "state_size": H, "output_size": dy,
               "dtype": "f32", "B": B, "tokens": tokens, "tokens_consumed": used, "max_steps": w.T, "steps": steps,
               "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "per_example_grads_per_sec": B / sec, "tokens_per_sec": used / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()), "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, {rec['per_example_grads_per_sec']:.0f} grads/s, "
            f"roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_conv(name, steps, warmup):
        w = pick(wl.CONV_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp = wl.make_conv_inputs(w)
        net = pfg.ConvNet.from_numpy(w.height, w.width, w.channels, inp.Wc, inp.bc, inp.Ws, inp.bs)
        X = torch.from_numpy(inp.X).to(dev)
        labels = torch.from_numpy(inp.labels).to(dev)
        f32 = dict(dtype=torch.float32, device=dev)
        B, dn = w.B, net.dense
        out = ([torch.empty((B,) + W.shape, **f32) for W in inp.Wc],
               [torch.empty((B, W.shape[3]), **f32) for W in inp.Wc],
               [torch.empty((B, dn.dims[l], dn.dims[l + 1]), **f32) for l in range(dn.L)],
               [torch.empty((B, dn.dims[l + 1]), **f32) for l in range(dn.L)], torch.empty((B,), **f32))
        norms = (w.call == "convnet_per_example_grad_norms")
        if norms:
            out = (torch.empty((B, net.nc + dn.L), **f32), torch.empty((B,), **f32), torch.empty((B,), **f32))
            ws = torch.empty(pfg.pfg_convnet_grad_norms_workspace_bytes(net, B), dtype=torch.uint8, device=dev)
            step = lambda: pfg.pfg_convnet_per_example_grad_norms(net, X, labels, out=out, workspace=ws)
        else:
            ws = torch.empty(pfg.pfg_convnet_workspace_bytes(net, B), dtype=torch.uint8, device=dev)
            step = lambda: pfg.pfg_convnet_per_example_grads(net, X, labels, out=out, workspace=ws)
        step()
        torch.cuda.synchronize()
        log(f"[bench] {name}: timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        if norms:
            values = sum(t.numel() for t in out)
        else:
            values = sum(t.numel() for group in out[:4] for t in group) + B
            # the dense weight gradients are the large output (4 bytes per value, written once); wide
            # layers leave in a kernel of their own, which is then the one to price
            wide = [l for l in range(dn.L) if is_wide(B, dn.dims[l], dn.dims[l + 1])]
            fam = "outer_product_wide" if wide else "outer_product"
            nbytes = 4 * B * sum(dn.dims[l] * dn.dims[l + 1] for l in (wide or range(dn.L)))
            if wide and round(kt[fam]["launches_per_step"]) != len(wide):
                raise RuntimeError(f"{len(wide)} launches of {fam} expected, {kt[fam]['launches_per_step']} recorded")
            per_ms = kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"]
            gbs = nbytes / kt[fam]["ms_per_step"] / 1e6
            roof = {"kernel": fam, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": None,
                    "bytes_per_launch": nbytes / kt[fam]["launches_per_step"], "ms_per_launch": per_ms,
                    "launches_per_step": kt[fam]["launches_per_step"]}
        # the conv products, against the fp32 MFMA peak
        hh, ww, cc = w.height, w.width, w.channels
        conv_flops = {"conv_gemm_forward": 0, "conv_gemm_filter": 0, "conv_gemm_cotangent": 0}
        direct = 0
        for i, (k, f) in enumerate(w.blocks):
            per = 2 * B * hh * ww * k * k * cc * f
            # a block with few taps per output goes from the image to the pooled output in one plain
            # ALU kernel (the library's rule, restated; the launch counts below check it): its
            # forward flops are not the matrix cores'
            taps = k * k * cc
            if taps <= 56 and f % 4 == 0 and taps * f <= 4096 and (k + 1) * (ww + k - 1) * cc <= 4096:
                direct += 1
            else:
                conv_flops["conv_gemm_forward"] += per
            conv_flops["conv_gemm_filter"] += per
            if i > 0:
                conv_flops["conv_gemm_cotangent"] += per
            hh, ww, cc = hh // 2, ww // 2, f
        seen = kt.get("conv_relu_pool", {}).get("launches_per_step", 0)
        if round(seen) != direct:
            raise RuntimeError(f"{direct} conv blocks expected in the image-to-pooled-output kernel, {seen} launched")
        conv_report = {fam2: {"flops_per_step": fl, "TFLOP/s": fl / kt[fam2]["ms_per_step"] / 1e9,
                              "mfma_frac": fl / kt[fam2]["ms_per_step"] / 1e9 / MFMA_PEAK_TFLOPS["f32"]}
                       for fam2, fl in conv_flops.items() if fam2 in kt and fl}
        if norms:
            # no large output is left: the slowest of the conv products is the kernel to price
            fam = max(conv_report, key=lambda f2: kt[f2]["ms_per_step"])
            tf = conv_report[fam]["TFLOP/s"]
            roof = {"kernel": fam, "bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["f32"],
                    "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                    "flops_per_launch": conv_report[fam]["flops_per_step"] / kt[fam]["launches_per_step"],
                    "ms_per_launch": kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"],
                    "launches_per_step": kt[fam]["launches_per_step"]}
        rec = {"workload": name, "call": w.call, "image": [w.height, w.width, w.channels],
               "blocks": [list(b) for b in w.blocks], "dense": list(w.dense), "dtype": "f32", "B": B,
               "steps": steps, "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "output_values": values, "output_GB": values * 4 / 1e9,
               "per_example_grads_per_sec": B / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()),
               "conv_products": conv_report, "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_cond_grads(name, steps, warmup):
        w = pick(wl.COND_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp = wl.make_cond_inputs(w)
        net = pfg.Cond.from_numpy(inp.pre, inp.w, inp.c0, inp.then_net, inp.else_net, w.act)
        X = torch.from_numpy(inp.X).to(dev)
        n = w.n
        labels = torch.from_numpy(np.random.Generator(np.random.Philox(wl.BASE_SEED + w.index + 900000))
                                  .integers(0, net.dout, size=n).astype(np.int32)).to(dev)
        f32 = dict(dtype=torch.float32, device=dev)
        out = {}
        nbytes = 0
        for nm, m in (("pre", net.pre), ("then", net.then_net), ("else", net.else_net)):
            out[nm] = ([torch.empty((n, m.dims[l], m.dims[l + 1]), **f32) for l in range(m.L)],
                       [torch.empty((n, m.dims[l + 1]), **f32) for l in range(m.L)])
            nbytes += 4 * n * sum(m.dims[l] * m.dims[l + 1] for l in range(m.L))
        out["loss"] = torch.empty((n,), **f32)
        out["cond"] = torch.empty((n,), dtype=torch.int32, device=dev)
        out["counts"] = torch.empty((2,), dtype=torch.int32, device=dev)
        ws = torch.empty(pfg.pfg_cond_grads_workspace_bytes(net, n), dtype=torch.uint8, device=dev)
        step = lambda: pfg.pfg_cond_per_example_grads(net, X, labels, out=out, workspace=ws)
        step()
        torch.cuda.synchronize()
        n_then, n_else = out["counts"].tolist()
        log(f"[bench] {name}: {n_then} then rows, {n_else} else rows; timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        # every gradient slice is written once (products or zeros): 4 bytes per value, all launches of the
        # outer-product family together
        fams = [f for f in kt if f.startswith("outer_product")]
        ms = sum(kt[f]["ms_per_step"] for f in fams)
        launches = sum(kt[f]["launches_per_step"] for f in fams)
        gbs = nbytes / ms / 1e6
        roof = {"kernel": "+".join(sorted(fams)), "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": nbytes / launches,
                "ms_per_launch": ms / launches, "launches_per_step": launches}
        rec = {"workload": name, "call": w.call, "pre": list(w.pre), "then": list(w.then_dims),
               "else": list(w.else_dims), "act": w.act, "dtype": "f32", "n": n, "n_then": n_then, "n_else": n_else,
               "steps": steps, "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "output_GB": nbytes / 1e9, "per_example_grads_per_sec": n / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()), "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_cond(name, steps, warmup):
        if wl.COND_WORKLOADS[name].call == "cond_per_example_grads":
            return measure_cond_grads(name, steps, warmup)
        w = pick(wl.COND_WORKLOADS, name)
        log(f"[bench] {name}: uploading inputs")
        inp = wl.make_cond_inputs(w)
        net = pfg.Cond.from_numpy(inp.pre, inp.w, inp.c0, inp.then_net, inp.else_net, w.act)
        X = torch.from_numpy(inp.X).to(dev)
        n = w.n
        out = (torch.empty((n, net.dout), dtype=torch.float32, device=dev),
               torch.empty((n,), dtype=torch.int32, device=dev), torch.empty((2,), dtype=torch.int32, device=dev))
        ws = torch.empty(pfg.pfg_cond_workspace_bytes(net, n), dtype=torch.uint8, device=dev)
        step = lambda: pfg.pfg_cond_forward(net, X, out=out, workspace=ws)
        step()
        torch.cuda.synchronize()
        n_then, n_else = out[2].tolist()
        log(f"[bench] {name}: {n_then} then rows, {n_else} else rows; timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        per_row = lambda dims: 2 * sum(dims[l] * dims[l + 1] for l in range(len(dims) - 1))
        dT = w.pre[-1]
        flops = {"cond_gemm_pre": n * per_row(w.pre), "cond_gemm_then": n_then * per_row((dT,) + w.then_dims),
                 "cond_gemm_else": n_else * per_row((dT,) + w.else_dims)}
        # the roofline counts the rows a branch really has, not the n rows its products are launched for
        fam = max(flops, key=flops.get)
        tf = flops[fam] / kt[fam]["ms_per_step"] / 1e9
        roof = {"kernel": fam, "bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["f32"],
                "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                "flops_per_step": flops[fam], "launches_per_step": kt[fam]["launches_per_step"],
                "ms_per_launch": kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"]}
        both = n * (per_row(w.pre) + per_row((dT,) + w.then_dims) + per_row((dT,) + w.else_dims))
        rec = {"workload": name, "call": "cond_forward", "pre": list(w.pre), "then": list(w.then_dims),
               "else": list(w.else_dims), "act": w.act, "dtype": "f32", "n": n, "n_then": n_then,
               "n_else": n_else, "steps": steps, "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "rows_per_sec": n / sec, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()),
               "flops_per_step": sum(flops.values()),
               "flops_if_both_branches_ran_on_every_row": both, "roofline": roof}
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, roofline frac {roof['frac']:.3f}")
        return rec, inp

    def measure_lstm(name, steps, warmup):
        if name in wl.CONV_WORKLOADS:
            return measure_conv(name, steps, warmup)
        if name in wl.COND_WORKLOADS:
            return measure_cond(name, steps, warmup)
        w = pick(wl.LSTM_WORKLOADS, name)
        if w.call == "lstm_varlen_forward":
            return measure_varlen(name, steps, warmup)
        if w.call == "lstm_while_forward":
            return measure_while(name, steps, warmup)
        if w.call in ("lstm_while_per_example_grads", "lstm_while_per_example_grad_norms"):
            return measure_while_grads(name, steps, warmup)
        log(f"[bench] {name}: uploading inputs")
        inp = wl.make_lstm_inputs(w)
        net = pfg.Lstm.from_numpy(inp.W, inp.b, inp.Wout, inp.bout, w.T)
        X = torch.from_numpy(inp.X).to(dev)
        labels = torch.from_numpy(inp.labels).to(dev)
        f32 = dict(dtype=torch.float32, device=dev)
        B, S, T, dx, H, dy = w.B, w.S, w.T, w.dx, w.H, w.dy
        if w.call == "lstm_per_example_grads":
            outs = [torch.empty(sh, **f32) for sh in ((B, dx + H, 4 * H), (B, 4 * H), (B, H, dy),
                                                      (B, dy), (B,))]
            ws = torch.empty(pfg.pfg_lstm_workspace_bytes(net, "per_example_grads", B),
                             dtype=torch.uint8, device=dev)
            step = lambda: pfg.pfg_lstm_per_example_grads(net, X, labels, out=outs, workspace=ws)
            values = sum(t.numel() for t in outs)
        elif w.call == "lstm_per_example_grad_norms":
            outs = (torch.empty((B, 4), **f32), torch.empty((B,), **f32), torch.empty((B,), **f32))
            ws = torch.empty(pfg.pfg_lstm_workspace_bytes(net, "grad_norms", B), dtype=torch.uint8, device=dev)
            step = lambda: pfg.pfg_lstm_per_example_grad_norms(net, X, labels, out=outs, workspace=ws)
            values = 6 * B
        else:
            J = torch.empty((B, S, T, dx), **f32)
            ws = torch.empty(pfg.pfg_lstm_workspace_bytes(net, "jacobian_input", B, S),
                             dtype=torch.uint8, device=dev)
            step = lambda: pfg.pfg_lstm_jacobian_input(net, X, out=J, workspace=ws)
            values = J.numel()
        step()
        torch.cuda.synchronize()
        log(f"[bench] {name}: timing {steps} steps")
        sec = timed(step, steps, warmup)
        sec_graph = None
        if not args.no_graph:
            try:
                sec_graph = timed_graph(step, steps, warmup)
            except Exception as e:
                log(f"[bench] {name}: graph replay not measured ({e})")
        kt = kernel_times(step, steps)
        if w.call == "lstm_per_example_grads":
            # the weight gradient is the one large output: 4 bytes per value of dW
            fam = "outer_sum"
            nbytes = 4 * B * (dx + H) * 4 * H
            per_ms = kt[fam]["ms_per_step"] / kt[fam]["launches_per_step"]
            gbs = nbytes / kt[fam]["ms_per_step"] / 1e6
            roof = {"kernel": fam, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": None,
                    "bytes_per_launch": nbytes / kt[fam]["launches_per_step"], "ms_per_launch": per_ms,
                    "launches_per_step": kt[fam]["launches_per_step"]}
        elif w.call == "lstm_per_example_grad_norms":
            # no large output: the step is the sequential sweep; priced like the dense norm workloads
            # by the bytes the Gram kernel reads (x, h and dz of every step, once)
            fam = "lstm_grad_sqnorms"
            nbytes = 4 * B * T * (dx + H + 4 * H)
            gbs = nbytes / kt[fam]["ms_per_step"] / 1e6
            roof = {"kernel": fam, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": nbytes,
                    "ms_per_launch": kt[fam]["ms_per_step"], "launches_per_step": kt[fam]["launches_per_step"],
                    "note": "latency-bound chain of steps; the Gram kernel is a small part of it"}
        else:
            rows = B * S
            # one product per step: [dx_t | dh_{t-1}] = dz_t [W_x ; W_h]^T (no dh for the first step)
            fams = ("lstm_gemm_reverse",)
            flops = T * 2 * rows * 4 * H * dx + (T - 1) * 2 * rows * 4 * H * H
            ms = sum(kt[f]["ms_per_step"] for f in fams)
            launches = sum(kt[f]["launches_per_step"] for f in fams)
            tf = flops / ms / 1e9
            roof = {"kernel": "+".join(fams), "bound": "mfma", "achieved": tf,
                    "peak": MFMA_PEAK_TFLOPS["f32"], "unit": "TFLOP/s",
                    "frac": tf / MFMA_PEAK_TFLOPS["f32"], "traffic": None,
                    "flops_per_launch": flops / launches, "ms_per_launch": ms / launches,
                    "launches_per_step": launches}
        rec = {"workload": name, "call": w.call, "input_size": dx, "state_size": H, "output_size": dy,
               "unrolled_steps": T, "dtype": "f32", "B": B, "S": S, "steps": steps,
               "ms_per_step": sec * 1e3,
               "ms_per_step_graph_replay": None if sec_graph is None else sec_graph * 1e3,
               "output_values": values, "output_GB": values * 4 / 1e9, "kernels": kt,
               "kernel_ms_sum": sum(v["ms_per_step"] for v in kt.values()),
               "launches_per_step": sum(v["launches_per_step"] for v in kt.values()),
               "roofline": roof}
        if w.call == "lstm_per_example_grads":
            rec["per_example_grads_per_sec"] = B / sec
        elif w.call == "lstm_per_example_grad_norms":
            rec["per_example_grad_norms_per_sec"] = B / sec
        else:
            rec["jacobian_rows_per_sec"] = B * S / sec
            rec["jacobian_entries_per_sec"] = values / sec
        log(f"[bench] {name}: {rec['ms_per_step']:.4f} ms/step, roofline frac {roof['frac']:.3f}")
        return rec, inp

    if args.copy_reference:
        # out = src + 1 over 64 Mi float32: reads 256 MiB and writes 256 MiB per launch
        n = 64 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_reference": "torch.add(src, 1.0, out=dst)", "launches": args.steps,
                          "read_bytes_per_launch": 4 * n, "write_bytes_per_launch": 4 * n}))
        return

    if args.fill_reference:
        # what the device's memory absorbs from the plainest write stream, at the output sizes of the
        # measured workloads: the library's sequential fill (16-byte non-temporal stores; 4, 8, 16 and
        # 64 KiB per workgroup), torch's fill_ and torch's zero_ (a memset)
        rows = []
        for nbytes in (85 << 20, 268435456, 342360064, 1 << 30, 1681915904, 8 << 30, 34401681408):
            buf = torch.empty(nbytes // 4, dtype=torch.float32, device=dev)
            reps = max(3, min(args.steps, int(2e11 // nbytes)))
            rec = {"bytes": nbytes, "launches": reps}
            for name, fn in (("pfg_fill_4KiB_per_wg", lambda: pfg.pfg_fill_reference(buf, 1.0, 1)),
                             ("pfg_fill_8KiB_per_wg", lambda: pfg.pfg_fill_reference(buf, 1.0, 2)),
                             ("pfg_fill_16KiB_per_wg", lambda: pfg.pfg_fill_reference(buf, 1.0, 4)),
                             ("pfg_fill_64KiB_per_wg", lambda: pfg.pfg_fill_reference(buf, 1.0, 16)),
                             ("torch_fill_", lambda: buf.fill_(1.0)), ("torch_zero_", lambda: buf.zero_())):
                for _ in range(2):
                    fn()
                start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                best, total = float("inf"), 0.0
                for _ in range(reps):
                    start.record()
                    fn()
                    stop.record()
                    stop.synchronize()
                    ms = start.elapsed_time(stop)
                    best, total = min(best, ms), total + ms
                rec[name] = {"avg_GBps": nbytes * reps / total / 1e6, "best_GBps": nbytes / best / 1e6,
                             "avg_us": total / reps * 1e3, "timed_by": "events around the launch"}
                if name.startswith("pfg_"):
                    # the kernel's own begin-to-end time, from events attached to the dispatch
                    pfg.pfg_timing_reset()
                    pfg.pfg_timing_enable(True)
                    try:
                        for _ in range(reps):
                            fn()
                        torch.cuda.synchronize()
                    finally:
                        pfg.pfg_timing_enable(False)
                    cnt, ms = pfg.pfg_timing_query("fill_reference")
                    pfg.pfg_timing_reset()
                    rec[name] = {"avg_GBps": nbytes * cnt / ms / 1e6, "avg_us": ms / cnt * 1e3,
                                 "timed_by": "events attached to the dispatch"}
            log(f"[bench] fill {nbytes / 1e6:.0f} MB: " + ", ".join(
                f"{k} {v['avg_GBps']:.0f} GB/s" for k, v in rec.items() if isinstance(v, dict)))
            rows.append(rec)
            del buf
            torch.cuda.empty_cache()
        print(json.dumps({"fill_reference": rows, "hbm_peak_GBps": HBM_PEAK_GBS}), flush=True)
        return

    if args.launch_floor:
        # what a chain of dependent launches costs when the kernels do next to nothing: the library's
        # fill kernel on 4 KiB (one workgroup), launched back to back on one stream, eagerly and
        # replayed from a graph; and the same with one workgroup per compute unit (256 x 4 KiB)
        rows = []
        for nfloats in (1024, 256 * 1024):
            buf = torch.empty(nfloats, dtype=torch.float32, device=dev)
            chain = 100
            one = lambda: pfg.pfg_fill_reference(buf, 1.0, 1)
            def step():
                for _ in range(chain):
                    one()
            sec = timed(step, max(20, args.steps), 5)
            sec_graph = timed_graph(step, max(20, args.steps), 5)
            kt = kernel_times(step, 20)["fill_reference"]
            rows.append({"bytes_per_launch": 4 * nfloats, "chain": chain, "us_per_launch_eager": sec / chain * 1e6,
                         "us_per_launch_graph": sec_graph / chain * 1e6,
                         "kernel_us": kt["ms_per_step"] / kt["launches_per_step"] * 1e3})
            log(f"[bench] launch floor, {4 * nfloats} B per launch: {rows[-1]['us_per_launch_eager']:.2f} us eager, "
                f"{rows[-1]['us_per_launch_graph']:.2f} us from a graph, kernel itself {rows[-1]['kernel_us']:.2f} us")
        print(json.dumps({"launch_floor": rows}), flush=True)
        return

    if args.workload:
        fn = measure if args.workload in wl.WORKLOADS else measure_lstm
        rec, _ = fn(args.workload, args.steps, args.warmup)
        print(json.dumps(rec), flush=True)
        return

    # The headline is the largest configuration that fits one GPU: c4 (4096-4096-4096-10, GELU, bf16
    # inputs and weights, float32 accumulation and output, batch 256, 34.4 GB written per step).
    primary = "c4_gelu_bf16_grads"
    rec, inp = measure(primary, args.steps, args.warmup)
    detail = {primary: rec}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        w = wl.WORKLOADS[primary]
        onet = oracle.Net(inp.Ws, inp.bs, w.act)
        cores = oracle.num_threads()
        n_sub = min(w.B, max(8, cores))           # one example per thread and pass; ~0.5 GB of float64 each
        log(f"[bench] cpu_baseline: float64 oracle on the first {n_sub} examples of {primary}")
        oracle.per_example_grads(onet, inp.X[:1], inp.labels[:1])     # load / page in
        passes, t_cpu = 0, 0.0
        while passes < 2 or (t_cpu < 12.0 and passes < 2000):
            t0 = time.perf_counter()
            out = oracle.per_example_grads(onet, inp.X[:n_sub], inp.labels[:n_sub])
            t_cpu += time.perf_counter() - t0
            del out
            passes += 1
        cpu = {"value": n_sub * passes / t_cpu, "unit": "grads/s", "cores": cores, "kind": "oracle",
               "sample": f"{passes} passes over the first {n_sub} of {w.B} examples of {primary} "
                         f"(float64, OpenMP over examples, gradients kept in host memory, no "
                         f"comparison or copies timed), {t_cpu:.1f} s wall"}
        log(f"[bench] cpu_baseline: {cpu['value']:.2f} grads/s on {cores} threads")

    failed = []
    if not args.only_primary:
        for name, steps in (("c2_mnist_mlp_grads", max(20, args.steps * 10)),
                            ("c5_nested_weight_jacobian", max(20, args.steps * 10)),
                            ("c3_tanh_jacobian", max(3, args.steps)),
                            ("c2_mnist_mlp_grad_norms", max(20, args.steps * 10)),
                            ("c4_gelu_bf16_grad_norms", max(3, args.steps * 2)),
                            ("c6_tanh_hessian", max(3, args.steps)),
                            ("c7_lstm_grads", max(3, args.steps * 5)),
                            ("c7_lstm_grad_norms", max(3, args.steps * 5)),
                            ("c8_lstm_jacobian", max(3, args.steps)),
                            ("c9_lstm_varlen", max(3, args.steps)),
                            ("c12_lstm_while", max(3, args.steps)),
                            ("c14_lstm_while_grads", max(3, args.steps)),
                            ("c14_lstm_while_grad_norms", max(3, args.steps)),
                            ("c10_mnist_convnet_grads", max(3, args.steps)),
                            ("c10_mnist_convnet_grad_norms", max(3, args.steps)),
                            ("c11_cond_two_branches", max(3, args.steps * 2)),
                            ("c13_cond_grads", max(3, args.steps))):
            try:
                fn = measure if name in wl.WORKLOADS else measure_lstm
                timing_passes["n"] = 2
                detail[name], _ = fn(name, steps, max(1, min(max(args.warmup, 10), steps // 2)))
                detail[name]["timing"] = "fastest of 2 passes of `steps` steps"
            except Exception as e:
                log(f"[bench] {name}: FAILED: {e}")
                detail[name] = {"error": str(e)}
                failed.append(name)
            torch.cuda.empty_cache()

    # The full records (per-kernel tables of every workload) go to a file and, one workload a line,
    # to stderr; the last line of stdout is the compact headline record.
    detail_file = args.detail_file if os.path.isabs(args.detail_file) else os.path.join(ROOT, args.detail_file)
    try:
        os.makedirs(os.path.dirname(detail_file), exist_ok=True)
        with open(detail_file, "w") as f:
            json.dump(detail, f, indent=1)
    except OSError as e:
        log(f"[bench] detail file not written: {e}")
    for name, r in detail.items():
        log("[bench-detail] " + json.dumps({name: r}))

    def brief(r):
        if "error" in r:
            return {"error": r["error"][:80]}
        b = {"ms_per_step": round(r["ms_per_step"], 5), "frac": round(r["roofline"]["frac"], 4),
             "bound": r["roofline"]["bound"]}
        for key in ("per_example_grads_per_sec", "jacobian_entries_per_sec", "jacobian_rows_per_sec"):
            if key in r:
                b[key] = float(f"{r[key]:.4g}")
        return b

    w = wl.WORKLOADS[primary]
    roof = rec["roofline"]
    line = {
        "metric": "per_example_grads_per_sec", "value": rec["per_example_grads_per_sec"],
        "unit": "grads/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 in / f32 acc", "data": "synthetic",
        "config": {"workload": primary, "call": w.call, "dims": list(w.dims), "act": w.act,
                   "batch": w.B, "output_GB_per_step": round(rec["output_GB"], 3)},
        "roofline": {"kernel": roof["kernel"], "bound": roof["bound"], "achieved": roof["achieved"],
                     "peak": roof["peak"], "unit": roof["unit"], "frac": roof["frac"],
                     "traffic": roof["traffic"],
                     "traffic_source": None if roof["traffic"] is None else
                     "stored rocprofv3 counters (profiles/outer_product_hbm_traffic.txt), not re-measured in this run",
                     "bytes_per_launch": roof["bytes_per_launch"], "ms_per_launch": roof["ms_per_launch"],
                     "scope": "kernel only (HIP events around the dispatch); the whole step is ms_per_step"},
        "cpu_baseline": cpu,
        "whole_step_hbm_frac": rec["output_GB"] / (rec["ms_per_step"] * 1e-3) / HBM_PEAK_GBS,
        "other_configs": {k: brief(detail[k]) for k in ("c2_mnist_mlp_grads", "c3_tanh_jacobian",
                                                         "c5_nested_weight_jacobian") if k in detail},
        "detail": args.detail_file + " and the [bench-detail] lines on stderr",
    }
    text = json.dumps(line)
    for key in ("detail", "other_configs", "whole_step_hbm_frac"):      # the record must stay under 2 KB
        if len(text) < 2048:
            break
        line.pop(key, None)
        text = json.dumps(line)
    print(text, flush=True)
    if failed:
        sys.exit(f"bench.py: workloads failed: {', '.join(failed)}")


if __name__ == "__main__":
    main()
