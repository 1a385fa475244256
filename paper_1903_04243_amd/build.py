"""Build libpfg.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpfg.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["gemm.hip", "gemm_skinny.hip", "gemm_small16.hip", "gemm_shortk.hip", "writer.hip", "elementwise.hip", "lstm.hip", "conv.hip", "conv_mfma.hip", "cond.hip", "loop.hip", "head.hip", "pfg.hip",
           "pfg_lstm.hip", "pfg_cond.hip"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(CSRC, "gemm_device.h"),
           os.path.join(CSRC, "host.h"), os.path.join(os.path.dirname(HERE), "include", "pfg.h")]
# packed-fp32 arithmetic is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage",
         # an array indexed at run time must show up as scratch (and be refused below), not be moved
         # silently into LDS, which costs a read of the dispatch packet at every kernel start
         "-mllvm", "-disable-promote-alloca-to-lds"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    jobs = []
    objs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + HEADERS):
            jobs.append([hipcc] + FLAGS + ["-c", s, "-o", o])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
        # A kernel that needs scratch memory (an array indexed at run time, or register spills) pays
        # for it on every launch, which the latency-bound kernels here cannot afford: refuse it.
        name, bad = None, []
        for line in r.stderr.splitlines():
            if "Function Name:" in line:
                name = line.split("Function Name:")[1].split("[")[0].strip()
            elif "ScratchSize [bytes/lane]:" in line:
                size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
                if size:
                    bad.append(f"{name}: {size} bytes of scratch per lane")
        if bad:
            out = cmd[-1]
            if os.path.exists(out) and out.endswith(".o"):
                os.remove(out)
            raise RuntimeError("kernels that use scratch memory in " + cmd[-3] + ":\n" + "\n".join(bad))

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    if force or jobs or _stale(LIB, objs):
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
