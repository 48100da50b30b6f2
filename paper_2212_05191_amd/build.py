"""Build libsmile.so (HIP, gfx950) in-tree with hipcc: one object per source, compiled side by side, then linked."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsmile.so")
PEAKS = os.path.join(HERE, "peaks_probe")
SOURCES = ["smile_api.hip", "gate_logits.hip", "route.hip", "permute.hip", "expert_ffn.hip", "aux_loss.hip",
           "backward.hip", "gemm_transposed.hip", "router_grad_mfma.hip", "static_scratch.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # hipcc -O3 may form packed-fp32 instructions from scalar float code; keep them off
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def sources_to_compile(only, sources, objs, headers):
    """The sources an incremental build compiles: those asked for, plus every source whose object is missing or
    older than the newest header (struct layouts are shared between the objects, so such an object is stale
    whatever the caller asked for).  Names in `only` that are not library sources (the probe) pass through."""
    newest = max((os.path.getmtime(h) for h in headers), default=0.0)
    stale = [s for s, o in zip(sources, objs)
             if s not in only and (not os.path.exists(o) or os.path.getmtime(o) < newest)]
    return list(only) + stale


def build(verbose: bool = False, jobs: int | None = None, only: list[str] | None = None) -> str:
    """Compile every source (always: no staleness check) and link the library and the peak-rate probe.
    only: recompile just these sources (the other objects must exist from an earlier full build) and relink."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    if only is not None:
        headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
        headers += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
        only = sources_to_compile(only, SOURCES, objs, headers)
    cmds = [[hipcc, *FLAGS, *inc, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)
            if only is None or s in only]
    # the stand-alone microbenchmark of the chip's measured peak rates (no library code in it)
    if only is None or "peaks_probe.hip" in only:
        cmds.append([hipcc, *FLAGS, os.path.join(CSRC, "peaks_probe.hip"), "-o", PEAKS])
    jobs = jobs or min(len(cmds), max(1, min(16, os.cpu_count() or 1)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, only=sys.argv[1:] or None))
    sys.exit(0)
