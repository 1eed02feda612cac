"""Build the HIP shared library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librelax_rollout.so")
SOURCES = ["api.hip", "gemm.hip", "elementwise.hip", "attention.hip", "attention_decode.hip", "moe.hip", "sampling.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-Rpass-analysis=kernel-resource-usage"]


def _resource_problems(stderr):
    """Kernels that the compiler gave scratch memory, and loops it declined to unroll, from hipcc's remarks.  Both
    have cost a factor here (accumulators indexed at run time end up in scratch), so the build refuses them."""
    bad, name = [], "?"
    for l in stderr.splitlines():
        if "remark: Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n:
                bad.append("%s uses %d bytes of scratch per lane" % (name, n))
        elif "loop not unrolled" in l:
            bad.append(l.strip())
    return bad


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    bad = _resource_problems(r.stderr)
    # hipcc's host pass does not know the packed-fp32 feature switch and says so; that is harmless.  The resource
    # remarks are read above and not passed on.
    keep, skip = [], 0
    for l in r.stderr.splitlines():
        if "kernel-resource-usage" in l:
            skip = 2                                # the remark's source line and caret follow it
            continue
        if skip and (l.lstrip()[:1].isdigit() or l.lstrip().startswith("|")):
            skip -= 1
            continue
        skip = 0
        if "packed-fp32-ops" not in l:
            keep.append(l)
    err = "\n".join(keep)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, err))
    if bad:
        raise RuntimeError("build refused: %s\n%s" % (" ".join(cmd), "\n".join(bad)))
    if err.strip():
        sys.stderr.write(err + "\n")


def build(force: bool = True, verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "relax_rollout.h")]
    newest = max(os.path.getmtime(p) for p in deps)
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= newest:
        return LIB
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as ex:
        list(ex.map(_run, cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--if-stale" not in sys.argv, verbose=True)
