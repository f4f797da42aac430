"""Build libcrope.so (HIP, gfx950) in-tree with hipcc.  No torch extension machinery: the
library is a plain C-ABI shared object loaded with ctypes."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcrope.so")
SOURCES = ["crope_api.hip", "rope.hip", "attention.hip", "project.hip"]
# measurement aids of bench.py (an MFMA-only loop and a plain copy): a library of their own,
# so that nothing in libcrope.so exists only for the benchmark
CEILINGS_LIB = os.path.join(HERE, "libcrope_ceilings.so")
CEILINGS_SOURCE = "ceilings.hip"
# issue-level microbenchmark (a standalone executable): the instruction-rate figures quoted for the
# attention kernel's design come from it
ISSUE_BENCH = os.path.join(HERE, "issue_bench")
ISSUE_BENCH_SOURCE = "issue_bench.hip"
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(CEILINGS_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(CEILINGS_LIB))
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))] + \
           [os.path.join(HERE, "..", "include", "crope.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    objs = []
    procs = []
    cmd = ["hipcc", *FLAGS, "-shared", os.path.join(CSRC, CEILINGS_SOURCE), "-o", CEILINGS_LIB + ".tmp"]
    procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    cmd = ["hipcc", *[f for f in FLAGS if f not in ("-fPIC", "-fvisibility=hidden")],
           os.path.join(CSRC, ISSUE_BENCH_SOURCE), "-o", ISSUE_BENCH]
    procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    # link against libamdhip64 by soname only (no rpath): inside a torch process the
    # already-loaded runtime is used.
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB + ".tmp"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    os.replace(CEILINGS_LIB + ".tmp", CEILINGS_LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
