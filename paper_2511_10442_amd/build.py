"""Build libfastgraph_hip.so for gfx950 with hipcc (in-tree, next to this file).

    python -m paper_2511_10442_amd.build [--force]

Flags that matter for correctness:
  -ffp-contract=off   squared distances are sums of individually rounded float32 operations;
                      a fused multiply-add would change their last bit
  -Xclang -target-feature -Xclang -packed-fp32-ops   no packed float32 instructions
  -munsafe-fp-atomics hardware float32 atomic add in the backward kernel
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfastgraph_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-munsafe-fp-atomics", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", os.path.join(ROOT, "include"), "-I", CSRC]

QUERY_DIMS = range(2, 11)


def units():
    """(source, object, extra flags)"""
    out = [(os.path.join(CSRC, f + ".hip"), os.path.join(OBJ, f + ".o"), [])
           for f in ("fg_api", "fg_binning", "fg_backward", "fg_oc_helper")]
    for d in QUERY_DIMS:
        out.append((os.path.join(CSRC, "fg_query_inst.hip"), os.path.join(OBJ, "fg_query_d%d.o" % d),
                    ["-DFG_QUERY_D=%d" % d]))
    return out


def _newest_header() -> float:
    t = os.path.getmtime(os.path.join(ROOT, "include", "fastgraph.h"))
    for f in os.listdir(CSRC):
        if f.endswith(".hpp"):
            t = max(t, os.path.getmtime(os.path.join(CSRC, f)))
    return max(t, os.path.getmtime(os.path.abspath(__file__)))


def _compile(job):
    src, obj, extra = job
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l)          # host pass does not know the feature: harmless
    return r.returncode, obj, msgs


def build(force: bool = False, jobs: int | None = None, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()
    todo = []
    for src, obj, extra in units():
        stale = (not os.path.exists(obj)) or os.path.getmtime(obj) < max(os.path.getmtime(src), hdr)
        if force or stale:
            todo.append((src, obj, extra))
    if todo:
        jobs = jobs or min(8, os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "8")))
        with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
            for rc, obj, msgs in ex.map(_compile, todo):
                if verbose or rc != 0:
                    print(os.path.basename(obj), "rc=%d" % rc)
                    if msgs.strip():
                        print(msgs)
                if rc != 0:
                    raise RuntimeError("hipcc failed for %s" % obj)
    objs = [u[1] for u in units()]
    if todo or not os.path.exists(LIB):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
