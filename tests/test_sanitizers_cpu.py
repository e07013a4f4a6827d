"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code, run on the CPU only:
the C oracle (all entry points, edge paths) and the host side of the C ABI (argument validation, bin heuristics,
workspace layout arithmetic).  Nothing here touches a GPU; device code is never sanitized."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    return r.returncode, r.stdout + r.stderr


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_oracle")
    rc, out = run(["gcc", "-O1", "-g", "-std=gnu11", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
                   "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", exe,
                   os.path.join(HERE, "sanitize_oracle_main.c"), os.path.join(ROOT, "oracle", "knn_oracle.c"),
                   os.path.join(ROOT, "oracle", "oc_helper_oracle.c"), "-lm"])
    assert rc == 0, out
    rc, out = run([exe], env=ENV)
    assert rc == 0 and "failures=0" in out and "runtime error" not in out and "AddressSanitizer" not in out, out


def test_host_side_of_the_abi_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    from paper_2511_10442_amd import build as hip_build
    hip_build.build()                                   # the other translation units, as built for the library
    objs = [o for _, o, _ in hip_build.units() if not o.endswith("fg_api.o")]
    api = str(tmp_path / "fg_api_san.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    rc, out = run([hipcc, *hip_build.FLAGS, "-O1", "-g", *san, "-c", os.path.join(hip_build.CSRC, "fg_api.hip"), "-o", api])
    assert rc == 0, out
    drv = str(tmp_path / "drv.o")
    rc, out = run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                   "-I", os.path.join(ROOT, "include"), "-c", os.path.join(HERE, "sanitize_abi_main.c"), "-o", drv])
    assert rc == 0, out
    exe = str(tmp_path / "sanitize_abi")
    rc, out = run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                   "-o", exe, api, drv, *objs])
    assert rc == 0, out
    rc, out = run([exe], env=ENV)
    assert rc == 0 and "bad=0" in out and "runtime error" not in out and "AddressSanitizer" not in out, out
