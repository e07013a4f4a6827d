"""The register sorting / merging networks of the query kernel, run on the CPU: the header is
compiled for the host and compared with std::sort on random keys (with many duplicates and with
all-ones sentinels)."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_sorting_networks_on_host():
    src = os.path.join(ROOT, "tests", "sortnet_check.hip")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sortnet_check")
        subprocess.check_call(["/opt/rocm/bin/hipcc", "-O1", "-std=c++17", "--offload-arch=gfx950",
                               "-I", os.path.join(ROOT, "paper_2511_10442_amd", "csrc"), src, "-o", exe],
                              stderr=subprocess.DEVNULL)
        out = subprocess.run([exe], capture_output=True, text=True)
        assert out.returncode == 0 and "OK" in out.stdout, out.stdout + out.stderr
