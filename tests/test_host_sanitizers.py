"""The host planner of libhkv under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

csrc/hkv_api.hip (argument validation, cache layout, tile and share tables, budget allocation) is compiled
with the host sanitizers, linked with stand-ins for the kernel launchers and driven by a seeded fuzz
program (tests/host_sanitize/) through the entry points that plan without a device.  Any sanitizer
finding, or any answer that contradicts the header, fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SRC = os.path.join(ROOT, "tests", "host_sanitize")
CSRC = os.path.join(ROOT, "paper_2604_05887_amd", "csrc")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-3000:]}\n{res.stderr[-3000:]}"
    return res


@pytest.mark.skipif(not os.path.exists(HIPCC) or shutil.which("g++") is None, reason="needs hipcc and g++")
def test_host_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    inc = [f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}"]
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]
    common = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-unused-command-line-argument",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    api, stubs, fuzz, exe = (str(tmp_path / n) for n in ("api.o", "stubs.o", "fuzz.o", "fuzz_planner"))
    _run([HIPCC, *common, *san_host, *inc, "-c", os.path.join(CSRC, "hkv_api.hip"), "-o", api])
    _run([HIPCC, *common, "-x", "hip", *san_host, *inc, "-c", os.path.join(SRC, "launcher_stubs.cpp"), "-o", stubs])
    _run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", inc[0],
          "-c", os.path.join(SRC, "fuzz_planner.cpp"), "-o", fuzz])
    _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
          "-Wno-unused-command-line-argument", fuzz, stubs, api, "-o", exe])
    env = dict(os.environ)
    # another preloaded library may come first in the link order; leak checking would report the HIP runtime's own start-up
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    for seed in ("0", "12345"):
        res = _run([exe, "250", seed], env=env, timeout=300)
        assert "no finding" in res.stdout, res.stdout
