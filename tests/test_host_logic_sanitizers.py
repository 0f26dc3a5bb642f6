"""The library's host logic (descriptor validation, workspace layout, the planner of merged dispatches,
launch shapes, the selector) built with AddressSanitizer and UndefinedBehaviorSanitizer on the host side
and driven, without a GPU, over the benchmark chains at every batch bucket and segment cut and over
thousands of random descriptors, a quarter of them damaged: an out-of-bounds access, a signed overflow
or a planner that stops making progress ends the driver with a report, a non-zero status or a timeout.
Only chain.hip is rebuilt with the sanitizers; the kernels' host-side tables come from the in-tree library."""
import os
import subprocess

from paper_2503_19779_amd.build import FLAGS, LIB, build_library

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
       "-Xarch_host", "-fno-omit-frame-pointer"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout + res.stderr
    return res


def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    build_library(force=False)
    common = [f for f in FLAGS if f not in ("-shared", "-fPIC", "-O3")] + ["-O1", "-g"] + SAN
    chain_o, drv_o, exe = str(tmp_path / "chain.o"), str(tmp_path / "driver.o"), str(tmp_path / "host_logic_sanitized")
    _run([HIPCC] + common + ["-c", "-o", chain_o, os.path.join(ROOT, "paper_2503_19779_amd", "csrc", "chain.hip")])
    _run([HIPCC] + common + ["-c", "-x", "hip", "-o", drv_o, os.path.join(HERE, "host_logic_sanitizer_driver.cpp")])
    _run([HIPCC, "--offload-arch=gfx950", "--hip-link", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, drv_o, chain_o,
          LIB, "-Wl,-rpath," + os.path.dirname(LIB)])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=240)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host logic sanitizer driver: ok" in res.stdout
