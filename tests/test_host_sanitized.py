"""The host code of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The host translation unit (configuration checks, permutation tables, block budget, work tables) is
compiled with `-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined` (device code is not
instrumented), linked with the objects of the regular build and a C++ driver that walks every path
that runs without a GPU; any report of either sanitizer fails the test."""
import os
import subprocess

from paper_2512_24086_amd import build as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def test_host_abi_is_clean_under_asan_and_ubsan(tmp_path):
    build_dir = os.path.join(b.PKG, "_build")
    others = [os.path.join(build_dir, os.path.splitext(s)[0] + ".o") for s in b.SOURCES if s != "rf2_plan.cpp"]
    if not all(os.path.exists(o) for o in others):
        b.build(verbose=False)
    plan_o, drv_o, exe = (str(tmp_path / n) for n in ("rf2_plan_san.o", "driver.o", "host_abi_sanitized"))
    subprocess.run([b.hipcc(), *b.FLAGS, *SAN, "-c", os.path.join(b.CSRC, "rf2_plan.cpp"), "-o", plan_o],
                   check=True, capture_output=True)
    subprocess.run([b.hipcc(), *b.FLAGS, *SAN, "-c", os.path.join(ROOT, "tests", "host_abi_sanitized.cpp"), "-o", drv_o],
                   check=True, capture_output=True)
    subprocess.run([b.hipcc(), "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    plan_o, drv_o, *others, "-o", exe], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    out = run.stdout + run.stderr
    assert run.returncode == 0, out[-3000:]
    assert "HOST ABI CHECK PASSED" in run.stdout
    assert "AddressSanitizer" not in out and "runtime error" not in out and "LeakSanitizer" not in out, out[-3000:]
