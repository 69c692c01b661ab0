"""Host code of the library and the C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Every source of the library is compiled for the host alone (no device code is generated, so this takes seconds)
with both sanitizers, linked with the sanitized C oracle and tests/host_sanitize_driver.cpp into one executable, and
run: edge and random shapes through descriptor validation, tile enumeration, ranking and the per-process tile table
(also from 8 threads at once), random and malformed loop nests through the working-set analysis, malformed
descriptors and tiles through every entry point that must refuse them before touching the device, and the oracle on
exactly-sized buffers.  A sanitizer report aborts the run (halt_on_error), which fails the test."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2002_02145_amd", "csrc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{err}"


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc for the host pass of the .hip sources")
def test_host_code_under_address_and_undefined_sanitizers(tmp_path):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    clang = os.path.join(rocm, "llvm", "bin", "clang")
    srcs = sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        _run(["hipcc", "-x", "hip", "--cuda-host-only", "-c", os.path.join(CSRC, src), "-o", obj, "-O1", "-g",
              "-fno-omit-frame-pointer", "-std=c++17", "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC] + host_san)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, srcs))
    oracle_obj = str(tmp_path / "conv_oracle.o")
    _run([clang, "-c", os.path.join(ROOT, "oracle", "conv_oracle.c"), "-o", oracle_obj, "-O1", "-g", "-std=c99",
          "-fno-omit-frame-pointer"] + SAN)
    driver_obj = str(tmp_path / "driver.o")
    _run([clang + "++", "-c", os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), "-o", driver_obj, "-O1", "-g",
          "-std=c++17", "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include")] + SAN)
    exe = str(tmp_path / "host_sanitize_driver")
    # no HIP runtime is linked: the driver answers the few runtime entry points itself, and the handles of the
    # (absent) device code objects stay unresolved
    _run([clang + "++", "-o", exe, driver_obj, oracle_obj] + objs + SAN +
         ["-lpthread", "-lm", "-Wl,--unresolved-symbols=ignore-all"])
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "halt_on_error=1:abort_on_error=0:detect_leaks=1:strict_string_checks=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(r.stdout[-2000:])
    assert r.returncode == 0, f"driver exit {r.returncode}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    assert "host sanitizer driver: 0 errors" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
