"""The ABI's validation and workspace-sizing layer under AddressSanitizer and UndefinedBehaviorSanitizer:
the library is rebuilt with the sanitizers on its HOST code only (device code untouched), linked with
tests/abi_sanitize_driver.c, and the driver's battery of refused calls must run clean.  No GPU needed:
every call in the battery is rejected before anything is enqueued."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_17286_amd", "csrc")
OUT = os.path.join(ROOT, "paper_2506_17286_amd", "_build", "asan")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_validation_layer_is_clean_under_address_and_ub_sanitizers():
    from paper_2506_17286_amd import build as bld
    os.makedirs(OUT, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    objs, procs = [], []
    for src in bld.SOURCES:
        obj = os.path.join(OUT, src.rsplit(".", 1)[0] + ".o")
        objs.append(obj)
        procs.append(subprocess.Popen([HIPCC, *bld.FLAGS, *san, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj],
                                      stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out[-3000:]
    drv = os.path.join(OUT, "driver.o")
    subprocess.run([HIPCC, "-x", "c", "-fno-gpu-sanitize", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g",
                    "-I", os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, "tests", "abi_sanitize_driver.c"),
                    "-o", drv], check=True, capture_output=True, text=True)
    exe = os.path.join(OUT, "abi_sanitize_driver")
    link = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address,undefined", *objs, drv, "-o", exe],
                          capture_output=True, text=True)
    assert link.returncode == 0, link.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "all calls refused as expected" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
