"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer: every source is
rebuilt with the sanitizers on its host code (the device code is compiled as usual), linked with
tests/sanitize_driver.c, and the driver - which only makes calls the argument validation must reject,
plus the size queries - has to run clean.  No GPU is touched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_argument_validation_runs_clean_under_asan_and_ubsan(tmp_path):
    from paper_2602_08387_amd import build as b
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1", "-g"]
    procs, objs = [], []
    for src in b.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen([hipcc, *flags, *san, "-c", os.path.join(b.CSRC, src), "-o", obj],
                                      stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out[-3000:]
    drv = str(tmp_path / "driver.o")
    r = subprocess.run([hipcc, "-x", "c", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        "-c", os.path.join(ROOT, "tests", "sanitize_driver.c"), "-o", drv], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = str(tmp_path / "sanitize_driver")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        *objs, drv, "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "all calls rejected as expected" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
