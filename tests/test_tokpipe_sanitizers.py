"""The tokenization pipeline under AddressSanitizer + UndefinedBehaviorSanitizer and under
ThreadSanitizer: csrc/tokpipe.cpp is rebuilt with the sanitizers, linked with
tests/tokpipe_sanitize_driver.c, and the driver - several pipeline shapes over one synthetic corpus, the
reader, the error paths - has to run clean.  CPU only."""
import os
import subprocess

import pytest

from synth import text as st

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2602_08387_amd", "csrc", "tokpipe.cpp")
DRIVER = os.path.join(ROOT, "tests", "tokpipe_sanitize_driver.c")


@pytest.mark.parametrize("name,flags,env", [
    ("asan_ubsan", ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"],
     {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"}),
    ("tsan", ["-fsanitize=thread"], {"TSAN_OPTIONS": "halt_on_error=1"}),
])
def test_pipeline_runs_clean_under_sanitizers(tmp_path, name, flags, env):
    corpus = tmp_path / "corpus.jsonl"
    corpus.write_bytes(st.make_jsonl(7, 300, n_words=800, median_doc_words=60))
    obj, drv, exe = (str(tmp_path / n) for n in ("tokpipe.o", "driver.o", "driver"))
    for cmd in (["g++", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer", *flags, "-c", SRC, "-o", obj],
                ["gcc", "-O1", "-g", *flags, "-c", DRIVER, "-o", drv],
                ["g++", *flags, obj, drv, "-pthread", "-o", exe]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe, str(corpus), str(tmp_path)], capture_output=True, text=True, env=dict(os.environ, **env), timeout=300)
    if name == "tsan" and "unexpected memory mapping" in r.stderr:
        pytest.skip("ThreadSanitizer cannot run under this kernel's address-space layout")
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-3000:])
    assert "all runs agree" in r.stdout
    for word in ("runtime error", "AddressSanitizer", "LeakSanitizer", "ThreadSanitizer"):
        assert word not in r.stderr, r.stderr[-3000:]
