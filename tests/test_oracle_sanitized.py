"""The oracle's pins once more, in a child process that runs the C oracle built with
-fsanitize=address,undefined: an out-of-bounds read or write, a use after free, a signed overflow
or a misaligned access anywhere in oracle/sparrow_oracle.c on the pins' inputs (empty contexts,
ragged batches, trees, windows larger than the text domain) aborts the child.  The checker itself
has to be memory-safe before its verdicts on the GPU path mean anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_attention.py", "tests/test_oracle_accept.py", "tests/test_oracle_accept_sample.py",
        "tests/test_oracle_accept_sample_q.py",
        "tests/test_oracle_tree.py", "tests/test_oracle_commit.py", "tests/test_oracle_hsr.py"]


def test_oracle_pins_under_address_and_ub_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True,
                          check=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc ships no AddressSanitizer runtime"
    env = dict(os.environ)
    # the sanitizer runtime has to be in the process before the instrumented library is loaded;
    # whatever is preloaded already stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SPARROW_ORACLE_SANITIZE"] = "1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, "sanitized run of the oracle pins failed:\n" + tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    san = os.path.join(ROOT, "oracle", "libsparrow_oracle_san.so")
    assert os.path.exists(san), "the child did not build the sanitized oracle"
    # the instrumented library really carries the sanitizer's checks
    syms = subprocess.run(["nm", "-D", san], capture_output=True, text=True, check=True).stdout
    assert "__asan_report" in syms or "__asan_init" in syms
    assert "__ubsan_handle" in syms
