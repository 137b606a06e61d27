"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, on
the CPU): adr_oracle.c is built with -fsanitize=address,undefined and the whole pin suite plus
the stored tiny case run against that build in a child process.  Any out-of-bounds access,
use of freed memory, signed overflow or misaligned access in the oracle aborts the child.

That the leg bites is tested too: a copy of the source whose score buffer is one element short
passes every arithmetic pin in an ordinary build's terms, and must be stopped by the sanitizer."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adr_oracle.c")
SAN_FLAGS = ["-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-fno-omit-frame-pointer",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def runtime_library():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def run_pins(so, files):
    asan = runtime_library()
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    # (-s: a sanitizer report is written as the process dies, past pytest's own capture)
    # the sanitizer's runtime has to be in the process before the interpreter starts; whatever is
    # preloaded already stays, behind it
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, ADR_ORACLE_MUTANT=so, LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([sys.executable, "-m", "pytest", *[os.path.join(ROOT, "tests", f) for f in files],
                           "-x", "-q", "-s", "-m", "not gpu", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True,
                          text=True, timeout=900)


def test_pin_suite_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    so = str(tmp_path / "liboracle_san.so")
    subprocess.check_call(["gcc", *SAN_FLAGS, "-o", so, SRC, "-lm"])
    run = run_pins(so, ["test_oracle_pins.py", "test_golden.py"])
    report = run.stdout[-1500:] + run.stderr[-1500:]
    assert run.returncode == 0, report
    assert "AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr, report
    assert " passed" in run.stdout


def test_the_sanitizer_stops_a_planted_overrun(tmp_path):
    text = open(SRC).read()
    old = "(size_t)(max_L > 0 ? max_L : 1));"
    assert text.count(old) == 1, "the oracle's source no longer contains the line this case edits"
    c_file = tmp_path / "short_buffer.c"
    c_file.write_text(text.replace(old, "(size_t)(max_L > 1 ? max_L - 1 : 1));"))
    so = str(tmp_path / "libshort.so")
    subprocess.check_call(["gcc", *SAN_FLAGS, "-o", so, str(c_file), "-lm"])
    run = run_pins(so, ["test_oracle_pins.py"])
    assert run.returncode != 0, "a one-element heap overrun in the oracle went unnoticed"
    assert "AddressSanitizer" in run.stderr + run.stdout, (run.stdout[-800:], run.stderr[-800:])
