"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The oracle is the yardstick for every GPU result, so its own memory accesses and arithmetic
are checked too: its source is built with -fsanitize=address,undefined (any report aborts)
and the pin tests run against that build in a fresh process.  A copy with a planted read one
entry past the allocation table must fail the same way, which shows that the sanitizer is
really in the loop."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "fdy_oracle.cpp")
PINS = ["test_oracle_scan.py", "test_oracle_fingerprint.py", "test_oracle_materialize.py", "test_oracle_derive.py"]


def asan_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def build(src_text, out_dir, name):
    cpp = os.path.join(out_dir, name + ".cpp")
    lib = os.path.join(out_dir, name + ".so")
    with open(cpp, "w") as f:
        f.write(src_text)
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", cpp, "-o", lib])
    return lib


def run_pins(lib, runtime, files):
    # the sanitizer runtime has to be loaded before the interpreter's own allocations; leak
    # checking is off because the interpreter itself never frees everything
    env = dict(os.environ, FDY_ORACLE_LIB=lib, LD_PRELOAD=runtime,
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1")
    # -s: a report must reach this process's pipe, not a capture file that dies with the child
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider"] + [
        os.path.join(ROOT, "tests", f) for f in files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode, r.stdout + r.stderr


def test_pins_pass_under_the_sanitizers(tmp_path):
    runtime = asan_runtime()
    if runtime is None:
        pytest.skip("no AddressSanitizer runtime with this compiler")
    lib = build(open(SRC).read(), str(tmp_path), "sanitized")
    rc, text = run_pins(lib, runtime, PINS)
    assert rc == 0, text[-2000:]


def test_a_planted_out_of_bounds_read_is_reported(tmp_path):
    runtime = asan_runtime()
    if runtime is None:
        pytest.skip("no AddressSanitizer runtime with this compiler")
    src = open(SRC).read()
    old = "for (uint32_t i = 0; i < n_alloc; ++i)\n      if (w >= table[i].base && w - table[i].base < table[i].size) hit = i;"
    assert src.count(old) == 1
    new = old.replace("i < n_alloc", "i <= n_alloc")  # reads one entry past the table
    lib = build(src.replace(old, new), str(tmp_path), "planted")
    rc, text = run_pins(lib, runtime, ["test_oracle_scan.py"])
    assert rc != 0 and "AddressSanitizer" in text
