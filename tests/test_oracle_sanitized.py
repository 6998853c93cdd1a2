"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): ref_stream.c is built
with -fsanitize=address,undefined and the oracle's own pins are run against that build in a child process.
An out-of-bounds read in the checker would otherwise show up as a wrong expected value, or not at all."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ref_stream.c")


def test_ref_stream_pins_under_asan_ubsan(tmp_path):
    lib = str(tmp_path / "libref_stream_san.so")
    cc = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-fopenmp", "-fPIC", "-shared", "-std=c11", SRC, "-o", lib, "-lm"]
    r = subprocess.run(cc, capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("this compiler cannot build with -fsanitize=address,undefined: " + r.stderr[-300:])
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("no libasan runtime next to this compiler")
    env = dict(os.environ)
    # the sanitizer runtime has to be loaded before the (uninstrumented) interpreter's other libraries;
    # anything already preloaded stays preloaded behind it
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    env["REF_STREAM_LIB"] = lib
    env["OMP_NUM_THREADS"] = "4"
    child = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                            os.path.join(ROOT, "tests", "test_block_pins.py")],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=1200)
    out = child.stdout + child.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-3000:]
    assert child.returncode == 0, out[-3000:]
    assert " passed" in out
    # the child really ran the instrumented build
    probe = subprocess.run([sys.executable, "-c",
                            "from oracle import ref_stream as r; r._load(); import sys; "
                            "sys.exit(0 if 'libref_stream_san' in open('/proc/self/maps').read() else 1)"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0, probe.stderr[-2000:]
