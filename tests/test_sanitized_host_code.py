"""The CPU oracle and the host-only sequencer built with AddressSanitizer and
UndefinedBehaviorSanitizer (gcc, on the CPU) and driven by small native programs: exact-size heap
buffers for every message length class, long random event streams for the state machine.  The
oracle's tags from the sanitized build must equal the normal build's."""
import os
import shutil
import subprocess
import tempfile

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g",
       "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")


def _build_and_run(compiler, sources, extra):
    if shutil.which(compiler) is None:
        pytest.skip(compiler + " not available")
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "driver")
        build = subprocess.run([compiler] + SAN + extra + sources + ["-o", exe, "-pthread"],
                               stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if build.returncode != 0 and "sanitize" in build.stdout.lower():
            pytest.skip("sanitizer runtime not available: " + build.stdout[-200:])
        assert build.returncode == 0, build.stdout
        run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                             env=ENV, timeout=300)
        assert run.returncode == 0, (run.returncode, run.stderr[-2000:])
        assert "runtime error" not in run.stderr and "ERROR: " not in run.stderr, run.stderr[-2000:]
        return run.stdout


def test_oracle_under_sanitizers_gives_the_same_tags():
    out = _build_and_run("gcc", [os.path.join(NATIVE, "oracle_driver.c"),
                                 os.path.join(ROOT, "oracle", "gcm_oracle.c")], ["-std=c11"])
    lines = out.strip().splitlines()
    assert len(lines) == 3 * 5 * 12
    # replay the driver's generator to get the same inputs for the normal build
    state = [2463534242]

    def next_byte():
        s = state[0]
        s ^= (s << 13) & 0xFFFFFFFF
        s ^= s >> 17
        s ^= (s << 5) & 0xFFFFFFFF
        state[0] = s
        return (s >> 11) & 0xFF

    k = 0
    for key_len in (16, 24, 32):
        for v, iv_len in enumerate((12, 1, 8, 16, 60)):
            for idx, ln in enumerate((0, 1, 15, 16, 17, 31, 32, 33, 100, 1023, 1024, 1025)):
                alen = (idx * 7 + v) % 40
                key = bytes(next_byte() for _ in range(key_len))
                iv = bytes(next_byte() for _ in range(iv_len))
                aad = bytes(next_byte() for _ in range(alen))
                pt = bytes(next_byte() for _ in range(ln))
                _, tag = oracle.encrypt(key, iv, aad, pt)
                assert lines[k] == "%d %d %d %s" % (key_len, iv_len, ln, tag.hex()), lines[k]
                k += 1


def test_sequencer_under_sanitizers():
    out = _build_and_run("g++", [os.path.join(NATIVE, "seq_driver.cpp"),
                                 os.path.join(ROOT, "paper_2411_03357_amd", "csrc", "pgcm_seq.cpp")],
                         ["-std=c++17", "-I" + os.path.join(ROOT, "include")])
    assert out.startswith("actions ") and int(out.split()[1].rstrip(",")) > 100000
    assert out.strip().endswith("iv wrap byte 4")
