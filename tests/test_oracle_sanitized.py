"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, gcc): the
same source, built with -fsanitize=address,undefined, must pass the whole pin battery in a child
process that preloads the sanitizer runtime; and the sanitizer must really be watching - a copy of
the source with a planted off-by-one overrun (on the CPU) makes the child die with ASan's report."""
import os
import subprocess
import sys

import pytest

from oracle import pier_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    try:
        path = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _child_env(lib):
    preload = _asan_runtime()
    if os.environ.get("LD_PRELOAD"):
        preload = preload + ":" + os.environ["LD_PRELOAD"]
    return dict(os.environ, LD_PRELOAD=preload, PIER_ORACLE_LIB=lib,
                ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:verify_asan_link_order=0",
                UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


pytestmark = pytest.mark.skipif(_asan_runtime() is None, reason="gcc's AddressSanitizer runtime is not installed")


SAN_FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def build_sanitized(src, lib):
    """The oracle's source with the oracle's own flags (minus -O2) plus the sanitizers."""
    flags = [f for f in O.CFLAGS if f not in ("-O2", "-Wall", "-Wextra")]
    subprocess.check_call(["gcc", *SAN_FLAGS, *flags, "-w", "-o", lib, src, "-lm"])
    return lib


def test_pins_pass_on_the_sanitizer_build(tmp_path):
    lib = build_sanitized(os.path.join(ROOT, "oracle", "pier_oracle.c"), str(tmp_path / "libpier_oracle_san.so"))
    probe = ("from oracle import pier_oracle as O; O.default(); m = open('/proc/self/maps').read(); "
             "assert 'libasan' in m and 'libpier_oracle_san' in m and 'oracle/libpier_oracle.so' not in m")
    subprocess.run([sys.executable, "-c", probe], env=_child_env(lib), cwd=ROOT, check=True, timeout=120)
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       env=_child_env(lib), cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "passed" in r.stdout and "Sanitizer" not in r.stdout + r.stderr


def test_sanitizer_build_notices_a_planted_overrun(tmp_path):
    src = open(os.path.join(ROOT, "oracle", "pier_oracle.c")).read()
    target = "for (int64_t i = 0; i < n; ++i) acc = acc + (double)g[i] * (double)g[i];"
    assert src.count(target) == 1
    bad_c = tmp_path / "overrun.c"
    bad_c.write_text(src.replace(target, target.replace("i < n", "i <= n")))
    lib = build_sanitized(str(bad_c), str(tmp_path / "liboverrun_san.so"))
    code = ("import numpy as np; from oracle import pier_oracle as O; "
            "print(O.sumsq(np.ones(1000, np.float32)))")
    r = subprocess.run([sys.executable, "-c", code], env=_child_env(lib), cwd=ROOT, capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr and "heap-buffer-overflow" in r.stderr, r.stderr[-1500:]
