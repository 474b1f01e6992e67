"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer: a subset of the oracle pins
and of the host-side library checks runs in a child process that loads the instrumented build of
``oracle/vecinfer_oracle.c`` (the sanitizer runtime preloaded), so an out-of-bounds access or
undefined arithmetic anywhere on those paths aborts the child instead of passing silently."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# pins that between them reach every exported function of the C file
SUBSET = ("hadamard or smoothing or transform or encode or dequant or decode_attention or alg1 or merge or "
          "residual or kmeans or pack or wide or general")


def test_oracle_pins_under_asan_ubsan():
    lib = oracle.oracle.build_sanitized(force=True)
    assert os.path.exists(lib)
    env = dict(os.environ)
    env["VECINFER_ORACLE_SANITIZED"] = "1"
    pre = [oracle.oracle.sanitizer_runtime()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    # the interpreter itself is not instrumented: no leak check at exit, no link-order check
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "1"
    cmd = [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
           "-p", "no:cacheprovider", "-k", SUBSET]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    # the child really ran on the instrumented library
    probe = subprocess.run([sys.executable, "-c",
                            "import oracle, ctypes; oracle.hadamard(4); "
                            "print(open('/proc/self/maps').read().count('libvecinfer_oracle_san.so') > 0)"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert probe.returncode == 0 and probe.stdout.strip().endswith("True"), probe.stdout + probe.stderr
