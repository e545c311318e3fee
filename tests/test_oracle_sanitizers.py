"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: it is built with
-fsanitize=address,undefined (no recovery: the first finding aborts) and its pin tests are run against
that build in a child process.  An out-of-bounds access, a use of uninitialised stack through a bad
index, a signed overflow or a misaligned access in the oracle would make a parity comparison
meaningless without failing it; here it fails the run.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvq_oracle.c")
PINS = ["tests/test_oracle_quant.py", "tests/test_oracle_fp16_pack.py", "tests/test_oracle_signposts.py",
        "tests/test_oracle_rope_matvec.py", "tests/test_oracle_sink.py"]


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], stdout=subprocess.PIPE, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    so = str(tmp_path / "kvq_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-shared", "-fPIC", "-o", so, SRC,
                    "-lm"], check=True)
    # the interpreter is not instrumented, so the sanitizer runtime has to be loaded first; whatever is
    # already preloaded stays, behind it.  Leak checking is off: the interpreter's own allocations
    # would be reported at exit.
    preload = ":".join(p for p in (asan, os.environ.get("LD_PRELOAD", "")) if p)
    env = dict(os.environ, KVQ_ORACLE_LIB=so, LD_PRELOAD=preload, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *PINS],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "passed" in r.stdout
