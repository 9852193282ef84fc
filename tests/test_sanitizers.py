"""The oracle and the input generator under AddressSanitizer and UndefinedBehaviorSanitizer.

Both are built on the CPU with -fsanitize=address,undefined and the oracle's pin tests and the
generator's tests run against those builds in a subprocess (the mechanism of the mutation test):
an out-of-bounds access, a use after free, a signed overflow or a misaligned access anywhere
on the paths the pins exercise aborts the subprocess.
"""
import os
import subprocess
import sys

import oracle
from paper_2009_06693_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = ["tests/test_oracle_primitives.py", "tests/test_oracle_walks.py", "tests/test_oracle_khop_layer.py",
         "tests/test_oracle_edges.py", "tests/test_oracle_formats.py", "tests/test_inputs.py"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True,
                          check=True).stdout.strip()
    assert os.path.isabs(path) and os.path.exists(path), f"{name} not found next to gcc"
    return path


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    olib, glib = str(tmp_path / "oracle_san.so"), str(tmp_path / "graphgen_san.so")
    oracle.compile_oracle(os.path.join(ROOT, "oracle", "nd_oracle.c"), olib, sanitize=True)
    inputs.compile_generator(glib, sanitize=True)
    # the sanitizer runtime has to come first; whatever is preloaded already stays behind it
    preload = " ".join(x for x in (_runtime("libasan.so"), os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, ND_ORACLE_LIB=olib, ND_GRAPHGEN_LIB=glib, LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *TESTS]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout[-3000:] + r.stderr[-3000:])
    assert "passed" in r.stdout
