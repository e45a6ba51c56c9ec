"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The oracle is the yardstick of every parity test, so its own memory accesses and arithmetic are
checked too: its C source is built with -fsanitize=address,undefined, and every pin module
(attention, sampler, tree, paged cache and commit, distillation rows, greedy, solver) is run
against that build in a child process.  A sanitizer report ends the child with an error
(halt_on_error), which fails this test.  The sanitizer run-time has to be loaded before Python
itself, hence the child process with LD_PRELOAD.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "respec_oracle.c")
PIN_MODULES = ["test_oracle_attention.py", "test_oracle_sampler.py", "test_oracle_tree.py", "test_oracle_paged.py",
               "test_oracle_kd.py", "test_oracle_greedy.py", "test_oracle_solver.py"]


def test_every_pin_passes_on_the_sanitizer_build(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no AddressSanitizer run-time here")
    lib = tmp_path / "librespec_oracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", str(lib), SRC, "-lm"],
                   check=True)
    env = dict(os.environ)
    env.update({
        "RESPEC_ORACLE_LIBRARY": str(lib),
        "LD_PRELOAD": asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else ""),
        # (Python itself is not built for leak checking; the link-order check trips over any
        # other preloaded library)
        "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:abort_on_error=0",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "OMP_NUM_THREADS": "4",
    })
    cmd = [sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", "-m", "not gpu"] + \
          [os.path.join(ROOT, "tests", m) for m in PIN_MODULES]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
