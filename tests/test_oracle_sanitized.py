"""Host sanitizer leg: the oracle's pins once more, with fusco_oracle.c built under AddressSanitizer and
UndefinedBehaviorSanitizer.  CPU only.  The instrumented library needs the sanitizer runtime loaded before
anything else, so the pins run in a child interpreter that has it preloaded."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_plan.py", "tests/test_oracle_dispatch_combine.py", "tests/test_oracle_segments.py",
             "tests/test_balancer.py"]


def _sanitizer_env():
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    import oracle
    oracle.build(sanitized=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # leaks of the interpreter itself are not the subject; the link-order check would object to libraries
    # that the environment preloads ahead of the runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:exitcode=86"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env[oracle.SANITIZED_ENV] = "1"
    return env


def test_oracle_pins_pass_under_address_and_ub_sanitizers():
    env = _sanitizer_env()
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + PIN_FILES,
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = res.stdout[-3000:]
    assert "AddressSanitizer" not in res.stdout and "runtime error:" not in res.stdout, tail
    assert res.returncode == 0, tail
    assert " passed" in res.stdout, tail


def test_sanitized_oracle_does_catch_an_overrun():
    """The leg has teeth: a destination one row too short for what the oracle is asked to write is reported."""
    env = _sanitizer_env()
    code = (
        "import ctypes, numpy as np, oracle\n"
        "lib = oracle._load()\n"
        "x = np.arange(64, dtype=np.uint8).reshape(4, 16)\n"
        "pl = oracle.plan(np.array([[0], [1], [0], [1]], dtype=np.int32), 2, 2)\n"
        "slots = np.arange(4, dtype=np.int32)\n"
        "short = np.empty((3, 16), dtype=np.uint8)\n"          # four rows are written into room for three
        "p = lambda a: a.ctypes.data_as(ctypes.c_void_p)\n"
        "lib.fusco_oracle_dispatch_rows(p(x), ctypes.c_int64(16), pl.P, p(pl.send_src), p(pl.slot_send_row), p(slots), 4, p(short))\n"
        "print('not caught')\n")
    res = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode != 0 and "AddressSanitizer" in res.stdout and "not caught" not in res.stdout, res.stdout[-2000:]
