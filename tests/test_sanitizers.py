"""CPU sanitizer leg: the oracle (every pin of it) and the library's host-side argument checks run once more
against builds with AddressSanitizer and UndefinedBehaviorSanitizer (host code only; the device code of the
library is compiled as always and never runs here).  Each run is a child process with the matching ASan runtime
preloaded in front of whatever is preloaded already; a finding aborts the child, which fails the test."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_PINS = ["test_oracle_scoring.py", "test_oracle_update.py", "test_oracle_lstm.py", "test_oracle_trigger.py",
               "test_oracle_transfer.py", "test_oracle_workers_and_grids.py", "test_oracle_layer_counts.py",
               "test_oracle_independent_pins.py"]


def _run_pytest_child(files, env_extra, runtime):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = runtime + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    # Python itself is not instrumented: its allocations at exit are not leaks of ours, and something else may be
    # preloaded in front of the runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", f) for f in files]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    return res.stdout


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    from oracle import oracle as orc
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no ASan runtime here")
    lib = orc.build_sanitized()
    out = _run_pytest_child(ORACLE_PINS, {"AUTOBYTE_ORACLE_LIB": lib}, os.path.realpath(runtime))
    print(out.strip().splitlines()[-1])


def test_host_side_argument_checks_under_sanitizers():
    from paper_2112_13509_amd import build as b
    hipcc_dir = os.path.dirname(os.path.realpath(b.HIPCC))
    cands = glob.glob(os.path.join(hipcc_dir, "..", "lib", "llvm", "lib", "clang", "*", "lib", "linux",
                                   "libclang_rt.asan-x86_64.so")) + \
        glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not cands:
        pytest.skip("the HIP compiler ships no ASan runtime here")
    lib = b.build_host_sanitized()
    out = _run_pytest_child(["test_abi_host.py"], {"AUTOBYTE_LIB": lib}, os.path.realpath(cands[0]))
    print(out.strip().splitlines()[-1])
