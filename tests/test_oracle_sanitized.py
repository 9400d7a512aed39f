"""The oracle's pins, and the host-only paths of the C ABI, once more over builds with AddressSanitizer
and UndefinedBehaviorSanitizer (host code only, no GPU): an out-of-bounds access, a use after free or
undefined arithmetic anywhere on the paths walked aborts the child process."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_select_weights.py", "test_oracle_round.py", "test_oracle_dtur.py", "test_oracle_grad.py",
             "test_flip_matching.py", "test_inputs.py"]


def test_pins_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = oracle.build_sanitized(str(tmp_path / "liboracle_san.so"))
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ)
    env["DBW_ORACLE_LIB"] = lib
    # the interpreter is not instrumented, so the sanitizer runtime has to come first in the process;
    # whatever is already preloaded stays, after it
    env["LD_PRELOAD"] = ":".join(p for p in (asan, env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           "-k", "not full_shape"] + [os.path.join(ROOT, "tests", f) for f in PIN_FILES]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "liboracle_san" not in r.stderr, tail


def test_abi_host_paths_under_sanitizers(tmp_path):
    """The library's host code (argument checks, graph validation before any allocation, error strings,
    export table) built with the sanitizers, walked by the ABI tests that need no GPU."""
    from paper_2102_06280_amd import build as b
    runtime = b.sanitizer_runtime()
    assert os.path.exists(runtime), runtime
    lib = b.build_sanitized(str(tmp_path / "san"))
    env = dict(os.environ)
    env["DBW_LIB"] = lib
    env["LD_PRELOAD"] = ":".join(p for p in (runtime, env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_abi.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0 and "passed" in r.stdout, tail
