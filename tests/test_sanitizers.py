"""Host-side sanitizer runs (CPU only).

The C oracle is rebuilt with -fsanitize=address,undefined and the suite that
pins it runs against that build in a child process (the sanitizer runtime has to
be preloaded into the interpreter); any finding aborts the child.  The host half
of the device library (argument checks, model bookkeeping, workspace layout) is
built the same way with hipcc (-Xarch_host -fsanitize=...) and the boundary
tests that need no GPU run against it.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _preload(env, runtime):
    old = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + old if old else "")
    # leaks: the interpreter's own; link order: other preloaded libraries may come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return env


def _run(cmd, env):
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    return r.stdout


def test_oracle_pins_hold_under_address_and_ub_sanitizers():
    from oracle import rec_oracle as orc
    orc.build_sanitized(force=True)
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(runtime):
        pytest.skip("gcc has no libasan here")
    env = _preload(dict(os.environ), runtime)
    env[orc.SANITIZE_ENV] = "1"
    which = _run([sys.executable, "-c", "from oracle import rec_oracle as o; print(o.lib()._name)"], env)
    assert which.strip().endswith("librec_oracle_san.so"), which
    out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                "tests/test_oracle_pins.py"], env)
    assert " passed" in out and "failed" not in out, out[-2000:]


def test_library_host_code_under_address_and_ub_sanitizers():
    """The device library with instrumented host code: model creation and every
    argument check that needs no GPU (tests/test_abi.py) must run clean."""
    from paper_2203_07424_amd import build
    lib = build.build_host_sanitized()
    runtime = build.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no clang AddressSanitizer runtime here")
    env = _preload(dict(os.environ), runtime)
    env["REC_MI355X_LIBRARY"] = lib
    which = _run([sys.executable, "-c", "from paper_2203_07424_amd import binding as b; print(b._lib._name)"], env)
    assert which.strip().endswith("librec_mi355x_hostsan.so"), which
    out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_abi.py"], env)
    assert " passed" in out and "failed" not in out, out[-2000:]
