"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Builds the oracle and the C-ABI library a second time, into a temporary directory, with the host
side instrumented (the device code of the library is compiled as usual and never runs here), and
runs the CPU tests of the oracle pins, the residency manager, the per-expert packing and the ABI
surface in a child process that loads those builds.  Any invalid access or undefined operation in
the oracle's loops, the residency state machine, the packing of slot images or the argument
validation ends the child with a sanitizer report.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(900)
def test_cpu_suite_under_asan_and_ubsan(tmp_path):
    if os.environ.get("LD_PRELOAD"):
        pytest.skip("another preload is active in this environment; the sanitizer runtime has to come first")
    from oracle import build as oracle_build
    from paper_2605_13779_amd import build as hip_build
    try:
        runtime = hip_build.sanitizer_runtime()
        cc = hip_build.sanitizer_clang()
    except (OSError, subprocess.CalledProcessError, RuntimeError) as e:
        pytest.skip(f"no clang sanitizer runtime here: {e}")
    if not os.path.exists(runtime):
        pytest.skip("no clang sanitizer runtime here")
    lib = hip_build.build_sanitized(str(tmp_path))
    ora = oracle_build.build_sanitized(str(tmp_path), cc)
    env = dict(os.environ, LD_PRELOAD=runtime, MLORA_LIB=lib, MLORA_ORACLE_LIB=ora,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",        # the interpreter itself leaks by design
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    files = ["tests/test_oracle_pins.py", "tests/test_resident.py", "tests/test_abi_symbols.py", "tests/test_workloads.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=800)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert " passed" in r.stdout, tail
