"""CPU-only sanitizer runs of the host code: the oracle under AddressSanitizer + UndefinedBehaviorSanitizer (as a
driver executable on exact-size heap buffers, and as the library behind the oracle's own pin tests), and the HIP
library's host side (argument validation, launch planning, workspace sizing) under UBSan in trap mode, driven by the
ABI tests.  Each run is a child process: a finding ends it with a non-zero status."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _env(**extra):
    env = dict(os.environ)
    # the sanitizer runtime is a dependency of the oracle library, not of python: skip ASan's link-order check;
    # python itself is not leak-clean
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def test_oracle_selftest_under_asan_and_ubsan():
    import oracle
    exe = oracle.build_selftest()
    r = subprocess.run([exe], env=_env(OMP_NUM_THREADS="2"), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "self-test ok" in r.stdout


def test_oracle_pins_under_asan_and_ubsan():
    import oracle
    oracle.build_sanitized()
    files = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_attention.py", "test_oracle_consensus.py",
                                                      "test_oracle_prefill.py", "test_oracle_block_mask.py")]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + files,
                       env=_env(ORTHRUS_ORACLE_SANITIZE="1", OMP_NUM_THREADS="2"), cwd=ROOT, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:]


@pytest.mark.skipif(not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_host_api_validation_under_ubsan_traps():
    from paper_2605_12825_amd import build as hip_build
    lib = hip_build.build_library(host_ubsan=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi_cpu.py"), os.path.join(ROOT, "tests",
                                                                                     "test_balanced_partition_math.py")],
                       env=_env(ORTHRUS_LIBRARY=lib), cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:]
