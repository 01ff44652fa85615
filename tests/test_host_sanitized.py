"""The host-side logic of the library (argument checks, stash / workspace layout, schedule builder, GEMM planning,
dropout key) under AddressSanitizer + UndefinedBehaviorSanitizer: the library is rebuilt with both on its host
pass and the CPU-only ABI tests run against that build in a child process with the sanitizer runtime preloaded."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(900)
def test_host_abi_tests_pass_under_address_and_ub_sanitizers():
    from paper_2104_04473_amd import build as Bld
    lib = Bld.build(verbose=False, sanitize=True)
    runtime = Bld.sanitizer_runtime()
    assert os.path.exists(lib) and os.path.exists(runtime), (lib, runtime)
    env = dict(os.environ)
    env["PTDP_LIB"] = lib
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_host_abi.py")], cwd=ROOT, env=env, capture_output=True, text=True)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert " passed" in out
