"""The host layer (validation, planning, layout operators, describe, and the host-memory stand-ins of the integer
kernels) under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU tests that exercise it are run once more, in a
child process, against libaxe_hostcheck_san.so.  Host code only: the GPU kernels are not part of that library."""
import os
import subprocess
import sys

from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import build as BUILD

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_LIB = os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_hostcheck_san.so")
FILES = ["tests/test_host_plans.py", "tests/test_layout_algebra.py", "tests/test_describe.py", "tests/test_boundary.py"]


def test_host_layer_under_address_and_undefined_behaviour_sanitizers():
    if os.environ.get("AXE_TEST_HOST_LIB"):
        return                                             # this is the child run itself
    if not os.path.exists(SAN_LIB):
        BUILD.build_hostcheck_sanitized()
    env = dict(os.environ)
    rt = BUILD.sanitizer_runtime()
    assert os.path.exists(rt), rt
    env["LD_PRELOAD"] = ":".join(filter(None, [env.get("LD_PRELOAD", ""), rt]))      # (python itself is not instrumented)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["AXE_TEST_HOST_LIB"] = SAN_LIB
    p = subprocess.run([sys.executable, "-m", "pytest", *FILES, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = p.stdout[-4000:]
    assert "AddressSanitizer" not in p.stdout and "runtime error:" not in p.stdout, tail
    assert p.returncode == 0, tail
    assert " passed" in p.stdout, tail
