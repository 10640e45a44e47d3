import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the sanitizer pass (tests/test_host_sanitizers.py) re-runs the CPU tests of the host layer in a child process
    # against a build of that layer with AddressSanitizer and UndefinedBehaviorSanitizer
    san = os.environ.get("AXE_TEST_HOST_LIB")
    if san:
        from paper_2601_19092_amd import binding
        binding.LIB_PATH = san
        if "san" in os.path.basename(san):                 # the run is only worth something with the runtime in the process
            assert "libclang_rt.asan" in open("/proc/self/maps").read(), "sanitizer runtime not loaded"


@pytest.fixture(scope="session")
def golden():
    import json
    with open(os.path.join(ROOT, "tests", "golden", "paper_examples.json")) as f:
        return json.load(f)
