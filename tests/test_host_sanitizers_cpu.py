"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, on a machine WITHOUT a GPU: the
boundary tests (argument checks, host-only queries) are run in a child process against a build whose host side
is instrumented.  Never run where a GPU is visible (sanitizer builds stay off the GPU machines)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = """
import sys
sys.path.insert(0, %r)
from paper_2509_09424_amd import binding
binding.LIB_PATH = %r
import pytest
sys.exit(pytest.main(["-q", "-p", "no:cacheprovider", %r]))
"""


def _gpu_visible():
    try:
        import torch
        return torch.cuda.is_available()
    except ImportError:
        return False


@pytest.mark.skipif(_gpu_visible(), reason="sanitizer builds are for the CPU-only machine")
def test_boundary_under_host_sanitizers():
    from paper_2509_09424_amd import build
    lib = build.build_sanitized()
    env = dict(os.environ, LD_PRELOAD=build.sanitizer_runtime(), ASAN_OPTIONS="detect_leaks=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    code = CHILD % (ROOT, lib, os.path.join(ROOT, "tests", "test_abi_cpu.py"))
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-3000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-3000:]
