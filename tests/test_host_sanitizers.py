"""The library's host code under sanitizers (no GPU): the step walk and validator, the offset
allocator, the cost walk, the plan generator with its worker threads and the partition search
are compiled with AddressSanitizer + UBSan, and again with ThreadSanitizer, and driven by
csrc/host_check.cpp.  A finding of either makes the executable exit non-zero or print a report."""
import subprocess

import pytest

from paper_2505_05856_amd import build as bld


@pytest.mark.parametrize("kind", ["asan", "tsan"])
def test_host_entry_points_are_clean_under_sanitizers(kind):
    exe = bld.build_host_check(kind)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "host_check ok" in r.stdout
    for marker in ("ERROR: AddressSanitizer", "runtime error:", "WARNING: ThreadSanitizer", "LeakSanitizer"):
        assert marker not in out, out[-4000:]
