"""Host-side pieces of the library that need no GPU, built with gcc and run here:
the host tier's thread pool under the thread sanitizer and the address sanitizer."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2112_08541_amd", "csrc")
SRC = os.path.join(ROOT, "tests", "native", "pool_stress.cpp")


@pytest.mark.parametrize("sanitizer", ["thread", "address"])
def test_pool_stress_under_sanitizer(tmp_path, sanitizer):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / f"pool_{sanitizer}")
    subprocess.check_call([gxx, "-std=c++17", "-O1", "-g", f"-fsanitize={sanitizer}", "-pthread", "-I" + CSRC,
                           SRC, "-o", exe])
    for threads in ("1", "3", "8"):
        p = subprocess.run([exe, threads, "200"], capture_output=True, text=True, timeout=300)
        assert p.returncode == 0, p.stdout + p.stderr
        assert p.stdout.startswith("ok"), p.stdout + p.stderr
        assert "WARNING: ThreadSanitizer" not in p.stderr and "ERROR: AddressSanitizer" not in p.stderr, p.stderr
