"""The C++ decoding loops (Algorithm 1 on two host threads, synchronous
speculative decoding, autoregressive decoding) on a CPU stand-in backend:
output equals the verify model's greedy sequence under randomly perturbed
interleavings, with ThreadSanitizer watching the shared buffers."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cpu", "loops_test.cpp")


@pytest.mark.parametrize("sanitize", [True, False])
def test_loops_against_stand_in_backend(tmp_path, sanitize):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no g++")
    exe = str(tmp_path / "loops_test")
    flags = ["-std=c++17", "-O1", "-g"] + (["-fsanitize=thread"] if sanitize else ["-O2"])
    r = subprocess.run([gxx] + flags + [SRC, "-o", exe, "-lpthread"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe, "16" if sanitize else "200"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "OK" in r.stdout and "WARNING: ThreadSanitizer" not in r.stderr
