"""Host model of the lock-free candidate insertion and the single-owner merge (Sec. 3.1.1),
run under ThreadSanitizer.  The model (tests/model/lockfree_insert_model.cpp) is plain C++ on
std::atomic<uint64_t>; it shares no code with the GPU library or the oracle."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "model", "lockfree_insert_model.cpp")


def _build(tmp_path, sanitize):
    exe = str(tmp_path / ("model_tsan" if sanitize else "model"))
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-pthread", SRC, "-o", exe]
    if sanitize:
        cmd.insert(1, "-fsanitize=thread")
    subprocess.run(cmd, check=True)
    return exe


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
@pytest.mark.parametrize("sanitize", (True, False))
def test_lockfree_insert_and_merge_model(tmp_path, sanitize):
    exe = _build(tmp_path, sanitize)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert r.stdout.strip().endswith("OK")
    assert "ThreadSanitizer" not in r.stderr
