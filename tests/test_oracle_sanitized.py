"""The oracle's pins once more, in a child process, against a build of the oracle instrumented
with AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU is involved): an
out-of-bounds access, a use after free, a signed overflow or a misaligned access anywhere in the
oracle aborts the child. The ASan runtime has to be the first library the child loads, so it is put
in front of whatever the environment already preloads."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    try:
        path = subprocess.check_output(["g++", "-print-file-name=libasan.so"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_asan_and_ubsan():
    rt = _asan_runtime()
    if rt is None:
        pytest.skip("no AddressSanitizer runtime next to g++")
    env = dict(os.environ)
    env["AIBX_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter's own leaks are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    files = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_")
                   and f.endswith(".py") and f != os.path.basename(__file__))
    assert len(files) >= 7
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
           *[os.path.join("tests", f) for f in files]]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "liboracle_san.so" in _loaded_marker(env), "the child did not load the instrumented oracle"


def _loaded_marker(env):
    """Which oracle library a child with this environment loads."""
    code = "import oracle; oracle._load(); print(oracle._LIB)"
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True,
                          timeout=300).stdout
