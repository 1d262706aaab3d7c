"""The CPU safety net: the oracle and the host-only part of the library (flat-slice helper, decomposer,
metadata checks, Worst-Fit deduplication) built with g++ -fsanitize=address,undefined, and the CPU tests
that exercise them run against those builds in a child process.  A sanitizer report makes the child fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no libasan.so beside gcc")
    d = tmp_path_factory.mktemp("san")
    oracle_lib, host_lib = str(d / "liboracle_san.so"), str(d / "libbcp_host_san.so")
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-shared", "-fPIC", "-pthread"] + SAN +
                          [os.path.join(ROOT, "oracle", "reshard_oracle.cpp"), "-o", oracle_lib])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-shared", "-fPIC"] + SAN +
                          ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2407_20143_amd", "csrc"),
                           os.path.join(ROOT, "paper_2407_20143_amd", "csrc", "bcp_host.cpp"), "-o", host_lib])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=oracle_lib, BCP_HOST_LIB_OVERRIDE=host_lib,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = ":".join(p for p in (asan, os.environ.get("LD_PRELOAD", "")) if p)
    return env


def _run(env, files, extra=()):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu and not needs_full_lib"]
    r = subprocess.run(cmd + list(extra) + [os.path.join(ROOT, "tests", f) for f in files], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert " passed" in r.stdout


def test_oracle_pins_under_sanitizers(sanitized):
    _run(sanitized, ["test_oracle_pins.py", "test_oracle_convert.py"])


def test_host_only_library_code_under_sanitizers(sanitized):
    _run(sanitized, ["test_host_logic.py", "test_host_validate.py", "test_dedup.py"])


def test_a_planted_overrun_is_reported(sanitized, tmp_path):
    """The net itself: the same build line and environment catch an out-of-bounds read."""
    src = tmp_path / "bad.cpp"
    src.write_text('#include <cstdlib>\nextern "C" int peek(int i) { int* a = (int*)malloc(16); int v = a[i]; free(a); return v; }\n')
    lib = tmp_path / "libbad.so"
    subprocess.check_call(["g++", "-shared", "-fPIC"] + SAN + [str(src), "-o", str(lib)])
    r = subprocess.run([sys.executable, "-c", f"import ctypes; ctypes.CDLL({str(lib)!r}).peek(4)"], env=sanitized,
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and ("heap-buffer-overflow" in r.stderr or "runtime error" in r.stderr)
