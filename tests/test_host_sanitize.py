"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the library's descriptor validation,
size arithmetic, split planning and multiply-shift division (tests/host/host_checks.cpp, which includes the
library's own headers), and the C oracle's loops on exactly sized arrays (tests/host/oracle_checks.c)."""
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(map(str, cmd))}\n{res.stdout[-3000:]}\n{res.stderr[-3000:]}"
    return res.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_library_host_logic_under_sanitizers(tmp_path):
    exe = tmp_path / "host_checks"
    _run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", str(ROOT / "include"),
          str(ROOT / "tests" / "host" / "host_checks.cpp"), "-o", str(exe)])
    out = _run([str(exe)], env={"ASAN_OPTIONS": "detect_leaks=1", "UBSAN_OPTIONS": "print_stacktrace=1"})
    assert "host checks passed" in out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host compiler")
def test_oracle_under_sanitizers(tmp_path):
    exe = tmp_path / "oracle_checks"
    _run(["gcc", "-std=c11", *SAN, "-fopenmp", str(ROOT / "oracle" / "ss_oracle.c"), str(ROOT / "tests" / "host" / "oracle_checks.c"),
          "-lm", "-o", str(exe)])
    out = _run([str(exe)], env={"ASAN_OPTIONS": "detect_leaks=0", "UBSAN_OPTIONS": "print_stacktrace=1", "OMP_NUM_THREADS": "2"})
    assert "oracle checks passed" in out
