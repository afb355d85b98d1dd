"""Builds the C-ABI library (HIP, gfx950 only) in-tree: paper_2411_00288_amd/libss.so.

Every translation unit under csrc/ is compiled to an object of its own, in parallel, and the objects are linked
into one shared library.  `build()` recompiles everything; `build(incremental=True)` (a convenience while working on
one file) reuses objects whose source, headers and flags have not changed.
"""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libss.so"
OBJDIR = HERE / "_build"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         # packed-fp32 instructions have produced silently wrong results on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def sources() -> list[Path]:
    return sorted(CSRC.glob("*.hip"))


def _run(cmd: list[str]) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 target feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed: {' '.join(cmd)}\n{err}")
    return err


def _stamp(src: Path, flags: list[str]) -> str:
    h = hashlib.sha256(" ".join(flags).encode())
    for f in [src, *sorted(CSRC.glob("*.h")), HERE.parent / "include" / "ss.h"]:
        h.update(f.read_bytes())
    return h.hexdigest()


def build(verbose: bool = False, extra_flags: list[str] | None = None, incremental: bool = False,
          out: Path | None = None, jobs: int | None = None) -> Path:
    flags = [*FLAGS, *(extra_flags or []), "-I", str(HERE.parent / "include")]
    OBJDIR.mkdir(exist_ok=True)
    out = Path(out) if out else LIB
    tag = hashlib.sha256(" ".join(flags).encode()).hexdigest()[:8]

    def compile_one(src: Path) -> Path:
        obj = OBJDIR / f"{src.stem}.{tag}.o"
        stamp_file = obj.with_suffix(".stamp")
        stamp = _stamp(src, flags) if incremental else None
        if incremental and obj.exists() and stamp_file.exists() and stamp_file.read_text() == stamp:
            return obj
        cmd = [HIPCC, *flags, "-c", str(src), "-o", str(obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        err = _run(cmd)
        if verbose and err.strip():
            print(err, file=sys.stderr)
        if incremental:
            stamp_file.write_text(stamp)
        return obj

    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, sources()))
    tmp = out.with_suffix(f".tmp{os.getpid()}.so")
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *map(str, objs), "-o", str(tmp)])
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
