"""Builds libembedpart.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libembedpart.so"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(CSRC.glob("*.hip"))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_lib(verbose: bool = False, extra_flags=()) -> Path:
    """Compile every .hip file under csrc/ (one hipcc per file, side by side) and link them into one
    shared library (always rebuilds).  The objects live in a temporary folder, not in the tree."""
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="embedpart_build_") as tmp:
        objs = [str(Path(tmp) / (src.stem + ".o")) for src in sources()]
        with ThreadPoolExecutor(max_workers=min(8, len(objs))) as pool:
            jobs = [pool.submit(_run, [HIPCC, *compile_flags, *extra_flags, "-c", str(src), "-o", obj], verbose)
                    for src, obj in zip(sources(), objs)]
            for job in jobs:
                job.result()
        _run([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", str(LIB)], verbose)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
