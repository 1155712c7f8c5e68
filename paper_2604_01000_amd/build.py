"""Builds libembedpart.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import hashlib
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
# Per source file, on top of FLAGS.  kmeans_small.hip: its hand-pipelined loops run one wave per SIMD and are bound by
# instruction issue; this scheduling strategy leaves fewer idle and wait instructions in them (the order the
# kernel pins with scheduling barriers stays).
FILE_FLAGS = {
    "kmeans_small.hip": ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp", "-mllvm", "-amdgpu-mfma-vgpr-form"],
}


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


def _stamp(src: Path, flags) -> str:
    """What an object file depends on: its source, every header beside it and in include/, and the flags."""
    h = hashlib.sha256(" ".join(flags).encode())
    for f in [src, *sorted(CSRC.glob("*.h")), *sorted((PKG.parent / "include").glob("*.h"))]:
        h.update(f.read_bytes())
    return h.hexdigest()


def build_lib(verbose: bool = False, extra_flags=(), object_cache: Path | None = None) -> Path:
    """Compile every .hip file under csrc/ (one hipcc per file, side by side) and link them into one
    shared library.  By default everything is compiled again and the objects live in a temporary folder,
    not in the tree; with `object_cache` (a folder outside the tree) an object whose source, headers and
    flags have not changed is taken from there instead."""
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="embedpart_build_") as tmp:
        where = Path(object_cache) if object_cache else Path(tmp)
        where.mkdir(parents=True, exist_ok=True)
        todo, objs = [], []
        for src in sources():
            obj, stamp_file = where / (src.stem + ".o"), where / (src.stem + ".stamp")
            objs.append(str(obj))
            file_flags = FILE_FLAGS.get(src.name, [])
            stamp = _stamp(src, [*compile_flags, *file_flags, *extra_flags])
            if object_cache and obj.exists() and stamp_file.exists() and stamp_file.read_text() == stamp:
                continue
            todo.append((src, obj, stamp_file, stamp, file_flags))
        with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as pool:
            jobs = [pool.submit(_run, [HIPCC, *compile_flags, *file_flags, *extra_flags, "-c", str(src), "-o", str(obj)], verbose)
                    for src, obj, _, _, file_flags in todo]
            for job in jobs:
                job.result()
        for _, _, stamp_file, stamp, _ in todo:
            stamp_file.write_text(stamp)
        _run([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", str(LIB)], verbose)
    return LIB


if __name__ == "__main__":
    # `python -m paper_2604_01000_amd.build [object cache folder]`
    print(build_lib(verbose=True, object_cache=Path(sys.argv[1]) if len(sys.argv) > 1 else None))
