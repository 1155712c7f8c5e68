"""ctypes front end of the fp64 CPU oracle (``embedpart_oracle.c``).

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares no
code with the HIP library and never imports it.

Every function takes and returns numpy arrays; embeddings are handed over as
the exact fp32 values the device sees (a bf16 matrix is widened first, which is
exact).  See the C file's header for the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "embedpart_oracle.c"
_LIB = _HERE / "liboracle.so"

FLAG_FINAL_REASSIGN = 1
FLAG_BF16_CENTROIDS = 2


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (plain -O2, OpenMP for the per-point loop)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               str(_SRC), "-o", str(_LIB), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(str(_LIB))
        p = C.c_void_p
        L.or_version.restype = C.c_int
        L.or_init_indices.argtypes = [C.c_uint64, C.c_int64, C.c_int32, p]
        L.or_init_indices.restype = C.c_int
        L.or_round_bf16.argtypes = [C.c_double]
        L.or_round_bf16.restype = C.c_double
        L.or_assign.argtypes = [C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, p, C.c_int, p, p, p]
        L.or_assign.restype = C.c_double
        L.or_update.argtypes = [C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, p, p, p]
        L.or_update.restype = C.c_int32
        L.or_validate_labels.argtypes = [C.c_int64, C.c_int32, p, p]
        L.or_validate_labels.restype = None
        L.or_lloyd.argtypes = [C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, C.c_int32, p, C.c_int,
                               p, p, p, p, p]
        L.or_lloyd.restype = C.c_int
        L.or_lloyd_bounds.argtypes = [C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, C.c_int32, p, C.c_int, C.c_int,
                                      p, p, p, p, p, p, p]
        L.or_lloyd_bounds.restype = C.c_int
        L.or_sampled_kmeans.argtypes = [C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, C.c_int64, p, C.c_int32,
                                        C.c_int, p, p, p, p, p]
        L.or_sampled_kmeans.restype = C.c_int
        L.or_partition_quality.argtypes = [C.c_int64, C.c_int32, p, p, p, p, p]
        L.or_partition_quality.restype = C.c_int
        L.or_edge_cut_ratio.argtypes = [C.c_int64, C.c_int64]
        L.or_edge_cut_ratio.restype = C.c_double
        L.or_vertex_balance.argtypes = [C.c_int32, p]
        L.or_vertex_balance.restype = C.c_double
        L.or_balance.argtypes = [C.c_int64, C.c_int32, p, p, C.c_int32, C.c_double, C.c_uint64, C.c_int32, p, p]
        L.or_balance.restype = C.c_int
        L.or_permutation.argtypes = [C.c_int64, C.c_int32, p, p, p]
        L.or_permutation.restype = C.c_int
        L.or_edge_gap_sum.argtypes = [C.c_int64, p, p, p]
        L.or_edge_gap_sum.restype = C.c_uint64
        L.or_vertex_bandwidth_sum.argtypes = [C.c_int64, p, p, p]
        L.or_vertex_bandwidth_sum.restype = C.c_uint64
        L.or_reorder_csr.argtypes = [C.c_int64, p, p, p, p, p]
        L.or_reorder_csr.restype = C.c_int
        _lib = L
    return _lib


def threads() -> int:
    """Threads the assignment loop will use (OpenMP default unless OMP_NUM_THREADS is set)."""
    v = os.environ.get("OMP_NUM_THREADS")
    return int(v) if v else (os.cpu_count() or 1)


def set_threads(count: int) -> None:
    """Number of OpenMP threads of the following calls (timing aid of the benchmark's CPU baseline:
    the arithmetic and its order inside a thread's share do not depend on it)."""
    lib()
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(count))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _x32(X):
    X = np.asarray(X)
    if X.dtype != np.float32 or X.ndim != 2 or X.strides[1] != 4 or X.strides[0] % 4:
        X = np.ascontiguousarray(X, dtype=np.float32)
    return X, X.strides[0] // 4


def init_indices(seed: int, n: int, k: int) -> np.ndarray:
    idx = np.empty(k, dtype=np.int64)
    if lib().or_init_indices(seed & (2**64 - 1), n, k, _ptr(idx)) != 0:
        raise ValueError("init_indices: need 1 <= k <= n")
    return idx


def round_bf16(v) -> np.ndarray:
    f = lib().or_round_bf16
    return np.vectorize(lambda t: f(float(t)), otypes=[np.float64])(np.asarray(v, dtype=np.float64))


def assign(X, Cc, round_bf16: bool = False):
    """Returns (labels int32[n], best f64[n], second f64[n], objective)."""
    X, ld = _x32(X)
    Cc = np.ascontiguousarray(Cc, dtype=np.float64)
    n, d = X.shape
    k = Cc.shape[0]
    assert Cc.shape == (k, d)
    labels = np.empty(n, dtype=np.int32)
    best = np.empty(n, dtype=np.float64)
    second = np.empty(n, dtype=np.float64)
    obj = lib().or_assign(n, d, k, _ptr(X), ld, _ptr(Cc), int(round_bf16), _ptr(labels), _ptr(best), _ptr(second))
    return labels, best, second, obj


def update(X, labels, C_prev):
    """Returns (C f64[k,d], counts int64[k], number of empty clusters)."""
    X, ld = _x32(X)
    Cn = np.array(C_prev, dtype=np.float64, order="C", copy=True)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n, d = X.shape
    k = Cn.shape[0]
    assert labels.shape == (n,) and (n == 0 or (labels.min() >= 0 and labels.max() < k))
    counts = np.empty(k, dtype=np.int64)
    empty = lib().or_update(n, d, k, _ptr(X), ld, _ptr(labels), _ptr(Cn), _ptr(counts))
    return Cn, counts, empty


def validate_labels(labels, k: int):
    """Returns (number of labels outside [0, k), index of the first one or n)."""
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    out = np.empty(2, dtype=np.int64)
    lib().or_validate_labels(labels.shape[0], k, _ptr(labels), _ptr(out))
    return int(out[0]), int(out[1])


def lloyd(X, k: int, iters: int, idx, flags: int = 0):
    """Returns dict(C, labels, counts, obj_hist, obj_final)."""
    X, ld = _x32(X)
    n, d = X.shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    assert idx.shape == (k,)
    Cc = np.empty((k, d), dtype=np.float64)
    labels = np.empty(n, dtype=np.int32)
    counts = np.zeros(k, dtype=np.int64)
    hist = np.empty(max(iters, 1), dtype=np.float64)
    fin = C.c_double(float("nan"))
    rc = lib().or_lloyd(n, d, k, _ptr(X), ld, iters, _ptr(idx), flags, _ptr(Cc), _ptr(labels), _ptr(counts),
                        _ptr(hist), C.addressof(fin))
    if rc != 0:
        raise ValueError("lloyd: bad arguments")
    return dict(C=Cc, labels=labels, counts=counts, obj_hist=hist[:iters], obj_final=fin.value)


def lloyd_bounds(X, k: int, iters: int, idx, flags: int = 0, audit: bool = False):
    """Lloyd rounds with bounds and incremental sums.  Returns dict(C, labels, counts, obj_hist, skipped, moved,
    violations); with audit every skipped point is searched anyway and `violations` counts the labels that
    would have changed."""
    X, ld = _x32(X)
    n, d = X.shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    assert idx.shape == (k,)
    Cc = np.empty((k, d), dtype=np.float64)
    labels = np.empty(n, dtype=np.int32)
    counts = np.zeros(k, dtype=np.int64)
    hist = np.empty(max(iters, 1), dtype=np.float64)
    skipped = np.zeros(max(iters, 1), dtype=np.int64)
    moved = np.zeros(max(iters, 1), dtype=np.int64)
    viol = C.c_int64(0)
    rc = lib().or_lloyd_bounds(n, d, k, _ptr(X), ld, iters, _ptr(idx), flags, int(audit), _ptr(Cc), _ptr(labels),
                               _ptr(counts), _ptr(hist), _ptr(skipped), _ptr(moved), C.addressof(viol))
    if rc != 0:
        raise ValueError("lloyd_bounds: bad arguments")
    return dict(C=Cc, labels=labels, counts=counts, obj_hist=hist[:iters], skipped=skipped[:iters],
                moved=moved[:iters], violations=viol.value)


def sampled_kmeans(X, k: int, iters: int, rows, flags: int = 0):
    """Centroids trained on the rows `rows` of X (first k of them as initial centroids), then every row
    assigned.  Returns dict(C, labels, counts, obj_hist, obj_full)."""
    X, ld = _x32(X)
    n, d = X.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    m = rows.shape[0]
    Cc = np.empty((k, d), dtype=np.float64)
    labels = np.empty(n, dtype=np.int32)
    counts = np.zeros(k, dtype=np.int64)
    hist = np.empty(max(iters, 1), dtype=np.float64)
    full = C.c_double(float("nan"))
    rc = lib().or_sampled_kmeans(n, d, k, _ptr(X), ld, m, _ptr(rows), iters, flags, _ptr(Cc), _ptr(labels),
                                 _ptr(counts), _ptr(hist), C.addressof(full))
    if rc != 0:
        raise ValueError("sampled_kmeans: bad arguments")
    return dict(C=Cc, labels=labels, counts=counts, obj_hist=hist[:iters], obj_full=full.value)


def _csr(rowptr, colidx):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    return rowptr, colidx


def partition_quality(rowptr, colidx, labels, k: int):
    """Returns (cut, sizes int64[k]); cut counts stored CSR entries."""
    rowptr, colidx = _csr(rowptr, colidx)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n = rowptr.shape[0] - 1
    assert labels.shape == (n,)
    cut = C.c_int64(0)
    sizes = np.empty(k, dtype=np.int64)
    rc = lib().or_partition_quality(n, k, _ptr(rowptr), _ptr(colidx), _ptr(labels), C.addressof(cut), _ptr(sizes))
    if rc != 0:
        raise ValueError("partition_quality: label or column index out of range")
    return cut.value, sizes


def edge_cut_ratio(cut: int, nnz: int) -> float:
    return lib().or_edge_cut_ratio(cut, nnz)


def vertex_balance(sizes) -> float:
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    return lib().or_vertex_balance(sizes.shape[0], _ptr(sizes))


def balance(rowptr, labels, k: int, beta: float, seed: int, max_rounds: int = 64, vclass=None, class_id: int = 0):
    """Balancing of one vertex class (Alg. 3 loop + Alg. 4).  Returns (new labels int32[n], stats int64[3] =
    rounds run, vertices moved, partitions still overloaded)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    out = np.array(labels, dtype=np.int32, copy=True)
    n = rowptr.shape[0] - 1
    assert out.shape == (n,)
    vc = None if vclass is None else np.ascontiguousarray(vclass, dtype=np.uint8)
    stats = np.zeros(3, dtype=np.int64)
    rc = lib().or_balance(n, k, _ptr(rowptr), None if vc is None else _ptr(vc), class_id, float(beta),
                          seed & (2**64 - 1), max_rounds, _ptr(out), _ptr(stats))
    if rc != 0:
        raise ValueError("balance: bad arguments")
    return out, stats


def permutation(labels, k: int):
    """Returns (new_id int32[n], order int32[n])."""
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n = labels.shape[0]
    new_id = np.empty(n, dtype=np.int32)
    order = np.empty(n, dtype=np.int32)
    if lib().or_permutation(n, k, _ptr(labels), _ptr(new_id), _ptr(order)) != 0:
        raise ValueError("permutation: label out of range")
    return new_id, order


def edge_gap_sum(rowptr, colidx, new_id=None) -> int:
    rowptr, colidx = _csr(rowptr, colidx)
    if new_id is not None:
        new_id = np.ascontiguousarray(new_id, dtype=np.int32)
    return lib().or_edge_gap_sum(rowptr.shape[0] - 1, _ptr(rowptr), _ptr(colidx), _ptr(new_id))


def vertex_bandwidth_sum(rowptr, colidx, new_id=None) -> int:
    rowptr, colidx = _csr(rowptr, colidx)
    if new_id is not None:
        new_id = np.ascontiguousarray(new_id, dtype=np.int32)
    return lib().or_vertex_bandwidth_sum(rowptr.shape[0] - 1, _ptr(rowptr), _ptr(colidx), _ptr(new_id))


def reorder_csr(rowptr, colidx, new_id):
    """The graph rewritten under the new ids: returns (new_rowptr int64[n+1], new_colidx int32[nnz]); row
    new_id[v] holds the neighbours of v under their new ids, ascending."""
    rowptr, colidx = _csr(rowptr, colidx)
    new_id = np.ascontiguousarray(new_id, dtype=np.int32)
    n = rowptr.shape[0] - 1
    assert new_id.shape == (n,)
    new_rowptr = np.empty(n + 1, dtype=np.int64)
    new_colidx = np.empty(colidx.shape[0], dtype=np.int32)
    if lib().or_reorder_csr(n, _ptr(rowptr), _ptr(colidx), _ptr(new_id), _ptr(new_rowptr), _ptr(new_colidx)) != 0:
        raise ValueError("reorder_csr: new_id is not a permutation, or a column index is out of range")
    return new_rowptr, new_colidx
