"""Thin ctypes binding of libembedpart.so: argument marshalling only.

Every function has the name and the argument order of the C entry point it wraps (see
``include/embedpart.h``) and takes torch tensors that live on the GPU; torch is used
for device memory and the current stream, nothing else.  There is no CPU fallback: a
missing library or a non-zero return code raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libembedpart.so"

EP_F32, EP_BF16, EP_F16 = 0, 1, 2
EP_RUN_FINAL_REASSIGN, EP_RUN_BOUNDS = 1, 2
EP_UPDATE_ACCUMULATE, EP_UPDATE_FINALIZE = 1, 2
EP_OK, EP_EINVAL, EP_EUNSUPPORTED, EP_EWORKSPACE, EP_EHIP = 0, -1, -2, -3, -4
EP_MAX_D, EP_MAX_K, EP_MAX_N = 1024, 65536, 1 << 31   # limits stated in the header
EP_BALANCE_MAX_K, EP_BALANCE_MAX_ROUNDS = 255, 1024
EP_NOALLOC_SCRATCH_BYTES = 34 * 1024 * 1024

SYMBOLS = (
    "ep_version", "ep_strerror", "ep_last_hip_error", "kmeans_init_indices", "kmeans_workspace_bytes",
    "kmeans_init", "kmeans_assign", "kmeans_update", "ep_validate_labels", "kmeans_run", "kmeans_run_workspace_bytes", "kmeans_run_searched", "kmeans_run_noalloc",
    "kmeans_sampled_workspace_bytes",
    "kmeans_run_sampled", "graph_workspace_bytes",
    "partition_quality", "partition_permutation", "edge_gap_sum", "vertex_bandwidth_sum",
    "balance_workspace_bytes", "partition_balance", "graph_reorder_workspace_bytes", "graph_reorder",
    "cluster_and_balance_workspace_bytes", "cluster_and_balance",
    "ep_profile_arm", "ep_profile_count", "ep_bench_copy", "ep_bench_mfma_bf16", "ep_bench_fold",
)
EP_PROF_LLOYD_MAIN, EP_PROF_UPDATE_SUMS, EP_PROF_EDGE_SWEEP = 1, 2, 3


class ep_problem(C.Structure):
    _fields_ = [("n", C.c_int64), ("ld", C.c_int64), ("d", C.c_int32), ("k", C.c_int32),
                ("dtype", C.c_int32), ("reserved", C.c_int32)]


class ep_phase2(C.Structure):
    _fields_ = [("beta", C.c_double * 3), ("seed", C.c_uint64), ("iters", C.c_int32), ("max_rounds", C.c_int32),
                ("sample_rows", C.c_int64)]


class EmbedPartError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code}, hip error {lib().ep_last_hip_error()})")


_lib = None


def lib() -> C.CDLL:
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(str(_LIB_PATH))
        vp, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
        pp = C.POINTER(ep_problem)
        L.ep_version.restype = C.c_int
        L.ep_strerror.argtypes, L.ep_strerror.restype = [C.c_int], C.c_char_p
        L.ep_last_hip_error.restype = C.c_int
        L.kmeans_init_indices.argtypes = [u64, i64, i32, vp]
        L.kmeans_workspace_bytes.argtypes = [pp, C.POINTER(sz)]
        L.kmeans_init.argtypes = [pp, vp, vp, vp, vp, sz, vp]
        L.kmeans_assign.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.kmeans_update.argtypes = [pp, vp, vp, vp, vp, vp, C.c_int, vp, sz, vp]
        L.ep_validate_labels.argtypes = [i64, i32, vp, vp, vp]
        L.kmeans_run.argtypes = [pp, vp, i32, vp, vp, vp, vp, C.c_int, vp, sz, vp]
        L.kmeans_run_workspace_bytes.argtypes = [pp, i32, C.c_int, C.POINTER(sz)]
        L.kmeans_run_searched.argtypes = [pp, i32, C.c_int, vp, sz, vp, vp]
        L.kmeans_run_noalloc.argtypes = [pp, vp, i32, vp, vp, vp, vp, C.c_int, vp]
        L.kmeans_sampled_workspace_bytes.argtypes = [pp, i64, C.POINTER(sz)]
        L.kmeans_run_sampled.argtypes = [pp, vp, i64, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.graph_workspace_bytes.argtypes = [i64, i64, i32, C.POINTER(sz)]
        L.partition_quality.argtypes = [i64, i64, i32, vp, C.c_int, vp, vp, vp, vp, vp, sz, vp]
        L.partition_permutation.argtypes = [i64, i32, vp, vp, vp, vp, sz, vp]
        L.balance_workspace_bytes.argtypes = [i64, C.POINTER(sz)]
        L.partition_balance.argtypes = [i64, i32, vp, C.c_int, vp, i32, C.c_double, C.c_uint64, i32, vp, vp, vp, sz, vp]
        L.edge_gap_sum.argtypes = [i64, i64, vp, C.c_int, vp, vp, vp, vp, sz, vp]
        L.vertex_bandwidth_sum.argtypes = [i64, i64, vp, C.c_int, vp, vp, vp, vp, sz, vp]
        L.graph_reorder_workspace_bytes.argtypes = [i64, i64, C.POINTER(sz)]
        L.cluster_and_balance_workspace_bytes.argtypes = [C.POINTER(ep_problem), i64, C.POINTER(sz)]
        L.cluster_and_balance.argtypes = [C.POINTER(ep_problem), vp, vp, C.c_int, vp, C.POINTER(ep_phase2), vp, vp, vp,
                                          vp, vp, vp, sz, vp]
        L.graph_reorder.argtypes = [i64, i64, vp, C.c_int, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ep_profile_arm.argtypes = [vp, C.c_int, C.c_int]
        L.ep_bench_copy.argtypes = [vp, vp, sz, vp]
        L.ep_bench_mfma_bf16.argtypes = [vp, i32, vp, vp]
        L.ep_bench_fold.argtypes = [vp, i32, i32, C.c_int, vp, vp, vp]
        for name in SYMBOLS:
            if name not in ("ep_strerror",):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().ep_strerror(code).decode()


def _check(code: int, what: str):
    if code != EP_OK:
        raise EmbedPartError(code, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def problem(X: torch.Tensor, k: int) -> ep_problem:
    """ep_problem for a 2-D float32 / bfloat16 / float16 tensor with unit column stride."""
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be 2-D with contiguous rows")
    if X.dtype == torch.float32:
        dt = EP_F32
    elif X.dtype == torch.bfloat16:
        dt = EP_BF16
    elif X.dtype == torch.float16:
        dt = EP_F16
    else:
        raise ValueError("X must be float32, bfloat16 or float16")
    return ep_problem(n=X.shape[0], ld=X.stride(0), d=X.shape[1], k=k, dtype=dt, reserved=0)


def ep_version() -> int:
    return lib().ep_version()


def kmeans_init_indices(seed: int, n: int, k: int) -> torch.Tensor:
    idx = torch.empty(k, dtype=torch.int64)
    _check(lib().kmeans_init_indices(seed & (2**64 - 1), n, k, C.c_void_p(idx.data_ptr())), "kmeans_init_indices")
    return idx


def kmeans_workspace_bytes(p: ep_problem) -> int:
    out = C.c_size_t(0)
    _check(lib().kmeans_workspace_bytes(C.byref(p), C.byref(out)), "kmeans_workspace_bytes")
    return out.value


def graph_workspace_bytes(n: int, nnz: int, k: int) -> int:
    out = C.c_size_t(0)
    _check(lib().graph_workspace_bytes(n, nnz, k, C.byref(out)), "graph_workspace_bytes")
    return out.value


def workspace(nbytes: int, device) -> torch.Tensor:
    """A 256-byte aligned device buffer of at least nbytes (torch's allocator aligns to 512)."""
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def kmeans_init(p, X, idx_host, Cc, ws):
    idx_host = idx_host.contiguous()
    assert idx_host.device.type == "cpu" and idx_host.dtype == torch.int64
    _check(lib().kmeans_init(C.byref(p), _ptr(X), _ptr(idx_host), _ptr(Cc), _ptr(ws), ws.numel(), _stream()),
           "kmeans_init")


def kmeans_assign(p, X, Cc, labels, min_d2, objective, ws):
    _check(lib().kmeans_assign(C.byref(p), _ptr(X), _ptr(Cc), _ptr(labels), _ptr(min_d2), _ptr(objective),
                               _ptr(ws), ws.numel(), _stream()), "kmeans_assign")


def kmeans_update(p, X, labels, C_prev, C_out, counts, flags, ws):
    _check(lib().kmeans_update(C.byref(p), _ptr(X), _ptr(labels), _ptr(C_prev), _ptr(C_out), _ptr(counts), flags,
                               _ptr(ws), ws.numel(), _stream()), "kmeans_update")


def ep_validate_labels(n, k, labels, result):
    _check(lib().ep_validate_labels(n, k, _ptr(labels), _ptr(result), _stream()), "ep_validate_labels")


def kmeans_run(p, X, iters, Cc, labels, counts, objective_hist, flags, ws):
    _check(lib().kmeans_run(C.byref(p), _ptr(X), iters, _ptr(Cc), _ptr(labels), _ptr(counts), _ptr(objective_hist),
                            flags, _ptr(ws), ws.numel(), _stream()), "kmeans_run")


def kmeans_run_workspace_bytes(p: ep_problem, iters: int, flags: int) -> int:
    out = C.c_size_t(0)
    _check(lib().kmeans_run_workspace_bytes(C.byref(p), iters, flags, C.byref(out)), "kmeans_run_workspace_bytes")
    return out.value


def kmeans_run_searched(p, iters, flags, ws, searched):
    _check(lib().kmeans_run_searched(C.byref(p), iters, flags, _ptr(ws), ws.numel(), _ptr(searched), _stream()),
           "kmeans_run_searched")


def kmeans_run_noalloc(p, X, iters, Cc, labels, counts, objective_hist, flags):
    _check(lib().kmeans_run_noalloc(C.byref(p), _ptr(X), iters, _ptr(Cc), _ptr(labels), _ptr(counts),
                                    _ptr(objective_hist), flags, _stream()), "kmeans_run_noalloc")


def kmeans_sampled_workspace_bytes(p: ep_problem, m: int) -> int:
    out = C.c_size_t(0)
    _check(lib().kmeans_sampled_workspace_bytes(C.byref(p), m, C.byref(out)), "kmeans_sampled_workspace_bytes")
    return out.value


def kmeans_run_sampled(p, X, sample_rows_host, iters, Cc, labels, counts, objective_hist, ws):
    rows = sample_rows_host.contiguous()
    assert rows.device.type == "cpu" and rows.dtype == torch.int64
    _check(lib().kmeans_run_sampled(C.byref(p), _ptr(X), rows.numel(), _ptr(rows), iters, _ptr(Cc), _ptr(labels),
                                    _ptr(counts), _ptr(objective_hist), _ptr(ws), ws.numel(), _stream()),
           "kmeans_run_sampled")


def balance_workspace_bytes(n: int) -> int:
    out = C.c_size_t(0)
    _check(lib().balance_workspace_bytes(n, C.byref(out)), "balance_workspace_bytes")
    return out.value


def partition_balance(n, k, rowptr, vclass, class_id, beta, seed, max_rounds, labels, stats, ws):
    _check(lib().partition_balance(n, k, _ptr(rowptr), _is_i64(rowptr), _ptr(vclass), class_id, float(beta),
                                   seed & (2**64 - 1), max_rounds, _ptr(labels), _ptr(stats), _ptr(ws), ws.numel(),
                                   _stream()), "partition_balance")


def _is_i64(rowptr):
    if rowptr.dtype == torch.int64:
        return 1
    if rowptr.dtype == torch.int32:
        return 0
    raise ValueError("rowptr must be int32 or int64")


def partition_quality(n, nnz, k, rowptr, colidx, labels, cut, sizes, ws):
    _check(lib().partition_quality(n, nnz, k, _ptr(rowptr), _is_i64(rowptr), _ptr(colidx), _ptr(labels), _ptr(cut),
                                   _ptr(sizes), _ptr(ws), ws.numel(), _stream()), "partition_quality")


def partition_permutation(n, k, labels, new_id, order, ws):
    _check(lib().partition_permutation(n, k, _ptr(labels), _ptr(new_id), _ptr(order), _ptr(ws), ws.numel(),
                                       _stream()), "partition_permutation")


def edge_gap_sum(n, nnz, rowptr, colidx, new_id, gap_sum, ws):
    _check(lib().edge_gap_sum(n, nnz, _ptr(rowptr), _is_i64(rowptr), _ptr(colidx), _ptr(new_id), _ptr(gap_sum),
                              _ptr(ws), ws.numel(), _stream()), "edge_gap_sum")


def vertex_bandwidth_sum(n, nnz, rowptr, colidx, new_id, bw_sum, ws):
    _check(lib().vertex_bandwidth_sum(n, nnz, _ptr(rowptr), _is_i64(rowptr), _ptr(colidx), _ptr(new_id),
                                      _ptr(bw_sum), _ptr(ws), ws.numel(), _stream()), "vertex_bandwidth_sum")


def phase2_options(beta, seed: int, iters: int, max_rounds: int, sample_rows: int = 0) -> ep_phase2:
    return ep_phase2((C.c_double * 3)(*[float(b) for b in beta]), seed & (2**64 - 1), iters, max_rounds, sample_rows)


def cluster_and_balance_workspace_bytes(p: ep_problem, sample_rows: int = 0) -> int:
    out = C.c_size_t(0)
    _check(lib().cluster_and_balance_workspace_bytes(C.byref(p), sample_rows, C.byref(out)),
           "cluster_and_balance_workspace_bytes")
    return out.value


def cluster_and_balance(p, X, rowptr, vclass, opt, rows_host, Cc, labels, counts, stats, ws):
    rows_host = rows_host.contiguous()
    assert rows_host.device.type == "cpu" and rows_host.dtype == torch.int64
    _check(lib().cluster_and_balance(C.byref(p), _ptr(X), _ptr(rowptr), _is_i64(rowptr), _ptr(vclass), C.byref(opt),
                                     _ptr(rows_host), _ptr(Cc), _ptr(labels), _ptr(counts), _ptr(stats), _ptr(ws),
                                     ws.numel(), _stream()), "cluster_and_balance")


def graph_reorder_workspace_bytes(n: int, nnz: int) -> int:
    out = C.c_size_t(0)
    _check(lib().graph_reorder_workspace_bytes(n, nnz, C.byref(out)), "graph_reorder_workspace_bytes")
    return out.value


def graph_reorder(n, nnz, rowptr, colidx, new_id, order, new_rowptr, new_colidx, ws):
    assert new_rowptr.dtype == rowptr.dtype
    _check(lib().graph_reorder(n, nnz, _ptr(rowptr), _is_i64(rowptr), _ptr(colidx), _ptr(new_id), _ptr(order),
                               _ptr(new_rowptr), _ptr(new_colidx), _ptr(ws), ws.numel(), _stream()), "graph_reorder")


def ep_bench_copy(dst, src):
    """Plain device copy of src into dst (same size, multiple of 16 bytes): a kernel of known traffic."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().ep_bench_copy(_ptr(dst), _ptr(src), nbytes, _stream()), "ep_bench_copy")


def ep_bench_fold(partials, parts, elems, mode, ticket, out):
    """`parts` workgroups write `elems` partials each; mode 0 nothing more, 1 the last workgroup to arrive adds them
    up behind a ticket, 2 a second launch adds them up."""
    assert partials.numel() >= parts * elems and out.numel() >= elems and ticket.numel() >= 1
    _check(lib().ep_bench_fold(_ptr(partials), parts, elems, mode, _ptr(ticket), _ptr(out), _stream()), "ep_bench_fold")


EP_BENCH_MFMA_OPERAND_BYTES = 65536
EP_BENCH_MFMA_FLOP_PER_ITER = 512.0 * 4 * 16 * 32768


def ep_bench_mfma_bf16(operands, iters, sink):
    """16 * iters bf16 matrix instructions per wave on 65,536 bytes of operands (device): the pipe's rate alone."""
    assert operands.numel() * operands.element_size() >= EP_BENCH_MFMA_OPERAND_BYTES and operands.is_contiguous()
    _check(lib().ep_bench_mfma_bf16(_ptr(operands), iters, _ptr(sink), _stream()), "ep_bench_mfma_bf16")
