"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, rejects bad arguments before any HIP call, and derives the seeded initial rows
exactly as the oracle does."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2604_01000_amd import embedpart as ep

INCLUDE = Path(__file__).resolve().parent.parent / "include"
HEADER = INCLUDE / "embedpart.h"
BENCH_HEADER = INCLUDE / "embedpart_bench.h"


def _declared_functions():
    assert sorted(h.name for h in INCLUDE.glob("*.h")) == ["embedpart.h", "embedpart_bench.h"]
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text() + BENCH_HEADER.read_text(), flags=re.S)
    text = re.sub(r"typedef struct.*?\}\s*\w+;", "", text, flags=re.S)
    return set(re.findall(r"\b(?:int|const char \*)\s*(\w+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    declared = _declared_functions()
    assert declared == set(ep.SYMBOLS)
    L = ep.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert ep.ep_version() >= 100
    assert ep.strerror(0) == "ok" and "workspace" in ep.strerror(ep.EP_EWORKSPACE)
    assert ep.strerror(-99) == "unknown error code"


def test_binding_constants_equal_the_header():
    text = HEADER.read_text() + BENCH_HEADER.read_text()
    defines = dict(re.findall(r"#define\s+(EP_\w+)\s+\(?(-?\d+)\)?\s", text))
    for name in ("EP_OK", "EP_EINVAL", "EP_EUNSUPPORTED", "EP_EWORKSPACE", "EP_EHIP", "EP_F32", "EP_BF16", "EP_F16",
                 "EP_RUN_FINAL_REASSIGN", "EP_RUN_BOUNDS", "EP_UPDATE_ACCUMULATE", "EP_UPDATE_FINALIZE", "EP_MAX_D", "EP_MAX_K", "EP_BALANCE_MAX_K", "EP_BALANCE_MAX_ROUNDS", "EP_PROF_LLOYD_MAIN", "EP_PROF_UPDATE_SUMS",
                 "EP_PROF_EDGE_SWEEP"):
        assert int(defines[name]) == getattr(ep, name), name
    assert "((int64_t)1 << 31)" in text and ep.EP_MAX_N == 1 << 31


def _prob(**kw):
    base = dict(n=1000, ld=128, d=128, k=8, dtype=ep.EP_F32, reserved=0)
    base.update(kw)
    return ep.ep_problem(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), ep.EP_EINVAL), (dict(k=0), ep.EP_EINVAL), (dict(d=0), ep.EP_EINVAL),
    (dict(k=1001), ep.EP_EINVAL), (dict(ld=64), ep.EP_EINVAL), (dict(ld=130), ep.EP_EINVAL),
    (dict(reserved=1), ep.EP_EINVAL), (dict(dtype=7), ep.EP_EUNSUPPORTED),
    (dict(d=4096, ld=4096), ep.EP_EUNSUPPORTED), (dict(n=2**31), ep.EP_EINVAL),
    (dict(n=10**6, k=70000), ep.EP_EUNSUPPORTED),
])
def test_bad_problems_are_rejected_on_the_host(kw, code):
    L = ep.lib()
    p = _prob(**kw)
    out = C.c_size_t(0)
    assert L.kmeans_workspace_bytes(C.byref(p), C.byref(out)) == code
    fake = C.c_void_p(0x1000)
    assert L.kmeans_run(C.byref(p), fake, 3, fake, fake, fake, None, 0, fake, 1 << 40, None) == code
    assert L.kmeans_run_noalloc(C.byref(p), fake, 3, fake, fake, fake, None, 0, None) == code
    if kw != dict(k=1001):   # a row range of a larger matrix may hold fewer rows than there are clusters
        assert L.kmeans_assign(C.byref(p), fake, fake, fake, None, None, fake, 1 << 40, None) == code
        assert L.kmeans_update(C.byref(p), fake, fake, fake, fake, fake, 2, fake, 1 << 40, None) == code


def test_null_pointers_workspace_and_flags():
    L = ep.lib()
    p = _prob()
    need = ep.kmeans_workspace_bytes(p)
    assert need > 0 and need % 256 == 0
    fake, ws = C.c_void_p(0x1000), C.c_void_p(0x100000)
    assert L.kmeans_workspace_bytes(None, None) == ep.EP_EINVAL
    assert L.kmeans_workspace_bytes(C.byref(p), None) == ep.EP_EINVAL
    assert L.kmeans_assign(C.byref(p), None, fake, fake, None, None, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_assign(C.byref(p), C.c_void_p(0x1004), fake, fake, None, None, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_assign(C.byref(p), fake, None, fake, None, None, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_assign(C.byref(p), fake, fake, None, None, None, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_assign(C.byref(p), fake, fake, fake, None, None, None, need, None) == ep.EP_EWORKSPACE
    assert L.kmeans_assign(C.byref(p), fake, fake, fake, None, None, ws, need - 1, None) == ep.EP_EWORKSPACE
    assert L.kmeans_assign(C.byref(p), fake, fake, fake, None, None, C.c_void_p(0x100010), need, None) == ep.EP_EWORKSPACE
    assert L.kmeans_update(C.byref(p), fake, None, fake, fake, fake, 2, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_update(C.byref(p), fake, fake, fake, fake, None, 2, ws, need, None) == ep.EP_EINVAL   # finalizing
    assert L.kmeans_update(C.byref(p), fake, fake, fake, None, fake, 3, ws, need, None) == ep.EP_EINVAL   # needs outputs
    assert L.kmeans_update(C.byref(p), fake, fake, fake, fake, fake, 4, ws, need, None) == ep.EP_EINVAL   # unknown flag
    assert L.kmeans_update(C.byref(p), fake, fake, None, None, None, 1, None, need, None) == ep.EP_EWORKSPACE
    assert L.ep_validate_labels(0, 4, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_validate_labels(10, 0, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_validate_labels(10, 4, None, fake, None) == ep.EP_EINVAL
    assert L.ep_validate_labels(10, 4, fake, C.c_void_p(0x1004), None) == ep.EP_EINVAL
    assert L.kmeans_run(C.byref(p), fake, -1, fake, fake, fake, None, 0, ws, need, None) == ep.EP_EINVAL
    assert L.kmeans_run(C.byref(p), fake, 1, fake, fake, fake, None, 8, ws, need, None) == ep.EP_EINVAL
    assert L.ep_bench_fold(None, 8, 64, 0, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_fold(fake, 0, 64, 0, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_fold(fake, 8, 60, 0, fake, fake, None) == ep.EP_EINVAL      # not a multiple of 8
    assert L.ep_bench_fold(fake, 8, 64, 3, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_fold(fake, 4096, 64, 1, fake, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_mfma_bf16(None, 1, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_mfma_bf16(fake, 0, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_mfma_bf16(fake, (1 << 22) + 1, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_mfma_bf16(C.c_void_p(0x1008), 1, fake, None) == ep.EP_EINVAL
    assert L.ep_bench_mfma_bf16(fake, 1, None, None) == ep.EP_EINVAL
    idx = (C.c_int64 * 8)(*range(8))
    assert L.kmeans_init(C.byref(p), fake, None, fake, ws, need, None) == ep.EP_EINVAL
    idx[3] = 1000                                            # row index out of range
    assert L.kmeans_init(C.byref(p), fake, idx, fake, ws, need, None) == ep.EP_EINVAL


def test_sampled_run_rejects_bad_arguments():
    L = ep.lib()
    p = _prob()                                              # n = 1000, k = 8
    out = C.c_size_t(0)
    assert L.kmeans_sampled_workspace_bytes(C.byref(p), 7, C.byref(out)) == ep.EP_EINVAL      # m < k
    assert L.kmeans_sampled_workspace_bytes(C.byref(p), 1001, C.byref(out)) == ep.EP_EINVAL   # m > n
    assert L.kmeans_sampled_workspace_bytes(C.byref(p), 64, None) == ep.EP_EINVAL
    need = ep.kmeans_sampled_workspace_bytes(p, 64)
    assert need > ep.kmeans_workspace_bytes(p) + 64 * 128 * 4 and need % 256 == 0
    fake, ws = C.c_void_p(0x1000), C.c_void_p(0x100000)
    rows = (C.c_int64 * 64)(*range(64))
    args = lambda **kw: [kw.get("p", C.byref(p)), kw.get("X", fake), kw.get("m", 64), kw.get("rows", rows),
                         kw.get("iters", 3), kw.get("C", fake), kw.get("labels", fake), kw.get("counts", fake), None,
                         kw.get("ws", ws), kw.get("bytes", need), None]
    assert L.kmeans_run_sampled(*args(rows=None)) == ep.EP_EINVAL
    assert L.kmeans_run_sampled(*args(m=7)) == ep.EP_EINVAL
    assert L.kmeans_run_sampled(*args(iters=-1)) == ep.EP_EINVAL
    assert L.kmeans_run_sampled(*args(labels=None)) == ep.EP_EINVAL
    assert L.kmeans_run_sampled(*args(counts=None)) == ep.EP_EINVAL
    assert L.kmeans_run_sampled(*args(ws=None)) == ep.EP_EWORKSPACE
    assert L.kmeans_run_sampled(*args(bytes=need - 1)) == ep.EP_EWORKSPACE
    rows[5] = 1000                                           # row index out of range
    assert L.kmeans_run_sampled(*args()) == ep.EP_EINVAL
    rows[5] = -1
    assert L.kmeans_run_sampled(*args()) == ep.EP_EINVAL


def test_balance_rejects_bad_arguments():
    L = ep.lib()
    fake, ws = C.c_void_p(0x1000), C.c_void_p(0x100000)
    out = C.c_size_t(0)
    assert L.balance_workspace_bytes(0, C.byref(out)) == ep.EP_EINVAL
    assert L.balance_workspace_bytes(10, None) == ep.EP_EINVAL
    need = ep.balance_workspace_bytes(1000)
    assert need >= 3 * 4 * 1000 and need % 256 == 0
    call = lambda **kw: L.partition_balance(kw.get("n", 1000), kw.get("k", 8), kw.get("rowptr", fake), 0, None, 0,
                                            kw.get("beta", 1.05), 7, kw.get("rounds", 8), kw.get("labels", fake),
                                            kw.get("stats", fake), kw.get("ws", ws), kw.get("bytes", need), None)
    assert call(n=0) == ep.EP_EINVAL
    assert call(k=0) == ep.EP_EINVAL
    assert call(k=256) == ep.EP_EUNSUPPORTED
    assert call(rowptr=None) == ep.EP_EINVAL
    assert call(labels=None) == ep.EP_EINVAL
    assert call(stats=None) == ep.EP_EINVAL
    assert call(beta=0.99) == ep.EP_EINVAL
    assert call(beta=float("nan")) == ep.EP_EINVAL
    assert call(rounds=-1) == ep.EP_EINVAL
    assert call(rounds=ep.EP_BALANCE_MAX_ROUNDS + 1) == ep.EP_EINVAL
    assert call(ws=None) == ep.EP_EWORKSPACE
    assert call(bytes=need - 1) == ep.EP_EWORKSPACE


def test_graph_calls_reject_bad_arguments():
    L = ep.lib()
    fake, ws = C.c_void_p(0x1000), C.c_void_p(0x100000)
    out = C.c_size_t(0)
    assert L.graph_workspace_bytes(0, 10, 4, C.byref(out)) == ep.EP_EINVAL
    assert L.graph_workspace_bytes(10, -1, 4, C.byref(out)) == ep.EP_EINVAL
    assert L.graph_workspace_bytes(10, 10, 0, C.byref(out)) == ep.EP_EINVAL
    assert L.graph_workspace_bytes(10, 10, 1 << 20, C.byref(out)) == ep.EP_EUNSUPPORTED
    need = ep.graph_workspace_bytes(1000, 5000, 8)
    assert need > 0
    args = (1000, 5000, 8, fake, 0, fake, fake, fake, fake)
    assert L.partition_quality(*args, None, need, None) == ep.EP_EWORKSPACE
    assert L.partition_quality(*args, ws, need - 1, None) == ep.EP_EWORKSPACE
    assert L.partition_quality(1000, 5000, 8, None, 0, fake, fake, fake, fake, ws, need, None) == ep.EP_EINVAL
    assert L.partition_quality(1000, 5000, 8, fake, 0, None, fake, fake, fake, ws, need, None) == ep.EP_EINVAL
    assert L.partition_quality(1000, 5000, 0, fake, 0, fake, fake, fake, fake, ws, need, None) == ep.EP_EINVAL
    assert L.partition_quality(1000, 5000, 8, fake, 0, fake, fake, None, fake, ws, need, None) == ep.EP_EINVAL
    assert L.partition_permutation(1000, 8, None, fake, fake, ws, need, None) == ep.EP_EINVAL
    assert L.partition_permutation(1000, 8, fake, fake, fake, None, need, None) == ep.EP_EWORKSPACE
    assert L.edge_gap_sum(1000, 5000, fake, 0, fake, None, None, ws, need, None) == ep.EP_EINVAL
    assert L.vertex_bandwidth_sum(1000, 5000, fake, 1, fake, None, fake, None, need, None) == ep.EP_EWORKSPACE
    assert ep.lib().ep_last_hip_error() == 0                 # nothing above reached the HIP runtime


@pytest.mark.parametrize("seed,n,k", [(0, 10, 10), (1, 20_000, 4), (2, 170_000, 8), (3, 2_450_000, 16),
                                       (5, 111_000_000, 64), (2**63 + 11, 5000, 4999), (3, 2_450_000, 16_384)])
def test_seeded_rows_match_the_oracle(seed, n, k):
    got = ep.kmeans_init_indices(seed, n, k).numpy()
    np.testing.assert_array_equal(got, oracle.init_indices(seed, n, k))
    assert len(set(got.tolist())) == k


def test_seeded_rows_reject_k_above_n():
    with pytest.raises(ep.EmbedPartError):
        ep.kmeans_init_indices(0, 3, 4)


def test_graph_reorder_rejects_bad_arguments():
    L = ep.lib()
    fake, fake2, ws = C.c_void_p(0x1000), C.c_void_p(0x2000), C.c_void_p(0x100000)
    out = C.c_size_t(0)
    assert L.graph_reorder_workspace_bytes(0, 10, C.byref(out)) == ep.EP_EINVAL
    assert L.graph_reorder_workspace_bytes(10, -1, C.byref(out)) == ep.EP_EINVAL
    assert L.graph_reorder_workspace_bytes(10, 10, None) == ep.EP_EINVAL
    need = ep.graph_reorder_workspace_bytes(100_000, 5_000_000)
    assert need >= 8 * (5_000_000 // 4096 + 100_000 // 2048) and need % 256 == 0
    call = lambda **kw: L.graph_reorder(kw.get("n", 100_000), kw.get("nnz", 5_000_000), kw.get("rowptr", fake),
                                        kw.get("i64", 0), kw.get("colidx", fake), kw.get("new_id", fake),
                                        kw.get("order", fake), kw.get("new_rowptr", fake2),
                                        kw.get("new_colidx", fake2), kw.get("ws", ws), kw.get("bytes", need), None)
    assert call(n=0) == ep.EP_EINVAL
    assert call(nnz=-1) == ep.EP_EINVAL
    assert call(rowptr=None) == ep.EP_EINVAL
    assert call(colidx=None) == ep.EP_EINVAL
    assert call(colidx=C.c_void_p(0x1004)) == ep.EP_EINVAL              # 16-byte alignment of the column array
    assert call(new_id=None) == ep.EP_EINVAL
    assert call(order=None) == ep.EP_EINVAL
    assert call(new_rowptr=None) == ep.EP_EINVAL
    assert call(new_colidx=None) == ep.EP_EINVAL
    assert call(new_rowptr=fake) == ep.EP_EINVAL                        # in place is not supported
    assert call(new_colidx=fake) == ep.EP_EINVAL
    assert call(nnz=1 << 31, bytes=1 << 40) == ep.EP_EINVAL             # 32-bit offsets cannot hold it
    assert call(ws=None) == ep.EP_EWORKSPACE
    assert call(bytes=need - 1) == ep.EP_EWORKSPACE


def test_cluster_and_balance_rejects_bad_arguments():
    L = ep.lib()
    fake, ws = C.c_void_p(0x1000), C.c_void_p(0x100000)
    out = C.c_size_t(0)
    p = ep.ep_problem(5000, 64, 64, 8, ep.EP_F32, 0)
    assert L.cluster_and_balance_workspace_bytes(C.byref(p), -1, C.byref(out)) == ep.EP_EINVAL
    assert L.cluster_and_balance_workspace_bytes(C.byref(p), 4, C.byref(out)) == ep.EP_EINVAL      # fewer than k rows
    assert L.cluster_and_balance_workspace_bytes(C.byref(p), 5001, C.byref(out)) == ep.EP_EINVAL
    assert L.cluster_and_balance_workspace_bytes(C.byref(p), 0, None) == ep.EP_EINVAL
    need = ep.cluster_and_balance_workspace_bytes(p)
    assert need >= ep.kmeans_workspace_bytes(p) + ep.balance_workspace_bytes(5000)
    assert ep.cluster_and_balance_workspace_bytes(p, 1000) > need - ep.kmeans_workspace_bytes(p)
    rows = (C.c_int64 * 8)(*range(8))

    def call(**kw):
        opt = ep.phase2_options(kw.get("beta", (1.05, 1.05, 1.1)), 3, kw.get("iters", 5), kw.get("rounds", 8),
                                kw.get("sample", 0))
        return L.cluster_and_balance(C.byref(kw.get("p", p)), kw.get("X", fake), kw.get("rowptr", fake), 0, None,
                                     C.byref(opt) if kw.get("opt", True) else None, kw.get("rows", rows),
                                     kw.get("C", fake), kw.get("labels", fake), kw.get("counts", fake),
                                     kw.get("stats", fake), kw.get("ws", ws), kw.get("bytes", need), None)

    assert call(opt=False) == ep.EP_EINVAL
    assert call(stats=None) == ep.EP_EINVAL
    assert call(rowptr=None) == ep.EP_EINVAL
    assert call(beta=(1.05, 0.5, 1.1)) == ep.EP_EINVAL
    assert call(rounds=ep.EP_BALANCE_MAX_ROUNDS + 1) == ep.EP_EINVAL
    assert call(sample=4) == ep.EP_EINVAL
    assert call(X=None) == ep.EP_EINVAL
    assert call(C=None) == ep.EP_EINVAL
    assert call(rows=None) == ep.EP_EINVAL
    assert call(ws=None) == ep.EP_EWORKSPACE
    assert call(bytes=need - 1) == ep.EP_EWORKSPACE
    big = ep.ep_problem(5000, 64, 64, 300, ep.EP_F32, 0)
    assert call(p=big) == ep.EP_EUNSUPPORTED                                  # balancing: partition-scale k only


def test_bench_refuses_more_than_one_gpu():
    """The benchmark covers one GPU; asking for more ends with a message and a non-zero status before
    anything touches a device."""
    import subprocess
    import sys
    from pathlib import Path
    bench = Path(__file__).resolve().parents[1] / "bench.py"
    proc = subprocess.run([sys.executable, str(bench), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert proc.returncode != 0
    assert "ONE GPU" in (proc.stderr + proc.stdout)
