"""kmeans_run_noalloc (the entry point that allocates nothing: its workspace is a static device
array inside the library) against kmeans_run with a caller-owned workspace, through the C ABI.
The two share their kernels, so every output must be equal bit for bit; the calls are made one
after the other on the same GPU, each with a smaller input than the one before, so that stale
contents of the shared array from a larger problem would show."""
import ctypes as C
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2604_01000_amd import embedpart as ep
from paper_2604_01000_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(n, d, k, dtype, seed):
    w = replace(synth.WORKLOADS["arxiv_like"].scaled(n), d=d, k=k, seed=seed,
                dtype="bf16" if dtype == torch.bfloat16 else "f32")
    X = synth.embeddings(w, DEV)
    if d % 4:   # rows must start 16-byte aligned: a view into a matrix with a padded row stride
        padded = torch.zeros((n, (d + 3) // 4 * 4), dtype=X.dtype, device=DEV)
        padded[:, :d] = X
        X = padded[:, :d]
    return X, ep.kmeans_init_indices(seed, n, k)


def _run(X, k, idx, iters, flags, static):
    n, d = X.shape
    p = ep.problem(X, k)
    ws = ep.workspace(ep.kmeans_workspace_bytes(p), DEV)
    Cc = torch.empty((k, d), dtype=torch.float32, device=DEV)
    labels = torch.full((n + 64,), -7, dtype=torch.int32, device=DEV)    # 64 canary entries behind the output
    counts = torch.full((k + 8,), -7, dtype=torch.int64, device=DEV)
    hist = torch.full((iters + 1 + 8,), -7.0, dtype=torch.float64, device=DEV)
    ep.kmeans_init(p, X, idx, Cc, ws)
    if static:
        del ws
        ep.kmeans_run_noalloc(p, X, iters, Cc, labels, counts, hist, flags)
    else:
        ep.kmeans_run(p, X, iters, Cc, labels, counts, hist, flags, ws)
    torch.cuda.synchronize()
    assert (labels[n:] == -7).all() and (counts[k:] == -7).all() and (hist[iters + 1:] == -7.0).all()
    return Cc.cpu().numpy(), labels[:n].cpu().numpy(), counts[:k].cpu().numpy(), hist[:iters + 1].cpu().numpy()


CALLS = [   # each smaller than the one before; the last is a shape of the generic kernels
    (50_000, 128, 64, torch.float32, 4, 0),
    (20_011, 128, 16, torch.bfloat16, 3, ep.EP_RUN_FINAL_REASSIGN),
    (7_001, 64, 8, torch.float32, 5, 0),
    (3_000, 10, 5, torch.float32, 3, ep.EP_RUN_FINAL_REASSIGN),
]


def test_noalloc_equals_kmeans_run_on_calls_in_a_row():
    want = []
    for i, (n, d, k, dtype, iters, flags) in enumerate(CALLS):
        X, idx = _inputs(n, d, k, dtype, 40 + i)
        want.append(_run(X, k, idx, iters, flags, static=False))
    for rep in range(2):   # the second pass starts from the array as the smallest problem left it
        for i, (n, d, k, dtype, iters, flags) in enumerate(CALLS):
            X, idx = _inputs(n, d, k, dtype, 40 + i)
            got = _run(X, k, idx, iters, flags, static=True)
            for g, w_, name in zip(got, want[i], ("C", "labels", "counts", "objective_hist")):
                if name == "objective_hist" and not flags:
                    g, w_ = g[:iters], w_[:iters]   # [iters] is written only with the re-assign flag
                np.testing.assert_array_equal(g, w_, err_msg=f"call {i} pass {rep}: {name}")
            assert got[1].min() >= 0 and got[1].max() < k and got[2].sum() == n


def test_noalloc_rejects_what_does_not_fit():
    L = ep.lib()
    X = torch.zeros((1000, 128), dtype=torch.float32, device=DEV)
    out = torch.zeros(4096, dtype=torch.int64, device=DEV)
    # a shape whose workspace grows with n (rows sorted by label for the update): 30 M rows cannot fit 34 MB
    big = ep.ep_problem(n=30_000_000, ld=128, d=128, k=100, dtype=ep.EP_F32, reserved=0)
    assert ep.kmeans_workspace_bytes(big) > ep.EP_NOALLOC_SCRATCH_BYTES
    rc = L.kmeans_run_noalloc(C.byref(big), C.c_void_p(X.data_ptr()), 1, C.c_void_p(out.data_ptr()),
                              C.c_void_p(out.data_ptr()), C.c_void_p(out.data_ptr()), None, 0, None)
    assert rc == ep.EP_EWORKSPACE
    # the largest shapes of the fused kernels fit at any n
    for d, k, dt in ((128, 64, ep.EP_F32), (128, 64, ep.EP_BF16), (256, 16, ep.EP_F32), (256, 16, ep.EP_BF16)):
        p = ep.ep_problem(n=2_000_000_000, ld=d, d=d, k=k, dtype=dt, reserved=0)
        assert ep.kmeans_workspace_bytes(p) <= ep.EP_NOALLOC_SCRATCH_BYTES
