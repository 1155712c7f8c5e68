"""The synthetic inputs have the stated shape and structure, and the oracle's cut
counter sees the planted block structure (a statistical cross-check of both)."""
import numpy as np
import torch

import oracle
from paper_2604_01000_amd import synth


def _check_csr(rowptr, colidx, n):
    rp = rowptr.numpy().astype(np.int64)
    ci = colidx.numpy()
    assert rp[0] == 0 and rp[-1] == len(ci) and np.all(np.diff(rp) >= 0)
    assert ci.min() >= 0 and ci.max() < n
    src = np.repeat(np.arange(n), np.diff(rp))
    assert not np.any(src == ci), "no self loops"
    key = src.astype(np.int64) * n + ci
    assert np.all(np.diff(key) > 0), "rows sorted, no duplicate entries"
    rev = ci.astype(np.int64) * n + src
    assert np.array_equal(np.sort(rev), key), "symmetric"
    return rp, ci


def test_tiny_workload_shape_and_planted_cut():
    w = synth.WORKLOADS["tiny"]
    X = synth.embeddings(w)
    assert X.shape == (20_000, 64) and X.dtype == torch.float32
    assert torch.equal(X, synth.embeddings(w)), "seeded"
    rowptr, colidx, blocks = synth.sbm_graph(w)
    assert rowptr.dtype == torch.int32 and colidx.dtype == torch.int32
    rp, ci = _check_csr(rowptr, colidx, w.n)
    assert abs(rp[-1] / w.n - 10.0) < 0.2
    cut, sizes = oracle.partition_quality(rp, ci, blocks.numpy().astype(np.int32), w.components)
    assert abs(cut / rp[-1] - 7.0 / 27.0) < 0.01           # 20:1 over 8 equal blocks
    assert sizes.sum() == w.n


def test_relu_bf16_and_powerlaw_variants():
    w = synth.WORKLOADS["products_reorder"].scaled(30_000)
    X = synth.embeddings(w)
    assert X.dtype == torch.bfloat16 and X.shape == (30_000, 128) and float(X.min()) == 0.0
    rowptr, colidx, blocks = synth.sbm_graph(w)
    assert rowptr.dtype == torch.int64
    rp, ci = _check_csr(rowptr, colidx, w.n)
    deg = np.diff(rp)
    assert deg.max() > 8 * deg.mean(), "heavy-tailed degrees"
    cut, _ = oracle.partition_quality(rp, ci, blocks.numpy().astype(np.int32), w.components)
    assert abs(cut / rp[-1] - 0.25) < 0.02


def test_embeddings_follow_the_mixture():
    w = synth.WORKLOADS["tiny"]
    X = synth.embeddings(w).double()
    blocks = synth.block_labels(w)
    means = synth.component_means(w).double()
    for g in range(w.components):
        sel = X[blocks == g]
        assert abs(len(sel) - w.n / w.components) < 0.1 * w.n / w.components
        assert (sel.mean(0) - means[g]).abs().max() < 0.15
        assert abs(float(sel.var(0).mean()) - 1.0) < 0.05
