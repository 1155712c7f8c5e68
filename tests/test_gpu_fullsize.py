"""The benchmark configurations at full size, in the launch configuration bench.py times.

Where the oracle can follow the whole run it does (products_like); where it cannot (k = 16,384:
1e14 flop per run; 111 M points: 57 GB of embeddings), the device results are checked on sampled
outputs the oracle computes one by one (nearest centroid of sampled points against all centroids,
means of sampled clusters) and through properties that hold at any size (counts = histogram of
labels, sizes sum to n, objective non-increasing); the integer graph outputs are compared in full.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import embedpart as ep
from paper_2604_01000_amd import synth

from parity import (CENTROID_RTOL, DEV, Graph, Kmeans, centroid_rel_err, centroids_used, check_free_running,
                    label_mismatches)

pytestmark = pytest.mark.gpu


def _sampled_round_check(X, km, C_before, got, k, bf16, rng, n_points=4096, n_clusters=24):
    """One device round checked on samples: labels of sampled points against the oracle's search over
    all k centroids, and the means / counts of sampled clusters against the oracle's update."""
    n = X.shape[0]
    rows = np.unique(np.concatenate([rng.integers(0, n, size=n_points), np.arange(min(n, 257)),
                                     np.arange(max(0, n - 131), n)]))
    Xs = X[torch.from_numpy(rows).to(DEV)].to("cpu", torch.float32).numpy()
    used = centroids_used(C_before, bf16)
    want, best, _, _ = oracle.assign(Xs, used)
    differing, unexcused = label_mismatches(Xs, used, got["labels"][rows], want, best)
    assert unexcused == 0, f"{unexcused} of {differing} sampled labels differ and are not near-ties"
    labels = got["labels"]
    assert labels.min() >= 0 and labels.max() < k
    counts = np.bincount(labels, minlength=k)
    np.testing.assert_array_equal(got["counts"], counts)
    assert counts.sum() == n
    labels_dev = torch.from_numpy(labels).to(DEV)
    for j in rng.choice(k, size=min(k, n_clusters), replace=False):
        members = torch.nonzero(labels_dev == int(j)).squeeze(1)
        if members.numel() == 0:
            np.testing.assert_array_equal(got["C"][j], np.asarray(C_before, dtype=np.float32)[j])
            continue
        # the oracle's mean of the members, taken over chunks of 2^20 rows so that the host never holds more
        # (the chunks' means are put together with their counts in fp64)
        total, seen = np.zeros(X.shape[1]), 0
        for lo in range(0, members.numel(), 1 << 20):
            Xm = X[members[lo:lo + (1 << 20)]].to("cpu", torch.float32).numpy()
            C_or, cnt_or, _ = oracle.update(Xm, np.zeros(len(Xm), dtype=np.int32), np.zeros((1, X.shape[1])))
            total += C_or[0] * float(cnt_or[0])
            seen += int(cnt_or[0])
        assert seen == counts[j]
        assert centroid_rel_err(got["C"][j:j + 1], (total / seen)[None, :]) <= CENTROID_RTOL
    return differing


def _all_rounds(X, w, bf16, rng, sampled_rounds, n_points, n_clusters_last):
    """The `iters` rounds the benchmark times, one device round at a time: every round's counts are the
    histogram of its labels and add up to n, the objective never rises, and the rounds named in
    `sampled_rounds` (the last one among them) are checked on samples against the oracle."""
    idx = oracle.init_indices(w.seed, w.n, w.k)
    km = Kmeans(X, w.k).init(idx)
    objs, got, C_before = [], None, None
    for t in range(w.iters):
        C_before = km.C.cpu().numpy().astype(np.float64)
        got = km.run(1)
        counts = np.bincount(got["labels"], minlength=w.k)
        np.testing.assert_array_equal(got["counts"], counts)
        assert counts.sum() == w.n and got["labels"].min() >= 0 and got["labels"].max() < w.k
        objs.append(got["obj_hist"][0])
        note = ""
        if t in sampled_rounds:
            last = t == w.iters - 1
            d = _sampled_round_check(X, km, C_before, got, w.k, bf16, rng, n_points=n_points,
                                     n_clusters=n_clusters_last if last else 3)
            note = f", sampled labels differing {d}"
        print(f"{w.name} round {t + 1}: objective {objs[-1]:.6e}, empty clusters {int((counts == 0).sum())}{note}",
              flush=True)
    assert all(b <= a * (1 + 1e-9) for a, b in zip(objs, objs[1:])), objs      # non-increasing over all rounds
    return km, got, C_before


def _graph_check(w, labels_np, k, reorder=False):
    rowptr, colidx, _ = synth.sbm_graph(w, DEV)
    gr = Graph(rowptr, colidx, k_max=max(k, 1))
    labels = torch.from_numpy(labels_np).to(DEV)
    cut, sizes = gr.quality(labels, k)
    cut_or, sizes_or = oracle.partition_quality(gr.rp_np, gr.ci_np, labels_np, k)
    assert cut == cut_or
    np.testing.assert_array_equal(sizes, sizes_or)
    if reorder:
        new_id, order = gr.permutation(labels, k)
        new_or, order_or = oracle.permutation(labels_np, k)
        np.testing.assert_array_equal(new_id.cpu().numpy(), new_or)
        np.testing.assert_array_equal(order.cpu().numpy(), order_or)
        assert gr.gap_sum(new_id) == oracle.edge_gap_sum(gr.rp_np, gr.ci_np, new_or)
        assert gr.gap_sum(None) == oracle.edge_gap_sum(gr.rp_np, gr.ci_np)
        nrp, nci = gr.reorder(new_id, order)                 # the graph rewritten under pi, in full
        nrp_or, nci_or = oracle.reorder_csr(gr.rp_np, gr.ci_np, new_or)
        np.testing.assert_array_equal(nrp, nrp_or)
        np.testing.assert_array_equal(nci, nci_or)
    return cut_or / max(gr.nnz, 1)


def _entry_hash(rows, cols):
    """Order-free 64-bit fingerprint of a multiset of (row, column) pairs (int64 arithmetic wraps)."""
    h = (rows.to(torch.int64) * 1_000_003 + cols.to(torch.int64)) * -7046029254386353131
    return int((h ^ (h >> 29)).sum().item())


def _reorder_property_check(w, labels_np, k):
    """graph_reorder where the oracle cannot follow (1.6e9 entries): row starts against a prefix sum by
    the tensor library, every row ascending, the multiset of (row, column) pairs equal to the relabelled
    input, and the gap / bandwidth sums carried over."""
    rowptr, colidx, _ = synth.sbm_graph(w, DEV)
    gr = Graph(rowptr, colidx, k_max=k)
    new_id, order = gr.permutation(torch.from_numpy(labels_np).to(DEV), k)
    new_rowptr, new_colidx = torch.full_like(rowptr, -7), torch.full_like(colidx, -7)
    ws = ep.workspace(ep.graph_reorder_workspace_bytes(gr.n, gr.nnz), DEV)
    ep.graph_reorder(gr.n, gr.nnz, gr.rowptr, gr.colidx, new_id, order, new_rowptr, new_colidx, ws)
    torch.cuda.synchronize()
    deg = rowptr[1:] - rowptr[:-1]
    deg_new = deg[order.long()]
    assert new_rowptr[0].item() == 0
    assert torch.equal(new_rowptr[1:], torch.cumsum(deg_new, 0).to(rowptr.dtype))
    starts = torch.zeros(gr.nnz + 1, dtype=torch.bool, device=DEV)
    starts[new_rowptr[:-1][deg_new > 0].long()] = True
    assert bool(((new_colidx[1:] >= new_colidx[:-1]) | starts[1:-1]).all())
    del starts
    ids = torch.arange(gr.n, dtype=torch.int32, device=DEV)
    want = _entry_hash(torch.repeat_interleave(new_id, deg), new_id[colidx.long()])
    got = _entry_hash(torch.repeat_interleave(ids, deg_new), new_colidx)
    assert got == want
    g2 = Graph(new_rowptr, new_colidx, k_max=k)
    assert g2.gap_sum(None) == gr.gap_sum(new_id)
    assert g2.bandwidth_sum(None) == gr.bandwidth_sum(new_id)


def test_products_like_full():
    w = synth.WORKLOADS["products_like"]
    X = synth.embeddings(w, DEV)
    idx = oracle.init_indices(w.seed, w.n, w.k)
    flips = check_free_running(X, w.k, w.iters, idx)
    print(f"products_like: {flips} labels differed from the oracle over {w.iters} rounds")
    got = Kmeans(X, w.k).init(idx).run(w.iters)
    ecr = _graph_check(w, got["labels"], w.k)
    print(f"products_like: edge-cut ratio {ecr:.4f}")


def test_products_reorder_full():
    w = synth.WORKLOADS["products_reorder"]
    X = synth.embeddings(w, DEV)
    rng = np.random.default_rng(7)
    km, got, _ = _all_rounds(X, w, True, rng, sampled_rounds={0, 1, 2, w.iters - 1}, n_points=4096, n_clusters_last=24)
    full = Kmeans(X, w.k).init(oracle.init_indices(w.seed, w.n, w.k)).run(w.iters)   # the driver equals its steps
    np.testing.assert_array_equal(full["labels"], got["labels"])
    np.testing.assert_array_equal(full["C"], got["C"])
    # the permutation, the gap sums and the rewritten graph of the FINAL labelling against the oracle's integer routines
    _graph_check(w, got["labels"], w.k, reorder=True)


def test_papers_like_full():
    w = synth.WORKLOADS["papers_like"]
    free, total = torch.cuda.mem_get_info()
    if free < 150 * 2**30:
        pytest.skip("needs about 150 GB of free device memory")
    X = synth.embeddings(w, DEV)
    rng = np.random.default_rng(11)
    km, got, C_before = _all_rounds(X, w, False, rng, sampled_rounds={0, 1, w.iters - 1}, n_points=16384,
                                    n_clusters_last=16)
    # a contiguous slice of the last round follows the oracle exactly: same rows, same centroids, lockstep
    lo, hi = 55_000_000, 55_000_000 + (1 << 18)
    Xs = X[lo:hi].to("cpu", torch.float32).numpy()
    used = centroids_used(C_before, False)
    want, best, _, _ = oracle.assign(Xs, used)
    differing, unexcused = label_mismatches(Xs, used, got["labels"][lo:hi], want, best)
    assert unexcused == 0
    labels_np = got["labels"]
    del X, km
    torch.cuda.empty_cache()
    ecr = _graph_check(w, labels_np, w.k)
    print(f"papers_like: edge-cut ratio {ecr:.4f}")
    _reorder_property_check(w, labels_np, w.k)


def test_maximum_k_and_maximum_d():
    """The limits of the header: k = 65,536 clusters (bf16 matrix-core path: 2,048 centroid tiles, codes up to
    8 * 2047 + 7) checked on sampled points and clusters, and d = 1,024 columns (generic path) in full."""
    rng = np.random.default_rng(65536)
    k, d, n = ep.EP_MAX_K, 64, ep.EP_MAX_K + 4_123
    gen = torch.Generator().manual_seed(99)
    X = (2.0 * torch.randn((64, d), generator=gen)[torch.randint(0, 64, (n,), generator=gen)]
         + torch.randn((n, d), generator=gen)).clamp_min(0).to(torch.bfloat16).to(DEV)
    idx = oracle.init_indices(5, n, k)
    km = Kmeans(X, k).init(idx)
    C0 = km.C.cpu().numpy().astype(np.float64)
    got = km.run(1)
    _sampled_round_check(X, km, C0, got, k, True, rng, n_points=1024, n_clusters=64)
    assert np.isfinite(got["obj_hist"][0])

    n2, d2, k2 = 700, ep.EP_MAX_D, 7
    X2 = torch.randn((n2, d2), generator=gen).to(DEV)
    check_free_running(X2, k2, 3, oracle.init_indices(6, n2, k2))
