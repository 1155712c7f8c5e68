"""GPU parity of the integer graph calls: bit-exact against the oracle's plain loops."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import synth

from parity import DEV, Graph

pytestmark = pytest.mark.gpu


def _labels(n, k, seed, skew=False):
    g = torch.Generator().manual_seed(seed)
    if skew:                                              # unbalanced sizes, some partitions empty
        lab = (torch.rand(n, generator=g) ** 3 * k).long().clamp_(max=k - 1)
        lab[lab == k // 2] = 0
    else:
        lab = torch.randint(0, k, (n,), generator=g)
    return lab.to(torch.int32)


def _check_all(gr: Graph, labels: torch.Tensor, k: int):
    lab_np = labels.numpy()
    cut, sizes = gr.quality(labels.to(DEV), k)
    cut_or, sizes_or = oracle.partition_quality(gr.rp_np, gr.ci_np, lab_np, k)
    assert cut == cut_or
    np.testing.assert_array_equal(sizes, sizes_or)
    new_id, order = gr.permutation(labels.to(DEV), k)
    new_or, order_or = oracle.permutation(lab_np, k)
    np.testing.assert_array_equal(new_id.cpu().numpy(), new_or)
    np.testing.assert_array_equal(order.cpu().numpy(), order_or)
    assert gr.gap_sum(None) == oracle.edge_gap_sum(gr.rp_np, gr.ci_np)
    assert gr.gap_sum(new_id) == oracle.edge_gap_sum(gr.rp_np, gr.ci_np, new_or)
    assert gr.bandwidth_sum(None) == oracle.vertex_bandwidth_sum(gr.rp_np, gr.ci_np)
    assert gr.bandwidth_sum(new_id) == oracle.vertex_bandwidth_sum(gr.rp_np, gr.ci_np, new_or)


@pytest.mark.parametrize("name,n", [("tiny", None), ("arxiv_like", None), ("products_like", 150_000),
                                    ("papers_like", 300_000)])
def test_graph_calls_on_workload_graphs(name, n):
    w = synth.WORKLOADS[name]
    w = w if n is None else w.scaled(n)
    rowptr, colidx, blocks = synth.sbm_graph(w)
    gr = Graph(rowptr, colidx)
    _check_all(gr, blocks.to(torch.int32), w.components)             # planted blocks
    _check_all(gr, _labels(w.n, w.k, 1), w.k)
    _check_all(gr, _labels(w.n, 1000, 2, skew=True), 1000)           # two-pass sort, empty partitions
    _check_all(gr, torch.zeros(w.n, dtype=torch.int32), 1)           # one partition: nothing cut


def test_graph_with_empty_rows_hubs_and_ragged_sizes():
    rng = np.random.default_rng(0)
    n = 10_007
    deg = rng.integers(0, 6, size=n)
    deg[rng.random(n) < 0.3] = 0                                     # many isolated vertices
    deg[[5, 4000, n - 1]] = [3000, 7000, 1]                           # hubs and a non-empty last row
    deg[:3] = 0                                                      # graph starts with empty rows
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    colidx = rng.integers(0, n, size=rowptr[-1]).astype(np.int32)     # directed, repeats allowed
    for dtype in (torch.int32, torch.int64):
        gr = Graph(torch.from_numpy(rowptr).to(dtype), torch.from_numpy(colidx))
        _check_all(gr, _labels(n, 7, 3), 7)
        _check_all(gr, _labels(n, 16_384, 4), 16_384)


def test_graph_without_edges_and_single_vertex():
    gr = Graph(torch.zeros(6, dtype=torch.int32), torch.zeros(0, dtype=torch.int32))
    cut, sizes = gr.quality(torch.tensor([0, 1, 1, 2, 2], dtype=torch.int32, device=DEV), 3)
    assert cut == 0 and sizes.tolist() == [1, 2, 2]
    assert gr.gap_sum(None) == 0 and gr.bandwidth_sum(None) == 0
    gr = Graph(torch.tensor([0, 1], dtype=torch.int64), torch.tensor([0], dtype=torch.int32))   # one self loop
    _check_all(gr, torch.zeros(1, dtype=torch.int32), 1)


def test_out_of_range_labels_are_skipped_not_read_out_of_bounds():
    w = synth.WORKLOADS["tiny"]
    rowptr, colidx, _ = synth.sbm_graph(w)
    gr = Graph(rowptr, colidx)
    lab = _labels(w.n, 4, 9)
    bad = lab.clone()
    bad[::5] = 1 << 20
    bad[1::9] = -3
    cut, sizes = gr.quality(bad.to(DEV), 4)
    ok = ((bad >= 0) & (bad < 4)).numpy()
    src = np.repeat(np.arange(w.n), np.diff(gr.rp_np))
    both = ok[src] & ok[gr.ci_np]
    b = bad.numpy()
    assert cut == int(np.count_nonzero(both & (b[src] != b[gr.ci_np])))
    assert sizes.tolist() == np.bincount(b[ok], minlength=4).tolist()


@pytest.mark.parametrize("rowptr_i64", [True, False])
def test_cut_count_through_buckets_on_a_graph_beyond_the_caches(rowptr_i64):
    """6.4 M vertices: the cut count goes through buckets of column ranges (two buckets of 2^20 vertices and more,
    a ragged last one).  Hubs, empty rows, labels outside [0, k) and every k the byte labels allow, bit-exact
    against the oracle; then a graph whose columns all fall into one bucket, and one with column indices out of range."""
    from paper_2604_01000_amd import embedpart as ep
    n = 6_400_123
    w = synth.WORKLOADS["papers_like"].scaled(n)
    rowptr, colidx, blocks = synth.sbm_graph(w, DEV)
    rp = rowptr.cpu().numpy().astype(np.int64)
    ci = colidx.cpu().numpy().copy()
    rng = np.random.default_rng(5)
    hub = rng.integers(0, n, size=300_000).astype(np.int32)          # one row of 300,000 entries, many rows emptied
    deg = np.diff(rp)
    deg[rng.random(n) < 0.2] = 0
    keep = np.repeat(deg > 0, np.diff(rp))
    ci = ci[keep]
    rp = np.concatenate([[0], np.cumsum(deg)])
    at = int(rp[n // 3])
    ci = np.concatenate([ci[:at], hub, ci[at:]])
    rp[n // 3 + 1:] += len(hub)
    assert rp[-1] == len(ci) and len(ci) >= 4 * n
    gr = Graph(torch.from_numpy(rp).to(torch.int64 if rowptr_i64 else torch.int32), torch.from_numpy(ci))
    assert ep.graph_workspace_bytes(n, len(ci), 64) >= 4 * len(ci)    # the record buffer is part of the workspace
    for k, seed in ((64, 1), (2, 2), (255, 3)):
        lab = _labels(n, k, seed)
        cut, sizes = gr.quality(lab.to(DEV), k)
        cut_or, sizes_or = oracle.partition_quality(gr.rp_np, gr.ci_np, lab.numpy(), k)
        assert cut == cut_or
        np.testing.assert_array_equal(sizes, sizes_or)
    bad = _labels(n, 7, 4)
    bad[::5] = 1 << 20
    bad[1::9] = -3
    cut, sizes = gr.quality(bad.to(DEV), 7)
    ok = ((bad >= 0) & (bad < 7)).numpy()
    src = np.repeat(np.arange(n), np.diff(gr.rp_np))
    b = bad.numpy()
    assert cut == int(np.count_nonzero(ok[src] & ok[gr.ci_np] & (b[src] != b[gr.ci_np])))
    # k = 256 does not fit a byte: the plain sweep, same answer as the oracle
    lab = _labels(n, 256, 6)
    cut, _ = gr.quality(lab.to(DEV), 256)
    assert cut == oracle.partition_quality(gr.rp_np, gr.ci_np, lab.numpy(), 256)[0]
    # every column in the first bucket
    ci2 = (gr.ci_np % 1000).astype(np.int32)
    gr2 = Graph(torch.from_numpy(gr.rp_np).to(torch.int64 if rowptr_i64 else torch.int32), torch.from_numpy(ci2))
    lab = _labels(n, 9, 8)
    assert gr2.quality(lab.to(DEV), 9)[0] == oracle.partition_quality(gr2.rp_np, ci2, lab.numpy(), 9)[0]
    # column indices outside [0, n) are skipped by every pass of the bucketed path (the header's contract); the
    # expected count is the definition over the remaining entries
    ci3 = gr.ci_np.copy()
    pick = rng.choice(len(ci3), size=4_000, replace=False)
    ci3[pick[:1_500]] = -7
    ci3[pick[1_500:3_000]] = n + 11
    ci3[pick[3_000:]] = np.iinfo(np.int32).max
    del gr2
    gr3 = Graph(torch.from_numpy(gr.rp_np).to(torch.int64 if rowptr_i64 else torch.int32), torch.from_numpy(ci3))
    lab = _labels(n, 64, 10)
    inside = (ci3 >= 0) & (ci3 < n)
    l = lab.numpy()
    assert gr3.quality(lab.to(DEV), 64)[0] == int(np.count_nonzero(inside & (l[src] != l[np.where(inside, ci3, 0)])))
