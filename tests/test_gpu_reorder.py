"""GPU parity of graph_reorder (the graph rewritten under the new vertex ids): bit-exact against the
oracle, on the synthetic workloads' graphs and on shapes that hit every path of the kernel: rows
longer than a window and longer than several LDS tiles, runs of empty rows, windows without a row
start, both offset widths."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import embedpart as ep
from paper_2604_01000_amd import synth

from parity import DEV, Graph

pytestmark = pytest.mark.gpu


def _check(rowptr: torch.Tensor, colidx: torch.Tensor, labels: np.ndarray, k: int):
    gr = Graph(rowptr, colidx, k_max=k)
    new_id, order = gr.permutation(torch.from_numpy(labels).to(DEV), k)
    new_or, _ = oracle.permutation(labels, k)
    np.testing.assert_array_equal(new_id.cpu().numpy(), new_or)
    nrp, nci = gr.reorder(new_id, order)
    nrp_or, nci_or = oracle.reorder_csr(gr.rp_np, gr.ci_np, new_or)
    np.testing.assert_array_equal(nrp, nrp_or)
    np.testing.assert_array_equal(nci, nci_or)
    return gr, new_id, nrp, nci


def _csr_from_rows(rows, n, i64):
    deg = np.array([len(r) for r in rows], dtype=np.int64)
    rowptr = np.concatenate([[0], np.cumsum(deg)])
    colidx = np.concatenate([np.asarray(r, dtype=np.int32) for r in rows]) if deg.sum() else np.zeros(0, np.int32)
    return torch.from_numpy(rowptr.astype(np.int64 if i64 else np.int32)), torch.from_numpy(colidx.astype(np.int32))


@pytest.mark.parametrize("name,n", [("tiny", None), ("arxiv_like", None), ("products_like", 150_000),
                                    ("papers_like", 300_000)])
def test_reorder_matches_oracle_on_workload_graphs(name, n):
    w = synth.WORKLOADS[name]
    if n is not None:
        w = w.scaled(n)
    rowptr, colidx, blocks = synth.sbm_graph(w, "cpu")
    rng = np.random.default_rng(w.seed)
    labels = rng.integers(0, w.k, w.n).astype(np.int32)
    gr, new_id, nrp, nci = _check(rowptr, colidx, labels, w.k)
    # the metrics of (G, pi) are those of the rewritten graph under the identity
    g2 = Graph(torch.from_numpy(nrp), torch.from_numpy(nci))
    assert g2.gap_sum(None) == gr.gap_sum(new_id)
    assert g2.bandwidth_sum(None) == gr.bandwidth_sum(new_id)


@pytest.mark.parametrize("i64", [False, True])
def test_reorder_long_rows_empty_rows_and_ragged_windows(i64):
    """Vertices joined to 70,001 / 40,000 / 20,000 / 4,097 / 4,096 others (more than two LDS tiles with two
    levels of global merging, more than one tile, just over and exactly one window), 30,000 isolated
    vertices in runs, unsorted rows with parallel entries, a self-loop."""
    rng = np.random.default_rng(17 + i64)
    n = 110_000
    rows = [[] for _ in range(n)]
    for v, deg in [(5, 70_001), (60_000, 40_000), (60_001, 20_000), (99_999, 4_097), (100_000, 4_096), (3, 9_000)]:
        rows[v] = rng.choice(n, size=deg, replace=False).tolist()
    for v in rng.choice(80_000, size=50_000, replace=False):
        if not rows[v]:
            rows[v] = rng.integers(0, n, size=int(rng.integers(1, 40))).tolist()    # parallel entries possible
    rows[7] = [7, 7, 2, 109_999, 0]
    rowptr, colidx = _csr_from_rows(rows, n, i64)
    for k, labels in [(8, rng.integers(0, 8, n).astype(np.int32)),
                      (1, np.zeros(n, dtype=np.int32)),                              # identity permutation
                      (300, (np.arange(n) % 300).astype(np.int32))]:
        _check(rowptr, colidx, labels, k)


def test_reorder_one_very_long_row():
    """A vertex joined to 300,001 others (19 LDS tiles, five levels of merging on global memory) among
    short rows, int64 offsets."""
    rng = np.random.default_rng(31)
    n = 400_000
    deg = rng.integers(0, 6, n)
    deg[123_456] = 300_001
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    colidx = rng.integers(0, n, int(rowptr[-1])).astype(np.int32)
    labels = rng.integers(0, 50, n).astype(np.int32)
    _check(torch.from_numpy(rowptr), torch.from_numpy(colidx), labels, 50)


def test_reorder_small_and_degenerate():
    rng = np.random.default_rng(23)
    # one vertex with a self-loop; two vertices; no edges at all; one entry
    for rows in ([[0]], [[1], [0]], [[], [], []], [[], [2], []], [[1, 1, 1], [0, 0, 0]]):
        n = len(rows)
        rowptr, colidx = _csr_from_rows(rows, n, False)
        labels = rng.integers(0, 2, n).astype(np.int32)
        _check(rowptr, colidx, labels, 2)
    # exactly one window, one window + 1, rows ending exactly on window boundaries
    for deg in (4096, 4097, 2048):
        n = 3 * deg + 5
        rows = [rng.integers(0, n, size=deg).tolist() if v % deg == 0 and v < 3 * deg else [] for v in range(n)]
        rowptr, colidx = _csr_from_rows(rows, n, True)
        _check(rowptr, colidx, rng.integers(0, 5, n).astype(np.int32), 5)


def test_reorder_rejects_a_non_permutation_without_writing():
    """order with a repeated row: the degrees do not add up to nnz, so no column is written (and nothing
    is read or written out of bounds); an out-of-range entry of order counts as an empty row."""
    w = synth.WORKLOADS["tiny"]
    rowptr, colidx, _ = synth.sbm_graph(w, "cpu")
    gr = Graph(rowptr, colidx, k_max=4)
    new_id = torch.arange(w.n, dtype=torch.int32)
    order = new_id.clone()
    deg = np.diff(gr.rp_np)
    a = int(np.argmax(deg))
    b = int(np.flatnonzero((deg > 0) & (deg < deg[a]))[0])
    order[b] = a                                           # row a twice, row b never
    _, nci = gr.reorder(new_id.to(DEV), order.to(DEV))
    assert (nci == -7).all()
    order[b] = w.n + 5
    _, nci = gr.reorder(new_id.to(DEV), order.to(DEV))
    assert (nci == -7).all()
    with pytest.raises(ep.EmbedPartError):                 # outputs must not be the inputs
        ws = ep.workspace(ep.graph_reorder_workspace_bytes(gr.n, gr.nnz), DEV)
        ep.graph_reorder(gr.n, gr.nnz, gr.rowptr, gr.colidx, new_id.to(DEV), new_id.to(DEV), gr.rowptr,
                         torch.empty_like(gr.colidx), ws)
