"""Pins for the oracle's graph metrics (CPU only): closed-form cuts, adjacency-matrix
brute force, the stated ranges of ECR and vertex balance, permutation properties and
gap / bandwidth values computed by hand."""
import numpy as np
import pytest

import oracle


def csr_from_undirected(n, edges):
    """Both directions stored, rows sorted (plain python; independent of the generators)."""
    adj = [[] for _ in range(n)]
    for u, v in edges:
        adj[u].append(v)
        if u != v:
            adj[v].append(u)
    rowptr = [0]
    col = []
    for u in range(n):
        col += sorted(adj[u])
        rowptr.append(len(col))
    return np.array(rowptr, dtype=np.int64), np.array(col, dtype=np.int32)


def _golden_rows(path):
    rows = {}
    for line in path.read_text().splitlines():
        line = line.split("#")[0].split()
        if line:
            rows[line[0]] = line[1:]
    return rows


def test_closed_form_cuts(golden_dir):
    g = _golden_rows(golden_dir / "cut_closed_forms.txt")
    # path split in two halves
    n = int(g["path"][0])
    rp, ci = csr_from_undirected(n, [(i, i + 1) for i in range(n - 1)])
    cut, sizes = oracle.partition_quality(rp, ci, np.repeat([0, 1], n // 2), 2)
    assert cut == int(g["path"][2]) and sizes.tolist() == [n // 2, n // 2]
    # cycle in contiguous arcs
    n = int(g["cycle"][0])
    rp, ci = csr_from_undirected(n, [(i, (i + 1) % n) for i in range(n)])
    cut, sizes = oracle.partition_quality(rp, ci, np.arange(n) // 3, 4)
    assert cut == int(g["cycle"][2]) and sizes.tolist() == [3, 3, 3, 3]
    assert oracle.vertex_balance(sizes) == 1.0
    # complete graph
    n = int(g["complete"][0])
    rp, ci = csr_from_undirected(n, [(i, j) for i in range(n) for j in range(i + 1, n)])
    cut, sizes = oracle.partition_quality(rp, ci, np.array([0, 0, 0, 1, 1, 2]), 3)
    assert cut == int(g["complete"][2]) == n * n - (sizes ** 2).sum()
    # perfect matching, endpoints apart: every edge cut
    n = int(g["matching"][0])
    rp, ci = csr_from_undirected(n, [(2 * i, 2 * i + 1) for i in range(n // 2)])
    cut, sizes = oracle.partition_quality(rp, ci, np.arange(n) % 2, 2)
    assert cut == int(g["matching"][2]) == rp[-1]
    assert oracle.edge_cut_ratio(cut, int(rp[-1])) == 1.0
    # one part: nothing cut, balance = k
    cut, sizes = oracle.partition_quality(rp, ci, np.zeros(n, dtype=np.int32), 4)
    assert cut == int(g["anygraph"][1]) and oracle.edge_cut_ratio(cut, int(rp[-1])) == 0.0
    assert oracle.vertex_balance(sizes) == 4.0


@pytest.mark.parametrize("seed", range(6))
def test_cut_matches_adjacency_matrix(seed):
    rng = np.random.default_rng(seed)
    n, k = int(rng.integers(2, 13)), int(rng.integers(1, 5))
    A = np.triu(rng.random((n, n)) < 0.4, 1)
    edges = [(int(u), int(v)) for u, v in zip(*np.nonzero(A))]
    rp, ci = csr_from_undirected(n, edges)
    labels = rng.integers(0, k, size=n).astype(np.int32)
    S = A | A.T
    want = int((S & (labels[:, None] != labels[None, :])).sum())
    cut, sizes = oracle.partition_quality(rp, ci, labels, k)
    assert cut == want
    assert sizes.tolist() == [int((labels == p).sum()) for p in range(k)]
    assert 0.0 <= oracle.edge_cut_ratio(cut, max(int(rp[-1]), 1)) <= 1.0
    assert 1.0 <= oracle.vertex_balance(sizes) <= k


def test_self_loops_never_cut_and_parallel_entries_count():
    rowptr = np.array([0, 3, 5], dtype=np.int64)
    colidx = np.array([0, 1, 1, 0, 0], dtype=np.int32)      # 0: self loop + (0,1) twice; 1: (1,0) twice
    cut, _ = oracle.partition_quality(rowptr, colidx, np.array([0, 1]), 2)
    assert cut == 4


def test_out_of_range_labels_are_rejected():
    rp, ci = csr_from_undirected(3, [(0, 1), (1, 2)])
    with pytest.raises(ValueError):
        oracle.partition_quality(rp, ci, np.array([0, 2, 1]), 2)
    with pytest.raises(ValueError):
        oracle.permutation(np.array([0, -1, 1]), 2)


def test_permutation_properties():
    rng = np.random.default_rng(4)
    n, k = 500, 7
    labels = rng.integers(0, k, size=n).astype(np.int32)
    labels[labels == 3] = 2                                  # an empty partition in the middle
    new_id, order = oracle.permutation(labels, k)
    assert sorted(new_id.tolist()) == list(range(n))        # bijection
    np.testing.assert_array_equal(order[new_id], np.arange(n))
    sorted_labels = labels[order]
    assert np.all(np.diff(sorted_labels) >= 0)              # partitions consecutive, ascending
    for p in range(k):
        members = order[sorted_labels == p]
        assert np.all(np.diff(members) > 0)                 # original order kept inside a partition
    np.testing.assert_array_equal(order, np.argsort(labels, kind="stable"))


def test_gap_and_bandwidth_by_hand():
    n = 9
    rp, ci = csr_from_undirected(n, [(i, i + 1) for i in range(n - 1)])
    assert oracle.edge_gap_sum(rp, ci) == 2 * (n - 1)       # identity ids on a path
    assert oracle.vertex_bandwidth_sum(rp, ci) == n          # every vertex's farthest neighbour is 1 away
    # star with centre 0 and leaves 1..4: gaps 1,2,3,4 each stored twice; bandwidths 4,1,2,3,4
    rp, ci = csr_from_undirected(5, [(0, j) for j in range(1, 5)])
    assert oracle.edge_gap_sum(rp, ci) == 2 * (1 + 2 + 3 + 4)
    assert oracle.vertex_bandwidth_sum(rp, ci) == 4 + 1 + 2 + 3 + 4
    # relabel the centre to the middle: pi = [2,0,1,3,4] -> gaps 2,1,1,2
    pi = np.array([2, 0, 1, 3, 4], dtype=np.int32)
    assert oracle.edge_gap_sum(rp, ci, pi) == 2 * (2 + 1 + 1 + 2)
    assert oracle.vertex_bandwidth_sum(rp, ci, pi) == 2 + 2 + 1 + 1 + 2
    # isolated vertices contribute nothing
    rp2 = np.array([0, 0, 1, 2, 2], dtype=np.int64)
    ci2 = np.array([2, 1], dtype=np.int32)
    assert oracle.edge_gap_sum(rp2, ci2) == 2 and oracle.vertex_bandwidth_sum(rp2, ci2) == 2


@pytest.mark.parametrize("seed", range(4))
def test_gap_matches_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(3, 12))
    A = np.triu(rng.random((n, n)) < 0.5, 1)
    rp, ci = csr_from_undirected(n, [(int(u), int(v)) for u, v in zip(*np.nonzero(A))])
    pi = rng.permutation(n).astype(np.int32)
    S = A | A.T
    gaps = np.abs(pi[:, None].astype(np.int64) - pi[None, :]) * S
    assert oracle.edge_gap_sum(rp, ci, pi) == int(gaps.sum())
    assert oracle.vertex_bandwidth_sum(rp, ci, pi) == int(gaps.max(axis=1).sum())


def test_clustered_ids_shrink_gaps_on_a_block_graph():
    # two cliques whose vertices are interleaved: grouping them makes every gap small
    n = 12
    labels = (np.arange(n) % 2).astype(np.int32)
    edges = [(u, v) for u in range(n) for v in range(u + 1, n) if labels[u] == labels[v]]
    rp, ci = csr_from_undirected(n, edges)
    pi, _ = oracle.permutation(labels, 2)
    assert oracle.edge_gap_sum(rp, ci, pi) < oracle.edge_gap_sum(rp, ci)
    assert oracle.partition_quality(rp, ci, labels, 2)[0] == 0


# ---- the graph rewritten under the new ids ---------------------------------------------------


def _random_graph(rng, n, m, hub=None):
    """Random undirected multigraph-free edge list, optionally with one vertex joined to many."""
    e = set()
    while len(e) < m:
        u, v = (int(t) for t in rng.integers(0, n, 2))
        if u != v:
            e.add((min(u, v), max(u, v)))
    if hub is not None:
        e |= {(min(hub, v), max(hub, v)) for v in range(n) if v != hub and v % 3}
    return csr_from_undirected(n, sorted(e))


def test_reorder_worked_example(golden_dir):
    g = _golden_rows(golden_dir / "reorder_worked.txt")
    rp, ci = csr_from_undirected(5, [(0, 1), (0, 2), (0, 4), (1, 3), (2, 4)])
    new_id, _ = oracle.permutation(np.array(g["labels"], dtype=np.int32), 2)
    assert new_id.tolist() == [int(t) for t in g["new_id"]]
    nrp, nci = oracle.reorder_csr(rp, ci, new_id)
    assert nrp.tolist() == [int(t) for t in g["new_rowptr"]]
    assert nci.tolist() == [int(t) for t in g["new_colidx"]]


def test_reorder_is_the_permuted_matrix():
    """Rewriting under pi is P A P^T: a library's sparse fancy indexing, never the oracle's own loop."""
    sp = pytest.importorskip("scipy.sparse")
    rng = np.random.default_rng(3)
    for n, m, hub in [(40, 90, None), (300, 1500, 7), (1000, 400, 999)]:   # the last: many empty rows
        rp, ci = _random_graph(rng, n, m, hub)
        new_id = rng.permutation(n).astype(np.int32)
        order = np.argsort(new_id)
        A = sp.csr_matrix((np.ones(len(ci), dtype=np.int8), ci, rp), shape=(n, n))
        B = A[order][:, order].tocsr()
        B.sort_indices()
        nrp, nci = oracle.reorder_csr(rp, ci, new_id)
        np.testing.assert_array_equal(nrp, B.indptr)
        np.testing.assert_array_equal(nci, B.indices)


def test_reorder_carries_the_metrics_over():
    """Gap sum, bandwidth sum and cut of (G, pi) are those of the rewritten graph under the identity."""
    rng = np.random.default_rng(4)
    n, k = 500, 6
    rp, ci = _random_graph(rng, n, 2500, hub=11)
    labels = rng.integers(0, k, n).astype(np.int32)
    new_id, order = oracle.permutation(labels, k)
    nrp, nci = oracle.reorder_csr(rp, ci, new_id)
    assert oracle.edge_gap_sum(nrp, nci) == oracle.edge_gap_sum(rp, ci, new_id)
    assert oracle.vertex_bandwidth_sum(nrp, nci) == oracle.vertex_bandwidth_sum(rp, ci, new_id)
    cut, sizes = oracle.partition_quality(rp, ci, labels, k)
    cut2, sizes2 = oracle.partition_quality(nrp, nci, labels[order], k)
    assert cut2 == cut and sizes2.tolist() == sizes.tolist()
    assert (np.diff(labels[order]) >= 0).all()                     # partitions are contiguous id ranges
    np.testing.assert_array_equal(np.diff(nrp), np.diff(rp)[order])  # degrees travel with the vertices


def test_reorder_identity_inverse_and_multiplicity():
    rng = np.random.default_rng(5)
    n = 200
    rp, ci = _random_graph(rng, n, 700)
    ident = np.arange(n, dtype=np.int32)
    nrp, nci = oracle.reorder_csr(rp, ci, ident)          # rows already sorted: unchanged
    np.testing.assert_array_equal(nrp, rp)
    np.testing.assert_array_equal(nci, ci)
    pi = rng.permutation(n).astype(np.int32)
    inv = np.argsort(pi).astype(np.int32)
    brp, bci = oracle.reorder_csr(*oracle.reorder_csr(rp, ci, pi), inv)
    np.testing.assert_array_equal(brp, rp)
    np.testing.assert_array_equal(bci, ci)
    # unsorted rows, a parallel edge and a self-loop: sorted, multiplicity kept
    rp2 = np.array([0, 4, 5, 6], dtype=np.int64)
    ci2 = np.array([2, 1, 2, 0, 0, 0], dtype=np.int32)
    nrp, nci = oracle.reorder_csr(rp2, ci2, np.array([2, 0, 1], dtype=np.int32))
    assert nrp.tolist() == [0, 1, 2, 6] and nci.tolist() == [2, 2, 0, 1, 1, 2]
    with pytest.raises(ValueError):
        oracle.reorder_csr(rp2, ci2, np.array([0, 0, 1], dtype=np.int32))     # not a bijection
