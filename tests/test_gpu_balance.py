"""partition_balance on the GPU against the oracle: integer work and a counter-based draw, so every
label and every statistic must be equal bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import embedpart as ep
from paper_2604_01000_amd import synth

from parity import DEV

pytestmark = pytest.mark.gpu


def _device_balance(rowptr, labels, k, beta, seed, max_rounds, vclass=None, class_id=0):
    n = labels.shape[0]
    rp = rowptr.to(DEV) if torch.is_tensor(rowptr) else torch.from_numpy(np.asarray(rowptr)).to(DEV)
    lab = torch.from_numpy(np.asarray(labels, dtype=np.int32)).to(DEV)
    vc = None if vclass is None else torch.from_numpy(np.asarray(vclass, dtype=np.uint8)).to(DEV)
    stats = torch.full((3,), -7, dtype=torch.int64, device=DEV)
    ws = ep.workspace(ep.balance_workspace_bytes(n), DEV)
    ep.partition_balance(n, k, rp, vc, class_id, beta, seed, max_rounds, lab, stats, ws)
    torch.cuda.synchronize()
    return lab.cpu().numpy(), stats.cpu().numpy()


def _skewed_labels(n, k, seed):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.ones(k) * 0.5)
    return rng.choice(k, size=n, p=p).astype(np.int32)


@pytest.mark.parametrize("n,k,beta,rounds,i64", [
    (1, 1, 1.0, 4, False), (257, 2, 1.0, 8, False), (5_003, 8, 1.05, 16, False), (20_011, 64, 1.2, 16, True),
    (70_001, 255, 1.05, 32, True), (40_000, 5, 1.0, 1, False), (40_000, 5, 1.0, 0, False),
    # beyond 2^18 vertices the rounds run as a chain of launches instead of one
    (300_007, 16, 1.05, 16, True), (280_001, 6, 1.1, 8, False), (262_144, 40, 1.05, 16, False), (262_145, 40, 1.05, 16, False),
])
def test_balance_equals_oracle(n, k, beta, rounds, i64):
    rng = np.random.default_rng(n + k)
    deg = rng.integers(0, 40, n) * (rng.random(n) < 0.9)           # some isolated vertices, many ties
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64 if i64 else np.int32)
    labels = _skewed_labels(n, k, n)
    want, st_or = oracle.balance(rowptr, labels, k, beta, seed=n, max_rounds=rounds)
    got, st = _device_balance(rowptr, labels, k, beta, n, rounds)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(st, st_or)
    if rounds >= 16:
        assert st[2] == 0


@pytest.mark.parametrize("n,k,lo,hi", [(30_011, 200, 90, 400), (20_000, 8, 250, 3_000), (25_000, 64, 0, 600),
                                      (6_000, 3, 100_000, 2_000_000), (270_000, 8, 250, 3_000), (300_000, 200, 60, 400),
                                      (270_001, 3, 100_000, 2_000_000), (263_000, 64, 0, 16_000_000)])
def test_balance_with_large_degrees_equals_oracle(n, k, lo, hi):
    """Degrees beyond the exact bins of the degree histogram (min(256, 16384 / k) - 1 and up share the last bin):
    the range that holds the threshold degree is counted again with narrower bins, inside the one launch of the
    small graphs and as further launches of the chain beyond 2^18 vertices, until it is one degree wide.  All must
    pick the oracle's movers.  (Degrees stay below 2^24, beyond which the device treats them as equal.)"""
    rng = np.random.default_rng(n + k)
    deg = rng.integers(lo, hi, n).astype(np.int64)
    deg[rng.random(n) < 0.3] = rng.integers(0, 30, n)[: int((rng.random(n) < 0.3).sum())][0]   # and a block of small ones
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    labels = _skewed_labels(n, k, n + 1)
    want, st_or = oracle.balance(rowptr, labels, k, 1.05, seed=n, max_rounds=12)
    got, st = _device_balance(rowptr, labels, k, 1.05, n, 12)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(st, st_or)


def test_three_classes_in_sequence_on_a_benchmark_graph():
    """Alg. 3 as a whole on the arxiv-like workload: K-Means labels, then the three loops (training,
    validation, remaining vertices) one after the other on the same label vector."""
    w = synth.WORKLOADS["arxiv_like"]
    rowptr, _, blocks = synth.sbm_graph(w, DEV)
    rng = np.random.default_rng(5)
    vclass = rng.choice(3, size=w.n, p=[0.55, 0.15, 0.30]).astype(np.uint8)
    labels = (blocks.cpu().numpy() % w.k).astype(np.int32)
    labels[rng.random(w.n) < 0.3] = 0                                # an overloaded partition
    rp_np = rowptr.cpu().numpy()
    dev = torch.from_numpy(labels).to(DEV)
    ws = ep.workspace(ep.balance_workspace_bytes(w.n), DEV)
    vc = torch.from_numpy(vclass).to(DEV)
    ref = labels.copy()
    for cls, beta in ((0, 1.05), (1, 1.05), (2, 1.1)):
        stats = torch.zeros(3, dtype=torch.int64, device=DEV)
        ep.partition_balance(w.n, w.k, rowptr, vc, cls, beta, 99 + cls, 32, dev, stats, ws)
        torch.cuda.synchronize()
        ref, st_or = oracle.balance(rp_np, ref, w.k, beta, seed=99 + cls, max_rounds=32, vclass=vclass, class_id=cls)
        np.testing.assert_array_equal(dev.cpu().numpy(), ref)
        np.testing.assert_array_equal(stats.cpu().numpy(), st_or)
        assert st_or[2] == 0 and st_or[1] > 0
    sizes = np.bincount(ref, minlength=w.k)
    assert sizes.sum() == w.n


def test_balance_is_reproducible_and_leaves_a_balanced_partition_alone():
    n, k = 30_000, 16
    rowptr = np.arange(n + 1, dtype=np.int32) * 3
    labels = _skewed_labels(n, k, 1)
    a, sa = _device_balance(rowptr, labels, k, 1.05, 4, 16)
    b, sb = _device_balance(rowptr, labels, k, 1.05, 4, 16)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(sa, sb)
    c, sc = _device_balance(rowptr, a, k, 1.05, 4, 16)             # already balanced: nothing moves
    np.testing.assert_array_equal(c, a)
    np.testing.assert_array_equal(sc, [0, 0, 0])
    d, _ = _device_balance(rowptr, labels, k, 1.05, 5, 16)         # another seed: other destinations
    assert not np.array_equal(a, d)


@pytest.mark.parametrize("name,sample,with_classes", [("tiny", 0, True), ("arxiv_like", 0, False), ("tiny", 2048, True)])
def test_cluster_and_balance_is_phase_two_of_the_method(name, sample, with_classes):
    """The one-call form of the paper's Alg. 3 equals its parts bit for bit (same kernels, same order), and
    the balancing it performs is the oracle's applied to the labels the clustering produced."""
    from parity import Kmeans
    w = synth.WORKLOADS[name]
    X = synth.embeddings(w, DEV)
    rowptr, _, _ = synth.sbm_graph(w, DEV)
    rng = np.random.default_rng(w.seed)
    vclass_np = rng.choice(3, size=w.n, p=[0.5, 0.2, 0.3]).astype(np.uint8) if with_classes else None
    vclass = None if vclass_np is None else torch.from_numpy(vclass_np).to(DEV)
    beta, seed, rounds = (1.05, 1.1, 1.2), 77, 16
    rows = oracle.init_indices(w.seed, w.n, sample if sample else w.k)
    rows_t = torch.as_tensor(np.asarray(rows), dtype=torch.int64)

    p = ep.problem(X, w.k)
    Cc = torch.empty((w.k, w.d), dtype=torch.float32, device=DEV)
    labels = torch.full((w.n,), -7, dtype=torch.int32, device=DEV)
    counts = torch.full((w.k,), -7, dtype=torch.int64, device=DEV)
    stats = torch.full((9,), -7, dtype=torch.int64, device=DEV)
    ws = ep.workspace(ep.cluster_and_balance_workspace_bytes(p, sample), DEV)
    opt = ep.phase2_options(beta, seed, w.iters, rounds, sample)
    ep.cluster_and_balance(p, X, rowptr, vclass, opt, rows_t, Cc, labels, counts, stats, ws)
    torch.cuda.synchronize()

    # the parts, called one by one
    km = Kmeans(X, w.k)
    if sample:
        sws = ep.workspace(ep.kmeans_sampled_workspace_bytes(km.p, sample), DEV)
        ep.kmeans_run_sampled(km.p, X, rows_t, w.iters, km.C, km.labels, km.counts, None, sws)
    else:
        km.init(rows)
        ep.kmeans_run(km.p, X, w.iters, km.C, km.labels, km.counts, None, 0, km.ws)
    torch.cuda.synchronize()
    clustered = km.labels.cpu().numpy()
    assert torch.equal(Cc, km.C) and torch.equal(counts, km.counts)

    want, want_stats = clustered.copy(), []
    rp_np = rowptr.cpu().numpy().astype(np.int64)
    for cls in ([0, 1, 2] if with_classes else [2]):
        want, st = oracle.balance(rp_np, want, w.k, beta[cls], seed + cls, rounds, vclass_np, cls)
        want_stats.append(st)
    np.testing.assert_array_equal(labels.cpu().numpy(), want)
    got_stats = stats.cpu().numpy().reshape(3, 3)
    np.testing.assert_array_equal(got_stats[3 - len(want_stats):], np.stack(want_stats))
    sizes = np.bincount(want, minlength=w.k)
    if not with_classes:
        assert sizes.max() <= max(np.floor(beta[2] * w.n / w.k), np.ceil(w.n / w.k))
