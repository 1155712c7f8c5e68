"""Pins of the oracle's balancing step (EmbedPart paper, Alg. 3 loops with the migration policy of Alg. 4):
a hand-worked case (tests/golden/balance_worked.txt), properties that follow from the algorithm's text, an
independent selection of the movers, the sampling proportions, and the draw function restated with Python
integers."""
from pathlib import Path

import numpy as np
import pytest

import oracle

GOLDEN = Path(__file__).resolve().parent / "golden" / "balance_worked.txt"
M64 = (1 << 64) - 1


def _rowptr(deg):
    return np.concatenate([[0], np.cumsum(np.asarray(deg, dtype=np.int64))])


def _draw64(seed, rnd, v):
    z = (seed + ((rnd << 32) + v + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _capacity(total, k, beta):
    return max(int(np.floor(beta * float(total) / float(k))), -(-total // k))


def test_hand_worked_case_from_golden_file():
    """8 vertices, k = 2, beta = 1: partition 0 holds 6, partition 1 holds 2; capacity 4, so the two
    members of partition 0 with the smallest degree move, and partition 1 is the only destination."""
    rows = [l.split() for l in GOLDEN.read_text().splitlines() if l and not l.startswith("#")]
    deg = [int(r[1]) for r in rows]
    before = [int(r[2]) for r in rows]
    after = [int(r[3]) for r in rows]
    got, stats = oracle.balance(_rowptr(deg), before, 2, 1.0, seed=123)
    np.testing.assert_array_equal(got, after)
    np.testing.assert_array_equal(stats, [1, 2, 0])


def test_balanced_input_is_left_alone_and_bad_arguments():
    labels = np.arange(40) % 4
    got, stats = oracle.balance(_rowptr(np.ones(40)), labels, 4, 1.0, seed=1)
    np.testing.assert_array_equal(got, labels)
    np.testing.assert_array_equal(stats, [0, 0, 0])
    with pytest.raises(ValueError):
        oracle.balance(_rowptr(np.ones(40)), labels, 4, 0.9, seed=1)       # beta < 1 can never be met
    with pytest.raises(ValueError):
        oracle.balance(_rowptr(np.ones(40)), labels + 1, 4, 1.0, seed=1)   # label out of range


@pytest.mark.parametrize("n,k,beta,seed", [(5000, 8, 1.05, 3), (3001, 5, 1.0, 4), (20000, 64, 1.2, 5)])
def test_properties_and_independent_selection_of_the_movers(n, k, beta, seed):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 30, n)
    p = rng.dirichlet(np.ones(k) * 0.6)
    labels = rng.choice(k, size=n, p=p).astype(np.int32)
    rp = _rowptr(deg)
    # one round only: who moves is fully determined by degrees and ids
    one, st1 = oracle.balance(rp, labels, k, beta, seed=seed, max_rounds=1)
    L = np.bincount(labels, minlength=k)
    C = _capacity(n, k, beta)
    F = int(np.maximum(C - L, 0).sum())
    cumf = np.cumsum(np.maximum(C - L, 0))
    moved = np.nonzero(one != labels)[0]
    expect = []
    for i in range(k):
        if L[i] > C:
            members = np.nonzero(labels == i)[0]
            order = np.lexsort((members, deg[members]))            # degree first, then vertex id
            expect.extend(members[order[:L[i] - C]].tolist())
    # a mover may draw any underloaded partition but never its own (it is overloaded, f = 0 there)
    np.testing.assert_array_equal(np.sort(moved), np.sort(np.array(expect, dtype=np.int64)))
    assert st1[1] == len(expect) and (st1[0] == 1) == (len(expect) > 0)
    for v in moved[:200]:
        r = _draw64(seed, 0, int(v)) % F
        assert one[v] == int(np.searchsorted(cumf, r, side="right"))
    # run to the end: every load within capacity, totals kept
    done, st = oracle.balance(rp, labels, k, beta, seed=seed)
    Ld = np.bincount(done, minlength=k)
    assert Ld.sum() == n and Ld.max() <= C and st[2] == 0
    assert st[0] >= 1 and st[1] >= len(expect)


def test_only_the_named_class_moves_and_capacity_counts_that_class():
    rng = np.random.default_rng(9)
    n, k = 6000, 6
    labels = rng.choice(k, size=n, p=[0.4, 0.2, 0.1, 0.1, 0.1, 0.1]).astype(np.int32)
    vclass = rng.choice(3, size=n, p=[0.1, 0.05, 0.85]).astype(np.uint8)
    rp = _rowptr(rng.integers(1, 9, n))
    got, st = oracle.balance(rp, labels, k, 1.05, seed=2, vclass=vclass, class_id=1)
    other = vclass != 1
    np.testing.assert_array_equal(got[other], labels[other])
    loads = np.bincount(got[vclass == 1], minlength=k)
    assert loads.max() <= _capacity(int((vclass == 1).sum()), k, 1.05) and st[2] == 0


def test_destinations_follow_free_capacity():
    """Two underloaded partitions with free capacity 3 : 1 receive movers in about that proportion."""
    n = 40000
    labels = np.zeros(n, dtype=np.int32)
    labels[:4000] = 1          # partition 1: 4000, partition 2: 8000 (below), partition 0: the rest
    labels[4000:12000] = 2
    # capacity with beta = 1.0: ceil(40000 / 3) = 13334 -> free: 9334 and 5334; partition 0 sheds 14666
    got, st = oracle.balance(_rowptr(np.ones(n)), labels, 3, 1.0, seed=77, max_rounds=1)
    to1 = np.count_nonzero((labels == 0) & (got == 1))
    to2 = np.count_nonzero((labels == 0) & (got == 2))
    assert to1 + to2 == 28000 - 13334
    share = to1 / (to1 + to2)
    assert abs(share - 9334 / (9334 + 5334)) < 0.02
