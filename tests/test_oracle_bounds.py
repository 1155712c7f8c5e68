"""Pins of the oracle's Lloyd rounds with bounds and incremental sums (oracle.lloyd_bounds): they are the plain
Lloyd rounds reached with less work, so every result must equal oracle.lloyd's; a hand-worked case fixes which
points are skipped; an audit searches every skipped point and must find no label that would have changed."""
import numpy as np
import pytest

import oracle


def _golden(path):
    out = {}
    for line in path.read_text().splitlines():
        if line and not line.startswith("#"):
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def test_hand_worked_bounds_1d(golden_dir):
    g = _golden(golden_dir / "bounds_1d_worked.txt")
    X = np.array(g["points"], dtype=np.float32)[:, None]
    idx = np.array(g["init_rows"], dtype=np.int64)
    r = oracle.lloyd_bounds(X, 2, 4, idx, audit=False)
    assert r["skipped"].tolist() == g["skipped"]
    assert r["moved"].tolist() == g["moved"]
    assert r["labels"].tolist() == g["labels_round4"]
    np.testing.assert_allclose(r["C"][:, 0], g["centroids_round4"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["obj_hist"], g["objective"], rtol=1e-12)
    for t in (1, 2, 3):   # and round by round against the first hand-worked file
        h = _golden(golden_dir / "lloyd_1d_worked.txt")
        rt = oracle.lloyd_bounds(X, 2, t, idx)
        assert rt["labels"].tolist() == h[f"labels_round{t}"]
        np.testing.assert_allclose(rt["C"][:, 0], h[f"centroids_round{t}"], rtol=0, atol=1e-12)


def _mixture(n, d, comps, seed, relu=True, sigma=1.0):
    rng = np.random.default_rng(seed)
    means = 2.0 * rng.normal(size=(comps, d))
    X = means[rng.integers(0, comps, size=n)] + sigma * rng.normal(size=(n, d))
    if relu:
        X = np.maximum(X, 0.0)
    return X.astype(np.float32)


CASES = [  # n, d, k, components, iters, flags
    (3000, 16, 8, 12, 12, 0), (2000, 64, 4, 8, 10, 0), (4000, 8, 30, 20, 15, 0), (1500, 32, 64, 40, 8, 0),
    (2500, 128, 16, 47, 10, oracle.FLAG_BF16_CENTROIDS), (500, 3, 1, 2, 4, 0), (64, 5, 64, 3, 3, 0),
]


@pytest.mark.parametrize("n,d,k,comps,iters,flags", CASES)
def test_bounds_rounds_equal_plain_rounds(n, d, k, comps, iters, flags):
    X = _mixture(n, d, comps, seed=n + k)
    if flags & oracle.FLAG_BF16_CENTROIDS:
        X = oracle.round_bf16(X).astype(np.float32)
    idx = oracle.init_indices(n, n, k)
    plain = oracle.lloyd(X, k, iters, idx, flags=flags)
    for audit in (False, True):
        fast = oracle.lloyd_bounds(X, k, iters, idx, flags=flags, audit=audit)
        np.testing.assert_array_equal(fast["labels"], plain["labels"])
        np.testing.assert_array_equal(fast["counts"], plain["counts"])
        np.testing.assert_allclose(fast["C"], plain["C"], rtol=1e-11, atol=1e-11)      # sums kept between rounds
        np.testing.assert_allclose(fast["obj_hist"], plain["obj_hist"], rtol=1e-11)
        assert fast["violations"] == 0
        assert fast["skipped"][0] == 0 and fast["moved"][0] == n
        assert np.all(fast["skipped"] >= 0) and np.all(fast["skipped"] <= n)
    # the audit only looks: it changes nothing, and it counts the same points as skipped
    np.testing.assert_array_equal(oracle.lloyd_bounds(X, k, iters, idx, flags=flags, audit=True)["skipped"],
                                  fast["skipped"])


def test_every_prefix_of_rounds_equals_plain():
    X = _mixture(2000, 24, 10, seed=5)
    idx = oracle.init_indices(9, 2000, 6)
    for t in range(0, 9):
        plain, fast = oracle.lloyd(X, 6, t, idx), oracle.lloyd_bounds(X, 6, t, idx)
        np.testing.assert_array_equal(fast["labels"][:0 if t == 0 else None], plain["labels"][:0 if t == 0 else None])
        np.testing.assert_allclose(fast["C"], plain["C"], rtol=1e-11, atol=1e-11)


def test_bounds_do_skip_and_everything_is_skipped_at_the_fixed_point():
    """Well separated blobs: from the round after the labels stop changing, no point is searched."""
    rng = np.random.default_rng(2)
    means = 50.0 * rng.normal(size=(5, 6))
    X = (means[rng.integers(0, 5, size=3000)] + rng.normal(size=(3000, 6))).astype(np.float32)
    idx = oracle.init_indices(4, 3000, 5)
    r = oracle.lloyd_bounds(X, 5, 30, idx, audit=True)
    assert r["violations"] == 0
    still = np.nonzero(r["moved"] == 0)[0]
    assert len(still) >= 2
    assert np.all(r["skipped"][still[0] + 1:] == 3000)       # centroids stand still: every bound stands
    assert r["skipped"][1:].sum() > 0


def test_duplicate_centroids_and_exact_ties_are_never_skipped_wrongly():
    """Two identical initial centroids and points at equal distance from two centroids: the lowest index must
    keep winning, with bounds exactly as without."""
    X = np.array([[0, 0], [0, 0], [4, 0], [2, 0], [2, 3], [2, -3], [6, 1], [6, -1]], dtype=np.float32)
    idx = np.array([0, 1, 2], dtype=np.int64)                # centroids 0 and 1 coincide
    for t in range(1, 6):
        plain, fast = oracle.lloyd(X, 3, t, idx), oracle.lloyd_bounds(X, 3, t, idx, audit=True)
        np.testing.assert_array_equal(fast["labels"], plain["labels"])
        np.testing.assert_array_equal(fast["counts"], plain["counts"])
        assert fast["violations"] == 0


def test_bad_arguments():
    X = np.zeros((4, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.lloyd_bounds(X, 2, 1, np.array([0, 9], dtype=np.int64))
    with pytest.raises(ValueError):
        oracle.lloyd_bounds(X, 2, 1, np.array([0, 1], dtype=np.int64), flags=oracle.FLAG_FINAL_REASSIGN)
