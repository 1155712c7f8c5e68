"""Pins for the oracle's K-Means (CPU only).

Each test checks the oracle against something that is not the oracle: a hand-worked
run, an independent brute-force loop nest on exactly representable inputs, a closed
form, a textbook special case or an invariant of Lloyd's algorithm.  A dropped term,
a wrong sign, a swapped index or a transposed operand in the oracle fails at least
one of them.
"""
import itertools

import numpy as np
import pytest

import oracle


def _parse_golden(path):
    out = {}
    for line in path.read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def test_hand_worked_1d_run(golden_dir):
    g = _parse_golden(golden_dir / "lloyd_1d_worked.txt")
    X = np.array(g["points"], dtype=np.float32)[:, None]
    idx = np.array(g["init_rows"], dtype=np.int64)
    for rounds in (1, 2, 3):
        r = oracle.lloyd(X, 2, rounds, idx)
        assert r["labels"].tolist() == [int(v) for v in g[f"labels_round{rounds}"]]
        np.testing.assert_allclose(r["C"][:, 0], g[f"centroids_round{rounds}"], rtol=0, atol=1e-12)
        np.testing.assert_allclose(r["obj_hist"], g["objective"][:rounds], rtol=1e-13)
    assert r["counts"].tolist() == [int(v) for v in g["counts_round3"]]


def _brute_assign(X, C):
    """Independent nearest-centroid search: python loops, exact on small integers."""
    n, d = X.shape
    labels, best, second = [], [], []
    for i in range(n):
        dists = []
        for j in range(C.shape[0]):
            s = 0
            for m in range(d):
                s += (int(X[i, m]) - int(C[j, m])) ** 2
            dists.append(s)
        lo = min(dists)
        labels.append(dists.index(lo))          # first index of the minimum
        best.append(lo)
        rest = sorted(dists)
        second.append(rest[1] if len(rest) > 1 else np.inf)
    return np.array(labels), np.array(best, dtype=np.float64), np.array(second, dtype=np.float64)


@pytest.mark.parametrize("n,d,k,seed", [(64, 4, 5, 0), (50, 3, 2, 1), (33, 1, 7, 2), (40, 6, 1, 3)])
def test_assign_matches_brute_force_on_integers(n, d, k, seed):
    rng = np.random.default_rng(seed)
    X = rng.integers(-9, 10, size=(n, d)).astype(np.float32)
    C = rng.integers(-9, 10, size=(k, d)).astype(np.float64)
    labels, best, second, obj = oracle.assign(X, C)
    bl, bb, bs = _brute_assign(X, C)
    assert labels.tolist() == bl.tolist()
    np.testing.assert_array_equal(best, bb)
    np.testing.assert_array_equal(second, bs)
    assert obj == bb.sum()


def test_assign_is_not_transposed_or_sign_flipped():
    # One point, asymmetric coordinates: d2 to c0 = (1-4)^2 + (2-6)^2 = 25, to c1 = (1-0)^2 + (2-2)^2 = 1.
    X = np.array([[1.0, 2.0]], dtype=np.float32)
    C = np.array([[4.0, 6.0], [0.0, 2.0]])
    labels, best, second, obj = oracle.assign(X, C)
    assert labels.tolist() == [1] and best[0] == 1.0 and second[0] == 25.0 and obj == 1.0


def test_ties_go_to_the_lowest_index_and_duplicates_starve():
    X = np.array([[1.0], [3.0], [5.0]], dtype=np.float32)
    C = np.array([[0.0], [2.0], [2.0], [6.0]])            # x=1 ties c0/c1; c2 duplicates c1
    labels, best, second, _ = oracle.assign(X, C)
    assert labels.tolist() == [0, 1, 3]
    assert best.tolist() == [1.0, 1.0, 1.0] and second.tolist() == [1.0, 1.0, 9.0]
    Cn, counts, empty = oracle.update(X, labels, C)
    assert counts.tolist() == [1, 1, 0, 1] and empty == 1
    assert Cn[:, 0].tolist() == [1.0, 3.0, 2.0, 5.0]       # empty cluster keeps its centroid


def test_k1_gives_global_mean_and_total_variance():
    rng = np.random.default_rng(5)
    X = rng.normal(size=(500, 7)).astype(np.float32)
    r = oracle.lloyd(X, 1, 2, np.array([17]))
    mean = X.astype(np.float64).mean(axis=0)
    np.testing.assert_allclose(r["C"][0], mean, rtol=1e-12, atol=1e-14)
    # round 1 measures against row 17, round 2 against the mean (two-pass variance)
    np.testing.assert_allclose(r["obj_hist"][0], ((X.astype(np.float64) - X[17].astype(np.float64)) ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(r["obj_hist"][1], ((X.astype(np.float64) - mean) ** 2).sum(), rtol=1e-12)
    assert r["counts"].tolist() == [500] and set(r["labels"].tolist()) == {0}


def test_k_equals_n_is_the_identity():
    rng = np.random.default_rng(6)
    X = rng.normal(size=(23, 5)).astype(np.float32)
    r = oracle.lloyd(X, 23, 2, np.arange(23))
    assert r["labels"].tolist() == list(range(23))
    assert r["obj_hist"].tolist() == [0.0, 0.0]
    np.testing.assert_array_equal(r["C"], X.astype(np.float64))


def test_separated_blobs_are_recovered_in_one_round():
    rng = np.random.default_rng(7)
    centres = np.array([[0, 0, 0], [100, 0, 0], [0, 100, 0], [0, 0, 100]], dtype=np.float64)
    truth = rng.integers(0, 4, size=400)
    truth[:4] = [0, 1, 2, 3]                               # rows 0..3: one per blob, used as init
    X = (centres[truth] + 1e-3 * rng.normal(size=(400, 3))).astype(np.float32)
    r = oracle.lloyd(X, 4, 1, np.arange(4))
    assert r["labels"].tolist() == truth.tolist()
    for j in range(4):
        np.testing.assert_allclose(r["C"][j], X[truth == j].astype(np.float64).mean(axis=0), rtol=1e-12, atol=1e-12)


def _random_problem(seed, n=600, d=9, k=6):
    rng = np.random.default_rng(seed)
    means = 3.0 * rng.normal(size=(k + 2, d))
    X = (means[rng.integers(0, k + 2, size=n)] + rng.normal(size=(n, d))).astype(np.float32)
    idx = oracle.init_indices(seed, n, k)
    return X, idx, k


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_lloyd_invariants(seed):
    X, idx, k = _random_problem(seed)
    T = 12
    r = oracle.lloyd(X, k, T, idx)
    h = r["obj_hist"]
    assert np.all(h[1:] <= h[:-1] * (1 + 1e-15)), "objective must not increase"
    assert r["counts"].sum() == X.shape[0]
    assert r["labels"].min() >= 0 and r["labels"].max() < k
    np.testing.assert_array_equal(r["counts"], np.bincount(r["labels"], minlength=k))
    Xd = X.astype(np.float64)
    for j in range(k):                                     # centroids are the means of their points
        if r["counts"][j]:
            np.testing.assert_allclose(r["C"][j], Xd[r["labels"] == j].mean(axis=0), rtol=1e-12, atol=1e-13)
    # the objective of round t is the within-cluster scatter about the centroids of round t-1
    prev = oracle.lloyd(X, k, T - 1, idx)
    d2 = ((Xd - prev["C"][r["labels"]]) ** 2).sum()
    np.testing.assert_allclose(h[-1], d2, rtol=1e-12)
    # step by step equals the driver
    C = Xd[idx].copy()
    for t in range(T):
        labels, best, _, obj = oracle.assign(X, C)
        assert obj == h[t]
        C, counts, _ = oracle.update(X, labels, C)
    np.testing.assert_array_equal(C, r["C"])
    np.testing.assert_array_equal(labels, r["labels"])


def test_fixed_point_and_final_reassign():
    X, idx, k = _random_problem(21, n=300, d=4, k=3)
    a = oracle.lloyd(X, k, 60, idx)
    b = oracle.lloyd(X, k, 61, idx)
    np.testing.assert_array_equal(a["labels"], b["labels"])     # converged by then
    np.testing.assert_array_equal(a["C"], b["C"])
    c = oracle.lloyd(X, k, 3, idx, flags=oracle.FLAG_FINAL_REASSIGN)
    d4 = oracle.lloyd(X, k, 4, idx)
    np.testing.assert_array_equal(c["labels"], d4["labels"])    # extra assignment = next round's labels
    assert c["obj_final"] == d4["obj_hist"][3]
    np.testing.assert_array_equal(c["C"], oracle.lloyd(X, k, 3, idx)["C"])


def test_translation_and_permutation_equivariance():
    X, idx, k = _random_problem(31, n=400, d=5, k=4)
    X = np.round(X * 64) / 64                                   # dyadic values: the shift below is exact in fp32
    shift = np.array([8.0, -4.0, 2.0, 16.0, -32.0], dtype=np.float32)
    a = oracle.lloyd(X, k, 5, idx)
    b = oracle.lloyd(X + shift, k, 5, idx)
    np.testing.assert_array_equal(a["labels"], b["labels"])
    np.testing.assert_allclose(b["C"] - shift, a["C"], rtol=0, atol=1e-12)
    perm = np.random.default_rng(1).permutation(X.shape[0])
    inv = np.argsort(perm)
    c = oracle.lloyd(X[perm], k, 5, inv[idx])
    np.testing.assert_array_equal(c["labels"], a["labels"][perm])
    np.testing.assert_allclose(c["C"], a["C"], rtol=1e-12, atol=1e-13)


def test_row_stride_is_honoured():
    X, idx, k = _random_problem(41, n=100, d=6, k=3)
    wide = np.full((100, 10), 1e6, dtype=np.float32)
    wide[:, :6] = X
    a = oracle.lloyd(X, k, 4, idx)
    b = oracle.lloyd(wide[:, :6], k, 4, idx)                    # strided view, ld = 10
    np.testing.assert_array_equal(a["labels"], b["labels"])
    np.testing.assert_array_equal(a["C"], b["C"])


def test_init_indices_distinct_seeded_in_range():
    for n, k, seed in [(10, 10, 0), (20_000, 4, 1), (1000, 999, 7), (170_000, 8, 2)]:
        idx = oracle.init_indices(seed, n, k)
        assert len(set(idx.tolist())) == k and idx.min() >= 0 and idx.max() < n
        np.testing.assert_array_equal(idx, oracle.init_indices(seed, n, k))
    assert oracle.init_indices(1, 1000, 8).tolist() != oracle.init_indices(2, 1000, 8).tolist()
    with pytest.raises(ValueError):
        oracle.init_indices(0, 3, 4)


def test_init_indices_follow_splitmix64():
    # Independent restatement of the published generator with python integers.
    def stream(seed):
        s = seed
        while True:
            s = (s + 0x9E3779B97F4A7C15) % 2**64
            z = s
            z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % 2**64
            z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % 2**64
            yield z ^ (z >> 31)
    for seed, n, k in [(0, 5, 5), (1234567, 37, 20), (2**64 - 1, 1000, 16)]:
        picks = []
        for z in stream(seed):
            r = z % n
            if r not in picks:
                picks.append(r)
            if len(picks) == k:
                break
        assert oracle.init_indices(seed, n, k).tolist() == picks
    # first output of splitmix64 seeded with 0, as widely published
    assert next(stream(0)) == 0xE220A8397B1DCDAF


def test_bf16_rounding_is_nearest_even():
    import torch
    rng = np.random.default_rng(3)
    v = np.concatenate([rng.normal(size=2000) * 10.0 ** rng.integers(-6, 6, size=2000),
                        [0.0, 1.0, -1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 3.3895314e38]])
    got = oracle.round_bf16(v)
    want = torch.from_numpy(v).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(got, want)
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0                  # tie -> even mantissa
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6  # tie -> even mantissa (up)


def test_bf16_centroid_flag_only_changes_the_distances():
    X, idx, k = _random_problem(51, n=300, d=8, k=5)
    C = X.astype(np.float64)[idx] * 1.001
    la, ba, _, _ = oracle.assign(X, C, round_bf16=True)
    lb, bb, _, _ = oracle.assign(X, oracle.round_bf16(C))
    np.testing.assert_array_equal(la, lb)
    np.testing.assert_array_equal(ba, bb)
    r = oracle.lloyd(X, k, 3, idx, flags=oracle.FLAG_BF16_CENTROIDS)
    Xd = X.astype(np.float64)
    for j in range(k):                                          # the means stay full precision
        if r["counts"][j]:
            np.testing.assert_allclose(r["C"][j], Xd[r["labels"] == j].mean(axis=0), rtol=1e-12, atol=1e-13)


def test_exhaustive_optimum_is_never_beaten():
    # Lloyd's objective can only be >= the best over all k^n labelings (tiny case, exhaustive).
    rng = np.random.default_rng(9)
    X = rng.integers(-5, 6, size=(7, 2)).astype(np.float32)
    Xd = X.astype(np.float64)
    best = np.inf
    for lab in itertools.product(range(2), repeat=7):
        lab = np.array(lab)
        s = 0.0
        for j in range(2):
            pts = Xd[lab == j]
            if len(pts):
                s += ((pts - pts.mean(axis=0)) ** 2).sum()
        best = min(best, s)
    r = oracle.lloyd(X, 2, 10, np.array([0, 1]), flags=oracle.FLAG_FINAL_REASSIGN)
    assert r["obj_final"] >= best - 1e-9


# ---- sample-trained K-Means (paper, Sec. "Implementation") ---------------------------------------

def _blobs(n, d, g, seed):
    rng = np.random.default_rng(seed)
    means = 3.0 * rng.standard_normal((g, d))
    return (means[rng.integers(0, g, n)] + rng.standard_normal((n, d))).astype(np.float32)


def test_sampled_identity_sample_is_lloyd_plus_one_assignment():
    X = _blobs(400, 5, 4, 1)
    rows = np.arange(400)
    got = oracle.sampled_kmeans(X, 4, 6, rows)
    ref = oracle.lloyd(X, 4, 6, np.arange(4), flags=oracle.FLAG_FINAL_REASSIGN)
    np.testing.assert_array_equal(got["C"], ref["C"])
    np.testing.assert_array_equal(got["labels"], ref["labels"])
    np.testing.assert_array_equal(got["counts"], ref["counts"])
    np.testing.assert_array_equal(got["obj_hist"], ref["obj_hist"])
    assert got["obj_full"] == ref["obj_final"]


def test_sampled_labels_are_brute_force_nearest_and_training_sees_only_the_sample():
    X = _blobs(900, 3, 5, 2)
    rows = oracle.init_indices(7, 900, 120)
    got = oracle.sampled_kmeans(X, 5, 8, rows)
    # training = Lloyd on the gathered rows, first k rows as the start
    ref = oracle.lloyd(X[rows], 5, 8, np.arange(5))
    np.testing.assert_array_equal(got["C"], ref["C"])
    np.testing.assert_array_equal(got["counts"], ref["counts"])
    assert got["counts"].sum() == 120
    # labels of ALL rows: exhaustive nearest centroid in numpy fp64, lowest index on ties
    d2 = ((X[:, None, :].astype(np.float64) - got["C"][None, :, :]) ** 2).sum(axis=2)
    np.testing.assert_array_equal(got["labels"], d2.argmin(axis=1))
    assert abs(got["obj_full"] - d2.min(axis=1).sum()) <= 1e-9 * got["obj_full"]
    # rows outside the sample do not move the centroids
    X2 = X.copy()
    outside = np.setdiff1d(np.arange(900), rows)
    X2[outside] += 100.0
    again = oracle.sampled_kmeans(X2, 5, 8, rows)
    np.testing.assert_array_equal(again["C"], got["C"])
    np.testing.assert_array_equal(again["labels"][rows], got["labels"][rows])


def test_sampled_order_of_the_sample_names_the_start_and_bad_arguments():
    X = _blobs(300, 2, 3, 3)
    rows = oracle.init_indices(11, 300, 60)
    a = oracle.sampled_kmeans(X, 3, 0, rows)                       # no rounds: C = first k sample rows
    np.testing.assert_array_equal(a["C"], X[rows[:3]].astype(np.float64))
    with pytest.raises(ValueError):
        oracle.sampled_kmeans(X, 3, 2, rows[:2])                   # fewer sample rows than clusters
    with pytest.raises(ValueError):
        oracle.sampled_kmeans(X, 3, 2, np.array([0, 1, 2, 300]))   # row out of range


def test_validate_labels_hand_counted():
    """Ids outside [0, k) counted by hand: k = 3, labels 0 3 -1 2 5 1 -> three offenders (3, -1, 5), the first at
    index 1; a clean vector -> none, first = n."""
    assert oracle.validate_labels([0, 3, -1, 2, 5, 1], 3) == (3, 1)
    assert oracle.validate_labels([0, 1, 2, 2, 1], 3) == (0, 5)
    assert oracle.validate_labels([2, 2, 2], 2) == (3, 0)
    rng = np.random.default_rng(3)
    lab = rng.integers(-2, 9, size=1000).astype(np.int32)
    bad = np.nonzero((lab < 0) | (lab >= 7))[0]
    assert oracle.validate_labels(lab, 7) == (len(bad), int(bad[0]))
