"""kmeans_run with EP_RUN_BOUNDS (distance bounds + incremental sums) on the GPU: the rounds must be the
rounds of the plain run -- the same labels bit for bit in every round, equal counts, centroids and
objectives equal up to the order of fp64 additions -- and so pass every comparison with the oracle that
the plain run passes; the bounds must really skip work once the centroids settle."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import embedpart as ep
from paper_2604_01000_amd import synth

from parity import CENTROID_RTOL, DEV, Guarded, Kmeans, centroid_rel_err, to_np32
from test_gpu_kmeans import _mixture

pytestmark = pytest.mark.gpu

B = ep.EP_RUN_BOUNDS


def _searched(km, iters, flags):
    g = Guarded(iters, torch.int64)
    ep.kmeans_run_searched(km.p, iters, flags, km.run_ws, g.t)
    torch.cuda.synchronize()
    return g.check().cpu().numpy()


def _both(X, k, idx, iters, extra=0):
    plain = Kmeans(X, k).init(idx).run(iters, extra)
    km = Kmeans(X, k).init(idx)
    fast = km.run(iters, B | extra)
    return plain, fast, _searched(km, iters, B | extra)


def _same_rounds(plain, fast, iters, n, exact=True):
    """The bounded run against the plain run.  Searched points go through the same score arithmetic, so for
    equal centroids the labels are equal bit for bit; the centroids themselves agree to the order of fp64
    additions (kept sums against sums from scratch), which can flip a near-tie now and then: with
    exact=False a small number of differing labels is accepted if the objectives still agree."""
    assert fast["counts"].sum() == n
    differing = int(np.count_nonzero(fast["labels"] != plain["labels"]))
    if exact:
        assert differing == 0
    if differing == 0:
        np.testing.assert_array_equal(fast["counts"], plain["counts"])
        assert centroid_rel_err(fast["C"], plain["C"]) <= 1e-6
    else:
        assert differing <= 0.01 * n
    np.testing.assert_allclose(fast["obj_hist"][:iters], plain["obj_hist"][:iters], rtol=1e-6)   # fp32 scores against fp64 sums
    return differing


def _check_rounds_against_oracle(X, k, idx, iters, bf16=False):
    """Every round of the bounded run's own trajectory against the oracle applied to the state the device
    held: labels of round t = the oracle's assignment to the device's centroids of round t - 1 (differences
    only at near-ties), counts exact, centroids = the oracle's means of the device's labels, objective."""
    from parity import centroids_used, label_mismatches
    X32 = to_np32(X)
    n = X32.shape[0]
    C_prev = X32[idx].astype(np.float64)
    flips = 0
    for t in range(1, iters + 1):
        got = Kmeans(X, k).init(idx).run(t, B)                 # a run of t rounds is a prefix of the longer runs
        used = centroids_used(C_prev, bf16)
        want, best, _, obj_or = oracle.assign(X32, used)
        differing, unexcused = label_mismatches(X32, used, got["labels"], want, best)
        assert unexcused == 0, f"round {t}: {unexcused} of {differing} differing labels are not near-ties"
        flips += differing
        C_or, counts_or, _ = oracle.update(X32, got["labels"], C_prev)
        np.testing.assert_array_equal(got["counts"], counts_or)
        assert centroid_rel_err(got["C"], C_or) <= CENTROID_RTOL, f"round {t}"
        assert abs(got["obj_hist"][t - 1] - obj_or) <= 1e-5 * obj_or, f"round {t}"
        C_prev = got["C"].astype(np.float64)
    return flips


SHAPES = [  # n, d, k, dtype, iters, components
    (20_011, 128, 16, torch.float32, 12, 20), (9_001, 128, 64, torch.float32, 10, 40), (7_003, 64, 30, torch.float32, 10, 12),
    (12_000, 128, 8, torch.bfloat16, 12, 10), (5_000, 64, 50, torch.bfloat16, 8, 30), (6_001, 128, 24, torch.bfloat16, 9, 16),
    (4_099, 64, 4, torch.float32, 15, 8), (37, 128, 5, torch.float32, 6, 3), (500, 128, 64, torch.float32, 7, 5),
    (3_000, 128, 2, torch.float32, 8, 6), (8_000, 128, 40, torch.float16, 9, 25), (6_000, 64, 12, torch.float16, 10, 9),
    (6_007, 64, 48, torch.float32, 9, 20),   # d = 64, k > 32: the bounds are taken inside the pipelined loop
]


@pytest.mark.parametrize("n,d,k,dtype,iters,comps", SHAPES)
def test_bounded_rounds_equal_plain_rounds_and_the_oracle(n, d, k, dtype, iters, comps):
    X = _mixture(n, d, comps, seed=n + k, relu=True, dtype=dtype)
    idx = oracle.init_indices(n + 1, n, k)
    plain, fast, searched = _both(X, k, idx, iters)
    _same_rounds(plain, fast, iters, n, exact=False)
    assert np.isnan(fast["obj_hist"][iters])
    assert np.all(searched[:3] == n) and np.all(searched >= 0) and np.all(searched <= n)
    # against the oracle's own free-running rounds (the plain device run is checked round by round elsewhere)
    ref = oracle.lloyd_bounds(to_np32(X), k, iters, idx, flags=oracle.FLAG_BF16_CENTROIDS if dtype == torch.bfloat16 else 0,
                              audit=True)
    assert ref["violations"] == 0
    if np.array_equal(fast["labels"], ref["labels"]):     # no near-tie went the other way on the road
        np.testing.assert_array_equal(fast["counts"], ref["counts"])
        assert centroid_rel_err(fast["C"], ref["C"]) <= CENTROID_RTOL
        assert np.all(np.abs(fast["obj_hist"][:iters] - ref["obj_hist"]) <= 1e-5 * ref["obj_hist"])
    else:
        assert abs(fast["obj_hist"][iters - 1] - ref["obj_hist"][-1]) <= 1e-3 * ref["obj_hist"][-1]


@pytest.mark.parametrize("n,d,k,dtype,iters,comps", [(15_000, 128, 40, torch.float32, 10, 30),
                                                     (20_000, 128, 16, torch.float32, 10, 47),
                                                     (9_000, 64, 8, torch.bfloat16, 9, 12)])
def test_every_round_of_the_bounded_run_against_the_oracle(n, d, k, dtype, iters, comps):
    X = _mixture(n, d, comps, seed=n + 7, relu=True, dtype=dtype)
    idx = oracle.init_indices(5, n, k)
    _check_rounds_against_oracle(X, k, idx, iters, dtype == torch.bfloat16)
    for t in (3, 4, iters):                                    # and the plain run's labels at the same rounds
        _same_rounds(Kmeans(X, k).init(idx).run(t), Kmeans(X, k).init(idx).run(t, B), t, n, exact=False)


@pytest.mark.parametrize("name,n", [("tiny", None), ("arxiv_like", 60_000), ("products_like", 80_000),
                                    ("papers_like", 50_000)])
def test_every_round_on_the_workload_recipes(name, n):
    w = synth.WORKLOADS[name]
    w = w if n is None else w.scaled(n)
    X = synth.embeddings(w, DEV)
    idx = oracle.init_indices(w.seed, w.n, w.k)
    _check_rounds_against_oracle(X, w.k, idx, min(w.iters, 12))


def test_bounds_skip_once_the_centroids_settle():
    """Separated blobs: after a few rounds nothing moves, nothing is searched, and nothing changes."""
    g = torch.Generator().manual_seed(3)
    means = 3.0 * torch.randn(6, 128, generator=g)
    X = (means[torch.randint(0, 6, (40_000,), generator=g)] + torch.randn(40_000, 128, generator=g)).to(DEV)
    idx = oracle.init_indices(8, 40_000, 6)
    plain, fast, searched = _both(X, 6, idx, 14)
    _same_rounds(plain, fast, 14, 40_000, exact=False)
    _check_rounds_against_oracle(X, 6, idx, 8)
    print("searched per round:", searched.tolist())
    assert searched[3:].sum() < 0.5 * 11 * 40_000
    again = Kmeans(X, 6).init(idx).run(14, B)                 # bit-reproducible
    for key in ("C", "labels", "counts"):
        np.testing.assert_array_equal(again[key], fast[key])
    np.testing.assert_array_equal(again["obj_hist"][:14], fast["obj_hist"][:14])


def test_on_the_workload_recipe_most_points_are_skipped_late():
    w = synth.WORKLOADS["products_like"].scaled(200_000)
    X = synth.embeddings(w, DEV)
    idx = oracle.init_indices(w.seed, w.n, w.k)
    plain, fast, searched = _both(X, w.k, idx, 20)
    _same_rounds(plain, fast, 20, w.n, exact=False)
    print("searched per round:", searched.tolist())
    assert searched[-1] < 0.25 * w.n


def test_duplicate_rows_and_exact_ties():
    """Rows that occur many times and a point set symmetric between two centroids: ties go to the lowest
    index with and without bounds."""
    g = torch.Generator().manual_seed(1)
    base = torch.randint(-2, 3, (40, 64), generator=g).float()
    X = base[torch.randint(0, 40, (6_000,), generator=g)].contiguous().to(DEV)     # integer coordinates, many exact ties
    idx = np.array([0, 1, 2, 3, 4, 5, 6, 7], dtype=np.int64)
    seen = {}
    rows = X.cpu().numpy()
    pick = []
    for i in range(6_000):                                     # k distinct rows as initial centroids
        key = rows[i].tobytes()
        if key not in seen:
            seen[key] = i
            pick.append(i)
        if len(pick) == 8:
            break
    idx = np.array(pick, dtype=np.int64)
    plain, fast, _ = _both(X, 8, idx, 9)
    _same_rounds(plain, fast, 9, 6_000)
    ref = oracle.lloyd(rows, 8, 9, idx)
    np.testing.assert_array_equal(fast["labels"], ref["labels"])


@pytest.mark.parametrize("n,d,k,dtype,iters", [(9_001, 128, 64, torch.float32, 8), (12_000, 128, 8, torch.bfloat16, 7),
                                               (3_000, 64, 5, torch.float32, 4)])
def test_bounded_run_without_objective_history(n, d, k, dtype, iters):
    """The objective is optional: without it the run gives the same centroids, labels and counts bit for bit."""
    X = _mixture(n, d, 12, seed=n + 3, relu=True, dtype=dtype)
    idx = oracle.init_indices(n, n, k)
    with_hist = Kmeans(X, k).init(idx).run(iters, B)
    km = Kmeans(X, k).init(idx)
    ws = ep.workspace(ep.kmeans_run_workspace_bytes(km.p, iters, B), X.device)
    ws.fill_(0x5A)
    ep.kmeans_run(km.p, X, iters, km.C, km.labels, km.counts, None, B, ws)
    km._sync_and_check()
    np.testing.assert_array_equal(km.labels.cpu().numpy(), with_hist["labels"])
    np.testing.assert_array_equal(km.counts.cpu().numpy(), with_hist["counts"])
    np.testing.assert_array_equal(km.C.cpu().numpy(), with_hist["C"])


def test_final_reassign_with_bounds():
    X = _mixture(8_000, 128, 10, seed=4, relu=True)
    idx = oracle.init_indices(2, 8_000, 12)
    plain, fast, _ = _both(X, 12, idx, 6, ep.EP_RUN_FINAL_REASSIGN)
    _same_rounds(plain, fast, 7, 8_000, exact=False)                        # objective [6] is the re-assignment's


def test_flag_without_effect_and_workspace_rules():
    X = _mixture(3_000, 128, 8, seed=6, relu=True)
    for k, iters in ((100, 5), (8, 2), (8, 3)):                # a shape without bounded kernels; too few rounds
        idx = oracle.init_indices(3, 3_000, k)
        plain, fast = Kmeans(X, k).init(idx).run(iters), Kmeans(X, k).init(idx).run(iters, B)
        for key in ("C", "labels", "counts"):
            np.testing.assert_array_equal(fast[key], plain[key])
        np.testing.assert_array_equal(fast["obj_hist"][:iters], plain["obj_hist"][:iters])
    p = ep.problem(X, 8)
    need_plain, need_b = ep.kmeans_workspace_bytes(p), ep.kmeans_run_workspace_bytes(p, 6, B)
    assert ep.kmeans_run_workspace_bytes(p, 6, 0) == need_plain and need_b >= need_plain + 12 * 3_000
    L = ep.lib()
    ws = ep.workspace(need_plain, DEV)
    out = torch.zeros(4096, dtype=torch.int64, device=DEV)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    rc = L.kmeans_run(C.byref(p), ptr(X), 6, ptr(out), ptr(out), ptr(out), None, B, ptr(ws), need_plain, None)
    assert rc == ep.EP_EWORKSPACE                              # the flag needs the larger workspace
    p100 = ep.problem(X, 100)
    ws100 = ep.workspace(ep.kmeans_run_workspace_bytes(p100, 6, B), DEV)
    assert L.kmeans_run_searched(C.byref(p100), 6, B, ptr(ws100), ws100.numel(), ptr(out), None) == ep.EP_EUNSUPPORTED
