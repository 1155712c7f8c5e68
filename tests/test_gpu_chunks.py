"""Row ranges through the C ABI: a matrix handled chunk by chunk (kmeans_assign on row ranges,
kmeans_update with its accumulate / finalize flags) must give what the oracle gives on the whole
matrix, and the same bits on every run; ep_validate_labels against the oracle's count."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_01000_amd import embedpart as ep

from parity import CENTROID_RTOL, DEV, centroid_rel_err, centroids_used, label_mismatches, to_np32
from test_gpu_kmeans import _mixture

pytestmark = pytest.mark.gpu

CANARY = 64   # elements behind every output buffer that no call may touch


def _guarded(shape, dtype, fill):
    """(view of the first `shape` elements, whole buffer): the tail is checked after the calls."""
    n0 = shape[0] if isinstance(shape, tuple) else shape
    rest = shape[1:] if isinstance(shape, tuple) else ()
    whole = torch.full((n0 + CANARY,) + tuple(rest), fill, dtype=dtype, device=DEV)
    return whole[:n0], whole


def _tail_untouched(whole, n0, fill):
    return bool((whole[n0:] == fill).all())


# one shape per update path: fused small-k kernels (matrix-core sums; LDS sum tables), rows sorted by label
# (bf16 matrix-core path, fp32 sliced path, segments cut in parts), the generic kernels' partial sums
SHAPES = [(20_011, 128, 16, torch.float32), (9_001, 128, 64, torch.float32), (7_003, 64, 30, torch.bfloat16),
          (6_000, 128, 300, torch.bfloat16), (5_001, 128, 100, torch.float32), (4_000, 516, 20, torch.float32),
          (3_001, 20, 5, torch.float32)]


def _cuts(n, parts, rng):
    """Chunk boundaries: ragged sizes, one chunk smaller than k, multiples of 4 so that labels stay aligned."""
    inner = np.sort(rng.choice(np.arange(1, n // 4), size=parts - 1, replace=False)) * 4
    cuts = [0, *inner.tolist(), n]
    cuts.insert(2, cuts[1] + 8)          # a chunk of 8 rows
    return cuts


@pytest.mark.parametrize("n,d,k,dtype", SHAPES)
def test_chunked_update_equals_oracle_on_the_whole(n, d, k, dtype):
    X = _mixture(n, d, 6, seed=n + k, relu=True, dtype=dtype)
    X32 = to_np32(X)
    rng = np.random.default_rng(n)
    labels_np = rng.integers(0, k, size=n).astype(np.int32)
    labels_np[labels_np == 1] = 0                       # cluster 1 is empty in every chunk
    C_prev_np = rng.normal(size=(k, d)).astype(np.float32)
    C_or, counts_or, _ = oracle.update(X32, labels_np, C_prev_np.astype(np.float64))
    labels = torch.from_numpy(labels_np).to(DEV)
    C_prev = torch.from_numpy(C_prev_np).to(DEV)
    cuts = _cuts(n, 4, rng)
    biggest = max(b - a for a, b in zip(cuts, cuts[1:]))
    ws = ep.workspace(ep.kmeans_workspace_bytes(ep.problem(X[:max(biggest, k)], k)), DEV)
    runs = []
    for rep in range(2):
        ws.fill_(0xA5 if rep else 0x5A)                 # whatever the workspace held before
        C_out, C_whole = _guarded((k, d), torch.float32, -7.0)
        counts, counts_whole = _guarded(k, torch.int64, -7)
        for i, (a, b) in enumerate(zip(cuts, cuts[1:])):
            flags = (ep.EP_UPDATE_ACCUMULATE if i > 0 else 0) | (ep.EP_UPDATE_FINALIZE if b == n else 0)
            last = b == n
            ep.kmeans_update(ep.problem(X[a:b], k), X[a:b], labels[a:b], C_prev if last else None,
                             C_out if last else None, counts if last else None, flags, ws)
        torch.cuda.synchronize()
        assert _tail_untouched(C_whole, k, -7.0) and _tail_untouched(counts_whole, k, -7)
        runs.append((C_out.cpu().numpy(), counts.cpu().numpy()))
    np.testing.assert_array_equal(runs[0][1], counts_or)
    assert centroid_rel_err(runs[0][0], C_or) <= CENTROID_RTOL
    np.testing.assert_array_equal(runs[0][0][1], C_prev_np[1])          # the empty cluster keeps its centroid
    np.testing.assert_array_equal(runs[0][0], runs[1][0])               # bit-reproducible
    np.testing.assert_array_equal(runs[0][1], runs[1][1])
    # one call over the whole matrix: same counts, same means up to the order of the fp64 additions
    whole = torch.empty((k, d), dtype=torch.float32, device=DEV)
    cw = torch.empty(k, dtype=torch.int64, device=DEV)
    ep.kmeans_update(ep.problem(X, k), X, labels, C_prev, whole, cw, ep.EP_UPDATE_FINALIZE,
                     ep.workspace(ep.kmeans_workspace_bytes(ep.problem(X, k)), DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cw.cpu().numpy(), counts_or)
    assert centroid_rel_err(whole.cpu().numpy(), runs[0][0]) <= 1e-6


@pytest.mark.parametrize("n,d,k,dtype", [(20_011, 128, 16, torch.float32), (9_001, 128, 64, torch.float32),
                                         (6_000, 128, 300, torch.bfloat16), (3_001, 20, 5, torch.float32)])
def test_streamed_lloyd_rounds_equal_the_oracle(n, d, k, dtype):
    """A matrix that stays on the HOST and passes through the device one chunk at a time: three Lloyd
    rounds of chunked assignment + chunked update against the oracle's rounds on the whole matrix."""
    bf16 = dtype == torch.bfloat16
    X_host = _mixture(n, d, 8, seed=3 * n + k, relu=True, dtype=dtype).cpu()
    X32 = to_np32(X_host)
    idx = oracle.init_indices(17, n, k)
    C_np = X32[idx].astype(np.float64)
    rng = np.random.default_rng(k)
    cuts = _cuts(n, 3, rng)
    biggest = max(b - a for a, b in zip(cuts, cuts[1:]))
    chunk_buf = torch.empty((biggest, d), dtype=dtype, device=DEV)
    ws = ep.workspace(ep.kmeans_workspace_bytes(ep.problem(chunk_buf[:max(biggest, k)], k)), DEV)
    Cc = torch.from_numpy(C_np.astype(np.float32)).to(DEV)
    labels, labels_whole = _guarded(n, torch.int32, -7)
    counts = torch.empty(k, dtype=torch.int64, device=DEV)
    obj = torch.zeros(1, dtype=torch.float64, device=DEV)
    for t in range(3):
        used = centroids_used(Cc.cpu().numpy(), bf16)
        want, best, _, obj_or = oracle.assign(X32, used)
        total = 0.0
        for i, (a, b) in enumerate(zip(cuts, cuts[1:])):
            Xc = chunk_buf[:b - a]
            Xc.copy_(X_host[a:b])                         # the chunk's trip to the device
            pc = ep.problem(Xc, k)
            ep.kmeans_assign(pc, Xc, Cc, labels[a:b], None, obj, ws)
            flags = (ep.EP_UPDATE_ACCUMULATE if i > 0 else 0) | (ep.EP_UPDATE_FINALIZE if b == n else 0)
            ep.kmeans_update(pc, Xc, labels[a:b], Cc, Cc, counts, flags, ws)
            total += float(obj.item())                    # (synchronises: the buffer is free for the next chunk)
        got = labels.cpu().numpy()
        differing, unexcused = label_mismatches(X32, used, got, want, best)
        assert unexcused == 0, f"round {t}: {unexcused} of {differing} differing labels are not near-ties"
        assert abs(total - obj_or) <= 1e-5 * obj_or
        C_or, counts_or, _ = oracle.update(X32, got, C_np)
        np.testing.assert_array_equal(counts.cpu().numpy(), counts_or)
        assert centroid_rel_err(Cc.cpu().numpy(), C_or) <= CENTROID_RTOL
        C_np = Cc.cpu().numpy().astype(np.float64)
    assert _tail_untouched(labels_whole, n, -7)


def test_chunk_smaller_than_k_and_single_row():
    X = _mixture(300, 128, 4, seed=9)
    X32 = to_np32(X)
    k = 64
    Cc = torch.from_numpy(X32[oracle.init_indices(2, 300, k)]).to(DEV)
    ws = ep.workspace(ep.kmeans_workspace_bytes(ep.problem(X, k)), DEV)
    labels, whole = _guarded(300, torch.int32, -7)
    for a, b in ((0, 1), (4, 40), (40, 300)):            # 1, 36 and 260 rows against 64 centroids
        ep.kmeans_assign(ep.problem(X[a:b], k), X[a:b], Cc, labels[a:b], None, None, ws)
    # unaligned starts are the caller's business: assign rows 1..4 through an aligned staging buffer
    tmp = torch.full((4 + CANARY,), -7, dtype=torch.int32, device=DEV)
    ep.kmeans_assign(ep.problem(X[1:4], k), X[1:4], Cc, tmp, None, None, ws)
    torch.cuda.synchronize()
    assert bool((tmp[3:] == -7).all())
    labels[1:4] = tmp[:3]
    want, _, _, _ = oracle.assign(X32, Cc.cpu().numpy().astype(np.float64))
    np.testing.assert_array_equal(labels.cpu().numpy(), want)
    assert _tail_untouched(whole, 300, -7)


@pytest.mark.parametrize("n,k", [(1, 1), (1000, 7), (1_000_003, 64), (300_001, 16_384)])
def test_validate_labels_equals_oracle(n, k):
    rng = np.random.default_rng(n + k)
    clean = rng.integers(0, k, size=n).astype(np.int32)
    dirty = clean.copy()
    for pos, val in ((n // 3, k), (n // 2, -1), (n - 1, 2**31 - 1), (n // 3 + 5 if n > 10 else 0, -(2**31))):
        dirty[pos] = val
    result, whole = _guarded(2, torch.int64, -7)
    for lab in (clean, dirty):
        ep.ep_validate_labels(n, k, torch.from_numpy(lab).to(DEV), result)
        torch.cuda.synchronize()
        assert tuple(result.cpu().tolist()) == oracle.validate_labels(lab, k)
    assert _tail_untouched(whole, 2, -7)
    assert oracle.validate_labels(clean, k) == (0, n)
