#!/usr/bin/env python3
"""Benchmark of the EmbedPart clustering hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: seeded initial centroids, `iters` Lloyd rounds (kmeans_run), the integer
partition-quality sweep over the CSR graph (partition_quality) and, for the reordering
workload, the partition-sorted relabelling and its edge-gap sum.  The headline value is
point-iterations per second over whole steps (n * iters / step time).

Prints ONE JSON line.  `roofline` describes the kernel that reads X in every Lloyd round, timed
with HIP events that the library hands to each of its launches (ep_profile_arm; the launch stamps
them with the kernel's own begin and end) in a second pass of the same steps, so that the events
do not perturb the headline timing.  `cpu_baseline` is the fp64
oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch of the roofline kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (see profiles/), scaled by the copy-kernel calibration; None where not measured.
MEASURED_TRAFFIC_BYTES = {
    "arxiv_like": 90_006_646,            # profiles/lloyd_small_kernel_arxiv_like_hbm_traffic.txt
    "products_like": 1_285_319_468,      # profiles/lloyd_small_kernel_products_like_hbm_traffic.txt
    "products_reorder": 1_149_254_277,   # profiles/large_assign_kernel_products_reorder_hbm_traffic.txt
    "papers_like": 57_374_169_219,       # profiles/lloyd_small_kernel_papers_like_hbm_traffic.txt
}


class HipEvents:
    """hipEvent_t handles owned by the benchmark (created through the HIP runtime directly)."""

    def __init__(self, count: int):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.arr = (C.c_void_p * count)()
        for i in range(count):
            ev = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(ev)) == 0
            self.arr[i] = ev

    def elapsed_ms(self, i: int, j: int) -> float:
        out = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(out), self.arr[i], self.arr[j])
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return out.value

    def destroy(self):
        for ev in self.arr:
            self.hip.hipEventDestroy(C.c_void_p(ev))


def run_workload(name: str, steps: int, warmup: int, cpu_baseline: bool, variants: bool = True) -> dict:
    import numpy as np
    import torch

    from paper_2604_01000_amd import embedpart as ep
    from paper_2604_01000_amd import synth

    dev = "cuda:0"
    w = synth.WORKLOADS[name]
    reorder = w.name == "products_reorder"

    # ---- inputs, resident in HBM before anything is timed ----
    blocks = synth.block_labels(w)
    X = synth.embeddings(w, dev, blocks)
    rowptr, colidx, _ = synth.sbm_graph(w, dev, blocks)
    nnz = colidx.numel()
    idx = ep.kmeans_init_indices(w.seed, w.n, w.k)

    p = ep.problem(X, w.k)
    ws = ep.workspace(ep.kmeans_workspace_bytes(p), dev)
    gws = ep.workspace(ep.graph_workspace_bytes(w.n, nnz, w.k), dev)
    Cc = torch.empty((w.k, w.d), dtype=torch.float32, device=dev)
    labels = torch.empty(w.n, dtype=torch.int32, device=dev)
    counts = torch.empty(w.k, dtype=torch.int64, device=dev)
    hist = torch.zeros(w.iters + 1, dtype=torch.float64, device=dev)
    cut = torch.zeros(1, dtype=torch.int64, device=dev)
    sizes = torch.zeros(w.k, dtype=torch.int64, device=dev)
    new_id = torch.empty(w.n, dtype=torch.int32, device=dev) if reorder else None
    order = torch.empty(w.n, dtype=torch.int32, device=dev) if reorder else None
    gap = torch.zeros(1, dtype=torch.int64, device=dev)

    def step():
        ep.kmeans_init(p, X, idx, Cc, ws)
        ep.kmeans_run(p, X, w.iters, Cc, labels, counts, hist, 0, ws)
        ep.partition_quality(w.n, nnz, w.k, rowptr, colidx, labels, cut, sizes, gws)
        if reorder:
            ep.partition_permutation(w.n, w.k, labels, new_id, order, gws)
            ep.edge_gap_sum(w.n, nnz, rowptr, colidx, new_id, gap, gws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    value = w.n * w.iters / (elapsed / steps) / 1e6

    def timed_kernels(kernel_class: int, launches_per_step: int) -> float:
        """Mean duration (ms) of one kernel class over a further pass of the same steps."""
        launches = steps * launches_per_step
        evs = HipEvents(2 * launches)
        assert ep.lib().ep_profile_arm(evs.arr, 2 * launches, kernel_class) == 0
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        seen = ep.lib().ep_profile_count()
        ep.lib().ep_profile_arm(None, 0, 0)
        assert seen == launches, (seen, launches)
        ms = float(np.mean([evs.elapsed_ms(2 * i, 2 * i + 1) for i in range(launches)]))
        evs.destroy()
        return ms

    # ---- further passes of the same steps with events around one kernel class at a time ----
    kernel_ms = timed_kernels(ep.EP_PROF_LLOYD_MAIN, w.iters)
    sweep_ms = timed_kernels(ep.EP_PROF_EDGE_SWEEP, 2 if reorder else 1)

    # ---- the variant the paper runs: centroids trained on 2^9 rows per cluster, then one assignment of
    # ---- every row (kmeans_run_sampled); timed beside the headline, not part of it ----
    sampled = None
    m = min(w.n, 512 * w.k)
    if variants and m < w.n:
        rows = ep.kmeans_init_indices(w.seed + 1, w.n, m)
        sws = ep.workspace(ep.kmeans_sampled_workspace_bytes(p, m), dev)
        ep.kmeans_run_sampled(p, X, rows, w.iters, Cc, labels, counts, hist, sws)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            ep.kmeans_run_sampled(p, X, rows, w.iters, Cc, labels, counts, hist, sws)
        b.record()
        torch.cuda.synchronize()
        sampled_ms = a.elapsed_time(b) / steps
        sampled = dict(sample_rows=m, iters=w.iters, ms=sampled_ms, Mpts_per_s=w.n / (sampled_ms * 1e-3) / 1e6,
                       objective=float(hist[w.iters].item()))
        del sws
        # leave labels / counts / hist as the headline run produced them
        step()
        torch.cuda.synchronize()

    # ---- the balancing loops of the paper's Alg. 3 on the K-Means partition (partition-scale k only):
    # ---- three vertex classes (seeded: 55% / 15% / 30%), beta = 1.05, timed beside the headline ----
    balance = None
    if variants and w.k <= ep.EP_BALANCE_MAX_K:
        g = torch.Generator(device="cpu").manual_seed(w.seed + 7)
        vclass = torch.bucketize(torch.rand(w.n, generator=g), torch.tensor([0.55, 0.70])).to(torch.uint8).to(dev)
        bws = ep.workspace(ep.balance_workspace_bytes(w.n), dev)
        stats = torch.zeros((3, 3), dtype=torch.int64, device=dev)
        blabels = labels.clone()
        cut_b = torch.zeros(1, dtype=torch.int64, device=dev)
        sizes_b = torch.zeros(w.k, dtype=torch.int64, device=dev)

        def balance_all():
            blabels.copy_(labels)
            for cls in range(3):
                ep.partition_balance(w.n, w.k, rowptr, vclass, cls, 1.05, w.seed + cls, 16, blabels, stats[cls], bws)

        balance_all()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            balance_all()
        b.record()
        torch.cuda.synchronize()
        ep.partition_quality(w.n, nnz, w.k, rowptr, colidx, blabels, cut_b, sizes_b, gws)
        torch.cuda.synchronize()
        st = stats.cpu().numpy()
        balance = dict(ms=a.elapsed_time(b) / steps, beta=1.05, max_rounds=16, rounds=st[:, 0].tolist(),
                       moved=st[:, 1].tolist(), still_overloaded=st[:, 2].tolist(),
                       vertex_balance_before=int(sizes.max().item()) * w.k / w.n,
                       vertex_balance_after=int(sizes_b.max().item()) * w.k / w.n,
                       edge_cut_ratio_before=int(cut.item()) / max(nnz, 1),
                       edge_cut_ratio_after=int(cut_b.item()) / max(nnz, 1))
        del bws, blabels, vclass

    # ---- the graph rewritten under the new ids (the step that makes the reordering usable by a trainer),
    # ---- timed beside the headline on the reordering workload; the metrics must carry over ----
    rewrite = None
    if variants and reorder:
        rws = ep.workspace(ep.graph_reorder_workspace_bytes(w.n, nnz), dev)
        new_rowptr, new_colidx = torch.empty_like(rowptr), torch.empty_like(colidx)
        ep.graph_reorder(w.n, nnz, rowptr, colidx, new_id, order, new_rowptr, new_colidx, rws)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            ep.graph_reorder(w.n, nnz, rowptr, colidx, new_id, order, new_rowptr, new_colidx, rws)
        b.record()
        torch.cuda.synchronize()
        gap2 = torch.zeros(1, dtype=torch.int64, device=dev)
        ep.edge_gap_sum(w.n, nnz, new_rowptr, new_colidx, None, gap2, gws)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / steps
        rewrite = dict(ms=ms, Gentries_per_s=nnz / (ms * 1e-3) / 1e9,
                       gap_sum_carried_over=int(gap2.item()) == int(gap.item()))
        del rws, new_rowptr, new_colidx

    # ---- copy bandwidth of this machine, for context: a plain 16-byte-per-lane copy of X ----
    Y = torch.empty_like(X)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ep.ep_bench_copy(Y, X)
    a.record()
    for _ in range(5):
        ep.ep_bench_copy(Y, X)
    b.record()
    torch.cuda.synchronize()
    copy_ms = a.elapsed_time(b) / 5
    x_bytes = X.numel() * X.element_size()
    del Y

    elem = 2 if w.dtype == "bf16" else 4
    if reorder:   # dense contraction on the matrix cores: 2*n*k*d flop per launch
        flop = 2.0 * w.n * w.k * w.d
        roofline = dict(bound="mfma", achieved=flop / (kernel_ms * 1e-3) / 1e12, peak=2500.0, unit="TFLOP/s")
    else:         # streaming: X read once + one int32 label per point
        nbytes = w.n * (w.d * elem + 4)
        roofline = dict(bound="hbm", achieved=nbytes / (kernel_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get(w.name)
    roofline["kernel_ms"] = kernel_ms
    roofline["kernel"] = "lloyd round kernel that reads X (EP_PROF_LLOYD_MAIN)"
    sweep_bytes = 4 * nnz + rowptr.element_size() * (w.n + 1) + 4 * w.n
    reference = dict(copy_GBs=2 * x_bytes / (copy_ms * 1e-3) / 1e9, copy_bytes_moved=2 * x_bytes,
                     edge_sweep_ms=sweep_ms, edge_sweep_GBs=sweep_bytes / (sweep_ms * 1e-3) / 1e9,
                     edge_sweep_Gentries_per_s=nnz / (sweep_ms * 1e-3) / 1e9)

    torch.cuda.synchronize()
    result_labels = labels.cpu().numpy()
    quality = dict(edge_cut_ratio=int(cut.item()) / max(nnz, 1), vertex_balance=int(sizes.max().item()) * w.k / w.n,
                   objective=float(hist[w.iters - 1].item()), nnz=nnz)
    if reorder:
        quality["mean_edge_gap"] = (int(gap.item()) & (2**64 - 1)) / max(nnz, 1)

    # ---- the oracle on this machine's host cores ----
    cpu = None
    if cpu_baseline:
        import oracle
        sample_n = min(w.n, 1 << 18 if w.k > 64 else 1 << 22)
        sample_iters = w.iters if w.k <= 64 else 1
        Xs = X[:sample_n].to("cpu", torch.float32).numpy()
        kk = min(w.k, sample_n)
        idx = oracle.init_indices(w.seed, sample_n, kk)
        flags = oracle.FLAG_BF16_CENTROIDS if w.dtype == "bf16" else 0
        runs, spent = 0, 0.0
        while runs == 0 or (spent < 10.0 and runs < 100):     # short workloads are repeated: ~10 s of CPU work
            t0 = time.perf_counter()
            oracle.lloyd(Xs, kk, sample_iters, idx, flags=flags)
            spent += time.perf_counter() - t0
            runs += 1
        cpu = dict(value=runs * sample_n * sample_iters / spent / 1e6, unit="Mpts*iter/s", cores=oracle.threads(),
                   kind="oracle",
                   sample=f"first {sample_n} rows of the workload, k={kk}, {sample_iters} Lloyd rounds, "
                          f"{runs} run(s), {spent:.1f} s in all")

    return dict(metric="kmeans_point_iterations_per_s", value=value, unit="Mpts*iter/s", n_gpus=1, steps=steps,
                warmup=warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
                dtype="bf16" if w.dtype == "bf16" else "f32", data="synthetic",
                config=dict(workload=w.name, n=w.n, d=w.d, k=w.k, iters=w.iters, nnz=nnz,
                            step="kmeans_init + kmeans_run + partition_quality" +
                                 (" + partition_permutation + edge_gap_sum" if reorder else "")),
                roofline=roofline, cpu_baseline=cpu, reference=reference, quality=quality, sampled_variant=sampled, balance_variant=balance,
                reorder_variant=rewrite,
                labels_checksum=int(np.bitwise_xor.reduce(result_labels.astype(np.int64) * (np.arange(w.n) % 9973 + 1))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="arxiv_like",
                    help="tiny | arxiv_like | products_like | products_reorder | papers_like")
    ap.add_argument("--also", default="products_like",
                    help="comma-separated further workloads reported under 'more' (fewer steps); '' for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the sample-trained and the balancing legs (for profiles of the headline kernels alone)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    out = run_workload(args.workload, args.steps, args.warmup, not args.no_cpu_baseline, not args.no_variants)
    more = []
    for name in [v for v in args.also.split(",") if v and v != args.workload]:
        torch.cuda.empty_cache()
        more.append(run_workload(name, max(3, args.steps // 4), 1, False, not args.no_variants))
    if more:
        out["more"] = more
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
