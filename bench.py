#!/usr/bin/env python3
"""Benchmark of the EmbedPart clustering hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: seeded initial centroids, `iters` Lloyd rounds (kmeans_run), the integer
partition-quality sweep over the CSR graph (partition_quality) and, for the reordering
workload, the partition-sorted relabelling and its edge-gap sum.  The value is
point-iterations per second over whole steps (n * iters / step time).

Prints ONE JSON line.  The headline is the largest configuration that fits one GPU
(`papers_like`: 111 M x 128 fp32, k = 64); the other four configurations of the benchmark
definition follow under `more`, each a complete line of its own with fewer timed steps.
Every line carries
  roofline      the kernel that reads X in every Lloyd round, timed with HIP events that the
                library hands to each of its launches (the launch stamps them with the
                kernel's own begin and end) in a further pass of the same steps, so that the
                events do not perturb the step timing;
  edge_sweep    the same for the CSR sweep of partition_quality (and edge_gap_sum);
  cpu_baseline  the fp64 oracle timed on this machine's host cores, at all cores and at one
                thread, on a contiguous slice of the same rows sized for a few seconds each.
`traffic` is the HBM byte count of the kernel from the rocprofv3 counter summary under
profiles/ that `traffic_source` names (null when there is none): it is read from that file,
not measured by this run.  `frac` is against the published peak; `frac_of_measured` is the same
rate against what this machine sustains in this run (`measured_peak`: a plain copy of X for the
streaming kernels, the bf16 matrix instruction alone on rows of X for the matrix-core kernel).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import re
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16 matrix rate
FP32_PEAK_TFLOPS = 157.3       # MI355X published fp32 vector rate (the fp32 matrix rate is the same)
LLC_BYTES = 256 * 1024 * 1024  # memory-side cache: a matrix below this is not served by HBM after round 1

HEADLINE = "papers_like"
OTHERS = "tiny,arxiv_like,products_like,products_reorder"
# timed steps of the workloads under `more` (the headline takes --steps / --warmup)
MORE_STEPS = {"tiny": (50, 5), "arxiv_like": (20, 3), "products_like": (10, 2), "products_reorder": (3, 1),
              "papers_like": (3, 1)}


def mfma_alone(X, dev):
    """Rate of back-to-back bf16 matrix instructions (library's benchmark aid) on zeros and on rows of X."""
    import torch

    from paper_2604_01000_amd import embedpart as ep

    nval = ep.EP_BENCH_MFMA_OPERAND_BYTES // 2
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    out = dict(unit="TFLOP/s")
    iters = 40000
    for name, ops in (("zero_operands", torch.zeros(nval, dtype=torch.bfloat16, device=dev)),
                      ("rows_of_X_as_operands", X.reshape(-1)[:nval].contiguous())):
        ep.ep_bench_mfma_bf16(ops, iters, sink)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(3):
            ep.ep_bench_mfma_bf16(ops, iters, sink)
        b.record()
        torch.cuda.synchronize()
        out[name] = ep.EP_BENCH_MFMA_FLOP_PER_ITER * iters * 3 / (a.elapsed_time(b) * 1e-3) / 1e12
    return out


def probe_fold() -> dict:
    """The library's fold probe (include/embedpart_bench.h) at the shapes of the two small workloads: what a Lloyd
    round's second pass costs as a launch of its own and as work of the last workgroup to arrive."""
    import torch

    from paper_2604_01000_amd import embedpart as ep

    dev, reps, res = "cuda:0", 2000, []
    for name, parts, elems in (("tiny", 313, 4 * 64), ("arxiv_like", 512, 8 * 128)):
        partials = torch.empty(parts * elems, dtype=torch.float32, device=dev)
        out = torch.empty(elems, dtype=torch.float32, device=dev)
        ticket = torch.zeros(1, dtype=torch.int32, device=dev)
        us = {}
        for mode, key in ((0, "producer_alone_us"), (2, "producer_and_second_launch_us"), (1, "producer_with_fold_us")):
            for _ in range(20):
                ep.ep_bench_fold(partials, parts, elems, mode, ticket, out)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                ep.ep_bench_fold(partials, parts, elems, mode, ticket, out)
            b.record()
            torch.cuda.synchronize()
            us[key] = a.elapsed_time(b) * 1e3 / reps
        res.append(dict(shape_of=name, partials=parts, floats_per_partial=elems, **us,
                        second_launch_costs_us=us["producer_and_second_launch_us"] - us["producer_alone_us"],
                        fold_costs_us=us["producer_with_fold_us"] - us["producer_alone_us"]))
    return dict(probe="fold of the second pass into the round kernel", launches_per_figure=reps, results=res)


def profile_traffic(kernel: str, workload: str):
    """(bytes per launch, file) from the counter summary of `kernel` on `workload` under profiles/."""
    path = ROOT / "profiles" / f"{kernel}_{workload}_hbm_traffic.txt"
    if not path.exists():
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\[" + re.escape(kernel) + r"\]\s*=\s*(\d+)", path.read_text(), re.M)
    return (int(m.group(1)), f"profiles/{path.name}") if m else (None, None)


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


def oracle_baseline(w, X, idx, seconds: float) -> dict:
    """The oracle's Lloyd rounds (assignment, then update, against all k centroids) on the first rows
    of the workload, at all cores and at one thread.

    The slice is sized from a short probe so that each of the two timings takes about `seconds`;
    the full-size figure is an extrapolation (the oracle's cost is linear in the rows) and is
    labelled as one."""
    import numpy as np
    import torch

    import oracle

    bf16 = w.dtype == "bf16"
    cores = oracle.threads()
    C0 = X[idx.to(X.device)].to("cpu", torch.float32).numpy().astype(np.float64)   # the workload's initial centroids

    def timed(rows: int, iters: int, threads: int) -> float:
        Xs = X[:rows].to("cpu", torch.float32).numpy()
        Cc = C0
        oracle.set_threads(threads)
        t0 = time.perf_counter()
        for _ in range(iters):
            labels, _, _, _ = oracle.assign(Xs, Cc, round_bf16=bf16)
            Cc, _, _ = oracle.update(Xs, labels, Cc)
        dt = time.perf_counter() - t0
        oracle.set_threads(cores)
        return dt

    out = {}
    for threads in (cores, 1):
        probe_rows = int(min(w.n, max(64, 2_000_000_000 // (w.k * w.d * 40)) * threads))
        per_point_iter = max(timed(probe_rows, 1, threads), 1e-4) / probe_rows
        iters = w.iters if per_point_iter * w.iters * 4096 < seconds else 1
        rows = int(min(w.n, max(64, seconds / (per_point_iter * iters))))
        dt, runs = timed(rows, iters, threads), 1
        while dt < 0.5 * seconds and runs < 200:     # a workload shorter than the budget is repeated
            dt += timed(rows, iters, threads)
            runs += 1
        out[threads] = dict(rate=runs * rows * iters / dt / 1e6, rows=rows, iters=iters, seconds=dt, runs=runs)
    a, one = out[cores], out[1]
    return dict(value=a["rate"], unit="Mpts*iter/s", cores=cores, kind="oracle",
                value_1_thread=one["rate"],
                sample=f"Lloyd rounds (assign + update, all k={w.k} centroids) on the first {a['rows']} rows x {a['iters']} "
                       f"round(s) x {a['runs']} run(s), {a['seconds']:.1f} s at {cores} threads; first {one['rows']} rows x "
                       f"{one['iters']} round(s) x {one['runs']} run(s), {one['seconds']:.1f} s at 1 thread",
                full_size_seconds_extrapolated=dict(all_cores=w.n * w.iters / (a["rate"] * 1e6),
                                                    one_thread=w.n * w.iters / (one["rate"] * 1e6)))


def run_workload(name: str, steps: int, warmup: int, cpu_seconds: float, variants: bool = True) -> dict:
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

    def timed_kernels(kernel_class: int, launches_per_step: int, passes: int) -> float:
        """Mean duration (ms) of one kernel class over further passes of the same step."""
        launches = passes * launches_per_step
        evs = HipEvents(2 * launches)
        assert ep.lib().ep_profile_arm(evs.arr, 2 * launches, kernel_class) == 0
        for _ in range(passes):
            step()
        torch.cuda.synchronize()
        seen = ep.lib().ep_profile_count()
        ep.lib().ep_profile_arm(None, 0, 0)
        assert seen == launches, (seen, launches)
        ms = float(np.mean([evs.elapsed_ms(2 * i, 2 * i + 1) for i in range(launches)]))
        evs.destroy()
        return ms

    # ---- further passes of the same steps with events around one kernel class at a time ----
    passes = min(steps, 20)
    kernel_ms = timed_kernels(ep.EP_PROF_LLOYD_MAIN, w.iters, passes)
    sweep_ms = timed_kernels(ep.EP_PROF_EDGE_SWEEP, 2 if reorder else 1, passes)

    # ---- the variant the paper runs: centroids trained on 2^9 rows per cluster, then one assignment of
    # ---- every row (kmeans_run_sampled); timed beside the step, not part of it ----
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
        # leave labels / counts / hist as the step produces them
        step()
        torch.cuda.synchronize()

    # ---- the same Lloyd rounds with distance bounds and kept sums (EP_RUN_BOUNDS): points whose bounds show that
    # ---- their label cannot change are not read.  Timed beside the step (kmeans_init + kmeans_run only, with and
    # ---- without the flag); `searched` is the number of rows read in each round, bytes_read_per_round what that
    # ---- amounts to (a searched row + its label, plus 12 bytes of bounds and label per row in a bounded round;
    # ---- the third round, which takes the bounds, writes 8 bytes per row more than a plain one)
    bounded = None
    if variants:
        flags = ep.EP_RUN_BOUNDS
        try:
            bws = ep.workspace(ep.kmeans_run_workspace_bytes(p, w.iters, flags), dev)
            hist_b = torch.zeros(w.iters + 1, dtype=torch.float64, device=dev)
            labels_b = torch.empty_like(labels)
            counts_b = torch.empty_like(counts)
            C_b = torch.empty_like(Cc)
            searched = torch.zeros(w.iters, dtype=torch.int64, device=dev)

            def timed_runs(run_flags, lab, cnt, hst, Cx, wsx):
                ep.kmeans_init(p, X, idx, Cx, wsx)
                ep.kmeans_run(p, X, w.iters, Cx, lab, cnt, hst, run_flags, wsx)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(steps):
                    ep.kmeans_init(p, X, idx, Cx, wsx)
                    ep.kmeans_run(p, X, w.iters, Cx, lab, cnt, hst, run_flags, wsx)
                b.record()
                torch.cuda.synchronize()
                return a.elapsed_time(b) / steps

            ms_b = timed_runs(flags, labels_b, counts_b, hist_b, C_b, bws)
            ms_plain = timed_runs(0, labels, counts, hist, Cc, ws)
            ep.kmeans_run_searched(p, w.iters, flags, bws, searched)
            torch.cuda.synchronize()
            sr = searched.cpu().tolist()
            row_bytes = w.d * (2 if w.dtype == "bf16" else 4) + 4
            bounded = dict(ms=ms_b, ms_plain_rounds=ms_plain, speedup=ms_plain / ms_b,
                           Mpts_iter_per_s=w.n * w.iters / (ms_b * 1e-3) / 1e6, searched_per_round=sr,
                           bytes_read_per_round=[r * row_bytes + (12 * w.n if t > 2 else 0) for t, r in enumerate(sr)],
                           bytes_read_per_round_plain=w.n * row_bytes,
                           labels_differing_from_plain=int((labels_b != labels).sum().item()),
                           objective=float(hist_b[w.iters - 1].item()), objective_plain=float(hist[w.iters - 1].item()))
            del bws, labels_b
        except ep.EmbedPartError as e:      # the flag has no bounded kernels for this shape: the rounds run in full
            if e.code != ep.EP_EUNSUPPORTED:
                raise
            bounded = dict(note="no bounded kernels for this shape (k > 64): the flag is accepted and the rounds run in full")

    # ---- the balancing loops of the paper's Alg. 3 on the K-Means partition (partition-scale k only):
    # ---- three vertex classes (seeded: 55% / 15% / 30%), beta = 1.05, timed beside the step ----
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
    # ---- timed beside the step on the reordering workload; the metrics must carry over ----
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
        main_kernel = "large_assign_kernel"
        roofline = dict(bound="mfma", achieved=flop / (kernel_ms * 1e-3) / 1e12, peak=MFMA_BF16_PEAK_TFLOPS,
                        unit="TFLOP/s", algorithmic_flop_per_launch=flop)
        # What the matrix pipe sustains with nothing else going on, on all-zero operands and on rows of this
        # workload: the chip is power-limited in this instruction and the power follows the operand values.
        roofline["matrix_instruction_alone"] = mfma_alone(X, dev)
    else:         # streaming: X read once + one int32 label per point
        nbytes = w.n * (w.d * elem + 4)
        main_kernel = "lloyd_small_kernel"
        roofline = dict(bound="hbm", achieved=nbytes / (kernel_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                        algorithmic_bytes_per_launch=nbytes)
        if x_bytes <= LLC_BYTES:
            roofline["note"] = ("the matrix fits the 256 MB memory-side cache and is served from it after the first "
                                "round: the HBM peak is not this launch's bound, the fraction is quoted for reference")
        # The same launch against the other roofline of this shape: 2*n*k*d flop of fp32-accurate score arithmetic
        # per launch against the fp32 vector (= fp32 matrix) peak.  At k = 64, d = 128 plain fp32 arithmetic at 100%
        # of that peak would stop at 0.62 of the HBM figure; the kernel gets past it on the bf16 matrix instructions
        # (three-way split, six products per fp32 product).
        flop32 = 2.0 * w.n * w.k * w.d
        roofline["fp32_equivalent"] = dict(achieved=flop32 / (kernel_ms * 1e-3) / 1e12, peak=FP32_PEAK_TFLOPS,
                                           unit="TFLOP/s", frac=flop32 / (kernel_ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS,
                                           hbm_frac_if_fp32_bound=(nbytes / HBM_PEAK_GBS / 1e9) /
                                                                  (flop32 / FP32_PEAK_TFLOPS / 1e12))
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["traffic"], roofline["traffic_source"] = profile_traffic(main_kernel, w.name)
    roofline["kernel_ms"] = kernel_ms
    roofline["kernel"] = main_kernel + ": the kernel that reads X in every Lloyd round"
    # CSR sweep: 4 B per stored entry + the offsets + one label (or new id) per vertex, once
    sweep_bytes = 4 * nnz + rowptr.element_size() * (w.n + 1) + 4 * w.n
    # The library's rule for the cut count through buckets of column ranges (labels far beyond the caches,
    # rows not nearly empty); otherwise one sweep kernel gathers the labels directly.
    bucketed = not reorder and w.k <= 255 and w.n >= 6 * 1024 * 1024 and nnz >= 4 * w.n
    sweep_kernel = "bucket_cut_count" if bucketed else "edge_block_sweep_kernel"
    sweep_note = (": bucket_hist + bucket_scan + bucket_scatter + bucket_sweep kernels together" if bucketed
                  else ": mean of the cut sweep and the gap sweep" if reorder else "")
    edge_sweep = dict(bound="hbm", achieved=sweep_bytes / (sweep_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                      algorithmic_bytes_per_launch=sweep_bytes, kernel_ms=sweep_ms,
                      Gentries_per_s=nnz / (sweep_ms * 1e-3) / 1e9, kernel=sweep_kernel + sweep_note)
    edge_sweep["frac"] = edge_sweep["achieved"] / edge_sweep["peak"]
    edge_sweep["traffic"], edge_sweep["traffic_source"] = profile_traffic(sweep_kernel, w.name)
    reference = dict(copy_GBs=2 * x_bytes / (copy_ms * 1e-3) / 1e9, copy_bytes_moved=2 * x_bytes)
    # the same rates against what this machine was measured to sustain (frac stays the one against the published peak)
    if reorder:
        roofline["measured_peak"] = roofline["matrix_instruction_alone"]["rows_of_X_as_operands"]
        roofline["measured_peak_kind"] = "the bf16 matrix instruction alone on rows of X (power-limited clock)"
    else:
        roofline["measured_peak"] = reference["copy_GBs"]
        roofline["measured_peak_kind"] = "plain copy of X, bytes read + bytes written"
    roofline["frac_of_measured"] = roofline["achieved"] / roofline["measured_peak"]
    edge_sweep["frac_of_measured_copy"] = edge_sweep["achieved"] / reference["copy_GBs"]

    torch.cuda.synchronize()
    result_labels = labels.cpu().numpy()
    quality = dict(edge_cut_ratio=int(cut.item()) / max(nnz, 1), vertex_balance=int(sizes.max().item()) * w.k / w.n,
                   objective=float(hist[w.iters - 1].item()), nnz=nnz)
    if reorder:
        quality["mean_edge_gap"] = (int(gap.item()) & (2**64 - 1)) / max(nnz, 1)

    # ---- the oracle on this machine's host cores ----
    cpu = oracle_baseline(w, X, idx, cpu_seconds) if cpu_seconds > 0 else None

    return dict(metric="kmeans_point_iterations_per_s", value=value, unit="Mpts*iter/s", n_gpus=1, steps=steps,
                warmup=warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
                dtype="bf16" if w.dtype == "bf16" else "f32", data="synthetic",
                config=dict(workload=w.name, n=w.n, d=w.d, k=w.k, iters=w.iters, nnz=nnz,
                            step="kmeans_init + kmeans_run + partition_quality" +
                                 (" + partition_permutation + edge_gap_sum" if reorder else "")),
                roofline=roofline, edge_sweep=edge_sweep, cpu_baseline=cpu, reference=reference, quality=quality,
                sampled_variant=sampled, bounds_variant=bounded, balance_variant=balance, reorder_variant=rewrite,
                labels_checksum=int(np.bitwise_xor.reduce(result_labels.astype(np.int64) * (np.arange(w.n) % 9973 + 1))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=HEADLINE,
                    help="tiny | arxiv_like | products_like | products_reorder | papers_like")
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads reported under 'more'; '' for none "
                         "(default: the other four configurations)")
    ap.add_argument("--cpu-seconds", type=float, default=4.0,
                    help="CPU time of each oracle timing (two per workload: all cores, one thread); 0 = none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the sample-trained, balancing and graph-rewrite legs (for profiles of the step's kernels alone)")
    ap.add_argument("--probe", default=None, choices=["fold"],
                    help="run one of the library's benchmark probes instead of the workloads and print its figures")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.probe == "fold":
        print(json.dumps(probe_fold()))
        return 0
    cpu_seconds = 0.0 if args.no_cpu_baseline else args.cpu_seconds
    also = OTHERS if args.also is None else args.also
    out = run_workload(args.workload, args.steps, args.warmup, cpu_seconds, not args.no_variants)
    more = []
    for name in [v for v in also.split(",") if v and v != args.workload]:
        torch.cuda.empty_cache()
        s, wu = MORE_STEPS[name]
        more.append(run_workload(name, s, wu, cpu_seconds, not args.no_variants))
    if more:
        out["more"] = more
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
