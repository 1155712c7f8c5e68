"""Seeded synthetic inputs: GNN-like embeddings and stochastic-block-model graphs.

These stand in for the trained node embeddings and the public graphs the paper
evaluates on (Table 1 gives their vertex counts and mean degrees), none of which
are available here.  The module holds input generation only -- nothing of the
clustering or of the quality metrics -- and is the one piece of code that both
the HIP path's callers and the oracle's tests use.

Embeddings: row i belongs to mixture component g_i (uniform over G components);
component means are N(0, 4 I); x_i = mean[g_i] + N(0, I); optionally max(., 0)
to mimic post-activation hidden states; optionally rounded to bf16.
Graph: stochastic block model over the same component labels: a fixed number of
undirected pairs, each with its partner inside the source's block with
probability f_in and in another block otherwise; optional Pareto(alpha) vertex
weights make the degree distribution heavy-tailed; self-loops and duplicate
pairs are dropped; both directions are stored in CSR with sorted rows.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    d: int
    k: int
    iters: int
    components: int
    relu: bool
    dtype: str            # "f32" or "bf16"
    avg_degree: float     # mean stored CSR entries per row (before de-duplication)
    f_in: float           # fraction of pairs that stay inside a block
    powerlaw_alpha: float # 0 = uniform vertex weights
    rowptr_i64: bool
    seed: int

    def scaled(self, n: int, name: str | None = None) -> "Workload":
        """Same recipe at another vertex count (for slices and quick tests)."""
        return replace(self, n=n, name=name or f"{self.name}@n={n}")


# The five configurations of the benchmark definition, in its order.
WORKLOADS = {
    "tiny": Workload("tiny", 20_000, 64, 4, 10, 8, False, "f32", 10.0, 20.0 / 27.0, 0.0, False, 1),
    "arxiv_like": Workload("arxiv_like", 170_000, 128, 8, 20, 40, True, "f32", 14.0, 0.8, 0.0, False, 2),
    "products_like": Workload("products_like", 2_450_000, 128, 16, 20, 47, True, "f32", 50.0, 0.75, 2.1, True, 3),
    "products_reorder": Workload("products_reorder", 2_450_000, 128, 16_384, 10, 47, True, "bf16", 50.0, 0.75, 2.1,
                                 True, 3),
    "papers_like": Workload("papers_like", 111_000_000, 128, 64, 10, 172, True, "f32", 14.5, 0.7, 0.0, True, 5),
}


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + stream) & 0x7FFF_FFFF_FFFF_FFFF)
    return g


def block_labels(w: Workload) -> torch.Tensor:
    """Mixture component / SBM block of every vertex (int64, CPU, device-independent)."""
    return torch.randint(0, w.components, (w.n,), generator=_gen(w.seed, 11, "cpu"), dtype=torch.int64)


def component_means(w: Workload) -> torch.Tensor:
    """G x d component means, N(0, 4 I), generated on the CPU for any device."""
    return 2.0 * torch.randn(w.components, w.d, generator=_gen(w.seed, 12, "cpu"), dtype=torch.float32)


def embeddings(w: Workload, device="cpu", blocks: torch.Tensor | None = None,
               chunk_rows: int = 1 << 21) -> torch.Tensor:
    """N x d embedding matrix on `device`, dtype float32 or bfloat16 per the workload.

    Noise is drawn per chunk of rows from a generator seeded by (seed, chunk), so a
    chunk can be regenerated alone on the same device type.
    """
    dev = torch.device(device)
    blocks = block_labels(w) if blocks is None else blocks
    means = component_means(w).to(dev)
    out_dtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    X = torch.empty((w.n, w.d), dtype=out_dtype, device=dev)
    for ci, lo in enumerate(range(0, w.n, chunk_rows)):
        hi = min(lo + chunk_rows, w.n)
        g = _gen(w.seed, 1000 + ci, dev)
        x = torch.randn((hi - lo, w.d), generator=g, dtype=torch.float32, device=dev)
        x += means[blocks[lo:hi].to(dev)]
        if w.relu:
            x.clamp_(min=0.0)
        X[lo:hi] = x.to(out_dtype)
        del x
    return X


def sbm_graph(w: Workload, device="cpu", blocks: torch.Tensor | None = None):
    """CSR (rowptr, colidx) of the block-model graph; rowptr int32 or int64 per the workload.

    Returns (rowptr, colidx int32, blocks int64 on `device`).
    """
    dev = torch.device(device)
    blocks_cpu = block_labels(w) if blocks is None else blocks.cpu()
    blocks_d = blocks_cpu.to(dev)
    n, G = w.n, w.components
    m = int(n * w.avg_degree / 2)               # undirected pairs drawn

    # vertices grouped by block: pos -> vertex, block offsets and sizes
    by_block = torch.argsort(blocks_d, stable=True)
    size = torch.bincount(blocks_d, minlength=G)
    off = torch.cumsum(size, 0) - size

    g = _gen(w.seed, 21, dev)
    if w.powerlaw_alpha > 0:
        # Pareto(alpha) weights, scale 1:  w = U^(-1/alpha); capped so one vertex cannot dominate.
        u = torch.rand(n, generator=g, device=dev, dtype=torch.float64).clamp_(min=1e-12)
        wt = u.pow(-1.0 / w.powerlaw_alpha).clamp_(max=float(n) ** 0.5)
        cw = torch.cumsum(wt[by_block], 0)       # cumulative weight in block-sorted order
        total = cw[-1]
        start_w = torch.cat([cw.new_zeros(1), cw])[off]          # weight before each block
        block_w = torch.cat([cw.new_zeros(1), cw])[off + size] - start_w
        r = torch.rand(m, generator=g, device=dev, dtype=torch.float64) * total
        pos_u = torch.searchsorted(cw, r, right=True).clamp_(max=n - 1)
        src = by_block[pos_u]
    else:
        src = torch.randint(0, n, (m,), generator=g, device=dev)
    b = blocks_d[src]
    inside = torch.rand(m, generator=g, device=dev) < w.f_in
    r2 = torch.rand(m, generator=g, device=dev, dtype=torch.float64)

    # partner inside the block
    if w.powerlaw_alpha > 0:
        target = start_w[b] + r2 * block_w[b]
        pos_in = torch.searchsorted(cw, target, right=True)
        pos_in = torch.minimum(torch.maximum(pos_in, off[b]), off[b] + size[b] - 1)
    else:
        pos_in = off[b] + (r2 * size[b]).long().minimum(size[b] - 1)
    # partner outside: uniform over the n - size[b] vertices of the other blocks, which in
    # block-sorted order are the cyclic range that starts after block b
    others = (n - size[b]).clamp_(min=1)
    pos_out = (off[b] + size[b] + (r2 * others).long().minimum(others - 1)) % n
    dst = by_block[torch.where(inside, pos_in, pos_out)]
    del pos_in, pos_out, r2, inside, b

    keep = src != dst
    lo = torch.minimum(src, dst)[keep]
    hi = torch.maximum(src, dst)[keep]
    del src, dst, keep
    und = torch.unique(lo * n + hi)              # sorted, duplicates dropped
    del lo, hi
    a, c = und // n, und % n
    del und
    keys = torch.cat([a * n + c, c * n + a])
    del a, c
    keys = torch.sort(keys).values
    rows = keys // n
    colidx = (keys % n).to(torch.int32)
    del keys
    counts = torch.bincount(rows, minlength=n)
    del rows
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(counts, 0)
    if not w.rowptr_i64:
        assert int(rowptr[-1]) < 2**31
        rowptr = rowptr.to(torch.int32)
    return rowptr, colidx, blocks_d
