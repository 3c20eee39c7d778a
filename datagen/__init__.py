"""Seeded synthetic inputs shared by the oracle-side and the HIP-side tests.

Nothing here belongs to the method: this module only manufactures graphs,
feature tables and training splits with the shapes of the paper's datasets
(Table 2), which are not available offline.  Both sides consume the arrays this
module returns; neither side's arithmetic lives here.

Graph recipe (directed Chung-Lu, power-law expected degrees):
  * rank i has expected out-degree w_i = c * (i + i0)^(-1/(gamma-1)), with c and
    i0 chosen so that sum(w) = E_target and w_0 = floor(sqrt(E_target));
  * degree d_i = floor(w_i) + Bernoulli(frac(w_i)); a fraction `isolated` of the
    vertices is forced to degree 0 so that empty rows exist;
  * each out-edge's target rank is drawn by inverting the continuous CDF of the
    same law; ranks map to vertex ids through two independent random
    permutations (one for sources, one for targets), so hubs are scattered;
  * self-loops and duplicate (src, dst) pairs are dropped and every row is
    sorted, giving a simple graph in CSR form.
All draws come from a torch.Generator seeded by the caller; for a given seed,
torch build and device the result is reproducible.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    num_vertices: int
    num_edges: int          # target; the simple graph ends up slightly below
    gamma: float
    feat_dim: int
    feat_dtype: str         # "float32" | "float16"
    fanouts: tuple
    batch: int
    train_frac: float
    topo_frac: float        # share of 4E + 8V bytes given to the topology cache
    feat_frac: float        # share of V * D * elem bytes given to the feature cache
    index64: bool
    config_no: int

    @property
    def gen_seed(self): return 1000 + self.config_no
    @property
    def feat_seed(self): return 2000 + self.config_no
    @property
    def split_seed(self): return 3000 + self.config_no
    @property
    def base_seed(self): return 4000 + self.config_no


# The five workloads named by the benchmark definition (shapes follow Table 2's
# PR / PA rows and the stated fan-outs; fp16 and 3-hop variants are additions).
TINY = WorkloadSpec("tiny", 10_000, 200_000, 2.1, 128, "float32", (10, 5), 1024, 1.0, 0.2, 0.2, False, 1)
MID = WorkloadSpec("mid", 2_400_000, 62_000_000, 2.1, 100, "float32", (15, 10, 5), 8192, 0.10, 0.5, 0.3, False, 2)
LARGE = WorkloadSpec("large", 111_000_000, 1_600_000_000, 2.1, 128, "float32", (15, 10, 5), 8192, 0.01, 1.0, 1.0, True, 3)
SHARE = WorkloadSpec("share", 250_000_000, 8_000_000_000, 2.0, 128, "float16", (25, 10), 8192, 0.01, 1.0, 1.0, True, 4)
WIDE = WorkloadSpec("wide", 10_000_000, 400_000_000, 2.1, 1024, "float16", (20, 10), 4096, 0.10, 1.0, 0.25, False, 5)
WORKLOADS = {w.name: w for w in (TINY, MID, LARGE, SHARE, WIDE)}


def scaled(spec: WorkloadSpec, factor: float, name: str | None = None) -> WorkloadSpec:
    """Same shape with V and E multiplied by `factor` (average degree, gamma,
    row size, fan-outs, batch and cache ratios unchanged)."""
    from dataclasses import replace
    return replace(spec, name=name or f"{spec.name}@{factor:g}", num_vertices=max(1, int(spec.num_vertices * factor)),
                   num_edges=max(1, int(spec.num_edges * factor)))


def _series_sum(V: int, i0: float, beta: float) -> float:
    """sum_{i=0}^{V-1} (i + i0)^(-beta) by Euler-Maclaurin (i0 >> 1)."""
    a, b = i0, i0 + V - 1.0
    if abs(beta - 1.0) < 1e-12:
        integral = math.log(b / a)
    else:
        integral = (b ** (1 - beta) - a ** (1 - beta)) / (1 - beta)
    return integral + 0.5 * (a ** -beta + b ** -beta) + beta / 12.0 * (a ** (-beta - 1) - b ** (-beta - 1))


def _solve_law(V: int, E: int, gamma: float):
    """Return (c, i0, beta) with sum w = E and w_0 = floor(sqrt(E))."""
    beta = 1.0 / (gamma - 1.0)
    wmax = max(1.0, math.floor(math.sqrt(E)))
    lo, hi = 1.0, float(max(V, 4)) * 64
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        c = E / _series_sum(V, mid, beta)
        if c * mid ** -beta > wmax:
            lo = mid
        else:
            hi = mid
    i0 = math.sqrt(lo * hi)
    return E / _series_sum(V, i0, beta), i0, beta


def make_graph(spec: WorkloadSpec, device: str = "cpu", isolated: float = 0.001, chunk_edges: int = 1 << 26,
               indptr_out: np.ndarray | None = None, indices_alloc=None):
    """Build the CSR graph for `spec`.

    Returns (indptr, indices) as numpy arrays: indptr int64 if spec.index64 else
    int32 (V + 1 entries), indices int32.  `indices_alloc(n)` may supply the
    destination array (e.g. pinned host memory); it is asked for room for all
    draws and `indices` is the prefix the simple graph fills.  `indptr_out`
    (V + 1 entries of the right dtype) likewise receives the offsets.
    """
    V, E = spec.num_vertices, spec.num_edges
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(spec.gen_seed)
    c, i0, beta = _solve_law(V, E, spec.gamma)

    # expected degree by rank -> integer degree by rank
    deg_rank = torch.empty(V, dtype=torch.int64, device=dev)
    step = 1 << 24
    for lo in range(0, V, step):
        hi = min(V, lo + step)
        r = torch.arange(lo, hi, device=dev, dtype=torch.float64)
        w = c * (r + i0) ** (-beta)
        fl = torch.floor(w)
        u = torch.rand(hi - lo, generator=gen, device=dev, dtype=torch.float64)
        d = fl + (u < (w - fl)).to(torch.float64)
        dead = torch.rand(hi - lo, generator=gen, device=dev) < isolated
        d[dead] = 0
        deg_rank[lo:hi] = d.to(torch.int64)
    perm_src = torch.randperm(V, generator=gen, device=dev)   # rank -> source vertex id
    perm_dst = torch.randperm(V, generator=gen, device=dev)   # rank -> target vertex id
    deg = torch.empty(V, dtype=torch.int64, device=dev)
    deg[perm_src] = deg_rank                                  # requested out-degree per vertex id
    del deg_rank, perm_src

    a, b = i0, i0 + float(V)
    if abs(beta - 1.0) < 1e-12:
        def inv_cdf(u):
            return a * (b / a) ** u - a
    else:
        pa, pb = a ** (1 - beta), b ** (1 - beta)
        def inv_cdf(u):
            return (pa + u * (pb - pa)) ** (1.0 / (1 - beta)) - a

    # rows are produced in chunks of consecutive vertex ids holding <= chunk_edges draws
    csum = torch.cumsum(deg, 0)
    total_draws = int(csum[-1].item())
    bounds = [0]
    while bounds[-1] < V:
        base = int(csum[bounds[-1] - 1].item()) if bounds[-1] > 0 else 0
        nxt = int(torch.searchsorted(csum, torch.tensor(base + chunk_edges, device=dev), right=True).item())
        bounds.append(min(V, max(nxt, bounds[-1] + 1)))
    final_deg = torch.zeros(V, dtype=torch.int64, device=dev)
    # destination sized for the draws; the simple graph uses a prefix of it
    indices_full = indices_alloc(total_draws) if indices_alloc is not None else np.empty(total_draws, dtype=np.int32)
    dst_t = torch.from_numpy(indices_full) if total_draws else None
    at = 0
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        d = deg[lo:hi]
        n = int(d.sum().item())
        if n == 0:
            continue
        src = torch.repeat_interleave(torch.arange(lo, hi, device=dev, dtype=torch.int64), d)
        u = torch.rand(n, generator=gen, device=dev, dtype=torch.float64)
        rank = inv_cdf(u).floor().to(torch.int64).clamp_(0, V - 1)
        del u
        dst = perm_dst[rank]
        del rank
        keep = dst != src
        key = (src[keep] << 32) | dst[keep]
        del src, dst, keep
        key = torch.unique(key)                               # sorted: by row, then by column id
        final_deg[lo:hi] = torch.bincount((key >> 32) - lo, minlength=hi - lo)
        cols = (key & 0xFFFFFFFF).to(torch.int32)
        dst_t[at:at + cols.numel()].copy_(cols)
        at += cols.numel()
        del key, cols
    n_edges = int(final_deg.sum().item())
    assert at == n_edges
    indices = indices_full[:n_edges]
    idt = torch.int64 if spec.index64 else torch.int32
    assert spec.index64 or n_edges < 2 ** 31
    indptr_t = torch.zeros(V + 1, dtype=torch.int64, device=dev)
    indptr_t[1:] = torch.cumsum(final_deg, 0)
    if indptr_out is not None:
        torch.from_numpy(indptr_out).copy_(indptr_t.to(idt))
        indptr_np = indptr_out
    else:
        indptr_np = indptr_t.to(idt).cpu().numpy()
    return indptr_np, indices


def make_features(spec: WorkloadSpec, device: str = "cpu", out: np.ndarray | None = None, chunk_rows: int = 1 << 20):
    """[V, D] table of N(0,1) draws (fp32, or fp32 rounded to fp16)."""
    V, D = spec.num_vertices, spec.feat_dim
    npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
    tdt = torch.float32 if spec.feat_dtype == "float32" else torch.float16
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(spec.feat_seed)
    if out is None:
        out = np.empty((V, D), dtype=npdt)
    for lo in range(0, V, chunk_rows):
        hi = min(V, lo + chunk_rows)
        x = torch.randn(hi - lo, D, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        torch.from_numpy(out[lo:hi]).copy_(x)
    return out


def make_tablet(spec: WorkloadSpec) -> np.ndarray:
    """Training tablet: the first train_frac * V entries of a seeded permutation,
    already in epoch order (consecutive slices of `batch` are the mini-batches)."""
    gen = torch.Generator()
    gen.manual_seed(spec.split_seed)
    perm = torch.randperm(spec.num_vertices, generator=gen)
    n = max(1, int(round(spec.train_frac * spec.num_vertices)))
    return perm[:n].to(torch.int32).numpy().copy()


def budgets(spec: WorkloadSpec, num_edges: int):
    """Byte budgets for the topology and feature caches from the spec's ratios."""
    elem = 4 if spec.feat_dtype == "float32" else 2
    topo = int(spec.topo_frac * (4 * num_edges + 8 * spec.num_vertices))
    feat = int(spec.feat_frac * spec.num_vertices) * spec.feat_dim * elem
    return topo, feat


def tiny_graph(num_vertices: int, avg_degree: float, seed: int, max_degree: int | None = None):
    """Small uniform-random simple digraph for brute-force tests (numpy only)."""
    rng = np.random.default_rng(seed)
    rows = []
    indptr = [0]
    for v in range(num_vertices):
        d = int(rng.poisson(avg_degree))
        if max_degree is not None:
            d = min(d, max_degree)
        d = min(d, num_vertices - 1)
        cand = rng.choice(num_vertices - 1, size=d, replace=False)
        cand = np.sort(np.where(cand >= v, cand + 1, cand))
        rows.append(cand)
        indptr.append(indptr[-1] + d)
    indices = np.concatenate(rows).astype(np.int32) if rows else np.empty(0, np.int32)
    return np.asarray(indptr, dtype=np.int32), indices
