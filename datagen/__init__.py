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
Every random value is a pure function of (seed, stream, index): a Philox4x32-10
generator written here with exact integer tensor operations (it is this module's
own; neither the oracle nor the library shares it), so a graph, a feature table
or a tablet is the same whether it is generated on the CPU or on a GPU, in one
piece or in chunks.  The two smooth functions of the recipe (expected degree by
rank, inverse CDF of the target law) and the normal quantile function are
tabulated once on the host and interpolated linearly with separate, exactly
rounded multiply / add operations, so no device-dependent libm result ever
decides an integer.
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


# ---- counter-based random numbers ------------------------------------------
_M0, _M1, _W0, _W1, _MASK = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85, 0xFFFFFFFF
# streams (third counter word): one per kind of draw, so no two draws share a counter
_S_DEG, _S_DEAD, _S_PERM_SRC, _S_PERM_DST, _S_EDGE, _S_FEAT, _S_SPLIT = range(7)


def philox_rounds(c0, c1, c2, c3, k0: int, k1: int):
    """Philox4x32-10 (Salmon et al., SC'11): counter words as int64 tensors holding 32-bit values, key words
    as Python ints.  Returns the four output words as int64 tensors in [0, 2^32)."""
    k0, k1 = k0 & _MASK, k1 & _MASK
    for _ in range(10):
        # 32 x 32 -> 64-bit products: the operands are below 2^32, so the wrapped int64 product holds
        # the exact low 64 bits; an arithmetic shift followed by the mask recovers the high word
        p0 = c0 * _M0
        p1 = c2 * _M1
        hi0, lo0 = (p0 >> 32) & _MASK, p0 & _MASK
        hi1, lo1 = (p1 >> 32) & _MASK, p1 & _MASK
        c0 = hi1 ^ c1 ^ k0
        c2 = hi0 ^ c3 ^ k1
        c1, c3 = lo1, lo0
        k0, k1 = (k0 + _W0) & _MASK, (k1 + _W1) & _MASK
    return c0, c1, c2, c3


def philox4x32_10(idx: torch.Tensor, stream: int, seed: int):
    """One generator call per entry of idx: counter = (idx low word, idx high word, stream, 0),
    key = (seed low word, seed high word)."""
    return philox_rounds(idx & _MASK, (idx >> 32) & _MASK, torch.full_like(idx, stream & _MASK),
                         torch.zeros_like(idx), seed, seed >> 32)


def _uniform_pair(idx: torch.Tensor, stream: int, seed: int):
    """Two float64 uniforms in [0, 1) per index, each from 53 random bits (exact)."""
    w0, w1, w2, w3 = philox4x32_10(idx, stream, seed)
    a = ((w0 << 21) | (w1 >> 11)).to(torch.float64) * (2.0 ** -53)
    b = ((w2 << 21) | (w3 >> 11)).to(torch.float64) * (2.0 ** -53)
    return a, b


def _uniform(first: int, n: int, stream: int, seed: int, dev) -> torch.Tensor:
    """Uniforms number first .. first + n - 1 of a stream (two per generator call)."""
    lo, hi = first // 2, (first + n + 1) // 2
    a, b = _uniform_pair(torch.arange(lo, hi, device=dev, dtype=torch.int64), stream, seed)
    u = torch.stack((a, b), dim=1).reshape(-1)
    return u[first - 2 * lo:first - 2 * lo + n]


def _permutation(n: int, stream: int, seed: int, dev) -> torch.Tensor:
    """Permutation of 0 .. n-1: positions ordered by a 63-bit random key (ties by position)."""
    w0, w1, _, _ = philox4x32_10(torch.arange(n, device=dev, dtype=torch.int64), stream, seed)
    key = (w0 << 31) | (w1 >> 1)
    return torch.sort(key, stable=True).indices


class _Table:
    """A smooth function tabulated at knots + 1 evenly spaced points of [0, span) on the host and
    interpolated linearly on any device with separately rounded operations."""

    def __init__(self, fn, span: float, knots: int, dev, dtype=torch.float64):
        x = np.arange(knots + 1, dtype=np.float64) * (span / knots)
        self.values = torch.from_numpy(np.asarray(fn(x), dtype=np.float64)).to(dtype).to(dev)
        self.scale = knots / span
        self.knots = knots

    def __call__(self, x: torch.Tensor) -> torch.Tensor:
        pos = x * self.scale
        k = pos.floor().clamp_(0, self.knots - 1)
        t = pos - k
        k = k.to(torch.int64)
        lo, hi = self.values[k], self.values[k + 1]
        return lo + (hi - lo) * t


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
    seed = spec.gen_seed
    c, i0, beta = _solve_law(V, E, spec.gamma)
    knots = 1 << 20

    # expected degree by rank -> integer degree by rank
    weight = _Table(lambda r: c * (r + i0) ** (-beta), float(V), knots, dev)
    deg_rank = torch.empty(V, dtype=torch.int64, device=dev)
    step = 1 << 24
    for lo in range(0, V, step):
        hi = min(V, lo + step)
        w = weight(torch.arange(lo, hi, device=dev, dtype=torch.float64))
        fl = torch.floor(w)
        d = fl + (_uniform(lo, hi - lo, _S_DEG, seed, dev) < (w - fl)).to(torch.float64)
        d[_uniform(lo, hi - lo, _S_DEAD, seed, dev) < isolated] = 0
        deg_rank[lo:hi] = d.to(torch.int64)
    perm_src = _permutation(V, _S_PERM_SRC, seed, dev)        # rank -> source vertex id
    perm_dst = _permutation(V, _S_PERM_DST, seed, dev)        # rank -> target vertex id
    deg = torch.empty(V, dtype=torch.int64, device=dev)
    deg[perm_src] = deg_rank                                  # requested out-degree per vertex id
    del deg_rank, perm_src

    a, b = i0, i0 + float(V)
    if abs(beta - 1.0) < 1e-12:
        def inv_cdf_host(u):
            return a * (b / a) ** u - a
    else:
        pa, pb = a ** (1 - beta), b ** (1 - beta)
        def inv_cdf_host(u):
            return (pa + u * (pb - pa)) ** (1.0 / (1 - beta)) - a
    inv_cdf = _Table(inv_cdf_host, 1.0, knots, dev)

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
    drawn = 0
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        d = deg[lo:hi]
        n = int(d.sum().item())
        if n == 0:
            continue
        src = torch.repeat_interleave(torch.arange(lo, hi, device=dev, dtype=torch.int64), d)
        u = _uniform(drawn, n, _S_EDGE, seed, dev)              # draw number = position in the requested edge list
        drawn += n
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
    """[V, D] table of N(0,1) draws (fp32, or fp32 rounded to fp16).  Element number e = v * D + c uses word
    e mod 4 of generator call e div 4; the normal quantile function is tabulated on the host at 2^16 + 1
    points and interpolated in fp32."""
    V, D = spec.num_vertices, spec.feat_dim
    npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
    tdt = torch.float32 if spec.feat_dtype == "float32" else torch.float16
    dev = torch.device(device)
    if out is None:
        out = np.empty((V, D), dtype=npdt)

    def quantile(p):
        p = np.clip(p, 2.0 ** -33, 1.0 - 2.0 ** -33)
        return (torch.erfinv(torch.from_numpy(2.0 * p - 1.0)) * math.sqrt(2.0)).numpy()

    table = _Table(quantile, 1.0, 1 << 16, dev, dtype=torch.float32)
    for lo in range(0, V, chunk_rows):
        hi = min(V, lo + chunk_rows)
        first, n = lo * D, (hi - lo) * D
        c_lo, c_hi = first // 4, (first + n + 3) // 4
        words = torch.stack(philox4x32_10(torch.arange(c_lo, c_hi, device=dev, dtype=torch.int64), _S_FEAT,
                                          spec.feat_seed), dim=1).reshape(-1)[first - 4 * c_lo:first - 4 * c_lo + n]
        u = (words.to(torch.float32) + 0.5) * (2.0 ** -32)      # fp32 rounding of the word: the same on every device
        x = table(u.clamp_(0.0, 1.0 - 2.0 ** -24)).reshape(hi - lo, D).to(tdt)
        torch.from_numpy(out[lo:hi]).copy_(x)
    return out


def make_tablet(spec: WorkloadSpec, device: str = "cpu") -> np.ndarray:
    """Training tablet: the first train_frac * V entries of a seeded permutation,
    already in epoch order (consecutive slices of `batch` are the mini-batches)."""
    perm = _permutation(spec.num_vertices, _S_SPLIT, spec.split_seed, torch.device(device))
    n = max(1, int(round(spec.train_frac * spec.num_vertices)))
    return perm[:n].to(torch.int32).cpu().numpy().copy()


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
