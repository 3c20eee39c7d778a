"""Thin ctypes binding of liblegion_prep (argument marshalling only).

PyTorch supplies device memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the library cannot be
loaded, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
import weakref

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "liblegion_prep.so")
MAX_HOPS = 8
MAX_FANOUT = 64
STATIC_GATHER_MAX_IDS = 1 << 22


class LegionPrepError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"legion_prep status {status}: {text}")
        self.status = status


class _Graph(C.Structure):
    _fields_ = [("num_vertices", C.c_int64), ("num_edges", C.c_int64), ("indptr", C.c_void_p),
                ("indptr_bytes", C.c_int32), ("indices", C.c_void_p), ("features", C.c_void_p),
                ("feat_dim", C.c_int32), ("elem_bytes", C.c_int32)]


class CachePlan(C.Structure):
    _fields_ = [("n_topo", C.c_int64), ("topo_edges", C.c_int64), ("topo_bytes", C.c_uint64),
                ("n_feat", C.c_int64), ("feat_bytes", C.c_uint64)]


class PlanPoint(C.Structure):
    _fields_ = [("m_topo", C.c_uint64), ("m_feat", C.c_uint64), ("n_topo", C.c_int64), ("n_feat", C.c_int64),
                ("uncached_topo_hot", C.c_uint64), ("uncached_feat_hot", C.c_uint64)]


class _SampleOut(C.Structure):
    _fields_ = [("frontier", C.c_void_p * (MAX_HOPS + 1)), ("nbr", C.c_void_p * MAX_HOPS),
                ("cnt", C.c_void_p * MAX_HOPS), ("cap", C.c_int64 * (MAX_HOPS + 1)), ("n_frontier", C.c_void_p),
                ("gather_ids", C.c_void_p), ("gather_cap", C.c_int64), ("n_gather", C.c_void_p)]


class _BlocksOut(C.Structure):
    _fields_ = [("blk_indptr", C.c_void_p * MAX_HOPS), ("blk_src", C.c_void_p * MAX_HOPS),
                ("feat_row", C.c_void_p * (MAX_HOPS + 1))]


class Profile(C.Structure):
    _fields_ = [("n_sample", C.c_int64), ("n_partition", C.c_int64), ("n_hit", C.c_int64), ("n_miss", C.c_int64),
                ("ms_sample", C.c_double), ("ms_partition", C.c_double), ("ms_hit", C.c_double),
                ("ms_miss", C.c_double)]


EXPORTS = ["lgp_host_alloc", "lgp_host_free", "lgp_shuffle_tablet", "lgp_create", "lgp_destroy", "lgp_build_hotness", "lgp_get_presample_stats", "lgp_get_hotness",
           "lgp_set_hotness", "lgp_plan_cache", "lgp_search_cache_plan", "lgp_cslp", "lgp_build_cache", "lgp_build_clique_cache", "lgp_get_clique_plan",
           "lgp_gather_features_clique", "lgp_get_cache_plan", "lgp_get_cache", "lgp_get_cache_part", "lgp_reserve",
           "lgp_sample_khop", "lgp_sample_extract", "lgp_build_blocks", "lgp_gather_features", "lgp_gather_features_static", "lgp_set_overlap", "lgp_workspace_bytes", "lgp_check", "lgp_set_profiling", "lgp_get_profile",
           "lgp_strerror", "lgp_last_error"]

_lib = None


def load_library():
    """Load liblegion_prep.so.  It is built first if no built library exists, or if the one that
    exists was built from other sources than the ones in csrc/ and include/ now (a hash of the
    sources is stored beside the library), so an edit never runs against an old binary."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if not os.path.exists(_LIBPATH) or _build.is_stale():
        _build.build()
    L = C.CDLL(_LIBPATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    L.lgp_host_alloc.argtypes = [C.c_size_t, C.POINTER(vp)]
    L.lgp_host_free.argtypes = [vp]
    L.lgp_create.argtypes = [C.POINTER(_Graph), C.c_int, C.POINTER(vp)]
    L.lgp_destroy.argtypes = [vp]
    L.lgp_build_hotness.argtypes = [vp, vp, i64, i32, vp, i32, u64, i64, vp]
    L.lgp_get_presample_stats.argtypes = [vp, vp, vp]
    L.lgp_get_hotness.argtypes = [vp, vp, vp]
    L.lgp_set_hotness.argtypes = [vp, vp, vp]
    L.lgp_plan_cache.argtypes = [vp, u64, u64, C.POINTER(CachePlan), vp]
    L.lgp_search_cache_plan.argtypes = [vp, u64, u64, C.c_uint32, i32, vp, vp, vp]
    L.lgp_shuffle_tablet.argtypes = [C.c_int, vp, vp, i64, u64, C.c_uint32, vp]
    L.lgp_cslp.argtypes = [C.c_int, i32, i64, vp, vp, vp, vp, vp, vp, vp]
    L.lgp_build_cache.argtypes = [vp, u64, u64, vp]
    L.lgp_get_cache_plan.argtypes = [vp, C.POINTER(CachePlan)]
    L.lgp_get_cache.argtypes = [vp, vp, vp, vp, vp, vp]
    L.lgp_get_cache_part.argtypes = [vp, i32, i64, i64, vp]
    L.lgp_reserve.argtypes = [vp, i32, vp, i32]
    L.lgp_build_clique_cache.argtypes = [vp, i32, vp, vp, u64, u64, vp]
    L.lgp_get_clique_plan.argtypes = [vp, i32, C.POINTER(CachePlan)]
    L.lgp_gather_features_clique.argtypes = [vp, i32, vp, i64, vp, vp, vp, vp]
    L.lgp_sample_khop.argtypes = [vp, vp, i32, vp, i32, u64, C.POINTER(_SampleOut), vp]
    L.lgp_sample_extract.argtypes = [vp, vp, i32, vp, i32, u64, C.POINTER(_SampleOut), vp, vp, vp, vp]
    L.lgp_build_blocks.argtypes = [vp, vp, i32, vp, i32, C.POINTER(_SampleOut), C.POINTER(_BlocksOut), vp]
    L.lgp_gather_features.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.lgp_gather_features_static.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.lgp_set_overlap.argtypes = [vp, C.c_int]
    L.lgp_workspace_bytes.argtypes = [vp, i32, vp, i32, vp, vp]
    L.lgp_check.argtypes = [vp, vp]
    L.lgp_set_profiling.argtypes = [vp, C.c_int]
    L.lgp_get_profile.argtypes = [vp, C.POINTER(Profile)]
    L.lgp_strerror.argtypes = [C.c_int]
    L.lgp_strerror.restype = C.c_char_p
    L.lgp_last_error.argtypes = [vp]
    L.lgp_last_error.restype = C.c_char_p
    for name in EXPORTS[:-2]:
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def pinned_empty(shape, dtype) -> np.ndarray:
    """numpy array in pinned, GPU-addressable host memory (lgp_host_alloc)."""
    L = load_library()
    dtype = np.dtype(dtype)
    shape = (shape,) if np.isscalar(shape) else tuple(int(s) for s in shape)
    nbytes = int(np.prod(shape, dtype=np.int64)) * dtype.itemsize
    ptr = C.c_void_p()
    st = L.lgp_host_alloc(max(nbytes, 1), C.byref(ptr))
    if st != 0:
        raise LegionPrepError(st, f"pinned allocation of {nbytes} bytes failed")
    buf = (C.c_char * max(nbytes, 1)).from_address(ptr.value)
    arr = np.frombuffer(buf, dtype=dtype, count=int(np.prod(shape, dtype=np.int64))).reshape(shape)
    weakref.finalize(buf, L.lgp_host_free, ptr.value)
    return arr


def pinned_copy(a: np.ndarray) -> np.ndarray:
    out = pinned_empty(a.shape, a.dtype)
    out[...] = a
    return out


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def worst_case_sizes(num_vertices: int, n_seeds: int, fanouts):
    """need[h] for h = 0 .. n_hops and the gather-set bound, as the header defines them."""
    need = [int(n_seeds)]
    total = int(n_seeds)
    for h, f in enumerate(fanouts):
        samples = need[h] * int(f)
        total += samples
        need.append(min(num_vertices, samples))
    return need, min(num_vertices, total)


def shuffle_tablet(train_ids: torch.Tensor, seed: int, epoch: int, stream=None) -> torch.Tensor:
    """Batch generator: the tablet (int32 CUDA tensor) in the order of epoch `epoch`."""
    L = load_library()
    assert train_ids.is_cuda and train_ids.dtype == torch.int32 and train_ids.is_contiguous()
    out = torch.empty_like(train_ids)
    st = L.lgp_shuffle_tablet(train_ids.device.index or 0, train_ids.data_ptr(), out.data_ptr(), train_ids.numel(),
                              seed & (2**64 - 1), epoch, _stream_ptr(stream))
    if st != 0:
        raise LegionPrepError(st, L.lgp_strerror(st).decode())
    return out


def cslp(hot: torch.Tensor, stream=None):
    """Algorithm 1 on a [k_g, V] int32/uint32 CUDA tensor of hotness rows.
    Returns (acc int64[V], order, owner, queues int32[V]) as CUDA tensors and the host list of queue offsets."""
    L = load_library()
    assert hot.is_cuda and hot.dim() == 2 and hot.is_contiguous() and hot.element_size() == 4
    k_g, V = hot.shape
    dev = hot.device
    acc = torch.empty(V, dtype=torch.int64, device=dev)
    order = torch.empty(V, dtype=torch.int32, device=dev)
    owner = torch.empty(V, dtype=torch.int32, device=dev)
    queues = torch.empty(V, dtype=torch.int32, device=dev)
    offsets = (C.c_int64 * (k_g + 1))()
    st = L.lgp_cslp(dev.index or 0, k_g, V, hot.data_ptr(), acc.data_ptr(), order.data_ptr(), owner.data_ptr(),
                    queues.data_ptr(), C.addressof(offsets), _stream_ptr(stream))
    if st != 0:
        raise LegionPrepError(st, L.lgp_strerror(st).decode())
    return acc, order, owner, queues, list(offsets)


class SampleBuffers:
    """Device buffers for one lgp_sample_khop call, sized for the worst case."""

    def __init__(self, num_vertices: int, max_seeds: int, fanouts, device="cuda:0", last_frontier: bool = False):
        """last_frontier: also produce frontier[n_hops], the set reached by the last hop (needed by build_blocks)."""
        self.fanouts = [int(f) for f in fanouts]
        self.need, self.gather_cap = worst_case_sizes(num_vertices, max_seeds, self.fanouts)
        dev = torch.device(device)
        L = len(self.fanouts)
        self.last_frontier = last_frontier
        self.frontier = [None] + [torch.empty(self.need[h], dtype=torch.int32, device=dev) for h in range(1, L)]
        if last_frontier:
            self.frontier.append(torch.empty(self.need[L], dtype=torch.int32, device=dev))
        self.nbr = [torch.empty((self.need[h], self.fanouts[h]), dtype=torch.int32, device=dev) for h in range(L)]
        self.cnt = [torch.empty(self.need[h], dtype=torch.int32, device=dev) for h in range(L)]
        self.n_frontier = torch.zeros(L + 1, dtype=torch.int32, device=dev)
        self.gather_ids = torch.empty(self.gather_cap, dtype=torch.int32, device=dev)
        self.n_gather = torch.zeros(1, dtype=torch.int32, device=dev)
        o = _SampleOut()
        for h in range(L):
            o.frontier[h] = self.frontier[h].data_ptr() if h else None
            o.nbr[h] = self.nbr[h].data_ptr()
            o.cnt[h] = self.cnt[h].data_ptr()
            o.cap[h] = self.need[h]
        if last_frontier:
            o.frontier[L] = self.frontier[L].data_ptr()
            o.cap[L] = self.need[L]
        o.n_frontier = self.n_frontier.data_ptr()
        o.gather_ids = self.gather_ids.data_ptr()
        o.gather_cap = self.gather_cap
        o.n_gather = self.n_gather.data_ptr()
        self.c_struct = o

    def to_host(self, seeds: torch.Tensor):
        """Synchronise and return (frontier, nbr, cnt, gather_ids) trimmed to their actual sizes (numpy)."""
        n = self.n_frontier.cpu().tolist()
        L = len(self.fanouts)
        fr = [seeds.cpu().numpy()] + [self.frontier[h][:n[h]].cpu().numpy() for h in range(1, len(self.frontier))]
        nbr = [self.nbr[h][:n[h]].cpu().numpy() for h in range(L)]
        cnt = [self.cnt[h][:n[h]].cpu().numpy() for h in range(L)]
        ng = int(self.n_gather.item())
        return fr, nbr, cnt, self.gather_ids[:ng].cpu().numpy()


class BlockBuffers:
    """Device buffers for one lgp_build_blocks call, sized like the SampleBuffers they go with."""

    def __init__(self, sample: SampleBuffers):
        assert sample.last_frontier, "build_blocks needs SampleBuffers(..., last_frontier=True)"
        dev = sample.gather_ids.device
        L = len(sample.fanouts)
        self.sample = sample
        self.blk_indptr = [torch.empty(sample.need[h] + 1, dtype=torch.int64, device=dev) for h in range(L)]
        self.blk_src = [torch.empty(sample.need[h] * sample.fanouts[h], dtype=torch.int32, device=dev) for h in range(L)]
        self.feat_row = [torch.empty(sample.need[h], dtype=torch.int32, device=dev) for h in range(L + 1)]
        o = _BlocksOut()
        for h in range(L):
            o.blk_indptr[h] = self.blk_indptr[h].data_ptr()
            o.blk_src[h] = self.blk_src[h].data_ptr()
        for h in range(L + 1):
            o.feat_row[h] = self.feat_row[h].data_ptr()
        self.c_struct = o

    def to_host(self):
        """Synchronise and return (blk_indptr, blk_src, feat_row) trimmed to their actual sizes (numpy)."""
        n = self.sample.n_frontier.cpu().tolist()
        L = len(self.sample.fanouts)
        indptr = [self.blk_indptr[h][:n[h] + 1].cpu().numpy() for h in range(L)]
        src = [self.blk_src[h][:int(indptr[h][-1])].cpu().numpy() for h in range(L)]
        rows = [self.feat_row[h][:n[h]].cpu().numpy() for h in range(L + 1)]
        return indptr, src, rows


class Context:
    """One graph + feature table in pinned CPU memory, its caches and scratch on one GPU.

    indptr / indices / features: numpy arrays from pinned_empty / pinned_copy, or pinned
    torch tensors.  Method names mirror the C entry points.
    """

    def __init__(self, indptr, indices, features=None, device: int = 0):
        self._L = load_library()
        self._keep = (indptr, indices, features)
        def ptr(a):
            return a.data_ptr() if isinstance(a, torch.Tensor) else a.ctypes.data
        def isz(a):
            return a.element_size() if isinstance(a, torch.Tensor) else a.dtype.itemsize
        g = _Graph()
        g.num_vertices = int(indptr.shape[0]) - 1
        g.num_edges = int(indices.shape[0])
        g.indptr = ptr(indptr)
        g.indptr_bytes = isz(indptr)
        g.indices = ptr(indices) if g.num_edges else None
        if features is not None:
            g.features = ptr(features)
            g.feat_dim = int(features.shape[1])
            g.elem_bytes = isz(features)
            self.feat_torch_dtype = {2: torch.float16, 4: torch.float32}.get(g.elem_bytes, torch.uint8)
        self.num_vertices = g.num_vertices
        self.feat_dim = int(g.feat_dim)
        self.elem_bytes = int(g.elem_bytes)
        self.device = torch.device(f"cuda:{device}")
        h = C.c_void_p()
        st = self._L.lgp_create(C.byref(g), device, C.byref(h))
        if st != 0:
            raise LegionPrepError(st, self._L.lgp_strerror(st).decode())
        self._h = h
        self._fin = weakref.finalize(self, self._L.lgp_destroy, h)

    def close(self):
        self._fin()

    def _ok(self, st: int):
        if st != 0:
            raise LegionPrepError(st, self._L.lgp_strerror(st).decode() + " -- " +
                                  self._L.lgp_last_error(self._h).decode())

    @staticmethod
    def _fanouts(fanouts):
        return np.ascontiguousarray(fanouts, dtype=np.int32)

    def build_hotness(self, train_ids: torch.Tensor, batch: int, fanouts, base_seed: int, max_batches: int = -1,
                      stream=None):
        assert train_ids.is_cuda and train_ids.dtype == torch.int32 and train_ids.is_contiguous()
        fo = self._fanouts(fanouts)
        self._ok(self._L.lgp_build_hotness(self._h, train_ids.data_ptr(), train_ids.numel(), batch, fo.ctypes.data,
                                           fo.size, base_seed & (2**64 - 1), max_batches, _stream_ptr(stream)))

    def get_presample_stats(self):
        """(n_batches, n_expansions) of the last build_hotness."""
        nb, ne = C.c_int64(0), C.c_int64(0)
        self._ok(self._L.lgp_get_presample_stats(self._h, C.addressof(nb), C.addressof(ne)))
        return int(nb.value), int(ne.value)

    def get_hotness(self):
        topo = np.empty(self.num_vertices, dtype=np.uint32)
        feat = np.empty(self.num_vertices, dtype=np.uint32)
        self._ok(self._L.lgp_get_hotness(self._h, topo.ctypes.data, feat.ctypes.data))
        return topo, feat

    def set_hotness(self, topo: np.ndarray, feat: np.ndarray):
        topo = np.ascontiguousarray(topo, dtype=np.uint32)
        feat = np.ascontiguousarray(feat, dtype=np.uint32)
        assert topo.size == self.num_vertices and feat.size == self.num_vertices
        self._ok(self._L.lgp_set_hotness(self._h, topo.ctypes.data, feat.ctypes.data))

    def plan_cache(self, topo_budget: int, feat_budget: int, stream=None) -> CachePlan:
        p = CachePlan()
        self._ok(self._L.lgp_plan_cache(self._h, int(topo_budget), int(feat_budget), C.byref(p), _stream_ptr(stream)))
        return p

    def search_cache_plan(self, total_budget: int, n_tsum: int, cls_bytes: int = 64, n_alpha: int = 101, stream=None):
        """Returns (best_index, points): points is a numpy structured array, one entry per candidate alpha."""
        pts = (PlanPoint * n_alpha)()
        best = C.c_int32(-1)
        self._ok(self._L.lgp_search_cache_plan(self._h, int(total_budget), int(n_tsum), cls_bytes, n_alpha,
                                               C.addressof(pts), C.addressof(best), _stream_ptr(stream)))
        arr = np.frombuffer(pts, dtype=[("m_topo", np.uint64), ("m_feat", np.uint64), ("n_topo", np.int64),
                                         ("n_feat", np.int64), ("uncached_topo_hot", np.uint64),
                                         ("uncached_feat_hot", np.uint64)]).copy()
        return int(best.value), arr

    def build_cache(self, topo_budget: int, feat_budget: int, stream=None) -> CachePlan:
        self._ok(self._L.lgp_build_cache(self._h, int(topo_budget), int(feat_budget), _stream_ptr(stream)))
        return self.get_cache_plan()

    def build_clique_cache(self, topo_hot: torch.Tensor, feat_hot: torch.Tensor, topo_budget: int, feat_budget: int,
                           stream=None) -> list:
        """Cache of a simulated clique from two [k_g, V] hotness matrices; budgets are per member.
        Returns the members' plans."""
        for h in (topo_hot, feat_hot):
            assert h.is_cuda and h.is_contiguous() and h.dim() == 2 and h.shape[1] == self.num_vertices
            assert h.dtype in (torch.int32, torch.uint32) and h.shape[0] == topo_hot.shape[0]
        k_g = topo_hot.shape[0]
        self._ok(self._L.lgp_build_clique_cache(self._h, k_g, topo_hot.data_ptr(), feat_hot.data_ptr(),
                                                int(topo_budget), int(feat_budget), _stream_ptr(stream)))
        return [self.get_clique_plan(g) for g in range(k_g)]

    def get_clique_plan(self, member: int) -> CachePlan:
        p = CachePlan()
        self._ok(self._L.lgp_get_clique_plan(self._h, member, C.byref(p)))
        return p

    def get_cache_plan(self) -> CachePlan:
        p = CachePlan()
        self._ok(self._L.lgp_get_cache_plan(self._h, C.byref(p)))
        return p

    def get_cache(self, contents: bool = True):
        """(topo_ids, t_indptr, t_indices, feat_ids, feat_rows); the two content arrays are None if not asked for."""
        p = self.get_cache_plan()
        topo_ids = np.empty(p.n_topo, dtype=np.int32)
        t_indptr = np.empty(p.n_topo + 1, dtype=np.int64)
        feat_ids = np.empty(p.n_feat, dtype=np.int32)
        t_indices = np.empty(p.topo_edges, dtype=np.int32) if contents else None
        feat_rows = np.empty((p.n_feat, self.feat_dim * self.elem_bytes), dtype=np.uint8) if contents else None
        self._ok(self._L.lgp_get_cache(self._h, topo_ids.ctypes.data, t_indptr.ctypes.data,
                                       t_indices.ctypes.data if contents else None, feat_ids.ctypes.data,
                                       feat_rows.ctypes.data if contents else None))
        return topo_ids, t_indptr, t_indices, feat_ids, feat_rows

    def get_cache_part(self, which: int, first: int, count: int, out: np.ndarray | None = None) -> np.ndarray:
        """which = 0: cached column ids [first, first + count) (int32); which = 1: cached feature rows of ranks
        first .. first + count - 1 (uint8 [count, row_bytes]).  `out` may supply the destination."""
        if out is None:
            out = (np.empty(count, dtype=np.int32) if which == 0
                   else np.empty((count, self.feat_dim * self.elem_bytes), dtype=np.uint8))
        assert out.flags["C_CONTIGUOUS"] and out.nbytes >= count * (4 if which == 0 else self.feat_dim * self.elem_bytes)
        self._ok(self._L.lgp_get_cache_part(self._h, which, int(first), int(count), out.ctypes.data))
        return out

    def reserve(self, max_seeds: int, fanouts):
        """Size every per-batch scratch now; afterwards the per-batch calls never allocate or synchronise."""
        fo = self._fanouts(fanouts)
        self._ok(self._L.lgp_reserve(self._h, int(max_seeds), fo.ctypes.data, fo.size))

    def sample_khop(self, seeds: torch.Tensor, fanouts, rng_seed: int, out: SampleBuffers | None = None,
                    stream=None) -> SampleBuffers:
        assert seeds.is_cuda and seeds.dtype == torch.int32 and seeds.is_contiguous()
        fo = self._fanouts(fanouts)
        if out is None:
            out = SampleBuffers(self.num_vertices, seeds.numel(), fo.tolist(), self.device)
        self._ok(self._L.lgp_sample_khop(self._h, seeds.data_ptr(), seeds.numel(), fo.ctypes.data, fo.size,
                                         rng_seed & (2**64 - 1), C.byref(out.c_struct), _stream_ptr(stream)))
        return out

    def sample_extract(self, seeds: torch.Tensor, fanouts, rng_seed: int, out: SampleBuffers, rows: torch.Tensor,
                       groups: torch.Tensor | None = None, stats: torch.Tensor | None = None, stream=None):
        """sample_khop + gather_features of one batch with the extraction overlapped hop by hop; out.gather_ids
        receives the listing (seeds, then per hop the vertices it reached first), rows its feature rows."""
        assert seeds.is_cuda and seeds.dtype == torch.int32 and seeds.is_contiguous()
        assert rows.is_cuda and rows.is_contiguous() and rows.numel() * rows.element_size() >= out.gather_cap * self.feat_dim * self.elem_bytes
        fo = self._fanouts(fanouts)
        self._ok(self._L.lgp_sample_extract(self._h, seeds.data_ptr(), seeds.numel(), fo.ctypes.data, fo.size,
                                            rng_seed & (2**64 - 1), C.byref(out.c_struct), rows.data_ptr(),
                                            None if groups is None else groups.data_ptr(),
                                            None if stats is None else stats.data_ptr(), _stream_ptr(stream)))
        return out

    def build_blocks(self, seeds: torch.Tensor, fanouts, sample: SampleBuffers, out: BlockBuffers | None = None,
                     stream=None) -> BlockBuffers:
        fo = self._fanouts(fanouts)
        if out is None:
            out = BlockBuffers(sample)
        self._ok(self._L.lgp_build_blocks(self._h, seeds.data_ptr(), seeds.numel(), fo.ctypes.data, fo.size,
                                          C.byref(sample.c_struct), C.byref(out.c_struct), _stream_ptr(stream)))
        return out

    def gather_features(self, ids: torch.Tensor, n_dev: torch.Tensor | None = None, out: torch.Tensor | None = None,
                        stats: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
        n_max = ids.numel()
        if out is None:
            out = torch.empty((n_max, self.feat_dim), dtype=self.feat_torch_dtype, device=self.device)
        assert out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= n_max * self.feat_dim * self.elem_bytes
        self._ok(self._L.lgp_gather_features(self._h, ids.data_ptr(), n_max,
                                             None if n_dev is None else n_dev.data_ptr(), out.data_ptr(),
                                             None if stats is None else stats.data_ptr(), _stream_ptr(stream)))
        return out

    def gather_features_static(self, ids: torch.Tensor, n_dev: torch.Tensor | None, out: torch.Tensor,
                               stats: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        """gather_features through the library's fixed scratch block: allocates nothing, so `out` is required."""
        assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
        n_max = ids.numel()
        assert out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= n_max * self.feat_dim * self.elem_bytes
        self._ok(self._L.lgp_gather_features_static(self._h, ids.data_ptr(), n_max,
                                                    None if n_dev is None else n_dev.data_ptr(), out.data_ptr(),
                                                    None if stats is None else stats.data_ptr(), _stream_ptr(stream)))
        return out

    def gather_features_clique(self, member: int, ids: torch.Tensor, n_dev: torch.Tensor | None = None,
                               out: torch.Tensor | None = None, stats: torch.Tensor | None = None,
                               stream=None) -> torch.Tensor:
        """gather_features as clique member `member`; stats (int32[3]) = {n_local, n_miss, n_peer}."""
        assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
        n_max = ids.numel()
        if out is None:
            out = torch.empty((n_max, self.feat_dim), dtype=self.feat_torch_dtype, device=self.device)
        assert out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() >= n_max * self.feat_dim * self.elem_bytes
        assert stats is None or (stats.is_cuda and stats.dtype == torch.int32 and stats.numel() >= 3)
        self._ok(self._L.lgp_gather_features_clique(self._h, member, ids.data_ptr(), n_max,
                                                    None if n_dev is None else n_dev.data_ptr(), out.data_ptr(),
                                                    None if stats is None else stats.data_ptr(), _stream_ptr(stream)))
        return out

    def workspace_bytes(self, max_seeds: int, fanouts):
        """(fixed, scratch) bytes of HBM the library holds / will allocate for batches of this shape (caches excluded)."""
        fo = self._fanouts(fanouts)
        fixed, scratch = C.c_size_t(), C.c_size_t()
        self._ok(self._L.lgp_workspace_bytes(self._h, int(max_seeds), fo.ctypes.data, fo.size, C.byref(fixed),
                                             C.byref(scratch)))
        return fixed.value, scratch.value

    def check(self, stream=None):
        self._ok(self._L.lgp_check(self._h, _stream_ptr(stream)))

    def set_overlap(self, enable: bool):
        self._ok(self._L.lgp_set_overlap(self._h, int(bool(enable))))

    def set_profiling(self, mode):
        """False / 0 = off, True / 1 = every kernel group, 2 = the two row gathers only."""
        self._ok(self._L.lgp_set_profiling(self._h, int(mode)))

    def get_profile(self) -> Profile:
        p = Profile()
        self._ok(self._L.lgp_get_profile(self._h, C.byref(p)))
        return p


def concurrent_streams(n: int):
    """n torch streams whose work runs side by side.  A process owns a handful of hardware queues, two streams that
    land on the same one serialise, and the API does not say which do: so candidates are tried pairwise with a
    spin kernel per stream (two spins take the time of one only when the streams are concurrent).  Returns
    (streams, found): found is False when fewer than n mutually concurrent streams turned up among the
    candidates; the list is then filled up with streams that share a queue with another one."""
    cur = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    spin = 2_000_000      # about a millisecond

    def both(a, b) -> float:
        torch.cuda.synchronize()
        e0.record()
        for st in (a, b):
            st.wait_stream(cur)
            with torch.cuda.stream(st):
                torch.cuda._sleep(spin)
        cur.wait_stream(a)
        cur.wait_stream(b)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    candidates = [torch.cuda.Stream() for _ in range(12)]
    both(candidates[0], candidates[0])
    alone = min(both(c, c) for c in candidates[:2]) / 2
    chosen = [candidates[0]]
    for c in candidates[1:]:
        if len(chosen) == n:
            break
        if all(both(c, k) < 1.5 * alone for k in chosen):
            chosen.append(c)
    concurrent = len(chosen) == n
    chosen += [c for c in candidates if c not in chosen][:n - len(chosen)]
    return chosen, concurrent
