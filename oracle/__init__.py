"""CPU oracle (test infrastructure): ctypes access to ``legion_oracle.cpp``.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package.  It shares nothing with the HIP library.
All arrays are numpy arrays in host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "legion_oracle.cpp")
_LIB = os.path.join(_HERE, "liblegion_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (plain -O2, no tuning flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


class _Graph(C.Structure):
    _fields_ = [("num_vertices", C.c_int64), ("indptr", C.c_void_p), ("indptr_bytes", C.c_int32),
                ("indices", C.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
        gp = C.POINTER(_Graph)
        L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_philox4x32_10.restype = None
        L.orc_draw64.argtypes = [u64, i64, i32, i32]
        L.orc_draw64.restype = u64
        L.orc_sample_row.argtypes = [gp, i64, i32, i32, u64, vp]
        L.orc_sample_row.restype = i32
        L.orc_sample_khop.argtypes = [gp, vp, i64, vp, i32, u64]
        L.orc_sample_khop.restype = vp
        for name in ("orc_batch_frontier", "orc_batch_nbr", "orc_batch_cnt"):
            getattr(L, name).argtypes = [vp, i32]
            getattr(L, name).restype = vp
        L.orc_batch_frontier_size.argtypes = [vp, i32]
        L.orc_batch_frontier_size.restype = i64
        L.orc_batch_gather_size.argtypes = [vp]
        L.orc_batch_gather_size.restype = i64
        L.orc_batch_gather_ids.argtypes = [vp]
        L.orc_batch_gather_ids.restype = vp
        L.orc_block_of_hop.argtypes = [vp, i32, i32, vp, vp]
        L.orc_block_of_hop.restype = None
        L.orc_feature_rows.argtypes = [vp, i32, vp]
        L.orc_feature_rows.restype = None
        L.orc_hop_order.argtypes = [vp, i64, vp, vp]
        L.orc_hop_order.restype = i64
        L.orc_batch_free.argtypes = [vp]
        L.orc_batch_free.restype = None
        L.orc_build_hotness.argtypes = [gp, vp, i64, i32, vp, i32, u64, i64, vp, vp]
        L.orc_build_hotness.restype = i64
        L.orc_rank_by_hotness.argtypes = [vp, i64, vp]
        L.orc_rank_by_hotness.restype = None
        L.orc_plan_topo.argtypes = [gp, vp, u64]
        L.orc_plan_topo.restype = i64
        L.orc_plan_feat.argtypes = [i64, i64, u64]
        L.orc_plan_feat.restype = i64
        L.orc_fill_topo.argtypes = [gp, vp, i64, vp, vp]
        L.orc_fill_topo.restype = i64
        L.orc_fill_feat.argtypes = [vp, i64, vp, i64, vp]
        L.orc_fill_feat.restype = None
        L.orc_gather.argtypes = [vp, i64, vp, i64, vp]
        L.orc_gather.restype = None
        L.orc_count_hits.argtypes = [vp, i64, vp, i64, i64]
        L.orc_count_hits.restype = i64
        L.orc_search_cache_plan.argtypes = [gp, vp, vp, vp, vp, i64, u64, u64, C.c_uint32, i32, vp]
        L.orc_search_cache_plan.restype = i32
        L.orc_shuffle_tablet.argtypes = [vp, vp, i64, u64, C.c_uint32]
        L.orc_shuffle_tablet.restype = None
        L.orc_cslp.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp]
        L.orc_cslp.restype = None
        L.orc_queue_prefix_topo.argtypes = [gp, vp, i64, u64]
        L.orc_queue_prefix_topo.restype = i64
        L.orc_queue_prefix_feat.argtypes = [i64, i64, u64]
        L.orc_queue_prefix_feat.restype = i64
        L.orc_count_three_way.argtypes = [vp, i64, vp, i32, vp]
        L.orc_count_three_way.restype = None
        _lib = L
    return _lib


PLAN_POINT = np.dtype([("m_topo", np.uint64), ("m_feat", np.uint64), ("n_topo", np.int64), ("n_feat", np.int64),
                       ("uncached_topo_hot", np.uint64), ("uncached_feat_hot", np.uint64)])


def _p(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _copy(ptr: int, n: int) -> np.ndarray:
    if n == 0:
        return np.empty(0, dtype=np.int32)
    return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_int32)), shape=(n,)).copy()


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _load().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def draw64(rng_seed: int, v: int, hop: int, slot: int) -> int:
    return int(_load().orc_draw64(rng_seed & (2**64 - 1), v, hop, slot))


def shuffle_tablet(train_ids: np.ndarray, seed: int, epoch: int) -> np.ndarray:
    """Batch generator: the tablet in the order of epoch `epoch`."""
    train_ids = np.ascontiguousarray(train_ids, dtype=np.int32)
    out = np.empty_like(train_ids)
    _load().orc_shuffle_tablet(_p(train_ids), _p(out), train_ids.size, seed & (2**64 - 1), epoch)
    return out


def cslp(hot: np.ndarray):
    """Algorithm 1 on a [k_g, V] hotness matrix -> (acc, order, owner, queues, offsets)."""
    hot = np.ascontiguousarray(hot, dtype=np.uint32)
    k_g, V = hot.shape
    acc = np.empty(V, dtype=np.uint64)
    order = np.empty(V, dtype=np.int32)
    owner = np.empty(V, dtype=np.int32)
    queues = np.empty(V, dtype=np.int32)
    offsets = np.empty(k_g + 1, dtype=np.int64)
    _load().orc_cslp(k_g, V, _p(hot), _p(acc), _p(order), _p(owner), _p(queues), _p(offsets))
    return acc, order, owner, queues, offsets


@dataclass
class Batch:
    """Result of sampling one mini-batch.  frontier[0] is the seed list; frontier has one more entry than
    nbr / cnt (the set reached by the last hop).  With blocks=True the graph constructor's output is filled in too."""
    frontier: list = field(default_factory=list)
    nbr: list = field(default_factory=list)       # nbr[h]: [len(frontier[h]), fanouts[h]] int32, -1 padded
    cnt: list = field(default_factory=list)
    gather_ids: np.ndarray = None
    blk_indptr: list = field(default_factory=list)   # per hop: int64[len(frontier[h]) + 1]
    blk_src: list = field(default_factory=list)      # per hop: int32[edges], positions inside frontier[h + 1]
    feat_row: list = field(default_factory=list)     # per frontier: positions inside gather_ids
    hop_order: np.ndarray = None                     # extraction order of the intra-batch pipeline
    hop_seg: np.ndarray = None                       # its groups: [seg[h], seg[h + 1]) = seeds (h = 0), hop h's new vertices


class Oracle:
    """Holds one CSR graph (int32 or int64 offsets, int32 column ids) and an
    optional feature table ([V, D] array of any 2- or 4-byte dtype)."""

    def __init__(self, indptr: np.ndarray, indices: np.ndarray, features: np.ndarray | None = None):
        assert indptr.dtype in (np.int32, np.int64) and indices.dtype == np.int32
        self.indptr = np.ascontiguousarray(indptr)
        self.indices = np.ascontiguousarray(indices)
        self.features = None if features is None else np.ascontiguousarray(features)
        self.V = int(indptr.shape[0] - 1)
        self._g = _Graph(self.V, _p(self.indptr), self.indptr.dtype.itemsize, _p(self.indices) if indices.size else None)
        self._L = _load()

    @property
    def row_bytes(self) -> int:
        return int(self.features.shape[1] * self.features.dtype.itemsize)

    def sample_row(self, v: int, hop: int, f: int, rng_seed: int):
        out = np.empty(f, dtype=np.int32)
        cnt = self._L.orc_sample_row(C.byref(self._g), v, hop, f, rng_seed & (2**64 - 1), _p(out))
        return out, int(cnt)

    def sample_khop(self, seeds: np.ndarray, fanouts, rng_seed: int, blocks: bool = False) -> Batch:
        seeds = np.ascontiguousarray(seeds, dtype=np.int32)
        fo = np.asarray(fanouts, dtype=np.int32)
        h = self._L.orc_sample_khop(C.byref(self._g), _p(seeds), seeds.size, _p(fo), fo.size, rng_seed & (2**64 - 1))
        try:
            b = Batch()
            for hop in range(fo.size):
                n = int(self._L.orc_batch_frontier_size(h, hop))
                b.frontier.append(_copy(self._L.orc_batch_frontier(h, hop), n))
                b.nbr.append(_copy(self._L.orc_batch_nbr(h, hop), n * int(fo[hop])).reshape(n, int(fo[hop])))
                b.cnt.append(_copy(self._L.orc_batch_cnt(h, hop), n))
            n_last = int(self._L.orc_batch_frontier_size(h, fo.size))
            b.frontier.append(_copy(self._L.orc_batch_frontier(h, fo.size), n_last))
            b.gather_ids = _copy(self._L.orc_batch_gather_ids(h), int(self._L.orc_batch_gather_size(h)))
            b.hop_seg = np.zeros(fo.size + 2, dtype=np.int64)
            total = int(self._L.orc_hop_order(h, self.V, None, _p(b.hop_seg)))
            b.hop_order = np.empty(total, dtype=np.int32)
            self._L.orc_hop_order(h, self.V, _p(b.hop_order) if total else None, _p(b.hop_seg))
            if blocks:
                for hop in range(fo.size):
                    n = b.frontier[hop].size
                    indptr = np.zeros(n + 1, dtype=np.int64)
                    src = np.empty(int(b.cnt[hop].sum()), dtype=np.int32)
                    self._L.orc_block_of_hop(h, hop, int(fo[hop]), _p(indptr), _p(src) if src.size else None)
                    b.blk_indptr.append(indptr)
                    b.blk_src.append(src)
                for hop in range(fo.size + 1):
                    rows = np.empty(b.frontier[hop].size, dtype=np.int32)
                    self._L.orc_feature_rows(h, hop, _p(rows) if rows.size else None)
                    b.feat_row.append(rows)
        finally:
            self._L.orc_batch_free(h)
        return b

    def build_hotness(self, train_ids: np.ndarray, batch: int, fanouts, base_seed: int, max_batches: int = -1):
        train_ids = np.ascontiguousarray(train_ids, dtype=np.int32)
        fo = np.asarray(fanouts, dtype=np.int32)
        topo = np.empty(self.V, dtype=np.uint32)
        feat = np.empty(self.V, dtype=np.uint32)
        nb = self._L.orc_build_hotness(C.byref(self._g), _p(train_ids), train_ids.size, batch, _p(fo), fo.size,
                                       base_seed & (2**64 - 1), max_batches, _p(topo), _p(feat))
        return topo, feat, int(nb)

    def rank_by_hotness(self, hot: np.ndarray) -> np.ndarray:
        hot = np.ascontiguousarray(hot, dtype=np.uint32)
        order = np.empty(self.V, dtype=np.int32)
        self._L.orc_rank_by_hotness(_p(hot), self.V, _p(order))
        return order

    def plan_topo(self, order: np.ndarray, topo_budget: int) -> int:
        return int(self._L.orc_plan_topo(C.byref(self._g), _p(order), int(topo_budget)))

    def plan_feat(self, feat_budget: int) -> int:
        return int(self._L.orc_plan_feat(self.V, self.row_bytes, int(feat_budget)))

    def fill_topo(self, order: np.ndarray, n: int):
        t_indptr = np.empty(n + 1, dtype=np.int64)
        total = int(self._L.orc_fill_topo(C.byref(self._g), _p(order), n, _p(t_indptr), None))
        t_indices = np.empty(total, dtype=np.int32)
        self._L.orc_fill_topo(C.byref(self._g), _p(order), n, _p(t_indptr), _p(t_indices) if total else None)
        return t_indptr, t_indices

    def fill_feat(self, order: np.ndarray, n: int) -> np.ndarray:
        cache = np.empty((n, self.features.shape[1]), dtype=self.features.dtype)
        self._L.orc_fill_feat(_p(self.features), self.row_bytes, _p(order), n, _p(cache) if n else None)
        return cache

    def gather(self, ids: np.ndarray) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        out = np.empty((ids.size, self.features.shape[1]), dtype=self.features.dtype)
        self._L.orc_gather(_p(self.features), self.row_bytes, _p(ids), ids.size, _p(out) if ids.size else None)
        return out

    def search_cache_plan(self, topo_hot, feat_hot, order_t, order_f, total_budget: int, n_tsum: int, cls: int = 64,
                          n_alpha: int = 101):
        """Returns (best_index, points): points is a structured array with one entry per candidate alpha."""
        topo_hot = np.ascontiguousarray(topo_hot, dtype=np.uint32)
        feat_hot = np.ascontiguousarray(feat_hot, dtype=np.uint32)
        points = np.zeros(n_alpha, dtype=PLAN_POINT)
        best = self._L.orc_search_cache_plan(C.byref(self._g), _p(topo_hot), _p(feat_hot), _p(order_t), _p(order_f),
                                             self.row_bytes, int(total_budget), int(n_tsum), cls, n_alpha, _p(points))
        return int(best), points

    def clique_plan(self, topo_hot: np.ndarray, feat_hot: np.ndarray, topo_budget: int, feat_budget: int):
        """Caches of a clique: topo_hot / feat_hot are [k_g, V] hotness matrices, the budgets are per GPU.
        Returns (topo_ids, feat_ids): per GPU, the vertex ids its caches hold, in fill order."""
        topo_ids, feat_ids = [], []
        _, _, _, queues, offsets = cslp(topo_hot)
        for g in range(offsets.size - 1):
            q = np.ascontiguousarray(queues[offsets[g]:offsets[g + 1]])
            n = int(self._L.orc_queue_prefix_topo(C.byref(self._g), _p(q), q.size, int(topo_budget))) if q.size else 0
            topo_ids.append(q[:n].copy())
        _, _, _, queues, offsets = cslp(feat_hot)
        for g in range(offsets.size - 1):
            q = queues[offsets[g]:offsets[g + 1]]
            n = int(self._L.orc_queue_prefix_feat(q.size, self.row_bytes, int(feat_budget)))
            feat_ids.append(q[:n].copy())
        return topo_ids, feat_ids

    def count_three_way(self, ids: np.ndarray, feat_ids: list, member: int):
        """(local hits, misses, peer hits) of an id list for GPU `member`, given every GPU's cached feature ids."""
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        cached_by = np.full(self.V, -1, dtype=np.int32)
        for g, f in enumerate(feat_ids):
            cached_by[f] = g
        counts = np.zeros(3, dtype=np.int64)
        self._L.orc_count_three_way(_p(ids), ids.size, _p(cached_by), member, _p(counts))
        return int(counts[0]), int(counts[1]), int(counts[2])

    def count_hits(self, ids: np.ndarray, order: np.ndarray, n_cached: int) -> int:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        return int(self._L.orc_count_hits(_p(ids), ids.size, _p(order), n_cached, self.V))
