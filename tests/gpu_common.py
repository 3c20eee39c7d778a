"""Helpers for the GPU parity tests: build a workload once, hold both sides."""
from __future__ import annotations

import numpy as np
import torch

import datagen
import oracle
import paper_2305_16588_amd as lgp


class Workload:
    def __init__(self, spec, device_gen: str = "cpu", with_features: bool = True, features_on_device: bool = False):
        """features_on_device: keep the source feature table in HBM instead of pinned CPU memory (the
        library accepts a device pointer in its place).  Used when the table does not fit under the box's
        pinned-memory limit; the oracle still reads a host copy of the same bytes."""
        self.spec = spec
        idt = np.int64 if spec.index64 else np.int32
        self.indptr = lgp.pinned_empty(spec.num_vertices + 1, idt)
        _, self.indices = datagen.make_graph(spec, device=device_gen, indptr_out=self.indptr,
                                             indices_alloc=lambda n: lgp.pinned_empty(n, np.int32))
        self.features = None
        if with_features:
            npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
            if features_on_device:
                self.features = np.empty((spec.num_vertices, spec.feat_dim), npdt)
            else:
                self.features = lgp.pinned_empty((spec.num_vertices, spec.feat_dim), npdt)
            datagen.make_features(spec, device=device_gen, out=self.features)
        self.tablet = datagen.make_tablet(spec, device=device_gen)
        self.tablet_dev = torch.from_numpy(self.tablet).cuda()
        self.features_dev = None
        if with_features and features_on_device:
            self.features_dev = torch.empty((spec.num_vertices, spec.feat_dim), device="cuda",
                                            dtype=torch.float32 if spec.feat_dtype == "float32" else torch.float16)
            step = 1 << 22
            for lo in range(0, spec.num_vertices, step):
                self.features_dev[lo:lo + step].copy_(torch.from_numpy(self.features[lo:lo + step]))
        self.ctx = lgp.Context(self.indptr, self.indices,
                               self.features_dev if self.features_dev is not None else self.features)
        self.orc = oracle.Oracle(self.indptr, self.indices, self.features)
        self.V = spec.num_vertices
        self.E = int(self.indices.size)

    def batch(self, b: int):
        lo = b * self.spec.batch
        return self.tablet[lo:lo + self.spec.batch], self.tablet_dev[lo:lo + self.spec.batch]


def assert_batch_equal(ref: "oracle.Batch", got, tag=""):
    fr, nbr, cnt, gids = got
    for h in range(len(ref.nbr)):
        assert fr[h].shape == ref.frontier[h].shape and (fr[h] == ref.frontier[h]).all(), f"{tag} frontier[{h}]"
        assert nbr[h].shape == ref.nbr[h].shape and (nbr[h] == ref.nbr[h]).all(), f"{tag} nbr[{h}]"
        assert (cnt[h] == ref.cnt[h]).all(), f"{tag} cnt[{h}]"
    if len(fr) == len(ref.frontier):                       # the last frontier was asked for
        assert fr[-1].shape == ref.frontier[-1].shape and (fr[-1] == ref.frontier[-1]).all(), f"{tag} last frontier"
    assert gids.shape == ref.gather_ids.shape and (gids == ref.gather_ids).all(), f"{tag} gather_ids"


def assert_blocks_equal(ref: "oracle.Batch", got, tag=""):
    indptr, src, rows = got
    for h in range(len(ref.blk_indptr)):
        assert indptr[h].shape == ref.blk_indptr[h].shape and (indptr[h] == ref.blk_indptr[h]).all(), f"{tag} indptr[{h}]"
        assert src[h].shape == ref.blk_src[h].shape and (src[h] == ref.blk_src[h]).all(), f"{tag} blk_src[{h}]"
    for h in range(len(ref.feat_row)):
        assert rows[h].shape == ref.feat_row[h].shape and (rows[h] == ref.feat_row[h]).all(), f"{tag} feat_row[{h}]"
