"""Helpers for the GPU parity tests: build a workload once, hold both sides."""
from __future__ import annotations

import numpy as np
import torch

import datagen
import oracle
import paper_2305_16588_amd as lgp


class Workload:
    def __init__(self, spec, device_gen: str = "cpu", with_features: bool = True, indptr_dtype=None):
        self.spec = spec
        indptr, indices = datagen.make_graph(spec, device=device_gen)
        if indptr_dtype is not None:
            indptr = indptr.astype(indptr_dtype)
        self.indptr = lgp.pinned_copy(indptr)
        self.indices = lgp.pinned_copy(indices)
        self.features = None
        if with_features:
            npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
            self.features = lgp.pinned_empty((spec.num_vertices, spec.feat_dim), npdt)
            datagen.make_features(spec, device=device_gen, out=self.features)
        self.tablet = datagen.make_tablet(spec)
        self.tablet_dev = torch.from_numpy(self.tablet).cuda()
        self.ctx = lgp.Context(self.indptr, self.indices, self.features)
        self.orc = oracle.Oracle(self.indptr, self.indices, self.features)
        self.V = spec.num_vertices
        self.E = int(indices.size)

    def batch(self, b: int):
        lo = b * self.spec.batch
        return self.tablet[lo:lo + self.spec.batch], self.tablet_dev[lo:lo + self.spec.batch]


def assert_batch_equal(ref: "oracle.Batch", got, tag=""):
    fr, nbr, cnt, gids = got
    for h in range(len(ref.nbr)):
        assert fr[h].shape == ref.frontier[h].shape and (fr[h] == ref.frontier[h]).all(), f"{tag} frontier[{h}]"
        assert nbr[h].shape == ref.nbr[h].shape and (nbr[h] == ref.nbr[h]).all(), f"{tag} nbr[{h}]"
        assert (cnt[h] == ref.cnt[h]).all(), f"{tag} cnt[{h}]"
    assert gids.shape == ref.gather_ids.shape and (gids == ref.gather_ids).all(), f"{tag} gather_ids"
