"""The synthetic-input recipe: sizes, skew, structure (simple graph, sorted rows)."""
import numpy as np

import datagen


def test_tiny_graph_shape_and_structure():
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    assert indptr.dtype == np.int32 and indices.dtype == np.int32 and indptr.size == spec.num_vertices + 1
    E = indices.size
    assert abs(E - spec.num_edges) / spec.num_edges < 0.05
    deg = np.diff(indptr)
    assert (deg == 0).any() and (deg > max(spec.fanouts)).any()      # both sampler branches are exercised
    assert indices.min() >= 0 and indices.max() < spec.num_vertices
    src = np.repeat(np.arange(spec.num_vertices), deg)
    assert (src != indices).all()                                    # no self-loops
    key = src.astype(np.int64) << 32 | indices
    assert (np.diff(key) > 0).all()                                  # rows sorted, no duplicate edges
    a, b = datagen.make_graph(spec)
    assert (a == indptr).all() and (b == indices).all()              # reproducible


def test_degree_skew():
    spec = datagen.scaled(datagen.MID, 0.05)
    indptr, indices = datagen.make_graph(spec)
    deg = np.sort(np.diff(indptr))[::-1].astype(float)
    assert abs(indices.size - spec.num_edges) / spec.num_edges < 0.05
    # CCDF slope past the structural cut-off (ranks >> i0) should be near gamma - 1
    V = deg.size
    i1, i2 = int(V * 0.02), int(V * 0.5)
    slope = -(np.log(i2 / V) - np.log(i1 / V)) / (np.log(deg[i2]) - np.log(deg[i1]))
    assert abs(slope - (spec.gamma - 1)) < 0.15
    indeg = np.bincount(indices, minlength=V)
    assert indeg.max() > 50 * indeg.mean()                           # in-degree (= access hotness) is skewed too


def test_features_and_tablet():
    spec = datagen.TINY
    x = datagen.make_features(spec)
    assert x.shape == (10_000, 128) and x.dtype == np.float32
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1) < 0.01
    t = datagen.make_tablet(spec)
    assert t.dtype == np.int32 and sorted(t.tolist()) == list(range(10_000))
    w = datagen.scaled(datagen.WIDE, 1e-4)
    assert datagen.make_features(w).dtype == np.float16
    topo_b, feat_b = datagen.budgets(spec, 196_222)
    assert feat_b == 2000 * 512 and topo_b == int(0.2 * (4 * 196_222 + 80_000))
