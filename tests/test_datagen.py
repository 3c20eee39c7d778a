"""The synthetic-input recipe: sizes, skew, structure (simple graph, sorted rows), and that every array is a
pure function of (seed, index): the generator's known answers, independence of chunking, stored fingerprints."""
import importlib.util
import os

import numpy as np
import pytest
import torch

import datagen

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _fingerprint_tool():
    spec = importlib.util.spec_from_file_location("write_datagen_fingerprints",
                                                  os.path.join(GOLDEN, "write_datagen_fingerprints.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _stored():
    out = {}
    for line in open(os.path.join(GOLDEN, "datagen_fingerprints.txt")):
        if line.strip() and not line.startswith("#"):
            key, *fields = line.split()
            out[key] = dict(f.split("=") for f in fields)
    return out


def test_generator_known_answers():
    """datagen's own Philox4x32-10 against the generator's published vectors."""
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        ctr = [torch.tensor([x], dtype=torch.int64) for x in w[:4]]
        got = [int(x) for x in datagen.philox_rounds(*ctr, w[4], w[5])]
        assert got == w[6:]


def test_arrays_do_not_depend_on_chunking():
    spec = datagen.TINY
    a, b = datagen.make_graph(spec, chunk_edges=1 << 12), datagen.make_graph(spec)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
    assert (datagen.make_features(spec, chunk_rows=777) == datagen.make_features(spec)).all()


@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("mid", 0.05), ("wide", 0.002), ("large", 0.0002),
                                        ("share", 0.0001)])
def test_stored_fingerprints(name, scale):
    tool, want = _fingerprint_tool(), _stored()[f"small:{name}@{scale:g}"]
    spec = tool.small_spec(name, scale)
    indptr, indices = datagen.make_graph(spec)
    assert indices.size == int(want["E"]) and tool.digest(indptr, indices) == want["graph"]
    assert tool.digest(datagen.make_features(spec)) == want["features"]
    assert tool.digest(datagen.make_tablet(spec)) == want["tablet"]


@pytest.mark.gpu
@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("mid", 0.05), ("wide", 0.002), ("large", 0.0002),
                                        ("share", 0.0001)])
def test_gpu_generation_gives_the_same_arrays(name, scale):
    tool, want = _fingerprint_tool(), _stored()[f"small:{name}@{scale:g}"]
    spec = tool.small_spec(name, scale)
    indptr, indices = datagen.make_graph(spec, device="cuda")
    assert indices.size == int(want["E"]) and tool.digest(indptr, indices) == want["graph"]
    assert tool.digest(datagen.make_features(spec, device="cuda")) == want["features"]
    assert tool.digest(datagen.make_tablet(spec, device="cuda")) == want["tablet"]


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
    # standard normal shape beyond the first two moments: quantiles and the tails
    q = np.quantile(x.astype(np.float64).ravel(), [0.001, 0.0228, 0.1587, 0.5, 0.8413, 0.9772, 0.999])
    assert np.abs(q - np.array([-3.0902, -2.0, -1.0, 0.0, 1.0, 2.0, 3.0902])).max() < 0.02
