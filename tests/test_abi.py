"""The C-ABI library loads and exports every entry point the header declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "legion_prep.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lgp_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2305_16588_amd as lgp
    names = declared_functions()
    assert {"lgp_build_hotness", "lgp_build_cache", "lgp_sample_khop", "lgp_gather_features"} <= set(names)
    lib = lgp.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(lgp.binding.EXPORTS) == names            # the binding covers the whole header
    raw = ctypes.CDLL(os.path.join(ROOT, "paper_2305_16588_amd", "liblegion_prep.so"))
    raw.lgp_strerror.restype = ctypes.c_char_p
    assert raw.lgp_strerror(0) == b"ok" and b"worst case" in raw.lgp_strerror(-3)


def test_struct_layouts_match_the_header():
    import paper_2305_16588_amd as lgp
    b = lgp.binding
    assert ctypes.sizeof(b._Graph) == 56 and ctypes.sizeof(b.CachePlan) == 40 and ctypes.sizeof(b.Profile) == 64
    assert ctypes.sizeof(b._SampleOut) == 4 * 8 * b.MAX_HOPS + 2 * 8 + 4 * 8
    assert ctypes.sizeof(b._BlocksOut) == 3 * 8 * b.MAX_HOPS + 8
    hdr = open(os.path.join(ROOT, "include", "legion_prep.h")).read()
    assert f"#define LGP_MAX_HOPS {b.MAX_HOPS}" in hdr and f"#define LGP_MAX_FANOUT {b.MAX_FANOUT}" in hdr


def test_null_arguments_are_rejected_without_a_gpu():
    import paper_2305_16588_amd as lgp
    lib = lgp.load_library()
    assert lib.lgp_create(None, 0, None) == -1
    assert lib.lgp_destroy(None) == 0
    assert lib.lgp_sample_khop(None, None, 0, None, 0, 0, None, None) == -1
    assert lib.lgp_gather_features(None, None, 0, None, None, None, None) == -1
    assert lib.lgp_host_free(None) == 0
    assert lib.lgp_build_clique_cache(None, 2, None, None, 0, 0, None) == -1
    assert lib.lgp_get_clique_plan(None, 0, None) == -1
    assert lib.lgp_gather_features_clique(None, 0, None, 0, None, None, None, None) == -1
    assert lib.lgp_build_blocks(None, None, 0, None, 0, None, None, None) == -1
    assert lib.lgp_workspace_bytes(None, 1, None, 1, None, None) == -1


def test_worst_case_sizes():
    import paper_2305_16588_amd as lgp
    need, g = lgp.worst_case_sizes(2_400_000, 8192, (15, 10, 5))
    assert need == [8192, 122_880, 1_228_800, 2_400_000] and g == 2_400_000
    need, g = lgp.worst_case_sizes(10_000, 1024, (10, 5))
    assert need == [1024, 10_000, 10_000] and g == 10_000


def test_calls_fail_cleanly_when_no_gpu_is_present():
    """On a machine without a GPU every entry point that needs one returns an error code; nothing crashes
    and nothing falls back to the CPU."""
    import numpy as np
    import torch
    import paper_2305_16588_amd as lgp
    if torch.cuda.is_available():
        import pytest
        pytest.skip("a GPU is present")
    lib = lgp.load_library()
    b = lgp.binding
    indptr = np.array([0, 1, 2], dtype=np.int32)
    indices = np.array([1, 0], dtype=np.int32)
    g = b._Graph()
    g.num_vertices, g.num_edges = 2, 2
    g.indptr, g.indptr_bytes, g.indices = indptr.ctypes.data, 4, indices.ctypes.data
    h = ctypes.c_void_p()
    assert lib.lgp_create(ctypes.byref(g), 0, ctypes.byref(h)) < 0 and not h.value
    p = ctypes.c_void_p(123)
    assert lib.lgp_host_alloc(1024, ctypes.byref(p)) == -6 and not p.value
    offs = (ctypes.c_int64 * 2)()
    dummy = ctypes.c_void_p(8)
    assert lib.lgp_cslp(0, 1, 2, dummy, dummy, dummy, dummy, dummy, ctypes.addressof(offs), None) == -1
    assert lib.lgp_shuffle_tablet(0, dummy, dummy, 2, 1, 0, None) == -1
    g.indptr_bytes = 3
    assert lib.lgp_create(ctypes.byref(g), 0, ctypes.byref(h)) == -1          # bad offset width
    g.indptr_bytes, g.num_vertices = 4, 2**31
    assert lib.lgp_create(ctypes.byref(g), 0, ctypes.byref(h)) == -4          # too many vertices for int32 ids
    with __import__("pytest").raises(lgp.LegionPrepError):
        lgp.pinned_empty(16, np.int32)
