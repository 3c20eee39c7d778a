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


def test_worst_case_sizes():
    import paper_2305_16588_amd as lgp
    need, g = lgp.worst_case_sizes(2_400_000, 8192, (15, 10, 5))
    assert need == [8192, 122_880, 1_228_800, 2_400_000] and g == 2_400_000
    need, g = lgp.worst_case_sizes(10_000, 1024, (10, 5))
    assert need == [1024, 10_000, 10_000] and g == 10_000
