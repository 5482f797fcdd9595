"""CPU-side checks of the C-ABI library: it loads, exports every function that
include/gns.h declares, and its host-only entry points (workspace sizing,
capacities, argument validation) behave as documented.  No GPU work here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2106_06150_amd", "libgns.so")
HEADER = os.path.join(ROOT, "include", "gns.h")

if not os.path.exists(LIB):
    pytest.skip("libgns.so not built (run __graft_entry__.build())", allow_module_level=True)

from paper_2106_06150_amd import binding as B  # noqa: E402


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gns_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported():
    names = declared_functions()
    assert len(names) == 26, names
    lib = ctypes.CDLL(LIB)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTED) == names


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(B.gns_graph) == 64
    assert ctypes.sizeof(B.gns_config) == 4 + 32 + 32 + 4 + 8 + 4 + 4 + 4 + 4
    assert ctypes.sizeof(B.gns_block) == 72


def _graph(n=1000, nnz=5000, i64=0, feat=16):
    g = B.gns_graph()
    g.num_nodes, g.num_entries = n, nnz
    g.indptr, g.indices = 0x1000, 0x2000          # never dereferenced by the host-only calls
    g.indptr_is_i64 = i64
    g.feat_dim = feat
    g.feat_dev = 0x3000
    return g


def test_block_capacity_is_the_worst_case_growth():
    g = _graph(n=10_000_000, nnz=400_000_000, i64=1)
    c = B.make_config((15, 10, 5), (0, 0, 1), 50_000, 2048)
    assert B.gns_block_capacity(g, c, 0) == (2048, 2048 * 16, 2048 * 15)
    assert B.gns_block_capacity(g, c, 1) == (32768, 32768 * 11, 327680)
    assert B.gns_block_capacity(g, c, 2) == (360448, 360448 * 6, 1802240)
    small = _graph(n=300, nnz=900)
    c2 = B.make_config((10, 5), (0, 1), 30, 256)
    assert B.gns_block_capacity(small, c2, 0) == (256, 300, 2560)      # src clipped to n
    assert B.gns_block_capacity(small, c2, 1) == (300, 300, 1500)
    with pytest.raises(B.GnsError):
        B.gns_block_capacity(small, c2, 2)


def test_workspace_bytes_scale_and_validation():
    g = _graph()
    c = B.make_config((10, 5), (0, 1), 10, 256)
    w = B.gns_workspace_bytes(g, c)
    assert w > 0 and w % 256 == 0
    big = B.make_config((10, 5), (0, 1), 10, 1024)
    assert B.gns_workspace_bytes(g, big) > w
    for bad in [B.make_config((), (), 10, 256), B.make_config((0,), (0,), 0, 256), B.make_config((65,), (0,), 0, 256),
                B.make_config((5,), (7,), 0, 256), B.make_config((5,), (1,), 0, 256),
                B.make_config((5,), (1,), 2000, 256), B.make_config((5,), (0,), 0, 0)]:
        with pytest.raises(B.GnsError) as e:
            B.gns_workspace_bytes(g, bad)
        assert e.value.status == B.GNS_EINVAL
    too_many = _graph(n=1000, nnz=2 ** 31, i64=0)
    with pytest.raises(B.GnsError):
        B.gns_workspace_bytes(too_many, c)
    no_store = _graph()
    no_store.feat_dev = None
    with pytest.raises(B.GnsError):
        B.gns_workspace_bytes(no_store, c)


def test_null_context_calls_return_einval():
    lib = B.lib
    assert lib.gns_sample_cache(None, 1, 0, None) == B.GNS_EINVAL
    assert lib.gns_sample_blocks(None, 1, None, 1, None, None) == B.GNS_EINVAL
    assert lib.gns_gather_features(None, None, 0, None, None) == B.GNS_EINVAL
    assert lib.gns_aggregate(None, None, None, 1, None, None) == B.GNS_EINVAL
    assert lib.gns_cache_view(None, None, None, None, None) == B.GNS_EINVAL
    assert lib.gns_destroy(None) == B.GNS_OK
    assert lib.gns_profile_begin(None, 1, 4) == B.GNS_EINVAL
    assert isinstance(lib.gns_last_error(None), bytes)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2106_06150_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".hpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
