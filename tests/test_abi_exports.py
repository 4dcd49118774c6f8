"""The C-ABI library loads and exports every symbol the public header declares (no compute calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sensei.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sensei_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_named_entry_points():
    names = _declared()
    for must in ("sensei_gcn_layer", "sensei_gat_layer", "sensei_select"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2306_15155_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2306_15155_amd import build
        build.build()
    L = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_status_strings_and_names_need_no_gpu():
    from paper_2306_15155_amd import binding
    assert binding.status_string(0) == "ok"
    assert binding.status_string(3) == "workspace too small"
    assert binding.num_compositions(binding.KIND_GCN) == 6 and binding.num_compositions(binding.KIND_GAT) == 4
    assert [binding.composition_name(0, i) for i in range(6)] == list(binding.GCN_NAMES)
    assert [binding.composition_name(1, i) for i in range(4)] == list(binding.GAT_NAMES)


def test_host_only_queries_and_argument_checks_need_no_gpu():
    """Workspace queries are pure host arithmetic; a call with a null context is rejected before any HIP call."""
    import ctypes as C
    from paper_2306_15155_amd import binding
    L = binding.lib()
    A = binding.CsrStruct(1000, 1000, 50_000, 0x1000, 0x2000, None)  # pointers are never dereferenced by the queries
    n = C.c_size_t()
    sizes = {}
    for cid in range(6):
        assert L.sensei_gcn_workspace(C.byref(A), 64, 32, cid, C.byref(n)) == 0
        sizes[cid] = n.value
        assert n.value > 0 and n.value % 256 == 0
    assert sizes[0] == sizes[2] == sizes[4]         # aggregate-first ids: U plus one (possibly slice-major) copy of X
    assert L.sensei_gcn_workspace(C.byref(A), 64, 32, 6, C.byref(n)) == 2
    assert L.sensei_gcn_workspace(C.byref(A), 0, 32, 0, C.byref(n)) == 1
    assert L.sensei_gcn_workspace(None, 64, 32, 0, C.byref(n)) == 1
    for cid in range(4):
        assert L.sensei_gat_workspace(C.byref(A), 64, 32, cid, C.byref(n)) == 0 and n.value > 0
    assert L.sensei_gat_workspace(C.byref(A), 64, 32, 4, C.byref(n)) == 2
    assert L.sensei_sparse_workspace(C.byref(A), 128, C.byref(n)) == 0 and n.value > 0
    assert L.sensei_select_workspace(0, C.byref(A), 64, 32, C.byref(n)) == 0 and n.value > sizes[0]
    assert L.sensei_select_workspace(7, C.byref(A), 64, 32, C.byref(n)) == 1
    bad = binding.CsrStruct(-1, 10, 0, 0x1000, None, None)
    assert L.sensei_gcn_workspace(C.byref(bad), 64, 32, 0, C.byref(n)) == 1
    # null context: rejected on the host
    cid = C.c_int(-1)
    assert L.sensei_select(None, 0, C.byref(A), 64, 32, 0, C.byref(cid), None, None, 0, None) == 1
    assert L.sensei_degrees(None, C.byref(A), None, None, None) == 1
    assert L.sensei_profile_enable(None, 1) == 1
    assert L.sensei_destroy(None) == 0


def test_variant_layer_and_tile_queries_need_no_gpu():
    """Workspace and size queries of the variant layers and of the dense-tile split: host arithmetic and argument checks."""
    import ctypes as C
    from paper_2306_15155_amd import binding
    L = binding.lib()
    A = binding.CsrStruct(1000, 1000, 50_000, 0x1000, 0x2000, None)
    n = C.c_size_t()
    for cid in (0, 1):
        assert L.sensei_sgc_workspace(C.byref(A), 64, 32, cid, C.byref(n)) == 0 and n.value > 0
        assert L.sensei_tagcn_workspace(C.byref(A), 64, 32, 3, cid, C.byref(n)) == 0 and n.value > 0
        assert L.sensei_gatv2_workspace(C.byref(A), 64, 32, cid, C.byref(n)) == 0 and n.value > 0
    assert L.sensei_sgc_workspace(C.byref(A), 64, 32, 2, C.byref(n)) == 2
    assert L.sensei_tagcn_workspace(C.byref(A), 64, 32, 0, 0, C.byref(n)) == 1      # at least one hop
    assert L.sensei_tagcn_workspace(C.byref(A), 64, 32, 3, 5, C.byref(n)) == 2
    assert L.sensei_gatv2_workspace(C.byref(A), 0, 32, 0, C.byref(n)) == 1
    # more hops need more room only where the hops are kept side by side (aggregate first)
    L.sensei_tagcn_workspace(C.byref(A), 64, 32, 2, 0, C.byref(n)); two = n.value
    L.sensei_tagcn_workspace(C.byref(A), 64, 32, 4, 0, C.byref(n)); four = n.value
    assert four > two
    L.sensei_tagcn_workspace(C.byref(A), 64, 32, 2, 1, C.byref(n)); two = n.value
    L.sensei_tagcn_workspace(C.byref(A), 64, 32, 4, 1, C.byref(n)); four = n.value
    assert four == two
    assert L.sensei_tiles_bytes(C.byref(A), 0.09, 256, C.byref(n)) == 0 and n.value > 0 and n.value % 256 == 0
    small = n.value
    assert L.sensei_tiles_bytes(C.byref(A), 0.09, 512, C.byref(n)) == 0 and n.value > small   # wider operands, larger buffers
    assert L.sensei_tiles_bytes(C.byref(A), 0.0, 256, C.byref(n)) == 1
    assert L.sensei_tiles_bytes(C.byref(A), 1.5, 256, C.byref(n)) == 1
    assert L.sensei_tiles_bytes(C.byref(A), 0.09, 100, C.byref(n)) == 1                       # a multiple of 32
    assert L.sensei_tiles_info(None, None, None, None) == 1
    assert L.sensei_tiles_set_min_width(None, 64) == 1
    assert L.sensei_tiles_destroy(None) == 0
    out = C.c_void_p()
    assert L.sensei_tiles_create(None, C.byref(A), 0.09, 256, None, 0, None, C.byref(out)) == 1


def test_gat_backward_workspace_query_takes_both_patterns():
    """The query sees the pattern and its transpose as the layer call will (either may carry a dense-tile split); the transpose may
    be left out when it carries none.  Host arithmetic only."""
    import ctypes as C
    from paper_2306_15155_amd import binding
    L = binding.lib()
    A = binding.CsrStruct(1000, 1200, 50_000, 0x1000, 0x2000, None)
    At = binding.CsrStruct(1200, 1000, 50_000, 0x3000, 0x4000, None)
    n = C.c_size_t()
    assert L.sensei_gat_backward_workspace(C.byref(A), C.byref(At), 64, 32, C.byref(n)) == 0 and n.value > 0
    both = n.value
    assert L.sensei_gat_backward_workspace(C.byref(A), None, 64, 32, C.byref(n)) == 0 and n.value == both   # no split on either
    assert L.sensei_gat_backward_workspace(C.byref(A), C.byref(At), 64, 128, C.byref(n)) == 0 and n.value > both
    assert L.sensei_gat_backward_workspace(None, C.byref(At), 64, 32, C.byref(n)) == 1
    assert L.sensei_gat_backward_workspace(C.byref(A), C.byref(At), 0, 32, C.byref(n)) == 1
    assert L.sensei_gat_backward_workspace(C.byref(A), C.byref(At), 64, 32, None) == 1


def test_bench_refuses_more_than_one_gpu_before_touching_one():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout.strip() == ""
