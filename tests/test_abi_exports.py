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
