"""The offline stage (matrix IR -> association trees -> pruning -> annotation) against the counts the paper prints
for its two case studies and against the embedding-size rules the library's selector applies."""
import importlib.util
import os
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load():
    # loaded by path: the module is pure Python and must not need the GPU binding of the package
    spec = importlib.util.spec_from_file_location("sensei_association", os.path.join(ROOT, "paper_2306_15155_amd", "association.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules["sensei_association"] = mod
    spec.loader.exec_module(mod)
    return mod


def _golden():
    path = os.path.join(ROOT, "tests", "golden", "paper_counts.txt")
    return {k: int(v) for k, v in (l.split() for l in open(path) if l.strip() and not l.startswith("#"))}


def test_gcn_forest_matches_the_counts_of_the_case_study():
    m, gold = _load(), _golden()
    trees = m.generate_trees(m.gcn_ir())
    assert len(trees) == gold["gcn_trees_generated"]
    assert len({t.text() for t in trees}) == len(trees)
    promoted, pruned = m.prune(trees)
    assert len(pruned) == gold["gcn_trees_pruned"] and len(promoted) == gold["gcn_trees_promoted"]
    sets = {}
    for t, scen in promoted:
        assert len(scen) == 1            # each promoted tree serves exactly one embedding-size scenario
        sets.setdefault(scen[0], []).append(t)
    assert len(sets) == gold["gcn_sets"] and all(len(v) == 2 for v in sets.values())
    # the two rules the paper spells out are in the forest: the SDDMM of D.A.D and the value-less SpMM
    assert any("(D1 A D2)" in t.text() and ("SDDMM", "nnz") in t.prims for t in trees)
    assert any(("SpMM_u", "in") in t.prims for t in trees) and any(("SpMM_u", "out") in t.prims for t in trees)
    # the original implementation (Eq. 3) is re-discovered, and pruned in favour of broadcasts at one width
    eq3 = [t for t in trees if t.text() == "(D1 ((A (D2 H)) W))"]
    assert len(eq3) == 1 and eq3[0] in pruned


def test_every_tree_is_a_full_valid_association():
    m = _load()
    for t in m.generate_trees(m.gcn_ir()):
        text = t.text()
        assert [w.strip("()") for w in text.split()] == ["D1", "A", "D2", "H", "W"]          # operand order is kept
        kinds = [k for k, _ in t.prims]
        assert kinds.count("GEMM") == 1 and sum(k.startswith("SpMM") for k in kinds) == 1   # one update, one aggregation
        assert (t.attr, t.rows, t.cols) == ("dense", "n", "out")


def test_promoted_trees_are_the_library_compositions_with_the_same_conditions():
    m = _load()
    table = m.composition_table("gcn")
    assert sorted(name for name, _, _ in table) == ["DYN_AGG", "DYN_UPD", "PRE_AGG", "PRE_UPD"]
    for name, _, scen in table:
        cid = oracle.GCN_COMPOSITIONS.index(name)
        # candidate for f_in < f_out / f_in > f_out exactly when the selector's rule filter keeps it
        assert ("in<out" in scen) == (cid in oracle.select_rules("gcn", 32, 64))
        assert ("in>out" in scen) == (cid in oracle.select_rules("gcn", 64, 32))


def test_gat_has_two_compositions_and_recomputation_only_pays_for_growing_sizes():
    m, gold = _load(), _golden()
    trees = m.gat_trees()
    assert len(trees) == gold["gat_compositions"]
    by = {name: (expr, scen) for name, expr, scen in m.composition_table("gat")}
    assert set(by) == {"REUSE", "RECOMP"}
    assert set(by["REUSE"][1]) == {"in<out", "in>out"} and set(by["RECOMP"][1]) == {"in<out"}
    recomp = [t for t in trees if t.text() == "((alpha H) W)"][0]
    assert [k for k, _ in recomp.prims].count("GEMM") == gold["gat_recompute_gemms"]
    for name, (_, scen) in by.items():
        cid = oracle.GAT_COMPOSITIONS.index(name)
        assert ("in<out" in scen) == (cid in oracle.select_rules("gat", 32, 64))
        assert ("in>out" in scen) == (cid in oracle.select_rules("gat", 64, 32))
