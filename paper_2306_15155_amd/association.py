"""Offline stage of the method (Section 3.2-3.4 of the paper): from the matrix IR of a layer to its association trees,
the input-oblivious pruning, and the annotation of the promoted trees with the embedding-size scenario they serve.

The matrix IR after post-processing is one multi-operand multiplication whose leaves carry an attribute and a
sub-attribute (the paper's table of matrix attributes): ``dense data``, ``dense weight``, ``sparse weighted``,
``sparse unweighted``, ``sparse diagonal``.  A candidate association combines adjacent operands that one sparse or
dense primitive can evaluate; Algorithm 1 applies every candidate in turn and recurses until no candidate is left,
which enumerates every valid association tree.  The paper lists only two of its candidate rules; the set below is
the smallest one found that contains those two and reproduces the counts the paper states for its case studies
(GCN: 12 trees, 8 pruned, 4 promoted in 2 sets of 2; GAT: 2 compositions):

    diagonal . sparse . diagonal          -> sparse weighted   SDDMM (the diagonals become the dense vectors)
    diagonal . sparse unweighted          -> sparse weighted   SDDMM with one vector (row scaling of the pattern)
    sparse unweighted . diagonal          -> sparse weighted   SDDMM with one vector (column scaling)
    sparse unweighted . dense             -> dense             SpMM that ignores the values
    sparse weighted . dense               -> dense             SpMM
    diagonal . dense                      -> dense             row broadcast
    dense . dense weight                  -> dense             GEMM

Pruning (Section 3.3) compares primitive multisets under the two scenarios f_in < f_out and f_in > f_out: a tree is
unprofitable in a scenario if another tree uses a sub-multiset of its primitives on matrices that are nowhere larger,
or the same primitives on smaller matrices; trees unprofitable in both scenarios are dropped, the rest are promoted
and annotated with the scenario(s) in which they survive.

This module is host-side tooling around the library (it produces the composition table that ``sensei.h`` exposes as
ids); nothing on the GPU path imports it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

# ------------------------------------------------------------------ IR


@dataclass(frozen=True)
class Node:
    """A leaf matrix or an intermediate result; ``rows`` / ``cols`` are symbolic: 'n' (nodes), 'in', 'out'."""
    name: str
    attr: str            # 'dense' | 'sparse'
    sub: str             # 'data' | 'weight' | 'weighted' | 'unweighted' | 'diagonal'
    rows: str
    cols: str
    expr: str = ""       # fully parenthesised expression that produces it (leaves: the name)
    prims: Tuple[Tuple[str, str], ...] = ()  # primitives used so far: (primitive, symbolic size)

    def text(self) -> str:
        return self.expr or self.name


def leaf(name, attr, sub, rows, cols) -> Node:
    return Node(name, attr, sub, rows, cols, name, ())


def gcn_ir() -> List[Node]:
    """D~^-1/2 . A~ . D~^-1/2 . H . W after the row broadcasts became diagonal multiplications (Section 3.2)."""
    return [leaf("D1", "sparse", "diagonal", "n", "n"), leaf("A", "sparse", "unweighted", "n", "n"),
            leaf("D2", "sparse", "diagonal", "n", "n"), leaf("H", "dense", "data", "n", "in"), leaf("W", "dense", "weight", "in", "out")]


def gat_ir() -> List[Node]:
    """alpha . H . W: the attention matrix comes out of AttenCalc, which is opaque to re-association (Section 5.2)."""
    return [leaf("alpha", "sparse", "weighted", "n", "n"), leaf("H", "dense", "data", "n", "in"), leaf("W", "dense", "weight", "in", "out")]


# ------------------------------------------------------------------ candidate rules

def _combine(parts: List[Node], prim: str, size: str, attr: str, sub: str) -> Node:
    expr = "(" + " ".join(p.text() for p in parts) + ")"
    prims = tuple(sorted(sum((p.prims for p in parts), ()) + ((prim, size),)))
    return Node("I", attr, sub, parts[0].rows, parts[-1].cols, expr, prims)


def candidates(ir: List[Node]) -> List[Tuple[int, int, Node]]:
    """(first index, count, result) for every association of adjacent operands one primitive can evaluate."""
    out = []
    for i in range(len(ir)):
        a = ir[i]
        b: Optional[Node] = ir[i + 1] if i + 1 < len(ir) else None
        c: Optional[Node] = ir[i + 2] if i + 2 < len(ir) else None
        if b is None:
            continue
        diag = lambda x: x.attr == "sparse" and x.sub == "diagonal"          # noqa: E731
        sparse = lambda x: x.attr == "sparse" and x.sub != "diagonal"        # noqa: E731
        dense = lambda x: x.attr == "dense"                                  # noqa: E731
        if c is not None and diag(a) and sparse(b) and diag(c):
            out.append((i, 3, _combine([a, b, c], "SDDMM", "nnz", "sparse", "weighted")))
        if diag(a) and sparse(b) and b.sub == "unweighted":
            out.append((i, 2, _combine([a, b], "SDDMM", "nnz", "sparse", "weighted")))
        if sparse(a) and a.sub == "unweighted" and diag(b):
            out.append((i, 2, _combine([a, b], "SDDMM", "nnz", "sparse", "weighted")))
        if sparse(a) and dense(b):
            out.append((i, 2, _combine([a, b], "SpMM_u" if a.sub == "unweighted" else "SpMM_w", b.cols, "dense", "data")))
        if diag(a) and dense(b):
            out.append((i, 2, _combine([a, b], "RowBcast", b.cols, "dense", "data")))
        if dense(a) and dense(b) and b.sub == "weight":
            out.append((i, 2, _combine([a, b], "GEMM", "n*in*out", "dense", "data")))
    return out


def generate_trees(ir: List[Node]) -> List[Node]:
    """Algorithm 1: depth-first over the candidates; the forest holds one node per distinct association tree."""
    forest = {}

    def rec(cur: List[Node]):
        cands = candidates(cur)
        if not cands:
            if len(cur) == 1:
                forest.setdefault(cur[0].text(), cur[0])
            return
        for start, count, result in cands:
            rec(cur[:start] + [result] + cur[start + count:])

    rec(list(ir))
    return [forest[k] for k in sorted(forest)]


# ------------------------------------------------------------------ pruning and annotation

_ORDER = {"in<out": {"in": 0, "out": 1}, "in>out": {"in": 1, "out": 0}}


def _size_le(a: str, b: str, scenario: str) -> bool:
    """a <= b for two symbolic sizes of one primitive kind under the scenario."""
    if a == b:
        return True
    if a in ("in", "out") and b in ("in", "out"):
        return _ORDER[scenario][a] < _ORDER[scenario][b]
    return False


def _dominates(p: Node, q: Node, scenario: str) -> bool:
    """p makes q unprofitable: every primitive of p is matched by a distinct primitive of q of the same kind on a matrix
    that is at least as large, and q has a primitive more or a strictly larger matrix somewhere."""
    rest = list(q.prims)
    strictly = False
    for kind, size in p.prims:
        match = None
        for cand in rest:
            if cand[0] == kind and _size_le(size, cand[1], scenario):
                if match is None or _size_le(cand[1], match[1], scenario):
                    match = cand  # the tightest match leaves the larger ones for the other primitives
        if match is None:
            return False
        rest.remove(match)
        strictly = strictly or match[1] != size
    return strictly or bool(rest)


def prune(trees: List[Node]):
    """-> (promoted, pruned); promoted entries are (tree, scenarios in which no other tree dominates it)."""
    promoted, pruned = [], []
    for t in trees:
        alive = [s for s in ("in<out", "in>out") if not any(_dominates(o, t, s) for o in trees if o is not t)]
        (promoted if alive else pruned).append((t, alive))
    return promoted, [t for t, _ in pruned]


# ------------------------------------------------------------------ the library's composition ids

GCN_IDS = {
    "((D1 (A (D2 H))) W)": "DYN_AGG",
    "(D1 (A (D2 (H W))))": "DYN_UPD",
    "(((D1 A D2) H) W)": "PRE_AGG",
    "((D1 A D2) (H W))": "PRE_UPD",
}
GAT_IDS = {"(alpha (H W))": "REUSE", "((alpha H) W)": "RECOMP"}


def gat_trees() -> List[Node]:
    """Association trees of alpha . H . W plus what AttenCalc itself needs: Theta = H . W, one GEMM.  A tree that also
    forms (H W) shares it (the common-sub-expression pass of Section 3.3: reuse); a tree that does not pays for it on
    top of its own primitives (recomputation: two GEMMs)."""
    out = []
    for t in generate_trees(gat_ir()):
        if "(H W)" in t.text():
            out.append(t)
        else:
            out.append(Node(t.name, t.attr, t.sub, t.rows, t.cols, t.expr, tuple(sorted(t.prims + (("GEMM", "n*in*out"),)))))
    return out


def composition_table(kind: str):
    """The promoted trees of a layer with the name of the library composition that evaluates each and its annotation."""
    trees = generate_trees(gcn_ir()) if kind == "gcn" else gat_trees()
    promoted, _ = prune(trees)
    ids = GCN_IDS if kind == "gcn" else GAT_IDS
    return [(ids[t.text()], t.text(), tuple(scen)) for t, scen in promoted]
