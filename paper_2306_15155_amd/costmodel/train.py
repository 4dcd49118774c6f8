"""Fits the learned per-primitive cost models and writes the tables the library embeds.

    python -m paper_2306_15155_amd.costmodel.train [--csv profiles_mi355x.csv] [--holdout]

Two gradient-boosted regression-tree ensembles (squared loss, written here from the textbook algorithm: each tree
is fitted to the residuals of the ensemble so far, splits chosen greedily by variance reduction).  The target is the
log2 of the time per unit of first-order work (milliseconds per gathered float for SpMM, per multiply-add for GEMM):
trees are piecewise constant, and a constant rate between two grid points is a far better guess than a constant time:
    SpMM : log2 of rows, columns, stored entries, mean entries per row, density, width, largest row over mean row,
           second moment of the row lengths over the squared mean (two cheap measures of skew); flavour one-hot
    GEMM : log2 of n, k, m
The predicted time of a composition is the sum of its primitives' predictions plus the library's closed-form terms
for the streaming passes (Section 3.4: the cost of an association tree is the sum of the costs of its primitives).
"""
from __future__ import annotations

import argparse
import csv
import math
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
FLAVOURS = ("pattern", "weighted", "scaled", "softmax")
N_TREES, DEPTH, RATE, MIN_LEAF = 120, 4, 0.1, 4


def spmm_features(n_rows, n_cols, nnz, max_deg, sum_sq_deg, width, flavour):
    """Must match spmm_features() in csrc/api.hip, entry by entry."""
    nnz = max(float(nnz), 1.0)
    mean = nnz / max(n_rows, 1)
    f = [math.log2(max(n_rows, 1)), math.log2(max(n_cols, 1)), math.log2(nnz), math.log2(mean),
         math.log2(nnz / (max(n_rows, 1) * max(n_cols, 1))), math.log2(max(width, 1)),
         math.log2(max(float(max_deg), 1.0) / mean),                               # how far the largest row stands out
         math.log2(max(float(sum_sq_deg), 1.0) / max(n_rows, 1) / (mean * mean))]   # second moment of the row lengths over mean^2
    return f + [1.0 if flavour == name else 0.0 for name in FLAVOURS]


def spmm_work(nnz, width):
    return math.log2(max(float(nnz), 1.0) * max(width, 1))


def gemm_work(n, k, m):
    return math.log2(max(float(n), 1.0) * max(k, 1) * max(m, 1))


def gemm_features(n, k, m):
    return [math.log2(max(n, 1)), math.log2(max(k, 1)), math.log2(max(m, 1))]


# ------------------------------------------------------------------ gradient-boosted regression trees

def _best_split(X, r, idx):
    """Greedy split of the samples idx on residuals r: (gain, feature, threshold) maximising the variance reduction."""
    best = (0.0, -1, 0.0)
    n = idx.size
    tot = r[idx].sum()
    for f in range(X.shape[1]):
        order = idx[np.argsort(X[idx, f], kind="stable")]
        xs, rs = X[order, f], r[order]
        left = np.cumsum(rs)[:-1]
        cnt = np.arange(1, n)
        ok = (xs[1:] > xs[:-1]) & (cnt >= MIN_LEAF) & (n - cnt >= MIN_LEAF)
        if not ok.any():
            continue
        gain = left ** 2 / cnt + (tot - left) ** 2 / (n - cnt) - tot ** 2 / n
        gain = np.where(ok, gain, -1.0)
        k = int(np.argmax(gain))
        if gain[k] > best[0]:
            best = (float(gain[k]), f, float(0.5 * (xs[k] + xs[k + 1])))
    return best


def _grow(X, r, idx, depth, nodes):
    """Appends the subtree for idx to nodes -> index of its root.  Node: [feature (-1 = leaf), threshold, left, right, value]."""
    me = len(nodes)
    nodes.append([-1, 0.0, -1, -1, float(r[idx].mean()) * RATE])
    if depth == 0 or idx.size < 2 * MIN_LEAF:
        return me
    gain, f, thr = _best_split(X, r, idx)
    if f < 0 or gain <= 1e-12:
        return me
    go_left = X[idx, f] <= thr
    nodes[me][0], nodes[me][1] = f, thr
    nodes[me][2] = _grow(X, r, idx[go_left], depth - 1, nodes)
    nodes[me][3] = _grow(X, r, idx[~go_left], depth - 1, nodes)
    return me


def _predict_tree(nodes, root, X):
    out = np.empty(X.shape[0])
    for i in range(X.shape[0]):
        k = root
        while nodes[k][0] >= 0:
            k = nodes[k][2] if X[i, nodes[k][0]] <= nodes[k][1] else nodes[k][3]
        out[i] = nodes[k][4]
    return out


class Gbt:
    def __init__(self):
        self.base, self.nodes, self.roots = 0.0, [], []

    def fit(self, X, y):
        X, y = np.asarray(X, dtype=np.float64), np.asarray(y, dtype=np.float64)
        self.base = float(y.mean())
        pred = np.full(y.shape, self.base)
        idx = np.arange(y.size)
        for _ in range(N_TREES):
            root = _grow(X, y - pred, idx, DEPTH, self.nodes)
            self.roots.append(root)
            pred += _predict_tree(self.nodes, root, X)
        return self

    def predict(self, X):
        X = np.asarray(X, dtype=np.float64)
        out = np.full(X.shape[0], self.base)
        for root in self.roots:
            out += _predict_tree(self.nodes, root, X)
        return out


# ------------------------------------------------------------------ data

def load(path):
    spmm_x, spmm_y, gemm_x, gemm_y, layers, graph_of = [], [], [], [], [], []
    for row in csv.DictReader(open(path)):
        key = (row["family"], int(row["n_rows"]), int(row["nnz"]))
        ms = float(row["ms"])
        if row["rec"] == "spmm":
            spmm_x.append(spmm_features(int(row["n_rows"]), int(row["n_cols"]), int(row["nnz"]), int(row["max_deg"]), int(row["sum_sq_deg"]),
                                        int(row["width"]), row["flavour"]))
            spmm_y.append(math.log2(max(ms, 1e-4)) - spmm_work(int(row["nnz"]), int(row["width"])))
            graph_of.append(("spmm", key))
        elif row["rec"] == "gemm":
            gemm_x.append(gemm_features(int(row["n_rows"]), int(row["gemm_k"]), int(row["width"])))
            gemm_y.append(math.log2(max(ms, 1e-4)) - gemm_work(int(row["n_rows"]), int(row["gemm_k"]), int(row["width"])))
            graph_of.append(("gemm", key))
        else:
            layers.append(dict(key=key, kind=int(row["kind"]), comp=int(row["comp"]), f_in=int(row["f_in"]), f_out=int(row["f_out"]),
                               n_rows=int(row["n_rows"]), n_cols=int(row["n_cols"]), nnz=int(row["nnz"]), max_deg=int(row["max_deg"]),
                               sum_sq_deg=int(row["sum_sq_deg"]), ms=ms))
    keys = {"spmm": [k for t, k in graph_of if t == "spmm"], "gemm": [k for t, k in graph_of if t == "gemm"]}
    return np.array(spmm_x), np.array(spmm_y), np.array(gemm_x), np.array(gemm_y), layers, keys


def emit(models, path):
    """The ensembles as C++ tables: per model a flat node array (feature, threshold, left, right, value) and its tree roots."""
    with open(path, "w") as f:
        f.write("// Generated by paper_2306_15155_amd/costmodel/train.py from costmodel/profiles_mi355x.csv: gradient-boosted regression\n"
                "// trees predicting log2(milliseconds per unit of work) of a primitive on MI355X (SpMM: per gathered float, nnz * width;\n"
                "// GEMM: per multiply-add, n * k * m).  Do not edit by hand.\n")
        for name, m in models.items():
            f.write("static const GbtNode k%sNodes[] = {\n" % name)
            for feat, thr, left, right, val in m.nodes:
                f.write("    {%d, %d, %d, (float)%.9g, (float)%.9g},\n" % (feat, left, right, thr, val))
            f.write("};\nstatic const int k%sRoots[] = {%s};\n" % (name, ", ".join(str(r) for r in m.roots)))
            f.write("static const float k%sBase = (float)%.9g;\n" % (name, m.base))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--csv", default=os.path.join(HERE, "profiles_mi355x.csv"))
    ap.add_argument("--out", default=os.path.join(os.path.dirname(HERE), "csrc", "learned_model.inc"))
    ap.add_argument("--holdout", action="store_true", help="also fit on four fifths of the graphs and report the error on the rest")
    args = ap.parse_args()
    sx, sy, gx, gy, layers, keys = load(args.csv)
    print("samples: spmm %d, gemm %d, layers %d" % (sy.size, gy.size, len(layers)))
    if args.holdout:
        graphs = sorted(set(keys["spmm"]))
        test = set(graphs[2::5])
        for name, X, y, ks in (("spmm", sx, sy, keys["spmm"]), ("gemm", gx, gy, keys["gemm"])):
            mask = np.array([k in test for k in ks])
            m = Gbt().fit(X[~mask], y[~mask])
            err = np.abs(m.predict(X[mask]) - y[mask])
            print("%s hold-out (%d graphs, %d samples): median |log2 error| %.3f, 90th percentile %.3f -> x%.2f / x%.2f in time"
                  % (name, len(test), int(mask.sum()), np.median(err), np.percentile(err, 90), 2 ** np.median(err), 2 ** np.percentile(err, 90)))
    models = {"Spmm": Gbt().fit(sx, sy), "Gemm": Gbt().fit(gx, gy)}
    for name, X, y in (("Spmm", sx, sy), ("Gemm", gx, gy)):
        err = np.abs(models[name].predict(X) - y)
        print("%s fit: median |log2 error| %.3f, max %.3f, %d nodes" % (name, np.median(err), err.max(), len(models[name].nodes)))
    emit(models, args.out)
    print("wrote", args.out)


if __name__ == "__main__":
    main()
