"""Collects primitive timings on this GPU for the learned cost models.

    python -m paper_2306_15155_amd.costmodel.collect --out paper_2306_15155_amd/costmodel/profiles_mi355x.csv

For every graph of a grid of seeded synthetic graphs (uniform G(n, M) and skewed R-MAT, 2e4 .. 2e6 nodes, mean degree
4 .. 1024) and every pair of embedding sizes, each GCN and GAT composition is run through the C ABI with the
library's own timers on; what is written per run:
    spmm rows : graph features (rows, columns, stored entries, largest row, sum of squared row lengths), SpMM flavour,
                width, ms of the SpMM call inside the layer
    gemm rows : n, k, m, ms of each GEMM launch inside the layer
    layer rows: composition, sizes, ms of the whole layer (to check that the parts add up and to score selections)
"""
from __future__ import annotations

import argparse
import csv
import itertools
import sys
import time

FLAVOUR_GCN = {0: "pattern", 1: "pattern", 2: "scaled", 3: "pattern", 4: "weighted", 5: "weighted"}
WIDTH_PAIRS = [(32, 128), (128, 32), (64, 256), (256, 64), (128, 512), (512, 128), (100, 47), (602, 256), (256, 41), (128, 128)]


def graph_grid(quick: bool):
    """(family, n, mean degree): sizes bounded so that generating a graph on the host stays within seconds."""
    out = []
    for n in (20_000, 50_000, 100_000, 250_000, 500_000, 1_000_000, 2_000_000):
        for d in (4, 8, 16, 32, 64, 128, 256, 512, 1024):
            if d < n // 8 and n * d <= 65_000_000:
                for fam in ("er", "rmat"):
                    out.append((fam, n, d))
    return out[:6] if quick else out


def make_graph(synth, fam, n, deg, seed):
    pairs = n * deg // 2
    if fam == "er":
        return synth.erdos_renyi(seed, n, pairs)
    return synth.rmat(seed, n, int(pairs * 1.25))  # duplicates collapse: draw a quarter more


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    ap.add_argument("--quick", action="store_true", help="a handful of graphs only (to try the tool)")
    args = ap.parse_args()

    import numpy as np
    import torch

    import synth
    from paper_2306_15155_amd import KIND_GAT, KIND_GCN, Context, csr_struct

    dev = "cuda:0"
    ctx = Context(0)
    rows = []

    def ev():
        return torch.cuda.Event(enable_timing=True)

    t_start = time.time()
    for gi, (fam, n, deg) in enumerate(graph_grid(args.quick)):
        g = make_graph(synth, fam, n, deg, 1000 + gi)
        N, nnz = g.n_rows, g.nnz
        rp, ci = torch.from_numpy(g.row_ptr).to(dev), torch.from_numpy(g.col_idx).to(dev)
        A = csr_struct(N, N, rp, ci)
        dr, dc = ctx.degrees(A)
        r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
        Apre = csr_struct(N, N, rp, ci, ctx.gcn_precompute(A, r, c))
        degs = np.diff(g.row_ptr).astype(np.float64)
        feat = dict(family=fam, n_rows=N, n_cols=N, nnz=nnz, max_deg=int(degs.max()), sum_sq_deg=int((degs * degs).sum()))
        for f_in, f_out in WIDTH_PAIRS:
            if N * max(f_in, f_out) * 4 > 6e9:
                continue
            X = torch.rand((N, f_in), device=dev) * 2 - 1
            W = (torch.rand((f_in, f_out), device=dev) - 0.5) * 0.2
            a_l, a_r = torch.randn(f_out, device=dev) * 0.1, torch.randn(f_out, device=dev) * 0.1
            Y = torch.empty((N, f_out), device=dev)
            for kind, n_ids in ((KIND_GCN, 6), (KIND_GAT, 4)):
                for cid in range(n_ids):
                    def run():
                        if kind == KIND_GCN:
                            ctx.gcn_layer(Apre if cid >= 4 else A, r, c, X, W, cid, 1, out=Y)
                        else:
                            ctx.gat_layer(A, X, W, a_l, a_r, cid, 0.2, 1, out=Y)
                    run()
                    torch.cuda.synchronize()
                    ctx.profile_enable(True)
                    e0, e1 = ev(), ev()
                    e0.record()
                    run()
                    run()
                    e1.record()
                    torch.cuda.synchronize()
                    spmm, gemm = ctx.profile_read(0), ctx.profile_read(1)
                    ctx.profile_enable(False)
                    layer_ms = e0.elapsed_time(e1) / 2
                    agg = (cid in (0, 2, 4)) if kind == KIND_GCN else (cid in (1, 2))
                    width = f_in if agg else f_out
                    flavour = FLAVOUR_GCN[cid] if kind == KIND_GCN else "softmax"
                    rows.append(dict(feat, rec="spmm", kind=kind, comp=cid, f_in=f_in, f_out=f_out, flavour=flavour, width=width,
                                     ms=float(np.mean(spmm))))
                    per = len(gemm) // 2
                    if kind == KIND_GCN:
                        shapes = [(N, f_in, f_out)]
                    else:
                        shapes = [(N, f_in, f_out), (N, f_in, f_out)] if cid == 1 else [(N, f_in, f_out)]
                    for j in range(per):
                        gn, gk, gm = shapes[j]
                        rows.append(dict(feat, rec="gemm", kind=kind, comp=cid, f_in=f_in, f_out=f_out, flavour="", width=gm, gemm_k=gk,
                                         ms=float(np.mean(gemm[j::per]))))
                    rows.append(dict(feat, rec="layer", kind=kind, comp=cid, f_in=f_in, f_out=f_out, flavour=flavour, width=width, ms=layer_ms))
            del X, W, Y
        print("graph %d %s n=%d deg=%d nnz=%d  (%.0f s)" % (gi, fam, N, deg, nnz, time.time() - t_start), flush=True)
        del rp, ci, A, Apre
        torch.cuda.empty_cache()

    cols = ["rec", "family", "n_rows", "n_cols", "nnz", "max_deg", "sum_sq_deg", "kind", "comp", "f_in", "f_out", "flavour", "width", "gemm_k", "ms"]
    with open(args.out, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=cols)
        w.writeheader()
        for row in rows:
            out = {k: row.get(k, "") for k in cols}
            out["ms"] = "%.5g" % row["ms"]
            w.writerow(out)
    print("wrote %d rows to %s" % (len(rows), args.out))
    ctx.close()


if __name__ == "__main__":
    sys.exit(main())
