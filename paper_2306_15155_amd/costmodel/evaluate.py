"""Scores the selectors on graphs that are not in the training grid (in the manner of the paper's cost-model table):

    python -m paper_2306_15155_amd.costmodel.evaluate --out results.csv

For every graph and pair of embedding sizes every composition is timed; a selector's regret is the time of its pick
over the time of the fastest candidate the embedding-size rules allow, minus one (regret_*), and over the time of the
fastest of all callable ids, which the rules may have dropped (regret_all_*).
"""
from __future__ import annotations

import argparse
import csv
import sys
import time

GRAPHS = [("er", 35_000, 6), ("rmat", 35_000, 6), ("er", 35_000, 300), ("rmat", 35_000, 300), ("er", 150_000, 6), ("rmat", 150_000, 6),
          ("er", 150_000, 48), ("rmat", 150_000, 48), ("er", 150_000, 300), ("rmat", 150_000, 300), ("er", 700_000, 6), ("rmat", 700_000, 6),
          ("er", 700_000, 48), ("rmat", 700_000, 48), ("rmat", 233_000, 494)]
PAIRS = [(48, 192), (192, 48), (96, 96), (300, 40), (40, 300), (602, 256)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    import numpy as np
    import torch

    import synth
    from paper_2306_15155_amd import KIND_GAT, KIND_GCN, SELECT_AUTO, SELECT_LEARNED, SELECT_MODEL, Context, csr_struct
    from paper_2306_15155_amd.costmodel.collect import make_graph

    dev = "cuda:0"
    ctx = Context(0)
    rows = []
    t0 = time.time()
    for gi, (fam, n, deg) in enumerate(GRAPHS):
        g = make_graph(synth, fam, n, deg, 5000 + gi)
        N = g.n_rows
        rp, ci = torch.from_numpy(g.row_ptr).to(dev), torch.from_numpy(g.col_idx).to(dev)
        A = csr_struct(N, N, rp, ci)
        dr, dc = ctx.degrees(A)
        r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
        Apre = csr_struct(N, N, rp, ci, ctx.gcn_precompute(A, r, c))
        for f_in, f_out in PAIRS:
            X = torch.rand((N, f_in), device=dev) * 2 - 1
            W = (torch.rand((f_in, f_out), device=dev) - 0.5) * 0.2
            a_l, a_r = torch.randn(f_out, device=dev) * 0.1, torch.randn(f_out, device=dev) * 0.1
            Y = torch.empty((N, f_out), device=dev)
            for kind, name, n_ids in ((KIND_GCN, "gcn", 6), (KIND_GAT, "gat", 4)):
                ms = []
                for cid in range(n_ids):
                    def run():
                        if kind == KIND_GCN:
                            ctx.gcn_layer(Apre if cid >= 4 else A, r, c, X, W, cid, 1, out=Y)
                        else:
                            ctx.gat_layer(A, X, W, a_l, a_r, cid, 0.2, 1, out=Y)
                    run()
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    run()
                    run()
                    e1.record()
                    torch.cuda.synchronize()
                    ms.append(e0.elapsed_time(e1) / 2)
                pick_m, est_m = ctx.select(kind, A, f_in, f_out, SELECT_MODEL)
                pick_l, est_l = ctx.select(kind, A, f_in, f_out, SELECT_LEARNED)
                pick_a, _ = ctx.select(kind, A, f_in, f_out, SELECT_AUTO)
                allowed = [i for i, e in enumerate(est_m) if e >= 0]
                best = min(allowed, key=lambda i: ms[i])
                rows.append(dict(family=fam, n=N, nnz=g.nnz, layer=name, f_in=f_in, f_out=f_out, best=best, best_ms=round(ms[best], 4),
                                 pick_model=pick_m, regret_model=round(ms[pick_m] / ms[best] - 1, 4), pick_learned=pick_l,
                                 regret_learned=round(ms[pick_l] / ms[best] - 1, 4), pick_auto=pick_a,
                                 regret_auto=round(ms[pick_a] / ms[best] - 1, 4),
                                 regret_all_model=round(ms[pick_m] / min(ms) - 1, 4), regret_all_learned=round(ms[pick_l] / min(ms) - 1, 4),
                                 regret_all_auto=round(ms[pick_a] / min(ms) - 1, 4),
                                 err_model=round(est_m[pick_m] / ms[pick_m], 3), err_learned=round(est_l[pick_l] / ms[pick_l], 3)))
            del X, W, Y
        print("graph %d %s n=%d deg=%d (%.0f s)" % (gi, fam, N, deg, time.time() - t0), flush=True)
    with open(args.out, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=list(rows[0]))
        w.writeheader()
        w.writerows(rows)
    for key in ("model", "learned", "auto"):
        reg = np.array([r["regret_" + key] for r in rows])
        reg_all = np.array([r["regret_all_" + key] for r in rows])
        line = ("%-8s picks the fastest allowed id in %d of %d cases; regret mean %.3f, max %.3f, over 10 %% in %d cases; against all ids: mean %.3f, max %.3f, over 10 %% in %d"
                % (key, int((reg < 1e-9).sum()), reg.size, reg.mean(), reg.max(), int((reg > 0.10).sum()), reg_all.mean(), reg_all.max(), int((reg_all > 0.10).sum())))
        if key != "auto":
            err = np.abs(np.log2(np.array([r["err_" + key] for r in rows])))
            line += "; |log2(predicted / measured)| of the pick: median %.2f, max %.2f" % (np.median(err), err.max())
        print(line)
    ctx.close()


if __name__ == "__main__":
    sys.exit(main())
