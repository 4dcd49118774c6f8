#!/usr/bin/env python3
"""Benchmark of the GCN / GAT layer hot path on one MI355X.

A step is one pass of the whole hot path over the synthetic Reddit-shaped workload: GCN layer 1
(602->256, ReLU), GCN layer 2 (256->41) and one single-head GAT layer (602->256), each run in the
composition sensei_select picked for it.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line (see the design doc for the meaning of every field).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (nodes, R-MAT draws, f_in, hidden, classes)
    "c2_rmat233k": dict(n=233_000, draws=92_600_000, f_in=602, hidden=256, classes=41, seed=7),
    "c1_er10k": dict(n=10_000, pairs=50_000, f_in=64, hidden=32, classes=16, seed=1),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_rmat233k", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip timing every composition id")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run four 1 GiB device-to-device copies (a kernel of known traffic, for scaling rocprofv3 --pmc byte counters)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU sharding is a design note in DESIGN.md",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import synth
    from paper_2306_15155_amd import (ACT_NONE, ACT_RELU, GAT_NAMES, GCN_NAMES, KIND_GAT, KIND_GCN, SELECT_MODEL, SELECT_TIMED,
                                      Context, csr_struct)

    wl = WORKLOADS[args.workload]
    dev = "cuda:0"
    t0 = time.time()
    if "draws" in wl:
        g = synth.rmat(wl["seed"], wl["n"], wl["draws"])
    else:
        g = synth.erdos_renyi(wl["seed"], wl["n"], wl["pairs"])
    N, nnz = g.n_rows, g.nnz
    f_in, hid, cls = wl["f_in"], wl["hidden"], wl["classes"]
    X = synth.uniform(wl["seed"], 10, (N, f_in))
    W1 = synth.glorot(wl["seed"], 11, f_in, hid)
    W2 = synth.glorot(wl["seed"], 12, hid, cls)
    Wg = synth.glorot(wl["seed"], 13, f_in, hid)
    a_l = synth.normal(wl["seed"], 14, (hid,), 0.0, 0.1)
    a_r = synth.normal(wl["seed"], 15, (hid,), 0.0, 0.1)
    gen_s = time.time() - t0

    row_ptr, col_idx = torch.from_numpy(g.row_ptr).to(dev), torch.from_numpy(g.col_idx).to(dev)
    Xd, W1d, W2d, Wgd = (torch.from_numpy(a).to(dev) for a in (X, W1, W2, Wg))
    ald, ard = torch.from_numpy(a_l).to(dev), torch.from_numpy(a_r).to(dev)
    ctx = Context(0)
    A = csr_struct(N, N, row_ptr, col_idx)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- one-off setup (a0, a1), timed separately
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    dr, dc = ctx.degrees(A)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    ntil = ctx.gcn_precompute(A, r, c)
    e1.record()
    torch.cuda.synchronize()
    setup_ms = e0.elapsed_time(e1)
    Apre = csr_struct(N, N, row_ptr, col_idx, ntil)

    # ---- composition choice per layer (cost model: host arithmetic only)
    ts = time.perf_counter()
    id1, est1 = ctx.select(KIND_GCN, A, f_in, hid, SELECT_MODEL)
    id2, est2 = ctx.select(KIND_GCN, A, hid, cls, SELECT_MODEL)
    idg, estg = ctx.select(KIND_GAT, A, f_in, hid, SELECT_MODEL)
    select_model_ms = (time.perf_counter() - ts) * 1e3

    H1 = torch.empty((N, hid), device=dev)
    Y2 = torch.empty((N, cls), device=dev)
    Yg = torch.empty((N, hid), device=dev)

    def gcn(cid, Xin, Win, out, act):
        return ctx.gcn_layer(Apre if cid >= 4 else A, r, c, Xin, Win, cid, act, out=out)

    def step():
        gcn(id1, Xd, W1d, H1, ACT_RELU)
        gcn(id2, H1, W2d, Y2, ACT_NONE)
        ctx.gat_layer(A, Xd, Wgd, ald, ard, idg, 0.2, ACT_RELU, out=Yg)

    if args.copy_probe:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    spmm_ms = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step = total_ms / args.steps
    ms_per_layer = ms_per_step / 3.0

    # ---- roofline of the dominant kernel: the SpMM of GCN layer 1 (3 SpMM launches per step, in order)
    per_step = len(spmm_ms) // max(args.steps, 1)
    l1 = spmm_ms[0::per_step] if per_step else []
    spmm_l1_ms = float(np.mean(l1)) if l1 else float("nan")
    agg1 = id1 in (0, 2, 4)
    f_sp = f_in if agg1 else hid
    weighted = id1 >= 4
    # compulsory bytes of one launch: indices (+ values), row pointers, every gathered row once, output once,
    # plus the two scaling vectors when they are applied inside the kernel
    idx_bytes = nnz * (8 if weighted else 4) + 4 * (N + 1)
    algo_bytes = idx_bytes + 4 * f_sp * N + 4 * f_sp * N + (8 * N if id1 in (2, 3) else 0)
    gather_bytes = idx_bytes + 4 * f_sp * nnz + 4 * f_sp * N
    achieved = algo_bytes / (spmm_l1_ms * 1e-3) / 1e9
    traffic = None
    prof = os.path.join(ROOT, "profiles", "k_spmm_c2_rmat233k_pmc.txt")
    if args.workload == "c2_rmat233k" and os.path.exists(prof):
        for line in open(prof):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline = {"kernel": "k_spmm (GCN layer 1, F=%d, %s)" % (f_sp, GCN_NAMES[id1]), "bound": "hbm", "achieved": round(achieved, 1),
                "peak": 8000.0, "unit": "GB/s", "frac": round(achieved / 8000.0, 4), "traffic": traffic,
                "avg_launch_ms": round(spmm_l1_ms, 4), "algorithmic_bytes": algo_bytes,
                "gather_GBps_no_reuse": round(gather_bytes / (spmm_l1_ms * 1e-3) / 1e9, 1)}

    # ---- per-layer and per-composition times (outside the timed region)
    def time_fn(fn, iters=3):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters

    detail = {"layers": {
        "gcn1_%d_%d" % (f_in, hid): {"id": GCN_NAMES[id1], "ms": round(time_fn(lambda: gcn(id1, Xd, W1d, H1, ACT_RELU)), 4)},
        "gcn2_%d_%d" % (hid, cls): {"id": GCN_NAMES[id2], "ms": round(time_fn(lambda: gcn(id2, H1, W2d, Y2, ACT_NONE)), 4)},
        "gat_%d_%d" % (f_in, hid): {"id": GAT_NAMES[idg], "ms": round(time_fn(lambda: ctx.gat_layer(A, Xd, Wgd, ald, ard, idg, 0.2, ACT_RELU, out=Yg)), 4)},
    }, "setup_ms": round(setup_ms, 4), "select_model_ms": round(select_model_ms, 4), "graph": {"nodes": N, "nnz": nnz,
        "max_degree": int(np.diff(g.row_ptr).max()), "generate_s": round(gen_s, 2)}}
    if not args.no_sweep:
        sweep = {}
        for name, Xin, Win, out, act in (("gcn1", Xd, W1d, H1, ACT_RELU), ("gcn2", H1, W2d, Y2, ACT_NONE)):
            sweep[name] = {GCN_NAMES[i]: round(time_fn(lambda: gcn(i, Xin, Win, out, act), 2), 4) for i in range(6)}
        sweep["gat"] = {GAT_NAMES[i]: round(time_fn(lambda: ctx.gat_layer(A, Xd, Wgd, ald, ard, i, 0.2, ACT_RELU, out=Yg), 2), 4)
                        for i in range(4)}
        detail["all_compositions_ms"] = sweep
        regret = {}
        for name, picked, names in (("gcn1", id1, GCN_NAMES), ("gcn2", id2, GCN_NAMES), ("gat", idg, GAT_NAMES)):
            regret[name] = round(sweep[name][names[picked]] / min(sweep[name].values()) - 1.0, 4)
        detail["selector_regret"] = regret
        ts = time.perf_counter()
        idt, _ = ctx.select(KIND_GCN, A, f_in, hid, SELECT_TIMED)
        torch.cuda.synchronize()
        detail["select_timed"] = {"gcn1_pick": GCN_NAMES[idt], "overhead_ms": round((time.perf_counter() - ts) * 1e3, 3),
                                  "overhead_in_layers": round((time.perf_counter() - ts) * 1e3 / detail["layers"]["gcn1_%d_%d" % (f_in, hid)]["ms"], 2)}

    # ---- CPU baseline: the fp64 oracle, single thread, on a bounded row sample, extrapolated by row count
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_s = min(N, 24000 if N > 50_000 else N)
        rows = np.sort(synth.distinct_nodes(wl["seed"], 40, N, n_s)) if n_s < N else None
        scale = N / float(n_s)
        tc = time.perf_counter()
        Xh1 = oracle.gcn_layer(N, N, g.row_ptr, g.col_idx, X, W1, 1, rows=rows)
        t1 = time.perf_counter() - tc
        H1_host = synth.uniform(wl["seed"], 16, (N, hid), 0.0, 1.0)  # stand-in for the hidden activations
        tc = time.perf_counter()
        oracle.gcn_layer(N, N, g.row_ptr, g.col_idx, H1_host, W2, 0, rows=rows)
        t2 = time.perf_counter() - tc
        tc = time.perf_counter()
        Yg_ref = oracle.gat_layer(N, N, g.row_ptr, g.col_idx, X, Wg, a_l, a_r, 0.2, 1, rows=rows)
        t3 = time.perf_counter() - tc
        cpu = {"value": round((t1 + t2 + t3) * scale * 1e3 / 3.0, 1), "unit": "ms per layer (extrapolated by row count)",
               "cores": oracle.threads(False), "kind": "oracle",
               "sample": "%d uniformly drawn output rows of each of the 3 layers (of %d), %.1f s of CPU work" % (n_s, N, t1 + t2 + t3)}
        # the sampled oracle rows double as a full-size parity check of what was just timed
        sel = slice(None) if rows is None else torch.from_numpy(rows.astype(np.int64)).to(dev)
        err1 = float(np.max(np.abs(H1[sel].cpu().numpy() - Xh1) / (1.0 + np.abs(Xh1))))
        errg = float(np.max(np.abs(Yg[sel].cpu().numpy() - Yg_ref) / (1.0 + np.abs(Yg_ref))))
        detail["sampled_parity_max_scaled_err"] = {"gcn1": err1, "gat": errg}

    out = {"metric": "ms per GCN/GAT layer (mean over GCN 602->256, GCN 256->41, GAT 602->256)", "value": round(ms_per_layer, 4),
           "unit": "ms/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": args.workload, "graph": "R-MAT(0.57,0.19,0.19,0.05) symmetrised + self loops" if "draws" in wl else "G(n,M) + self loops",
                      "nodes": N, "nnz": nnz, "layers": "GCN %d->%d->%d, GAT %d->%d" % (f_in, hid, cls, f_in, hid),
                      "compositions": [GCN_NAMES[id1], GCN_NAMES[id2], GAT_NAMES[idg]]},
           "roofline": roofline, "cpu_baseline": cpu, "detail": detail}
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
