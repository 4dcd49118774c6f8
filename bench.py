#!/usr/bin/env python3
"""Benchmark of the GCN / GAT layer hot path on one MI355X.

A step is one pass of the whole hot path over a synthetic workload: every layer of the workload's
layer list, each run in the composition sensei_select picked for it.  The default workload is the
Reddit-shaped one (GCN 602->256 with ReLU, GCN 256->41, single-head GAT 602->256 on the 233k-node
R-MAT graph).  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _gcn(f_in, f_out, act, src):
    return dict(kind="gcn", f_in=f_in, f_out=f_out, act=act, src=src)


def _gat(f_in, f_out, act, src):
    return dict(kind="gat", f_in=f_in, f_out=f_out, act=act, src=src)


# src: "X" = the node features, an integer = output of that earlier layer of the list
WORKLOADS = {
    "c2_rmat233k": dict(graph="rmat", n=233_000, draws=92_600_000, seed=7, f_x=602, x="uniform",
                        layers=[_gcn(602, 256, 1, "X"), _gcn(256, 41, 0, 0), _gat(602, 256, 1, "X")]),
    "c3_rmat2450k": dict(graph="rmat", n=2_450_000, draws=84_000_000, seed=7, f_x=100, x="normal",
                         layers=[l for h in (32, 128, 512, 1024) for l in (_gcn(100, h, 1, "X"), _gcn(h, h, 0, -1))]),
    # shapes of the two extremes of the paper's graph table: very dense (98 k nodes, 1e8 stored entries) and
    # road-network-like (12 M nodes, about two links per node)
    "dense98k": dict(graph="er", n=98_000, pairs=50_000_000, seed=3, f_x=256, x="uniform",
                     layers=[_gcn(256, 64, 1, "X"), _gcn(64, 256, 0, 0), _gat(64, 256, 1, 0)]),
    "road12m": dict(graph="grid", side=3464, keep=0.53, seed=5, f_x=128, x="normal",
                    layers=[_gcn(128, 32, 1, "X"), _gcn(32, 128, 0, 0), _gat(32, 128, 1, 0)]),
    "c1_er10k": dict(graph="er", n=10_000, pairs=50_000, seed=1, f_x=64, x="uniform", layers=[_gcn(64, 32, 1, "X")]),
}


def _source_sha16():
    """Hash of the kernel sources: a counter summary under profiles/ is only quoted while it was taken from these very sources."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2306_15155_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".h")):
            h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()[:16]


def _profile_value(path, key):
    """'<key>: <number>' from a profile summary, or None when the file is missing or was taken from other kernel sources."""
    if not os.path.exists(path):
        return None
    sha, val = None, None
    for line in open(path):
        if line.startswith("source_sha16:"):
            sha = line.split(":")[1].strip()
        if line.startswith(key + ":"):
            val = float(line.split(":")[1])
    return val if sha == _source_sha16() else None


def _hip_runtime():
    """The HIP runtime already mapped into this process (ctypes handle), for counting the kernel nodes of a captured stream."""
    import ctypes
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            return ctypes.CDLL(line.split()[-1])
    return None


def _kernel_count(torch, fn):
    """Number of kernel launches of fn(): captured on a side stream into a HIP graph that is never launched, nodes counted."""
    import ctypes
    hip = _hip_runtime()
    if hip is None:
        return None
    fn()                                 # allocations and workspace growth happen outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph, n = ctypes.c_void_p(), ctypes.c_size_t(0)
    with torch.cuda.stream(side):
        st = ctypes.c_void_p(side.cuda_stream)
        if hip.hipStreamBeginCapture(st, 2) != 0:   # relaxed mode
            return None
        try:
            fn()
        finally:
            rc = hip.hipStreamEndCapture(st, ctypes.byref(graph))
    if rc != 0 or not graph:
        return None
    rc = hip.hipGraphGetNodes(graph, None, ctypes.byref(n))
    hip.hipGraphDestroy(graph)
    torch.cuda.synchronize()
    return int(n.value) if rc == 0 else None


def _time_fn(torch, fn, iters=3):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def _graph_replay_ms(torch, fn, iters=50):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    return _time_fn(torch, graph.replay, iters)


def _spmm_shape_of(kind, cid, f_in, f_out):
    """(columns the SpMM of this composition gathers, bytes per stored entry it reads, scaling vectors read inside it)."""
    if kind == "gcn":
        return (f_in if cid in (0, 2, 4) else f_out), (8 if cid >= 4 else 4), cid in (2, 3)
    return (f_out if cid in (0, 3) else f_in), 8, False


def _layer_report(torch, np, ctx, kind, A, Apre, N, nnz, r, c, Xd, Wd, att, f_in, f_out, act, out, iters=2):
    """Every composition id of one layer timed; the selector's pick with its regret (against the ids its rules allow and against
    all ids); SpMM and GEMM launches of the picked id timed by the library's HIP events, with the roofline each is held to."""
    from paper_2306_15155_amd import GAT_NAMES, GCN_NAMES, KIND_GAT, KIND_GCN, SELECT_MODEL
    names = GCN_NAMES if kind == "gcn" else GAT_NAMES
    k = KIND_GCN if kind == "gcn" else KIND_GAT

    def run(cid):
        if kind == "gcn":
            ctx.gcn_layer(Apre if cid >= 4 else A, r, c, Xd, Wd, cid, act, out=out)
        else:
            ctx.gat_layer(A, Xd, Wd, att[0], att[1], cid, 0.2, act, out=out)

    pick, est = ctx.select(k, A, f_in, f_out, SELECT_MODEL)
    ms = {names[cid]: round(_time_fn(torch, lambda: run(cid), iters), 4) for cid in range(len(names))}
    allowed = [names[cid] for cid, t in enumerate(est) if t >= 0]
    ctx.profile_enable(True)
    for _ in range(3):
        run(pick)
    torch.cuda.synchronize()
    sp, ge = ctx.profile_read(0), ctx.profile_read(1)
    ctx.profile_enable(False)
    rep = {"picked": names[pick], "ms": ms, "regret_vs_allowed": round(ms[names[pick]] / min(ms[n] for n in allowed) - 1.0, 4),
           "regret_vs_all_ids": round(ms[names[pick]] / min(ms.values()) - 1.0, 4)}
    if sp:
        f_sp, per_nnz, scaled = _spmm_shape_of(kind, pick, f_in, f_out)
        t = float(np.mean(sp[len(sp) // 3:])) * 1e-3
        idx = nnz * per_nnz + 4 * (N + 1) + (8 * N if scaled else 0)
        b_min, b_max = idx + 8 * f_sp * N, idx + 4 * f_sp * nnz + 4 * f_sp * N
        rep["spmm"] = {"f": f_sp, "ms": round(t * 1e3, 4), "B_min_GBps": round(b_min / t / 1e9, 1), "B_max_GBps": round(b_max / t / 1e9, 1),
                       "frac_of_hbm_peak_on_B_min": round(b_min / t / 8e12, 4)}
    if ge:
        per = len(ge) // 3
        t = float(np.max([np.mean(ge[j::per][1:]) for j in range(per)])) * 1e-3      # the longest GEMM launch of the layer
        flops = 2.0 * N * f_in * f_out
        by = 4.0 * (N * f_in + f_in * f_out + N * f_out)
        mult, peak, dtype = _gemm_matrix_core(N, f_in, f_out)
        bound = "mfma" if mult * flops / by > peak / 8e12 else "hbm"
        rep["gemm"] = {"ms": round(t * 1e3, 4), "tflops": round(flops / t / 1e12, 1), "flop_per_byte": round(flops / by, 1), "bound": bound,
                       "matrix_core": dtype, "frac": round(mult * flops / t / peak if bound == "mfma" else by / t / 8e12, 3)}
    run(pick)  # the picked composition's output stays in `out`
    return rep


def _gemm_matrix_core(n, k, m):
    """(matrix-core operations per fp32 multiply-add pair, dense peak of that instruction in op/s, description) of the kernel the
    library takes for an n x k by k x m product: the fp32 instruction, or six bf16 piece products per term for large products."""
    from paper_2306_15155_amd import binding
    if binding.gemm_kernel(n, k, m) == binding.GEMM_BF16_PIECES:
        return 6.0, 2.5e15, "bf16, three exact pieces per fp32 operand, six piece products per term"
    return 1.0, 157.3e12, "fp32"


def run_extras(args, torch, np, synth, oracle):
    """What the default run reports beside the headline workload, each under its own key of `detail`."""
    from paper_2306_15155_amd import Context, Panels, csr_struct
    dev = "cuda:0"
    out = {}
    ctx = Context(0)

    def upload(g):
        row_ptr, col_idx = torch.from_numpy(g.row_ptr).to(dev), torch.from_numpy(g.col_idx).to(dev)
        A = csr_struct(g.n_rows, g.n_cols, row_ptr, col_idx)
        dr, dc = ctx.degrees(A)
        r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
        ntil = ctx.gcn_precompute(A, r, c)
        return dict(row_ptr=row_ptr, col_idx=col_idx, r=r, c=c, ntil=ntil)

    def patterns(g, d, with_panels):
        panels = Panels(ctx, csr_struct(g.n_rows, g.n_cols, d["row_ptr"], d["col_idx"]), 0, tune=True) if with_panels else None
        d["panels"] = panels
        return (csr_struct(g.n_rows, g.n_cols, d["row_ptr"], d["col_idx"], None, panels),
                csr_struct(g.n_rows, g.n_cols, d["row_ptr"], d["col_idx"], d["ntil"], panels))

    def release():
        ctx.ws.buf = torch.empty(0, dtype=torch.uint8, device=dev)
        torch.cuda.empty_cache()

    # ---- hidden-size sweep on the 2.45 M-node graph (both layers, all six ids per size), then the sampled mini-batch drawn from it
    t0 = time.time()
    g = synth.rmat(7, 2_450_000, 84_000_000)
    N, nnz = g.n_rows, g.nnz
    X = synth.normal(7, 10, (N, 100))
    d = upload(g)
    A, Apre = patterns(g, d, True)
    Xd = torch.from_numpy(X).to(dev)
    rows = np.sort(np.unique(np.concatenate([[int(np.diff(g.row_ptr).argmax()), int(np.diff(g.row_ptr).argmin())],
                                            synth.distinct_nodes(7, 50, N, 1000)]))).astype(np.int32)
    sel = torch.from_numpy(rows.astype(np.int64)).to(dev)
    sweep = {"graph": {"nodes": N, "nnz": nnz, "max_degree": int(np.diff(g.row_ptr).max())}, "column_panels": d["panels"].count, "sizes": {}}
    for i, h in enumerate((32, 128, 512, 1024)):
        W1, W2 = synth.glorot(7, 100 + 2 * i, 100, h), synth.glorot(7, 101 + 2 * i, h, h)
        H1, H2 = torch.empty((N, h), device=dev), torch.empty((N, h), device=dev)
        l1 = _layer_report(torch, np, ctx, "gcn", A, Apre, N, nnz, d["r"], d["c"], Xd, torch.from_numpy(W1).to(dev), None, 100, h, 1, H1)
        ref = oracle.gcn_layer(N, N, g.row_ptr, g.col_idx, X, W1, 1, rows=rows, omp=True)
        got = H1[sel].cpu().numpy()
        l1["sampled_parity_max_scaled_err"] = float(np.max(np.abs(got - ref) / (1.0 + np.abs(ref))))
        l2 = _layer_report(torch, np, ctx, "gcn", A, Apre, N, nnz, d["r"], d["c"], H1, torch.from_numpy(W2).to(dev), None, h, h, 0, H2)
        sweep["sizes"][str(h)] = {"gcn_100_%d" % h: l1, "gcn_%d_%d" % (h, h): l2, "ms_per_layer_picked": round((l1["ms"][l1["picked"]] + l2["ms"][l2["picked"]]) / 2, 4)}
        del H1, H2
        release()
    sweep["parity_sample"] = "%d output rows of every 100->h layer (the longest row, a shortest one, 1,000 random) against the fp64 oracle" % rows.size
    sweep["seconds"] = round(time.time() - t0, 1)
    out["c3_rmat2450k_sweep"] = sweep
    del Xd, A, Apre
    # mini-batch: 1,024 seeds, fan-outs 10 then 25; the wide block runs first
    t0 = time.time()
    seeds = synth.distinct_nodes(7, 40, N, 1024)
    b2, ids1 = synth.sample_block(7, 41, g, seeds, 10)
    b1, ids0 = synth.sample_block(7, 42, g, ids1, 25)
    X0 = synth.normal_rows(7, 43, ids0, 100)
    W1, W2 = synth.glorot(7, 44, 100, 256), synth.glorot(7, 45, 256, 47)
    d1, d2 = upload(b1), upload(b2)
    (A1, A1p), (A2, A2p) = patterns(b1, d1, False), patterns(b2, d2, False)
    X0d, W1d, W2d = torch.from_numpy(X0).to(dev), torch.from_numpy(W1).to(dev), torch.from_numpy(W2).to(dev)
    H1, Y = torch.empty((b1.n_rows, 256), device=dev), torch.empty((b2.n_rows, 47), device=dev)
    from paper_2306_15155_amd import GCN_NAMES, KIND_GCN, SELECT_MODEL
    p1, p2 = ctx.select(KIND_GCN, A1, 100, 256, SELECT_MODEL)[0], ctx.select(KIND_GCN, A2, 256, 47, SELECT_MODEL)[0]

    def l1(cid):
        ctx.gcn_layer(A1p if cid >= 4 else A1, d1["r"], d1["c"], X0d, W1d, cid, 1, out=H1)

    def l2(cid):
        ctx.gcn_layer(A2p if cid >= 4 else A2, d2["r"], d2["c"], H1, W2d, cid, 0, out=Y)

    def chain():
        l1(p1)
        l2(p2)

    mb = {"blocks": {"wide": [b1.n_rows, b1.n_cols, b1.nnz], "narrow": [b2.n_rows, b2.n_cols, b2.nnz]},
          "picked": [GCN_NAMES[p1], GCN_NAMES[p2]],
          "eager_us_per_layer": round(_time_fn(torch, chain, 50) * 500.0, 2),
          "graph_replay_us_per_layer": round(_graph_replay_ms(torch, chain) * 500.0, 2),
          "per_id": {GCN_NAMES[cid]: {"wide_us": round(_time_fn(torch, lambda: l1(cid), 20) * 1e3, 2), "narrow_us": round(_time_fn(torch, lambda: l2(cid), 20) * 1e3, 2),
                                      "kernels_wide": _kernel_count(torch, lambda: l1(cid)), "kernels_narrow": _kernel_count(torch, lambda: l2(cid))}
                     for cid in range(6)}}
    chain()
    H1_ref = oracle.gcn_layer(b1.n_rows, b1.n_cols, b1.row_ptr, b1.col_idx, X0, W1, 1)
    Y_ref = oracle.gcn_layer(b2.n_rows, b2.n_cols, b2.row_ptr, b2.col_idx, H1_ref.astype(np.float32), W2, 0)
    mb["parity_max_scaled_err"] = float(np.max(np.abs(Y.cpu().numpy() - Y_ref) / (1.0 + np.abs(Y_ref))))
    mb["note"] = "latency bound: a fraction of roofline is not meaningful at this size"
    mb["seconds"] = round(time.time() - t0, 1)
    out["c5_minibatch"] = mb
    del g, d, d1, d2, X0d, H1, Y
    release()

    # ---- the 10,000-node graph: latency bound as well
    t0 = time.time()
    g = synth.erdos_renyi(1, 10_000, 50_000)
    X, W = synth.uniform(1, 10, (10_000, 64)), synth.glorot(1, 11, 64, 32)
    d = upload(g)
    A, Apre = patterns(g, d, False)
    Xd, Wd, Y = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev), torch.empty((10_000, 32), device=dev)

    def one(cid):
        ctx.gcn_layer(Apre if cid >= 4 else A, d["r"], d["c"], Xd, Wd, cid, 1, out=Y)

    pick = ctx.select(KIND_GCN, A, 64, 32, SELECT_MODEL)[0]
    c1 = {"picked": GCN_NAMES[pick],
          "per_id": {GCN_NAMES[cid]: {"eager_us": round(_time_fn(torch, lambda: one(cid), 50) * 1e3, 2),
                                      "graph_replay_us": round(_graph_replay_ms(torch, lambda: one(cid)) * 1e3, 2),
                                      "kernels": _kernel_count(torch, lambda: one(cid))} for cid in range(6)}}
    one(pick)
    ref = oracle.gcn_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, 1)
    c1["parity_max_scaled_err"] = float(np.max(np.abs(Y.cpu().numpy() - ref) / (1.0 + np.abs(ref))))
    c1["note"] = "latency bound (working set about 4 MB): a fraction of roofline is not meaningful at this size"
    c1["seconds"] = round(time.time() - t0, 1)
    out["c1_er10k"] = c1
    del g, d, Xd, Wd, Y
    release()

    # ---- the two extremes of the paper's graph table: road-network shape and very dense
    for name, make, f_x, shapes in (("road12m", lambda: synth.thinned_grid(5, 3464, 0.53), 128, ((128, 32), (32, 128))),
                                    ("dense98k", lambda: synth.erdos_renyi(3, 98_000, 50_000_000), 256, ((256, 64), (64, 256)))):
        t0 = time.time()
        g = make()
        N, nnz = g.n_rows, g.nnz
        X = synth.normal(5, 10, (N, f_x)) if name == "road12m" else synth.uniform(3, 10, (N, f_x))
        d = upload(g)
        A, Apre = patterns(g, d, True)
        Xd = torch.from_numpy(X).to(dev)
        rep = {"graph": {"nodes": N, "nnz": nnz, "max_degree": int(np.diff(g.row_ptr).max())}, "column_panels": d["panels"].count, "layers": {}}
        for j, (f_in, f_out) in enumerate(shapes):
            Xin = Xd[:, :f_in].contiguous()
            Wd = torch.from_numpy(synth.glorot(5, 100 + j, f_in, f_out)).to(dev)
            Y = torch.empty((N, f_out), device=dev)
            rep["layers"]["gcn_%d_%d" % (f_in, f_out)] = _layer_report(torch, np, ctx, "gcn", A, Apre, N, nnz, d["r"], d["c"], Xin, Wd, None, f_in, f_out, 1, Y)
            att = (torch.from_numpy(synth.normal(5, 200 + j, (f_out,), 0.0, 0.1)).to(dev), torch.from_numpy(synth.normal(5, 300 + j, (f_out,), 0.0, 0.1)).to(dev))
            rep["layers"]["gat_%d_%d" % (f_in, f_out)] = _layer_report(torch, np, ctx, "gat", A, Apre, N, nnz, d["r"], d["c"], Xin, Wd, att, f_in, f_out, 1, Y)
            del Xin, Wd, Y
        rep["seconds"] = round(time.time() - t0, 1)
        out[name] = rep
        del g, d, A, Apre, Xd
        release()
    torch.cuda.synchronize()
    ctx.close()
    return out


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)  # the iteration count of the paper's evaluation
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2_rmat233k", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip timing every composition id (and, unless --backward, the backward pass)")
    ap.add_argument("--backward", action="store_true", help="time the backward pass even with --no-sweep")
    ap.add_argument("--no-panels", action="store_true", help="do not build the column-panel copy of the graph")
    ap.add_argument("--panels", type=int, default=0, help="force the number of column panels (0 = let the library measure)")
    ap.add_argument("--tiles", type=float, default=0.07, help="dense-tile split of the hub region: least density of a kept tile (0 = off)")
    ap.add_argument("--tiles-min-width", type=int, default=64, help="narrowest SpMM (columns) that uses the dense-tile split")
    ap.add_argument("--tiles-remainder-panels", type=int, default=0,
                    help="column panels of the panel-major copy of the split's sparse remainder (0 = the library decides, 1 = none)")
    ap.add_argument("--tiles-min-share", type=float, default=1.0 / 3.0,
                    help="the split is attached to the pattern only if at least this share of the entries lies in kept tiles")
    ap.add_argument("--tiles-max-width", type=int, default=0,
                    help="widest SpMM operand (columns, rounded up to 32) the dense-tile split is built for; 0 = the widest layer dimension, at most 1024")
    ap.add_argument("--no-gather-probe", action="store_true", help="skip the L2-resident gather probe")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what the default run adds under detail beside the headline workload: the hidden-size sweep on the 2.45 M-node "
                         "graph, the sampled mini-batch, the 10,000-node graph, the road-shaped and the very dense graph")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run four 1 GiB device-to-device copies (a kernel of known traffic, for scaling rocprofv3 --pmc byte counters)")
    return ap.parse_args()


def headline(args):
    """The timed workload: returns the JSON line as a dict (every device tensor it used is released on return)."""
    import numpy as np
    import torch

    import synth
    from paper_2306_15155_amd import (GAT_NAMES, GCN_NAMES, KIND_GAT, KIND_GCN, SELECT_AUTO, SELECT_LEARNED, SELECT_MODEL, SELECT_TIMED, Context, Panels,
                                      csr_struct)

    wl = WORKLOADS[args.workload]
    layers = wl["layers"]
    dev = "cuda:0"
    seed = wl["seed"]
    t0 = time.time()
    if wl["graph"] == "rmat":
        g = synth.rmat(seed, wl["n"], wl["draws"])
    elif wl["graph"] == "grid":
        g = synth.thinned_grid(seed, wl["side"], wl["keep"])
    else:
        g = synth.erdos_renyi(seed, wl["n"], wl["pairs"])
    N, nnz = g.n_rows, g.nnz
    X = synth.uniform(seed, 10, (N, wl["f_x"])) if wl["x"] == "uniform" else synth.normal(seed, 10, (N, wl["f_x"]))
    Ws = [synth.glorot(seed, 100 + i, L["f_in"], L["f_out"]) for i, L in enumerate(layers)]
    att = [(synth.normal(seed, 200 + i, (L["f_out"],), 0.0, 0.1), synth.normal(seed, 300 + i, (L["f_out"],), 0.0, 0.1))
           if L["kind"] == "gat" else None for i, L in enumerate(layers)]
    gen_s = time.time() - t0

    row_ptr, col_idx = torch.from_numpy(g.row_ptr).to(dev), torch.from_numpy(g.col_idx).to(dev)
    Xd = torch.from_numpy(X).to(dev)
    Wd = [torch.from_numpy(w).to(dev) for w in Ws]
    attd = [None if a is None else (torch.from_numpy(a[0]).to(dev), torch.from_numpy(a[1]).to(dev)) for a in att]
    ctx = Context(0)
    A = csr_struct(N, N, row_ptr, col_idx)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- one-off set-up (degrees, D^-1/2 vectors, N~), timed separately
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    dr, dc = ctx.degrees(A)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    ntil = ctx.gcn_precompute(A, r, c)
    e1.record()
    torch.cuda.synchronize()
    setup_ms = e0.elapsed_time(e1)
    # optional column-panel copy of the pattern (the library decides from the graph whether to cut it at all)
    panels, panels_ms = None, 0.0
    if not args.no_panels:
        tp = time.perf_counter()
        panels = Panels(ctx, A, args.panels, tune=(args.panels == 0))
        torch.cuda.synchronize()
        panels_ms = (time.perf_counter() - tp) * 1e3  # includes the timed trials when the count is measured
        A = csr_struct(N, N, row_ptr, col_idx, None, panels)
    tiles, tiles_ms, tiles_attached = None, 0.0, False
    if args.tiles > 0:
        from paper_2306_15155_amd import Tiles
        tp = time.perf_counter()
        widest = args.tiles_max_width or min(1024, max(max(L["f_in"], L["f_out"]) for L in layers))
        tiles = Tiles(ctx, A, args.tiles, (widest + 31) // 32 * 32, args.tiles_min_width, args.tiles_remainder_panels)
        torch.cuda.synchronize()
        tiles_ms = (time.perf_counter() - tp) * 1e3
        # the split pays when a good part of the entries lies in kept tiles (measured: 64 % of them: SpMM call -25 %; 20 %: +5 %)
        tiles_attached = tiles.nnz_dense >= args.tiles_min_share * nnz
        if tiles_attached:
            A = csr_struct(N, N, row_ptr, col_idx, None, panels, tiles)
    Apre = csr_struct(N, N, row_ptr, col_idx, ntil, panels)

    # ---- composition choice per layer (cost model: host arithmetic only)
    ts = time.perf_counter()
    ids = [ctx.select(KIND_GCN if L["kind"] == "gcn" else KIND_GAT, A, L["f_in"], L["f_out"], SELECT_MODEL)[0] for L in layers]
    select_model_ms = (time.perf_counter() - ts) * 1e3

    outs = [torch.empty((N, L["f_out"]), device=dev) for L in layers]

    def src_of(i):
        s = layers[i]["src"]
        return Xd if s == "X" else outs[i + s if s < 0 else s]

    def run_layer(i, cid):
        L = layers[i]
        if L["kind"] == "gcn":
            ctx.gcn_layer(Apre if cid >= 4 else A, r, c, src_of(i), Wd[i], cid, L["act"], out=outs[i])
        else:
            ctx.gat_layer(A, src_of(i), Wd[i], attd[i][0], attd[i][1], cid, 0.2, L["act"], out=outs[i])

    def step():
        for i in range(len(layers)):
            run_layer(i, ids[i])

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
    marks = [ev() for _ in range(args.steps + 1)]
    e0.record()
    marks[0].record()
    for k in range(args.steps):
        step()
        marks[k + 1].record()
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    each_ms = [marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)]
    spmm_ms = ctx.profile_read(0)
    gemm_ms = ctx.profile_read(1)
    ctx.profile_enable(False)
    ms_per_step = total_ms / args.steps
    ms_per_layer = ms_per_step / len(layers)

    def name_of(i, cid=None):
        cid = ids[i] if cid is None else cid
        return (GCN_NAMES if layers[i]["kind"] == "gcn" else GAT_NAMES)[cid]

    def tag(i):
        return "%s%d_%d_%d" % (layers[i]["kind"], i, layers[i]["f_in"], layers[i]["f_out"])

    # ---- roofline of the dominant kernel: the SpMM launch (one per layer per step, in layer order) with the largest mean time
    per_step = len(layers)
    spmm_mean = [float(np.mean(spmm_ms[i::per_step])) for i in range(per_step)] if len(spmm_ms) == per_step * args.steps else []
    roofline = None
    if spmm_mean:
        k = int(np.argmax(spmm_mean))
        L, cid = layers[k], ids[k]
        if L["kind"] == "gcn":
            f_sp = L["f_in"] if cid in (0, 2, 4) else L["f_out"]
            weighted, scaled = cid >= 4, cid in (2, 3)
        else:
            f_sp = L["f_out"] if cid in (0, 3) else L["f_in"]
            weighted, scaled = True, False
        # compulsory bytes of one launch: indices (+ values), row pointers, every gathered row once, the output once,
        # plus the scaling vectors when they are applied inside the kernel
        idx_bytes = nnz * (8 if weighted else 4) + 4 * (N + 1)
        algo_bytes = idx_bytes + 4 * f_sp * N + 4 * f_sp * N + (8 * N if scaled else 0)
        gather_bytes = idx_bytes + 4 * f_sp * nnz + 4 * f_sp * N
        t_s = spmm_mean[k] * 1e-3
        # HBM-side bytes of one call from the rocprofv3 counter summary of this workload; null when the summary was not taken
        # from the kernel sources this run was built from
        traffic = _profile_value(os.path.join(ROOT, "profiles", "k_spmm_%s_pmc.txt" % args.workload), "traffic_bytes_per_launch %s" % tag(k))
        split = tiles_attached and tiles.n_tiles > 0 and f_sp >= args.tiles_min_width
        what = "SpMM call = hub tiles on the bf16 matrix cores (k_dense_tiles_bf / k_dense_tiles_attn_bf) + k_spmm on the sparse remainder + join" if split else "k_spmm"
        roofline = {"kernel": "%s (%s, F=%d, %s)" % (what, tag(k), f_sp, name_of(k)), "bound": "hbm",
                    "achieved": round(algo_bytes / t_s / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                    "frac": round(algo_bytes / t_s / 1e9 / 8000.0, 4), "traffic": traffic,
                    "avg_launch_ms": round(spmm_mean[k], 4), "algorithmic_bytes": algo_bytes,
                    "gather_GBps_no_reuse": round(gather_bytes / t_s / 1e9, 1),
                    "measured_traffic_GBps": None if traffic is None else round(traffic / t_s / 1e9, 1)}

    # ---- MFMA utilisation of the GEMM launch with the largest mean time, against the peak of the instruction its kernel uses
    gemm_info = None
    n_gemm = [2 if (L["kind"] == "gat" and ids[i] == 1) else 1 for i, L in enumerate(layers)]
    if len(gemm_ms) == sum(n_gemm) * args.steps:
        per, off, best = sum(n_gemm), 0, None
        for i, L in enumerate(layers):
            for j in range(n_gemm[i]):
                t = float(np.mean(gemm_ms[off + j::per]))
                if best is None or t > best[1]:
                    best = (i, t)
            off += n_gemm[i]
        i, t = best
        flops = 2.0 * N * layers[i]["f_in"] * layers[i]["f_out"]
        mult, peak, dtype = _gemm_matrix_core(N, layers[i]["f_in"], layers[i]["f_out"])
        gemm_info = {"kernel": "%s (%s, %dx%dx%d)" % ("k_gemm_bf" if mult > 1 else "k_gemm", tag(i), N, layers[i]["f_in"], layers[i]["f_out"]),
                     "avg_launch_ms": round(t, 4), "tflops": round(flops / t / 1e9, 1), "matrix_core": dtype,
                     "mfma_tflops": round(mult * flops / t / 1e9, 1), "mfma_peak_tflops": peak / 1e12,
                     "mfma_utilisation": round(mult * flops / t / 1e9 / (peak / 1e12), 3)}

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

    detail = {"layers": {tag(i): {"id": name_of(i), "ms": round(time_fn(lambda: run_layer(i, ids[i])), 4),
                                  "spmm_kernel_ms": round(spmm_mean[i], 4) if spmm_mean else None} for i in range(len(layers))},
              "step_ms_median": round(float(np.median(each_ms)), 4), "step_ms_min": round(float(np.min(each_ms)), 4),
              "gemm": gemm_info, "setup_ms": round(setup_ms, 4), "column_panels": None if panels is None else panels.count,
              "column_panels_min_width": None if panels is None else panels.min_width,
              "column_panels_setup_ms": round(panels_ms, 3),
              "dense_tiles": None if tiles is None else {"min_density": args.tiles, "tiles": tiles.n_tiles, "nnz_dense": tiles.nnz_dense,
                                                         "nnz_sparse": tiles.nnz_sparse, "setup_ms": round(tiles_ms, 3), "used": tiles_attached},
              "column_panels_trial_ms": None if panels is None or panels.tune_ms is None else [round(x, 3) for x in panels.tune_ms], "select_model_ms": round(select_model_ms, 4),
              "graph": {"nodes": N, "nnz": nnz, "max_degree": int(np.diff(g.row_ptr).max()), "generate_s": round(gen_s, 2)}}
    if not args.no_sweep:
        sweep, regret, regret_all = {}, {}, {}
        for i, L in enumerate(layers):
            n_ids = 6 if L["kind"] == "gcn" else 4
            sweep[tag(i)] = {name_of(i, cid): round(time_fn(lambda: run_layer(i, cid), 2), 4) for cid in range(n_ids)}
            allowed = [cid for cid, t in enumerate(ctx.select(KIND_GCN if L["kind"] == "gcn" else KIND_GAT, A, L["f_in"], L["f_out"],
                                                              SELECT_MODEL)[1]) if t >= 0]
            regret[tag(i)] = round(sweep[tag(i)][name_of(i)] / min(sweep[tag(i)][name_of(i, cid)] for cid in allowed) - 1.0, 4)
            regret_all[tag(i)] = round(sweep[tag(i)][name_of(i)] / min(sweep[tag(i)].values()) - 1.0, 4)
            run_layer(i, ids[i])  # leave the selected composition's output in place for later layers
        detail["all_compositions_ms"] = sweep
        detail["selector_regret"] = regret                      # against the fastest id the embedding-size rules allow
        detail["selector_regret_vs_all_ids"] = regret_all       # against the fastest of all callable ids
        # the same question to the learned per-primitive models (gradient-boosted trees fitted to MI355X timings)
        learned = {}
        for i, L in enumerate(layers):
            kind = KIND_GCN if L["kind"] == "gcn" else KIND_GAT
            pick, est = ctx.select(kind, A, L["f_in"], L["f_out"], SELECT_LEARNED)
            allowed = [cid for cid, t in enumerate(est) if t >= 0]
            best = min(sweep[tag(i)][name_of(i, cid)] for cid in allowed)
            learned[tag(i)] = {"pick": name_of(i, pick), "regret": round(sweep[tag(i)][name_of(i, pick)] / best - 1.0, 4),
                               "predicted_ms": round(est[pick], 4)}
        detail["selector_learned"] = learned
        L0 = layers[0]
        ts = time.perf_counter()
        idt, _ = ctx.select(KIND_GCN if L0["kind"] == "gcn" else KIND_GAT, A, L0["f_in"], L0["f_out"], SELECT_TIMED)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - ts) * 1e3
        detail["select_timed"] = {"layer": tag(0), "pick": name_of(0, idt), "overhead_ms": round(dt, 3),
                                  "overhead_in_layers": round(dt / detail["layers"][tag(0)]["ms"], 2)}
        # rules + model, with a timed trial only among candidates the model cannot separate (within 15 % of its cheapest)
        auto = {}
        for i, L in enumerate(layers):
            ts = time.perf_counter()
            ida, _ = ctx.select(KIND_GCN if L["kind"] == "gcn" else KIND_GAT, A, L["f_in"], L["f_out"], SELECT_AUTO)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - ts) * 1e3
            allowed_ms = [sweep[tag(i)][name_of(i, cid)] for cid, t in enumerate(ctx.select(KIND_GCN if L["kind"] == "gcn" else KIND_GAT, A, L["f_in"], L["f_out"],
                                                                                             SELECT_MODEL)[1]) if t >= 0]
            auto[tag(i)] = {"pick": name_of(i, ida), "regret": round(sweep[tag(i)][name_of(i, ida)] / min(allowed_ms) - 1.0, 4),
                            "overhead_ms": round(dt, 3), "overhead_in_layers": round(dt / detail["layers"][tag(i)]["ms"], 2)}
        detail["select_auto"] = auto

    # ---- training: backward of the GCN layers in both associations (symmetric pattern: it is its own transpose)
    if not args.no_sweep or args.backward:
        bwd = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gcn":
                continue
            dYt = torch.randn((N, L["f_out"]), device=dev)
            Ymask = outs[i] if L["act"] else None
            t = {nm: round(time_fn(lambda: ctx.gcn_backward(A, A, r, c, src_of(i), Wd[i], dYt, bid, Y=Ymask, activation=L["act"]), 2), 4)
                 for bid, nm in ((0, "BWD_AGG"), (1, "BWD_UPD"))}
            pick, _ = ctx.select_gcn_backward(A, L["f_in"], L["f_out"])
            t["picked"] = ("BWD_AGG", "BWD_UPD")[pick]
            t["regret"] = round(t[t["picked"]] / min(t["BWD_AGG"], t["BWD_UPD"]) - 1.0, 4)
            bwd[tag(i)] = t
            del dYt
        detail["gcn_backward_ms"] = bwd
        gat_bwd = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gat":
                continue
            tp = time.perf_counter()
            t_pos = ctx.transpose_positions(A, A)
            torch.cuda.synchronize()
            pos_ms = (time.perf_counter() - tp) * 1e3
            dYt = torch.randn((N, L["f_out"]), device=dev)
            Ymask = outs[i] if L["act"] else None
            gat_bwd[tag(i)] = {"ms": round(time_fn(lambda: ctx.gat_backward(A, A, t_pos, src_of(i), Wd[i], attd[i][0], attd[i][1], dYt, Y=Ymask,
                                                                            activation=L["act"]), 2), 4),
                               "transpose_positions_setup_ms": round(pos_ms, 3)}
            del dYt, t_pos
        detail["gat_backward_ms"] = gat_bwd

    # ---- K-hop simplified graph convolution on the shapes of the GCN layers (2 hops): both associations
    if not args.no_sweep:
        sgc = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gcn":
                continue
            tmp_out = torch.empty_like(outs[i])   # the outputs of the timed step stay as they are for the parity check below
            sgc[tag(i)] = {nm: round(time_fn(lambda: ctx.sgc_layer(A, r, c, src_of(i), Wd[i], 2, cid, L["act"], out=tmp_out), 2), 4)
                           for cid, nm in ((0, "AGG"), (1, "UPD"))}
            del tmp_out
        detail["sgc_2hop_ms"] = sgc
        tag2 = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gcn":
                continue
            W3 = torch.randn((3 * L["f_in"], L["f_out"]), device=dev) * 0.05
            tmp_out = torch.empty_like(outs[i])
            tag2[tag(i)] = {nm: round(time_fn(lambda: ctx.tagcn_layer(A, r, c, src_of(i), W3, 2, cid, L["act"], out=tmp_out), 2), 4)
                            for cid, nm in ((0, "AGG"), (1, "UPD"))}
            dYt = torch.randn((N, L["f_out"]), device=dev)
            for bid, nm in ((0, "BWD_AGG"), (1, "BWD_UPD")):
                tag2[tag(i)][nm] = round(time_fn(lambda: ctx.tagcn_backward(A, A, r, c, src_of(i), W3, 2, dYt, bid, Y=outs[i] if L["act"] else None,
                                                                           activation=L["act"]), 2), 4)
            pick, _ = ctx.select_khop_backward(A, L["f_in"], L["f_out"], 2, True)
            tag2[tag(i)]["backward_picked"] = ("BWD_AGG", "BWD_UPD")[pick]
            tag2[tag(i)]["backward_regret"] = round(tag2[tag(i)][tag2[tag(i)]["backward_picked"]] / min(tag2[tag(i)]["BWD_AGG"], tag2[tag(i)]["BWD_UPD"]) - 1.0, 4)
            del W3, tmp_out, dYt
        detail["tagcn_2hop_ms"] = tag2

    # ---- GATv2 on the shapes of the GAT layers (separate W_l and W_r): reuse and recompute
    if not args.no_sweep:
        v2 = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gat":
                continue
            Wl2 = torch.randn_like(Wd[i]) * 0.05
            att2 = torch.randn((L["f_out"],), device=dev) * 0.1
            tmp_out = torch.empty_like(outs[i])
            v2[tag(i)] = {nm: round(time_fn(lambda: ctx.gatv2_layer(A, src_of(i), Wl2, Wd[i], att2, cid, 0.2, L["act"], out=tmp_out), 2), 4)
                          for cid, nm in ((0, "REUSE"), (1, "RECOMP"))}
            t_pos = ctx.transpose_positions(A, A)
            dYt = torch.randn((N, L["f_out"]), device=dev)
            v2[tag(i)]["BACKWARD"] = round(time_fn(lambda: ctx.gatv2_backward(A, A, t_pos, src_of(i), Wl2, Wd[i], att2, dYt, Y=outs[i] if L["act"] else None,
                                                                              activation=L["act"]), 2), 4)
            del Wl2, att2, tmp_out, t_pos, dYt
        detail["gatv2_ms"] = v2
        # key-query attention (dot-product scores, 64-column queries and keys) on the same shapes: reuse and recompute
        kq = {}
        for i, L in enumerate(layers):
            if L["kind"] != "gat":
                continue
            Wq2, Wk2 = torch.randn((L["f_in"], 64), device=dev) * 0.05, torch.randn((L["f_in"], 64), device=dev) * 0.05
            tmp_out = torch.empty_like(outs[i])
            kq[tag(i)] = {nm: round(time_fn(lambda: ctx.dotgat_layer(A, src_of(i), Wq2, Wk2, Wd[i], 0.125, cid, L["act"], out=tmp_out), 2), 4)
                          for cid, nm in ((0, "REUSE"), (1, "RECOMP"))}
            t_pos = ctx.transpose_positions(A, A)
            dYt = torch.randn((N, L["f_out"]), device=dev)
            kq[tag(i)]["BACKWARD"] = round(time_fn(lambda: ctx.dotgat_backward(A, A, t_pos, src_of(i), Wq2, Wk2, Wd[i], 0.125, dYt,
                                                                               Y=outs[i] if L["act"] else None, activation=L["act"]), 2), 4)
            del Wq2, Wk2, tmp_out, t_pos, dYt
        detail["key_query_attention_ms"] = kq

    # ---- one training iteration of the GCN stack of the workload (the layers whose input is X or the previous layer):
    # forward with the selected compositions, backward with the associations the cost model picks; the first layer needs no dX
    if not args.no_sweep or args.backward:
        chain = [i for i, L in enumerate(layers) if L["kind"] == "gcn" and (L["src"] == "X" or L["src"] in (-1, i - 1))]
        chain = chain[:2] if len(chain) >= 2 and layers[chain[1]]["src"] in (-1, chain[0]) else chain[:1]
        bwd_pick = {i: ctx.select_gcn_backward(A, layers[i]["f_in"], layers[i]["f_out"], want_dx=(i != chain[0]))[0] for i in chain}
        dLast = torch.randn((N, layers[chain[-1]]["f_out"]), device=dev)

        def train_step():
            for i in chain:
                run_layer(i, ids[i])
            grad = dLast
            for i in reversed(chain):
                L = layers[i]
                dX, _ = ctx.gcn_backward(A, A, r, c, src_of(i), Wd[i], grad, bwd_pick[i], Y=outs[i] if L["act"] else None, activation=L["act"],
                                         want_dx=(i != chain[0]))
                grad = dX
        detail["gcn_training_iteration"] = {"layers": [tag(i) for i in chain], "ms": round(time_fn(train_step, 3), 4),
                                            "backward": {tag(i): ("BWD_AGG", "BWD_UPD")[bwd_pick[i]] for i in chain}}
        del dLast

    # ---- ceiling of the neighbour gather: the same SpMM kernel (value-less, F = 256) on a synthetic pattern whose
    # columns span only 8192 rows of the gathered matrix, so every 128-byte feature slice (1 MB) stays in one L2.
    # The rate it reaches bounds what any SpMM of this shape can consume, whatever the graph.
    if not args.no_gather_probe:
        from paper_2306_15155_amd import SPMM_PATTERN
        n_c, n_r, d, f_p = 8192, 65536, 512, 256
        rng = np.random.default_rng(7)
        start = rng.integers(0, n_c, n_r, dtype=np.int64)
        stride = rng.integers(0, n_c // 2, n_r, dtype=np.int64) * 2 + 1  # odd stride modulo a power of two: d distinct columns
        cols = ((start[:, None] + stride[:, None] * np.arange(d, dtype=np.int64)[None, :]) % n_c).astype(np.int32)
        cols.sort(axis=1)
        p_rp = torch.arange(0, (n_r + 1) * d, d, dtype=torch.int32, device=dev)
        p_ci = torch.from_numpy(cols.reshape(-1)).to(dev)
        p_B = torch.rand((n_c, f_p), device=dev)
        p_C = torch.empty((n_r, f_p), device=dev)
        p_A = csr_struct(n_r, n_c, p_rp, p_ci)
        p_ms = time_fn(lambda: ctx.spmm(p_A, SPMM_PATTERN, p_B, out=p_C), 5)
        p_rate = n_r * d * 4.0 * f_p / p_ms / 1e6
        detail["l2_resident_gather_probe"] = {"pattern": "%d x %d, %d entries per row" % (n_r, n_c, d), "f": f_p, "ms": round(p_ms, 4),
                                              "gather_GBps": round(p_rate, 1)}
        if roofline is not None:
            roofline["gather_frac_of_l2_resident_rate"] = round(roofline["gather_GBps_no_reuse"] / p_rate, 3)
        del p_rp, p_ci, p_B, p_C, cols

    # ---- SDDMM instances and the edge softmax as stand-alone calls on this graph: time by events, algorithmic bytes
    # (4 B column index + 4 B written per stored entry, the row pointers, the two node vectors), fraction of the HBM peak.
    # Each stored entry gathers one 4-byte scalar of a node vector that does not fit the 32 KB vector caches, i.e. one
    # 128-byte line from the L2: nnz * 128 B over the 64 B/clk/CU fill path of 256 CUs is the floor quoted beside it.
    if nnz >= (1 << 22):
        s_l = torch.rand(N, device=dev) - 0.5
        s_r = torch.rand(N, device=dev) - 0.5
        e_buf = torch.rand(nnz, device=dev) - 0.5
        a_buf = torch.empty(nnz, device=dev)
        ctx.ws.ensure(ctx.sparse_workspace(A, 1))
        fill_ms = nnz * 128.0 / (256 * 64 * 2.4e9) * 1e3
        edge = []
        for kname, fn, by in (("k_sddmm_norm (Eq. 4)", lambda: ctx.gcn_precompute(A, r, c), 8.0 * nnz + 4.0 * (N + 1) + 8.0 * N),
                              ("k_score (Eq. 2, k = 1)", lambda: ctx.sddmm_score(A, s_l, s_r), 8.0 * nnz + 4.0 * (N + 1) + 8.0 * N),
                              ("edge softmax: k_softmax_stats + k_softmax_fixup + k_softmax_alpha", lambda: ctx.edge_softmax(A, e_buf, out=a_buf),
                               12.0 * nnz + 8.0 * (N + 1) + 8.0 * N)):
            t = time_fn(fn, 5)
            edge.append({"kernel": kname, "bound": "hbm", "avg_call_ms": round(t, 4), "algorithmic_bytes": int(by), "achieved": round(by / t / 1e6, 1),
                         "peak": 8000.0, "unit": "GB/s", "frac": round(by / t / 1e6 / 8000.0, 4),
                         "line_fill_floor_ms": round(fill_ms, 4) if "softmax" not in kname else None})
        detail["edge_kernels"] = edge
        del s_l, s_r, e_buf, a_buf

    # ---- launch-bound workloads: the same step captured once in a HIP graph and replayed
    if N <= 50_000:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        with torch.cuda.graph(graph):
            step()
        detail["graph_replay_ms_per_layer"] = round(time_fn(graph.replay, 50) / len(layers), 5)
        detail["eager_ms_per_layer"] = round(time_fn(step, 50) / len(layers), 5)

    # ---- CPU baseline: the fp64 oracle as it stands, one thread, on a bounded sample of output rows of every layer,
    # extrapolated by row count.  Hidden inputs are seeded stand-ins so that nothing from the GPU reaches the oracle.
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        step()  # the outputs checked below are those of the timed configuration, whatever ran in between
        torch.cuda.synchronize()
        budget_rows = 72_000 if N > 50_000 else N * len(layers)
        n_s = min(N, max(500, budget_rows // len(layers)))
        if args.workload == "c3_rmat2450k":
            n_s = 3000
        rows = np.sort(synth.distinct_nodes(seed, 40, N, n_s)) if n_s < N else None
        scale = N / float(n_s)
        t_cpu, t_omp, errs = 0.0, 0.0, {}
        sel = slice(None) if rows is None else torch.from_numpy(rows.astype(np.int64)).to(dev)
        for i, L in enumerate(layers):
            from_x = L["src"] == "X"
            Xin = X if from_x else synth.uniform(seed, 400 + i, (N, L["f_in"]), 0.0, 1.0)
            tc = time.perf_counter()
            if L["kind"] == "gcn":
                ref = oracle.gcn_layer(N, N, g.row_ptr, g.col_idx, Xin, Ws[i], L["act"], rows=rows)
            else:
                ref = oracle.gat_layer(N, N, g.row_ptr, g.col_idx, Xin, Ws[i], att[i][0], att[i][1], 0.2, L["act"], rows=rows)
            t_cpu += time.perf_counter() - tc
            tc = time.perf_counter()  # the same source built with OpenMP (rows are independent), every host thread
            if L["kind"] == "gcn":
                oracle.gcn_layer(N, N, g.row_ptr, g.col_idx, Xin, Ws[i], L["act"], rows=rows, omp=True)
            else:
                oracle.gat_layer(N, N, g.row_ptr, g.col_idx, Xin, Ws[i], att[i][0], att[i][1], 0.2, L["act"], rows=rows, omp=True)
            t_omp += time.perf_counter() - tc
            if from_x:  # same inputs as the timed GPU layer: a full-size parity check of what was just timed
                got = outs[i][sel].cpu().numpy()
                errs[tag(i)] = float(np.max(np.abs(got - ref) / (1.0 + np.abs(ref))))
        cpu = {"value": round(t_cpu * scale * 1e3 / len(layers), 1), "unit": "ms per layer (extrapolated by row count)",
               "cores": oracle.threads(False), "kind": "oracle",
               "sample": "%d uniformly drawn output rows of each of the %d layers (of %d rows), %.1f s of CPU work" % (n_s, len(layers), N, t_cpu),
               "all_threads": {"value": round(t_omp * scale * 1e3 / len(layers), 1), "cores": oracle.threads(True),
                               "note": "same oracle source compiled with OpenMP over output rows, same sample"}}
        detail["sampled_parity_max_scaled_err"] = errs

    desc = ", ".join("%s %d->%d" % (L["kind"].upper(), L["f_in"], L["f_out"]) for L in layers)
    out = {"metric": "ms per GCN/GAT layer (mean over the %d layers of one step)" % len(layers), "value": round(ms_per_layer, 4),
           "unit": "ms/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": args.workload,
                      "graph": {"rmat": "R-MAT(0.57,0.19,0.19,0.05) symmetrised + self loops", "er": "G(n,M) + self loops",
                                "grid": "square grid, links kept with probability %s, + self loops" % wl.get("keep")}[wl["graph"]],
                      "nodes": N, "nnz": nnz, "layers": desc, "compositions": [name_of(i) for i in range(len(layers))]},
           "roofline": roofline, "cpu_baseline": cpu, "detail": detail}
    torch.cuda.synchronize()
    ctx.close()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; pass --gpus 1 (there is no multi-GPU path to measure)",
              file=sys.stderr)
        sys.exit(2)
    out = headline(args)
    if not args.no_extras:
        import numpy as np
        import torch

        import oracle
        import synth
        torch.cuda.empty_cache()
        t0 = time.time()
        out["detail"]["other_workloads"] = run_extras(args, torch, np, synth, oracle)
        out["detail"]["other_workloads"]["seconds"] = round(time.time() - t0, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
