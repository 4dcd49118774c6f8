"""GPU parity of the backward pass (through the C ABI) against the fp64 chain-rule oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2306_15155_amd import ACT_NONE, ACT_RELU, GCN_BWD_AGG, GCN_BWD_UPD, Context

from gpu_util import DeviceCSR, assert_close, dev, hub_and_empty_graph, rect_block

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = Context(0)
    yield c
    c.close()


GRAPHS = {
    "er": lambda: synth.erdos_renyi(41, 3000, 40_000),                 # symmetric, several chunks
    "rmat_hub": lambda: synth.rmat(42, 5000, 150_000),                 # skewed, rows crossing chunk boundaries
    "hub_empty": lambda: hub_and_empty_graph(43, 2500, 30_000, 1800, 40),  # not symmetric, empty rows, no self loops
    "rect": lambda: rect_block(44, 700, 4000, 9),                      # bipartite block
    "dense_small": lambda: synth.erdos_renyi(45, 600, 60_000),         # every row gathered often: slice-major path
}


def _inputs(g, f_in, f_out, seed):
    X = synth.uniform(seed, 10, (g.n_cols, f_in))
    W = synth.glorot(seed, 11, f_in, f_out)
    dY = synth.normal(seed, 12, (g.n_rows, f_out), 0.0, 1.0)
    return X, W, dY


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("widths", [(40, 24), (24, 40), (100, 41), (33, 130)])
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_gcn_backward_matches_chain_rule(ctx, name, widths, act):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out = widths
    X, W, dY = _inputs(g, f_in, f_out, 50 + f_in)
    Y = None
    if act == ACT_RELU:  # the mask comes from the forward output; both sides get the oracle's, rounded to fp32
        Y = oracle.gcn_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, 1).astype(np.float32)
    want_dx, want_dw = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=act)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    Yd = None if Y is None else dev(Y)
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        dX, dW = ctx.gcn_backward(A.s, At.s, r, c, dev(X), dev(W), dev(dY), bwd, Y=Yd, activation=act)
        assert_close(dX, want_dx, what=f"dX bwd {bwd}")
        assert_close(dW, want_dw, what=f"dW bwd {bwd}")
    # weight gradient only (first layer of a model)
    none, dW = ctx.gcn_backward(A.s, At.s, r, c, dev(X), dev(W), dev(dY), GCN_BWD_AGG, Y=Yd, activation=act, want_dx=False)
    assert none is None
    assert_close(dW, want_dw, what="dW only")


def test_gcn_backward_with_saved_aggregate_and_strided_operands(ctx):
    g = synth.rmat(46, 4000, 100_000)
    f_in, f_out = 52, 96
    X, W, dY = _inputs(g, f_in, f_out, 60)
    r64 = 1.0 / np.sqrt(np.maximum(np.diff(g.row_ptr), 1).astype(np.float64))
    U = oracle.row_broadcast(r64, oracle.spmm(g.row_ptr, g.col_idx, r64[g.col_idx], X)).astype(np.float32)  # symmetric: c = r
    want_dx, want_dw = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY)
    A = DeviceCSR(g)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    # operands as column slices of wider buffers (leading dimension > width, odd offsets)
    Xw = torch.zeros((g.n_cols, f_in + 7), device="cuda:0"); Xw[:, 3:3 + f_in] = dev(X)
    dYw = torch.zeros((g.n_rows, f_out + 5), device="cuda:0"); dYw[:, 1:1 + f_out] = dev(dY)
    Uw = torch.zeros((g.n_rows, f_in + 2), device="cuda:0"); Uw[:, 1:1 + f_in] = dev(U)
    dX, dW = ctx.gcn_backward(A.s, A.s, r, c, Xw[:, 3:3 + f_in], dev(W), dYw[:, 1:1 + f_out], GCN_BWD_UPD, U_saved=Uw[:, 1:1 + f_in])
    assert_close(dX, want_dx, what="dX saved U")
    assert_close(dW, want_dw, what="dW saved U")
    dX, dW = ctx.gcn_backward(A.s, A.s, r, c, Xw[:, 3:3 + f_in], dev(W), dYw[:, 1:1 + f_out], GCN_BWD_AGG)
    assert_close(dX, want_dx, what="dX strided")
    assert_close(dW, want_dw, what="dW strided")


def test_gcn_backward_on_a_dense_tile_split(ctx):
    """The transposed aggregation of the backward pass is a value-less SpMM too: with a tile split attached to the (here
    symmetric) pattern it takes the split path, and the gradients still match the chain rule."""
    from paper_2306_15155_amd import Tiles, csr_struct
    g = synth.rmat(48, 5000, 150_000)
    f_in, f_out = 72, 96
    X, W, dY = _inputs(g, f_in, f_out, 61)
    Y = oracle.gcn_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, 1).astype(np.float32)
    want_dx, want_dw = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=ACT_RELU)
    A = DeviceCSR(g)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0
    At = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        dX, dW = ctx.gcn_backward(At, At, r, c, dev(X), dev(W), dev(dY), bwd, Y=dev(Y), activation=ACT_RELU)
        assert_close(dX, want_dx, what=f"dX bwd {bwd}")
        assert_close(dW, want_dw, what=f"dW bwd {bwd}")
    T.close()


def test_gcn_backward_argument_checks(ctx):
    import ctypes
    from paper_2306_15155_amd import binding
    g = synth.erdos_renyi(47, 200, 600)
    A = DeviceCSR(g)
    X, W, dY = (torch.zeros(s, device="cuda:0") for s in ((200, 8), (8, 4), (200, 4)))
    dX, dW, ws = torch.zeros((200, 8), device="cuda:0"), torch.zeros((8, 4), device="cuda:0"), torch.zeros(1 << 22, dtype=torch.uint8, device="cuda:0")
    r = torch.ones(200, device="cuda:0")
    L = binding.lib()

    def call(bwd=0, act=0, Y=None, dXp=dX, wsb=ws.numel(), At=A.s):
        return L.sensei_gcn_backward(ctx._h, ctypes.byref(A.s), ctypes.byref(At), r.data_ptr(), r.data_ptr(), binding.mat_struct(X),
                                     binding.mat_struct(W), None if Y is None else Y.data_ptr(), 4, binding.mat_struct(dY), act, None, 0,
                                     dXp.data_ptr(), 8, dW.data_ptr(), 4, bwd, ws.data_ptr(), wsb, None)

    assert call() == 0
    assert call(bwd=2) == 2                       # unknown association
    assert call(act=1) == 1                       # ReLU without the forward output
    assert call(wsb=1024) == 3                    # workspace too small
    assert call(dXp=X) == 1                       # output aliases an input
    g2 = synth.erdos_renyi(48, 100, 300)
    assert call(At=DeviceCSR(g2).s) == 1          # transposed pattern of another shape
    torch.cuda.synchronize()


# ------------------------------------------------------------------ K-hop layer

SQUARE = ("er", "rmat_hub", "hub_empty", "dense_small")


@pytest.mark.parametrize("name", SQUARE)
@pytest.mark.parametrize("widths", [(40, 24), (24, 40), (33, 130)])
@pytest.mark.parametrize("k_hops", [1, 2, 3])
def test_sgc_backward_matches_chain_rule(ctx, name, widths, k_hops):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out = widths
    X, W, dY = _inputs(g, f_in, f_out, 80 + f_in + k_hops)
    for act in (ACT_NONE, ACT_RELU):
        Y = None
        if act == ACT_RELU:
            Y = oracle.sgc_layer(g.n_rows, g.row_ptr, g.col_idx, X, W, k_hops, 1).astype(np.float32)
        want_dx, want_dw = oracle.sgc_backward(g.n_rows, g.row_ptr, g.col_idx, X, W, k_hops, dY, Y=Y, act=act)
        A, At = DeviceCSR(g), DeviceCSR(gt)
        dr, dc = ctx.degrees(A.s)
        r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
        Yd = None if Y is None else dev(Y)
        for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
            dX, dW = ctx.sgc_backward(A.s, At.s, r, c, dev(X), dev(W), k_hops, dev(dY), bwd, Y=Yd, activation=act)
            assert_close(dX, want_dx, what=f"dX k={k_hops} bwd {bwd} act {act}")
            assert_close(dW, want_dw, what=f"dW k={k_hops} bwd {bwd} act {act}")
    none, dW = ctx.sgc_backward(A.s, At.s, r, c, dev(X), dev(W), k_hops, dev(dY), GCN_BWD_UPD, Y=Yd, activation=ACT_RELU, want_dx=False)
    assert none is None
    assert_close(dW, want_dw, what="dW only")


def test_sgc_backward_one_hop_is_the_gcn_backward_and_split_patterns_agree(ctx):
    """One hop runs exactly the kernels of the GCN backward (bit-equal outputs); with a tile split and with column panels
    attached to the symmetric pattern the hops take those paths and still match the chain rule."""
    from paper_2306_15155_amd import Panels, Tiles, csr_struct
    g = synth.rmat(49, 5000, 150_000)
    f_in, f_out = 72, 48
    X, W, dY = _inputs(g, f_in, f_out, 90)
    A = DeviceCSR(g)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        a = ctx.gcn_backward(A.s, A.s, r, c, dev(X), dev(W), dev(dY), bwd)
        a = [t.clone() for t in a]
        b = ctx.sgc_backward(A.s, A.s, r, c, dev(X), dev(W), 1, dev(dY), bwd)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    want_dx, want_dw = oracle.sgc_backward(g.n_rows, g.row_ptr, g.col_idx, X, W, 3, dY)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0
    P = Panels(ctx, A.s, 4)
    for At in (csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T), csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, P)):
        for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
            dX, dW = ctx.sgc_backward(At, At, r, c, dev(X), dev(W), 3, dev(dY), bwd)
            assert_close(dX, want_dx, what=f"dX bwd {bwd}")
            assert_close(dW, want_dw, what=f"dW bwd {bwd}")
    T.close()
    P.close()


def test_sgc_backward_argument_checks(ctx):
    g = synth.erdos_renyi(47, 200, 600)
    A = DeviceCSR(g)
    X, W, dY = (torch.zeros(s, device="cuda:0") for s in ((200, 8), (8, 4), (200, 4)))
    r = torch.ones(200, device="cuda:0")
    ctx.sgc_backward(A.s, A.s, r, r, X, W, 2, dY, GCN_BWD_AGG)
    with pytest.raises(RuntimeError):
        ctx.sgc_backward(A.s, A.s, r, r, X, W, 0, dY, GCN_BWD_AGG)      # at least one hop
    with pytest.raises(RuntimeError):
        ctx.sgc_backward(A.s, A.s, r, r, X, W, 2, dY, 2)                # two associations
    with pytest.raises(RuntimeError):
        ctx.sgc_backward(A.s, A.s, r, r, X, W, 2, dY, GCN_BWD_AGG, activation=ACT_RELU)   # ReLU without the forward output
    gr = rect_block(44, 70, 400, 9)
    Ar, Art = DeviceCSR(gr), DeviceCSR(synth.transpose(gr))
    with pytest.raises(RuntimeError):                                     # hops need a square pattern
        ctx.sgc_backward(Ar.s, Art.s, torch.ones(70, device="cuda:0"), torch.ones(400, device="cuda:0"), torch.zeros((400, 8), device="cuda:0"), W, 2,
                         torch.zeros((70, 4), device="cuda:0"), GCN_BWD_AGG)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ K-hop layer with a weight block per hop (TAGCN)

def _tagcn_inputs(g, f_in, f_out, k_hops, seed):
    X = synth.uniform(seed, 10, (g.n_cols, f_in))
    W = np.concatenate([synth.glorot(seed, 20 + k, f_in, f_out) for k in range(k_hops + 1)], axis=0)
    dY = synth.normal(seed, 12, (g.n_rows, f_out), 0.0, 1.0)
    return X, W, dY


@pytest.mark.parametrize("name", SQUARE)
@pytest.mark.parametrize("widths", [(40, 24), (24, 40), (33, 130), (41, 7)])
@pytest.mark.parametrize("k_hops", [0, 1, 2, 3])
def test_tagcn_backward_matches_chain_rule(ctx, name, widths, k_hops):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out = widths
    X, W, dY = _tagcn_inputs(g, f_in, f_out, k_hops, 120 + f_in + k_hops)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    for act in (ACT_NONE, ACT_RELU):
        Y = None
        if act == ACT_RELU:
            Y = oracle.tagcn_layer(g.n_rows, g.row_ptr, g.col_idx, X, W, k_hops, 1).astype(np.float32)
        want_dx, want_dw = oracle.tagcn_backward(g.n_rows, g.row_ptr, g.col_idx, X, W, k_hops, dY, Y=Y, act=act)
        Yd = None if Y is None else dev(Y)
        for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
            dX, dW = ctx.tagcn_backward(A.s, At.s, r, c, dev(X), dev(W), k_hops, dev(dY), bwd, Y=Yd, activation=act)
            assert_close(dX, want_dx, what=f"dX k={k_hops} bwd {bwd} act {act}")
            assert_close(dW, want_dw, what=f"dW k={k_hops} bwd {bwd} act {act}")
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        none, dW = ctx.tagcn_backward(A.s, At.s, r, c, dev(X), dev(W), k_hops, dev(dY), bwd, Y=Yd, activation=ACT_RELU, want_dx=False)
        assert none is None
        assert_close(dW, want_dw, what=f"dW only, bwd {bwd}")


def test_tagcn_backward_on_split_patterns_and_strided_operands(ctx):
    """With a tile split and with column panels attached to the symmetric pattern the hops take those paths; operands and results
    with leading dimensions larger than their widths."""
    from paper_2306_15155_amd import Panels, Tiles, csr_struct
    g = synth.rmat(49, 5000, 150_000)
    f_in, f_out, K = 72, 48, 2
    X, W, dY = _tagcn_inputs(g, f_in, f_out, K, 130)
    A = DeviceCSR(g)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    Y = oracle.tagcn_layer(g.n_rows, g.row_ptr, g.col_idx, X, W, K, 1).astype(np.float32)
    want_dx, want_dw = oracle.tagcn_backward(g.n_rows, g.row_ptr, g.col_idx, X, W, K, dY, Y=Y, act=1)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0
    P = Panels(ctx, A.s, 4)
    Xs = torch.zeros((g.n_cols, f_in + 5), device="cuda:0")
    Xs[:, :f_in] = dev(X)
    dYs = torch.zeros((g.n_rows, f_out + 3), device="cuda:0")
    dYs[:, :f_out] = dev(dY)
    for At in (csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T), csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, P)):
        for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
            dX, dW = ctx.tagcn_backward(At, At, r, c, Xs[:, :f_in], dev(W), K, dYs[:, :f_out], bwd, Y=dev(Y), activation=ACT_RELU)
            assert_close(dX, want_dx, what=f"dX bwd {bwd}")
            assert_close(dW, want_dw, what=f"dW bwd {bwd}")
    T.close()
    P.close()


def test_k_hop_backward_degenerate_patterns(ctx):
    """A pattern without entries (A^ = 0: only the hop-free term of TAGCN is left, the SGC layer and its gradients vanish) and a
    pattern without nodes (the weight gradient, a sum over no nodes, is zero)."""
    n, f_in, f_out, K = 50, 12, 7, 2
    none = np.empty(0, np.int32)
    g = synth.build_csr(n, n, none, none, False, False)
    X, W, dY = _tagcn_inputs(g, f_in, f_out, K, 140)
    A = DeviceCSR(g)
    ones = torch.ones(n, device="cuda:0")
    want_dx, want_dw = oracle.tagcn_backward(n, g.row_ptr, g.col_idx, X, W, K, dY)
    assert np.abs(want_dw[f_in:]).max() == 0.0 and np.abs(want_dw[:f_in]).max() > 0.0
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        dX, dW = ctx.tagcn_backward(A.s, A.s, ones, ones, dev(X), dev(W), K, dev(dY), bwd)
        assert_close(dX, want_dx, what=f"tagcn dX, bwd {bwd}")
        assert_close(dW, want_dw, what=f"tagcn dW, bwd {bwd}")
        dX, dW = ctx.sgc_backward(A.s, A.s, ones, ones, dev(X), dev(W[:f_in]), K, dev(dY), bwd)
        assert float(dX.abs().max()) == 0.0 and float(dW.abs().max()) == 0.0
    g0 = synth.build_csr(0, 0, none, none, False, False)
    A0 = DeviceCSR(g0)
    e = torch.empty(0, device="cuda:0")
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        for fn, Wd in ((ctx.tagcn_backward, dev(W)), (ctx.sgc_backward, dev(W[:f_in]))):
            dX, dW = fn(A0.s, A0.s, e, e, torch.empty((0, f_in), device="cuda:0"), Wd, K, torch.empty((0, f_out), device="cuda:0"), bwd)
            assert dX.shape == (0, f_in) and dW.shape == Wd.shape and float(dW.abs().max()) == 0.0
    torch.cuda.synchronize()


def test_khop_backward_selection_follows_the_widths(ctx):
    """The cost model's pick between the two associations of the K-hop backward: the hops run at the narrower width, for both layers,
    and the pick is the association that is measured faster where the widths differ by a factor of eight."""
    import time
    g = synth.rmat(99, 60_000, 3_000_000)
    A = DeviceCSR(g)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    for f_in, f_out, want in ((128, 16, GCN_BWD_AGG), (16, 128, GCN_BWD_UPD)):
        for tagcn in (False, True):
            pick, est = ctx.select_khop_backward(A.s, f_in, f_out, 2, tagcn)
            assert pick == want and len(est) == 2 and min(est) > 0, (f_in, f_out, tagcn, pick, est)
            X = torch.rand((g.n_cols, f_in), device="cuda:0")
            W = torch.rand(((3 if tagcn else 1) * f_in, f_out), device="cuda:0")
            dY = torch.randn((g.n_rows, f_out), device="cuda:0")
            fn = ctx.tagcn_backward if tagcn else ctx.sgc_backward
            ms = []
            for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
                fn(A.s, A.s, r, c, X, W, 2, dY, bwd)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(3):
                    fn(A.s, A.s, r, c, X, W, 2, dY, bwd)
                torch.cuda.synchronize()
                ms.append((time.perf_counter() - t0) / 3)
            assert ms[pick] <= 1.1 * min(ms), (f_in, f_out, tagcn, pick, ms)
    with pytest.raises(RuntimeError):
        ctx.select_khop_backward(A.s, 16, 16, -1, True)


def test_tagcn_backward_argument_checks(ctx):
    g = synth.erdos_renyi(47, 200, 600)
    A = DeviceCSR(g)
    X, W, dY = (torch.zeros(s, device="cuda:0") for s in ((200, 8), (24, 4), (200, 4)))
    r = torch.ones(200, device="cuda:0")
    ctx.tagcn_backward(A.s, A.s, r, r, X, W, 2, dY, GCN_BWD_AGG)
    with pytest.raises(RuntimeError):
        ctx.tagcn_backward(A.s, A.s, r, r, X, W, 1, dY, GCN_BWD_AGG)     # W holds three blocks, not two
    with pytest.raises(RuntimeError):
        ctx.tagcn_backward(A.s, A.s, r, r, X, W, 2, dY, 2)               # two associations
    with pytest.raises(RuntimeError):
        ctx.tagcn_backward(A.s, A.s, r, r, X, W, 2, dY, GCN_BWD_UPD, activation=ACT_RELU)   # ReLU without the forward output
    gr = rect_block(44, 70, 400, 9)
    Ar, Art = DeviceCSR(gr), DeviceCSR(synth.transpose(gr))
    with pytest.raises(RuntimeError):                                      # hops need a square pattern
        ctx.tagcn_backward(Ar.s, Art.s, torch.ones(70, device="cuda:0"), torch.ones(400, device="cuda:0"), torch.zeros((400, 8), device="cuda:0"), W, 2,
                           torch.zeros((70, 4), device="cuda:0"), GCN_BWD_AGG)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ GAT

@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("widths", [(40, 24), (24, 40), (70, 41), (33, 130)])
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_gat_backward_matches_chain_rule(ctx, name, widths, act):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out = widths
    X, W, dY = _inputs(g, f_in, f_out, 70 + f_in)
    a_l, a_r = synth.normal(71, 20, (f_out,), 0.0, 0.3), synth.normal(71, 21, (f_out,), 0.0, 0.3)
    Y = None
    if act == ACT_RELU:
        Y = oracle.gat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1).astype(np.float32)
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY, Y=Y, slope=0.2, act=act)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    pos = ctx.transpose_positions(A.s, At.s)
    # the map really is the transposition: entry k = (i, j) of A sits at row j, column i of At
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.row_ptr))
    p = pos.cpu().numpy()[:g.nnz]
    assert np.array_equal(gt.col_idx[p], rows) and np.array_equal(np.sort(p), np.arange(g.nnz))
    got = ctx.gat_backward(A.s, At.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY), Y=None if Y is None else dev(Y), activation=act)
    for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
        assert_close(gpu, ref, what=what)


def test_gat_backward_other_slope_and_weight_gradient_only(ctx):
    g = synth.rmat(72, 3000, 60_000)
    f_in, f_out = 48, 64
    X, W, dY = _inputs(g, f_in, f_out, 73)
    a_l, a_r = synth.normal(73, 20, (f_out,), 0.0, 0.5), synth.normal(73, 21, (f_out,), 0.0, 0.5)
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY, slope=0.05)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)  # symmetric pattern: its own transpose
    none, dW, dal, dar = ctx.gat_backward(A.s, A.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY), neg_slope=0.05, want_dx=False)
    assert none is None
    assert_close(dW, want[1], what="dW")
    assert_close(dal, want[2], what="da_l")
    assert_close(dar, want[3], what="da_r")


@pytest.mark.parametrize("widths", [(72, 96), (40, 130), (48, 24)])
def test_gat_backward_on_a_dense_tile_split(ctx, widths):
    """With a tile split attached to the pattern, the per-entry products <dP_i, Theta_j> of the entries inside kept tiles come
    from one dense product per tile and the others from the remainder; the gradients still match the chain rule.  The last
    width is below the split's minimum and takes the plain path."""
    from paper_2306_15155_amd import Tiles, csr_struct
    g = synth.rmat(74, 5000, 150_000)
    f_in, f_out = widths
    X, W, dY = _inputs(g, f_in, f_out, 75)
    a_l, a_r = synth.normal(75, 20, (f_out,), 0.0, 0.3), synth.normal(75, 21, (f_out,), 0.0, 0.3)
    Y = oracle.gat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1).astype(np.float32)
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY, Y=Y, slope=0.2, act=ACT_RELU)
    A = DeviceCSR(g)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0 and T.nnz_sparse > 0
    Ah = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    pos = ctx.transpose_positions(A.s, A.s)  # symmetric pattern: its own transpose
    # split on the pattern only, on the transposed pattern only (alpha^T . dP takes it), on both; the last one twice, so that
    # the second call meets the workspace the first one left behind
    for how, first, second in (("A", Ah, A.s), ("At", A.s, Ah), ("both", Ah, Ah), ("both again", Ah, Ah)):
        got = ctx.gat_backward(first, second, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY), Y=dev(Y), activation=ACT_RELU)
        for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
            assert_close(gpu, ref, what=f"{what}, split on {how}")
    T.close()


def test_gat_backward_on_a_dense_tile_split_with_large_logits(ctx):
    """Logits of up to +-24: the coefficients the transposed tile kernel forms are exp(e - max of the column's softmax row) / sum,
    never larger than one, whichever side of the split holds the row's maximum.  The large part of every logit is exact in fp32
    by construction (feature 0 holds small integers and only a_r sees it: W[0, 0] = 1, a_r[0] = 8, a_l[0] = 0, so
    s_r[j] = 8 X[j, 0] + terms below 1), which keeps the comparison about the kernels: with logits of that size formed by rounded
    dot products, fp32 input rounding alone would leave more than 1e-4 whatever the kernel does.  Both paths, the plain one and
    the split one, are held to the fp32 bar against the fp64 oracle."""
    from paper_2306_15155_amd import Tiles, csr_struct
    g = synth.rmat(78, 5000, 150_000)
    f_in, f_out = 32, 128
    X, W, dY = _inputs(g, f_in, f_out, 79)
    a_l, a_r = synth.normal(79, 20, (f_out,), 0.0, 0.03), synth.normal(79, 21, (f_out,), 0.0, 0.03)
    X[:, 0] = np.array([-3.0, -2.0, -1.0, 1.0, 2.0, 3.0], dtype=np.float32)[(np.arange(g.n_cols) * 7) % 6]
    W[0, :] = 0.0
    W[:, 0] = 0.0
    W[0, 0] = 1.0
    a_l[0], a_r[0] = 0.0, 8.0
    Th = X.astype(np.float64) @ W.astype(np.float64)
    s_l, s_r = Th @ a_l.astype(np.float64), Th @ a_r.astype(np.float64)
    assert np.abs(s_r).max() > 20.0 and np.abs(s_r).min() > 7.0 and np.abs(s_l).max() < 1.0   # large logits, none near the LeakyReLU kink
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY, slope=0.2)
    A = DeviceCSR(g)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0 and T.nnz_sparse > 0
    Ah = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    pos = ctx.transpose_positions(A.s, A.s)
    for how, first, second in (("plain", A.s, A.s), ("split", Ah, Ah)):
        got = ctx.gat_backward(first, second, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY))
        for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
            assert_close(gpu, ref, what=f"{what}, {how}, large logits")
    T.close()


def test_gat_backward_with_a_split_of_a_rectangular_transposed_pattern(ctx):
    """Fewer destinations than sources: the transposed pattern is a matrix of its own with its own tile split, whose rows are
    the sources and whose columns are the destinations."""
    from paper_2306_15155_amd import Tiles, csr_struct
    full = synth.rmat(76, 4500, 200_000)
    rp = full.row_ptr[:3001].copy()  # the first 3000 destinations of a power-law graph, all 4500 sources
    g = synth.CSR(3000, full.n_cols, rp, full.col_idx[:rp[-1]].copy())
    gt = synth.transpose(g)
    f_in, f_out = 56, 160
    X, W, dY = _inputs(g, f_in, f_out, 77)
    a_l, a_r = synth.normal(77, 20, (f_out,), 0.0, 0.3), synth.normal(77, 21, (f_out,), 0.0, 0.3)
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY, slope=0.2)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    T, Tt = Tiles(ctx, A.s, 0.05, 192, min_width=32), Tiles(ctx, At.s, 0.05, 192, min_width=32)
    assert T.n_tiles > 0 and Tt.n_tiles > 0
    Ah = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    Ath = csr_struct(gt.n_rows, gt.n_cols, At.row_ptr, At.col_idx, None, None, Tt)
    pos = ctx.transpose_positions(A.s, At.s)
    got = ctx.gat_backward(Ah, Ath, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY))
    for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
        assert_close(gpu, ref, what=what)
    T.close()
    Tt.close()


def test_transpose_positions_rejects_a_pattern_that_is_not_the_transpose(ctx):
    from paper_2306_15155_amd import SenseiError
    g = hub_and_empty_graph(74, 500, 3000, 200, 5)   # not symmetric
    A = DeviceCSR(g)
    with pytest.raises(SenseiError):
        ctx.transpose_positions(A.s, A.s)


# ------------------------------------------------------------------ degenerate shapes

@pytest.mark.parametrize("case", ["no_entries", "single_node", "width_one", "one_long_row"])
def test_backward_degenerate_cases(ctx, case):
    if case == "no_entries":       # rows without any stored entry: every gradient through the graph is zero
        e = np.empty(0, dtype=np.int32)
        g = synth.build_csr(50, 50, e, e, False, False)
        f_in, f_out = 6, 5
    elif case == "single_node":
        g = synth.self_loops_only(1)
        f_in, f_out = 3, 2
    elif case == "width_one":
        g = synth.erdos_renyi(81, 400, 1500)
        f_in, f_out = 1, 1
    else:                          # one row holding every column (spans many chunks), the others only their self edge
        n = 3000
        g = synth.build_csr(n, n, np.zeros(n, dtype=np.int32), np.arange(n, dtype=np.int32), False, True)
        f_in, f_out = 20, 36
    gt = synth.transpose(g)
    X, W, dY = _inputs(g, f_in, f_out, 90)
    a_l, a_r = synth.normal(91, 20, (f_out,), 0.0, 0.3), synth.normal(91, 21, (f_out,), 0.0, 0.3)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    want_dx, want_dw = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY)
    for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
        dX, dW = ctx.gcn_backward(A.s, At.s, r, c, dev(X), dev(W), dev(dY), bwd)
        assert_close(dX, want_dx, what=f"{case} gcn dX {bwd}")
        assert_close(dW, want_dw, what=f"{case} gcn dW {bwd}")
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY)
    pos = ctx.transpose_positions(A.s, At.s)
    got = ctx.gat_backward(A.s, At.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY))
    for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
        assert_close(gpu, ref, what=f"{case} gat {what}")
    if case == "no_entries":
        assert float(got[1].abs().max()) == 0.0 and float(dW.abs().max()) == 0.0


@pytest.mark.parametrize("split", [False, True])
def test_backward_can_be_captured_in_a_hip_graph(ctx, split):
    """The backward calls only enqueue kernels (fill kernels instead of memsets, no allocation of their own, no
    synchronisation): a captured training step replays to the same bits as the eager run, every time.  With a dense-tile
    split on the pattern the calls fork to the split's stream and join it again by events, which the capture records as
    dependencies of the graph."""
    from paper_2306_15155_amd import Tiles, csr_struct
    g = synth.rmat(95, 4000, 90_000)
    A = DeviceCSR(g)
    plain = A.s
    dr, dc = ctx.degrees(plain)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    f_in, f_out = (48, 40) if not split else (48, 136)
    T = None
    if split:
        T = Tiles(ctx, plain, 0.05, 160, min_width=32)
        assert T.n_tiles > 0
        A = type("Split", (), {"s": csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T), "keep": A})()
    X, W, dY = (dev(t) for t in _inputs(g, f_in, f_out, 96))
    a_l, a_r = dev(synth.normal(96, 20, (f_out,), 0.0, 0.3)), dev(synth.normal(96, 21, (f_out,), 0.0, 0.3))
    pos = ctx.transpose_positions(plain, plain)
    Y = ctx.gcn_layer(A.s, r, c, X, W, 3, ACT_RELU)

    def step():
        out = list(ctx.gcn_backward(A.s, A.s, r, c, X, W, dY, GCN_BWD_AGG, Y=Y, activation=ACT_RELU))
        out += list(ctx.gcn_backward(A.s, A.s, r, c, X, W, dY, GCN_BWD_UPD, Y=Y, activation=ACT_RELU))
        out += list(ctx.gat_backward(A.s, A.s, pos, X, W, a_l, a_r, dY))
        return out

    want = [t.clone() for t in step()]  # also sizes the workspace before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        got = step()
    for rep in range(3):
        for t in got:
            t.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep}"
        eager = step()  # eager work between replays
        torch.cuda.synchronize()
        for a, b in zip(eager, want):
            assert torch.equal(a, b)
    if T is not None:
        del graph
        T.close()


def test_variant_backwards_can_be_captured_in_a_hip_graph(ctx):
    """The same for the backward calls of the variant layers: a captured step replays to the bits of the eager run."""
    g = synth.rmat(97, 4000, 90_000)
    A = DeviceCSR(g)
    dr, dc = ctx.degrees(A.s)
    r, c = ctx.norm_vectors(dr), ctx.norm_vectors(dc)
    f_in, f_out, K = 24, 32, 2
    X, W, dY = (dev(t) for t in _inputs(g, f_in, f_out, 98))
    W3 = dev(np.concatenate([synth.glorot(98, 30 + k, f_in, f_out) for k in range(K + 1)], axis=0))
    Wq = dev(synth.glorot(98, 40, f_in, 16))
    a_l, a_r = dev(synth.normal(98, 20, (f_out,), 0.0, 0.3)), dev(synth.normal(98, 21, (f_out,), 0.0, 0.3))
    pos = ctx.transpose_positions(A.s, A.s)

    def step():
        out = []
        for bwd in (GCN_BWD_AGG, GCN_BWD_UPD):
            out += list(ctx.sgc_backward(A.s, A.s, r, c, X, W, K, dY, bwd))
            out += list(ctx.tagcn_backward(A.s, A.s, r, c, X, W3, K, dY, bwd))
        out += list(ctx.gat_backward_heads(A.s, A.s, pos, X, W, a_l, a_r, 4, dY))
        out += list(ctx.gatv2_backward(A.s, A.s, pos, X, W, W, a_l, dY))
        out += list(ctx.dotgat_backward(A.s, A.s, pos, X, Wq, Wq, W, 0.25, dY))
        return out

    want = [t.clone() for t in step()]  # also sizes the workspace before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        got = step()
    for rep in range(3):
        for t in got:
            t.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep}"
        eager = step()  # eager work between replays
        torch.cuda.synchronize()
        for a, b in zip(eager, want):
            assert torch.equal(a, b)


# ------------------------------------------------------------------ multi-head GAT

@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("shape", [(40, 24, 2), (24, 40, 5), (70, 41, 1), (33, 128, 2), (20, 96, 3), (24, 15, 3), (16, 130, 2)])
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_multi_head_gat_backward_matches_chain_rule(ctx, name, shape, act):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out, heads = shape
    X, W, dY = _inputs(g, f_in, f_out, 150 + f_in)
    a_l, a_r = synth.normal(151, 20, (f_out,), 0.0, 0.3), synth.normal(151, 21, (f_out,), 0.0, 0.3)
    Y = None
    if act == ACT_RELU:
        Y = oracle.gat_layer_heads(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, heads, 0.2, 1).astype(np.float32)
    want = oracle.gat_backward_heads(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, heads, dY, Y=Y, slope=0.2, act=act)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    pos = ctx.transpose_positions(A.s, At.s)
    got = ctx.gat_backward_heads(A.s, At.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), heads, dev(dY), Y=None if Y is None else dev(Y), activation=act)
    for gpu, ref, what in zip(got, want, ("dX", "dW", "da_l", "da_r")):
        assert_close(gpu, ref, what=what)


def test_multi_head_gat_backward_one_head_and_split_patterns(ctx):
    """One head is the single-head call (bit-equal); with a tile split attached the heads of 128 columns take the split paths."""
    from paper_2306_15155_amd import Tiles, csr_struct
    g = synth.rmat(152, 5000, 150_000)
    f_in, f_out = 48, 256
    X, W, dY = _inputs(g, f_in, f_out, 153)
    a_l, a_r = synth.normal(153, 20, (f_out,), 0.0, 0.3), synth.normal(153, 21, (f_out,), 0.0, 0.3)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    one = [t.clone() for t in ctx.gat_backward_heads(A.s, A.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), 1, dev(dY))]
    ref = ctx.gat_backward(A.s, A.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), dev(dY))
    assert all(torch.equal(a, b) for a, b in zip(one, ref))
    want = oracle.gat_backward_heads(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, a_l, a_r, 2, dY)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0
    At = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    none, dW, dal, dar = ctx.gat_backward_heads(At, At, pos, dev(X), dev(W), dev(a_l), dev(a_r), 2, dev(dY), want_dx=False)
    assert none is None
    for gpu, ref, what in zip((dW, dal, dar), want[1:], ("dW", "da_l", "da_r")):
        assert_close(gpu, ref, what=what)
    with pytest.raises(RuntimeError):
        ctx.gat_backward_heads(A.s, A.s, pos, dev(X), dev(W), dev(a_l), dev(a_r), 3, dev(dY))     # 3 does not divide 256
    T.close()


# ------------------------------------------------------------------ GATv2

def _gatv2_inputs(g, f_in, f_out, seed):
    """The derivative of LeakyReLU jumps where a component of U_ij = Theta_l[i] + Theta_r[j] is zero, and with millions of components some
    lie closer to zero than fp32 rounding of the projections (seen: one of 4.3 million at 1.3e-8, where the fp32 path and the fp64
    oracle took different branches and one column of dW_l moved by 2e-4).  X and the two weight matrices therefore take multiples
    of 1/64: products and sums of the projections are then exact in fp32 in any order, both sides see the same U, and take the
    same branch everywhere, also where U is exactly zero."""
    grid = lambda a: (np.round(a * 64.0) / 64.0).astype(np.float32)
    X = grid(synth.uniform(seed, 10, (g.n_cols, f_in)))
    W_l, W_r = grid(synth.glorot(seed, 13, f_in, f_out) * 2.0), grid(synth.glorot(seed, 11, f_in, f_out) * 2.0)
    att = synth.normal(seed, 20, (f_out,), 0.0, 0.3)
    dY = synth.normal(seed, 12, (g.n_rows, f_out), 0.0, 1.0)
    return X, W_l, W_r, att, dY


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("widths", [(40, 24), (24, 40), (70, 41), (20, 64)])
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_gatv2_backward_matches_chain_rule(ctx, name, widths, act):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, f_out = widths
    X, W_l, W_r, att, dY = _gatv2_inputs(g, f_in, f_out, 170 + f_in)
    assert np.count_nonzero(W_l) > W_l.size // 2
    Y = None
    if act == ACT_RELU:
        Y = oracle.gatv2_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, 0.2, 1).astype(np.float32)
    want = oracle.gatv2_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, dY, Y=Y, slope=0.2, act=act)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    pos = ctx.transpose_positions(A.s, At.s)
    got = ctx.gatv2_backward(A.s, At.s, pos, dev(X), dev(W_l), dev(W_r), dev(att), dev(dY), Y=None if Y is None else dev(Y), activation=act)
    for gpu, ref, what in zip(got, want, ("dX", "dW_l", "dW_r", "datt")):
        assert_close(gpu, ref, what=what)


def test_gatv2_backward_other_slope_shared_weights_and_strides(ctx):
    """Another slope; one weight matrix passed for both roles (its gradient is the sum of the two returned); operands and results with
    leading dimensions larger than their widths; weight gradients only."""
    g = synth.rmat(172, 3000, 60_000)
    f_in, f_out = 48, 64
    X, W, _, att, dY = _gatv2_inputs(g, f_in, f_out, 173)
    want = oracle.gatv2_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, W, att, dY, slope=0.05)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)  # symmetric pattern: its own transpose
    Xs = torch.zeros((g.n_cols, f_in + 3), device="cuda:0")
    Xs[:, :f_in] = dev(X)
    Ws = torch.zeros((f_in, f_out + 8), device="cuda:0")
    Ws[:, :f_out] = dev(W)
    dYs = torch.zeros((g.n_rows, f_out + 4), device="cuda:0")
    dYs[:, :f_out] = dev(dY)
    dX, dWl, dWr, da = ctx.gatv2_backward(A.s, A.s, pos, Xs[:, :f_in], Ws[:, :f_out], Ws[:, :f_out], dev(att), dYs[:, :f_out], neg_slope=0.05)
    assert_close(dX, want[0], what="dX")
    assert_close(dWl, want[1], what="dW_l")
    assert_close(dWr, want[2], what="dW_r")
    assert_close(da, want[3], what="datt")
    none, dWl2, dWr2, da2 = ctx.gatv2_backward(A.s, A.s, pos, dev(X), dev(W), dev(W), dev(att), dev(dY), neg_slope=0.05, want_dx=False)
    assert none is None and torch.equal(dWl2, dWl) and torch.equal(dWr2, dWr) and torch.equal(da2, da)


def test_gatv2_backward_on_a_graph_of_millions_of_entries(ctx):
    """2 million stored entries, thousands of chunks, hub rows that span hundreds of them (their carries and fix-ups in every one
    of the SpMM-shaped sums), ReLU mask."""
    g = synth.rmat(176, 20_000, 2_000_000)
    assert g.nnz > 2_000_000 and np.diff(g.row_ptr).max() > 5000
    f_in, f_out = 32, 32
    X, W_l, W_r, att, dY = _gatv2_inputs(g, f_in, f_out, 177)
    Y = oracle.gatv2_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, 0.2, 1).astype(np.float32)
    want = oracle.gatv2_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, dY, Y=Y, slope=0.2, act=1)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    got = ctx.gatv2_backward(A.s, A.s, pos, dev(X), dev(W_l), dev(W_r), dev(att), dev(dY), Y=dev(Y), activation=ACT_RELU)
    for gpu, ref, what in zip(got, want, ("dX", "dW_l", "dW_r", "datt")):
        assert_close(gpu, ref, what=what)


def test_gatv2_backward_slope_one_is_the_gat_backward(ctx):
    """With slope 1 the score is att.Theta_l[i] + att.Theta_r[j]; the first term cancels in the softmax, so the layer is the GAT layer
    with W = W_r and a_r = att: nothing flows through W_l, and dX, dW_r, datt are that layer's dX, dW, da_r (its own oracle)."""
    g = synth.rmat(174, 2000, 30_000)
    f_in, f_out = 24, 40
    X, W_r, dY = _inputs(g, f_in, f_out, 175)
    W_l = synth.glorot(175, 13, f_in, f_out)
    att = synth.normal(175, 20, (f_out,), 0.0, 0.3)
    want = oracle.gat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_r, np.zeros(f_out, np.float32), att, dY, slope=1.0)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    dX, dWl, dWr, da = ctx.gatv2_backward(A.s, A.s, pos, dev(X), dev(W_l), dev(W_r), dev(att), dev(dY), neg_slope=1.0)
    assert_close(dX, want[0], what="dX")
    assert_close(dWr, want[1], what="dW_r")
    assert_close(da, want[3], what="datt")
    assert_close(dWl, np.zeros((f_in, f_out)), what="dW_l")


def test_gatv2_backward_argument_checks(ctx):
    g = synth.erdos_renyi(47, 200, 600)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    X, W, dY = (torch.zeros(s, device="cuda:0") for s in ((200, 8), (8, 4), (200, 4)))
    att = torch.zeros(4, device="cuda:0")
    ctx.gatv2_backward(A.s, A.s, pos, X, W, W, att, dY)
    with pytest.raises(RuntimeError):
        ctx.gatv2_backward(A.s, A.s, pos, X, W, torch.zeros((8, 5), device="cuda:0"), att, dY)      # the two projections differ in width
    with pytest.raises(RuntimeError):
        ctx.gatv2_backward(A.s, A.s, pos, X, W, W, att, dY, activation=ACT_RELU)                    # ReLU without the forward output
    with pytest.raises(RuntimeError):
        ctx.gatv2_backward(A.s, A.s, None, X, W, W, att, dY)                                         # no transposition map
    g2 = synth.erdos_renyi(48, 100, 300)
    with pytest.raises(RuntimeError):
        ctx.gatv2_backward(A.s, DeviceCSR(g2).s, pos, X, W, W, att, dY)                              # transposed pattern of another shape
    torch.cuda.synchronize()


# ------------------------------------------------------------------ key-query attention

def _kq_inputs(g, f_in, d_k, f_out, seed):
    X = synth.uniform(seed, 10, (g.n_cols, f_in))
    W_q, W_k, W_v = synth.glorot(seed, 14, f_in, d_k), synth.glorot(seed, 15, f_in, d_k), synth.glorot(seed, 16, f_in, f_out)
    dY = synth.normal(seed, 12, (g.n_rows, f_out), 0.0, 1.0)
    return X, W_q, W_k, W_v, dY


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("widths", [(40, 16, 24), (24, 40, 40), (70, 33, 41), (20, 64, 7)])
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_key_query_attention_backward_matches_chain_rule(ctx, name, widths, act):
    g = GRAPHS[name]()
    gt = synth.transpose(g)
    f_in, d_k, f_out = widths
    X, W_q, W_k, W_v, dY = _kq_inputs(g, f_in, d_k, f_out, 190 + f_in)
    scale = 1.0 / np.sqrt(d_k)
    Y = None
    if act == ACT_RELU:
        Y = oracle.dotgat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, 1).astype(np.float32)
    want = oracle.dotgat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, dY, Y=Y, act=act)
    A, At = DeviceCSR(g), DeviceCSR(gt)
    pos = ctx.transpose_positions(A.s, At.s)
    got = ctx.dotgat_backward(A.s, At.s, pos, dev(X), dev(W_q), dev(W_k), dev(W_v), float(scale), dev(dY), Y=None if Y is None else dev(Y),
                              activation=act)
    for gpu, ref, what in zip(got, want, ("dX", "dW_q", "dW_k", "dW_v")):
        assert_close(gpu, ref, what=what)


def test_key_query_attention_backward_large_graph_strides_and_weight_gradients_only(ctx):
    g = synth.rmat(192, 20_000, 2_000_000)
    f_in, d_k, f_out = 32, 16, 48
    X, W_q, W_k, W_v, dY = _kq_inputs(g, f_in, d_k, f_out, 193)
    Y = oracle.dotgat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.25, 1).astype(np.float32)
    want = oracle.dotgat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.25, dY, Y=Y, act=1)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    Xs = torch.zeros((g.n_cols, f_in + 3), device="cuda:0")
    Xs[:, :f_in] = dev(X)
    dYs = torch.zeros((g.n_rows, f_out + 4), device="cuda:0")
    dYs[:, :f_out] = dev(dY)
    got = ctx.dotgat_backward(A.s, A.s, pos, Xs[:, :f_in], dev(W_q), dev(W_k), dev(W_v), 0.25, dYs[:, :f_out], Y=dev(Y), activation=ACT_RELU)
    for gpu, ref, what in zip(got, want, ("dX", "dW_q", "dW_k", "dW_v")):
        assert_close(gpu, ref, what=what)
    none, dWq, dWk, dWv = ctx.dotgat_backward(A.s, A.s, pos, dev(X), dev(W_q), dev(W_k), dev(W_v), 0.25, dev(dY), Y=dev(Y), activation=ACT_RELU,
                                              want_dx=False)
    assert none is None and torch.equal(dWq, got[1]) and torch.equal(dWk, got[2]) and torch.equal(dWv, got[3])


def test_key_query_attention_backward_argument_checks(ctx):
    g = synth.erdos_renyi(47, 200, 600)
    A = DeviceCSR(g)
    pos = ctx.transpose_positions(A.s, A.s)
    X, Wq, Wv, dY = (torch.zeros(s, device="cuda:0") for s in ((200, 8), (8, 3), (8, 4), (200, 4)))
    ctx.dotgat_backward(A.s, A.s, pos, X, Wq, Wq, Wv, 0.5, dY)
    with pytest.raises(RuntimeError):
        ctx.dotgat_backward(A.s, A.s, pos, X, Wq, torch.zeros((8, 5), device="cuda:0"), Wv, 0.5, dY)      # queries and keys differ in width
    with pytest.raises(RuntimeError):
        ctx.dotgat_backward(A.s, A.s, pos, X, Wq, Wq, Wv, 0.5, dY, activation=ACT_RELU)                   # ReLU without the forward output
    with pytest.raises(RuntimeError):
        ctx.dotgat_backward(A.s, A.s, None, X, Wq, Wq, Wv, 0.5, dY)                                        # no transposition map
    with pytest.raises(RuntimeError):
        ctx.dotgat_backward(A.s, A.s, pos, X, Wq, Wq, Wv, 0.5, torch.zeros((200, 5), device="cuda:0"))    # dY of another width
    torch.cuda.synchronize()


def test_attention_variant_backward_without_output_rows(ctx):
    """A block with sources but no destinations: no output depends on anything, every gradient is zero."""
    none = np.empty(0, np.int32)
    g = synth.build_csr(0, 6, none, none, False, False)
    A, At = DeviceCSR(g), DeviceCSR(synth.transpose(g))
    X = torch.ones((6, 5), device="cuda:0")
    W, Wq = torch.ones((5, 4), device="cuda:0"), torch.ones((5, 3), device="cuda:0")
    att = torch.ones(4, device="cuda:0")
    dY = torch.empty((0, 4), device="cuda:0")
    for got in (ctx.gatv2_backward(A.s, At.s, None, X, W, W, att, dY), ctx.dotgat_backward(A.s, At.s, None, X, Wq, Wq, W, 0.5, dY)):
        assert got[0].shape == (6, 5)
        assert all(float(t.abs().max()) == 0.0 for t in got)
    torch.cuda.synchronize()
