"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself
(dense brute force, closed forms, invariants, library routines on special cases)."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth
from oracle import dense


def _rand_graph(seed, n, pairs):
    return synth.erdos_renyi(seed, n, pairs)


def _rect_block(seed, n_rows, n_cols, per_row):
    """Bipartite block: destinations are the first n_rows columns, each with a self edge."""
    rng = np.random.default_rng(seed)
    u = np.repeat(np.arange(n_rows), per_row)
    v = rng.integers(0, n_cols, size=u.size)
    return synth.build_csr(n_rows, n_cols, u, v, False, True)


def _close(a, b, tol=1e-10):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    assert np.max(np.abs(a - b) / (1.0 + np.abs(b))) < tol


# --------------------------------------------------------------- Eq. 1 / Eq. 2

@pytest.mark.parametrize("weighted", [False, True])
def test_spmm_matches_dense_definition(weighted):
    g = _rand_graph(3, 60, 150)
    rng = np.random.default_rng(0)
    B = rng.standard_normal((60, 7))
    val = rng.standard_normal(g.nnz) if weighted else None
    A = dense.dense_pattern(60, 60, g.row_ptr, g.col_idx)
    if weighted:
        A[A != 0] = val  # row-major order of the non-zeros == CSR order (columns ascending)
    _close(oracle.spmm(g.row_ptr, g.col_idx, val, B), dense.spmm_dense(A, B), 1e-12)


def test_spmm_matches_scipy():
    g = _rand_graph(4, 300, 2000)
    rng = np.random.default_rng(1)
    B = rng.standard_normal((300, 13))
    val = rng.standard_normal(g.nnz)
    M = sp.csr_matrix((val, g.col_idx, g.row_ptr), shape=(300, 300))
    _close(oracle.spmm(g.row_ptr, g.col_idx, val, B), M @ B, 1e-12)


def test_sddmm_matches_dense_definition():
    g = _rand_graph(5, 50, 120)
    rng = np.random.default_rng(2)
    b, c = rng.standard_normal(50), rng.standard_normal(50)
    D = dense.sddmm_dense(dense.dense_pattern(50, 50, g.row_ptr, g.col_idx), b[:, None], c[:, None])
    got = oracle.sddmm_mul(g.row_ptr, g.col_idx, None, b, c)
    for i in range(50):
        for k in range(g.row_ptr[i], g.row_ptr[i + 1]):
            assert abs(got[k] - D[i, g.col_idx[k]]) < 1e-14
    # an operand swap (b_j * c_i) must be visible: the pattern is symmetric but b != c
    wrong = oracle.sddmm_mul(g.row_ptr, g.col_idx, None, c, b)
    assert np.max(np.abs(wrong - got)) > 1e-3


def test_gemm_special_cases_and_library():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((37, 11))
    W = rng.standard_normal((11, 5))
    _close(oracle.gemm(A, W), A @ W, 1e-13)
    _close(oracle.gemm(A, np.eye(11)), A, 1e-15)
    assert np.all(oracle.gemm(A, np.zeros((11, 4))) == 0.0)
    _close(oracle.gemv(A, W[:, 0]), A @ W[:, 0], 1e-13)


# ------------------------------------------------------------------ GCN layer

@pytest.mark.parametrize("act", [0, 1])
def test_gcn_layer_matches_dense_brute_force(act):
    g = _rand_graph(6, 120, 400)
    X = synth.uniform(6, 10, (120, 9))
    W = synth.glorot(6, 11, 9, 5)
    A = dense.dense_pattern(120, 120, g.row_ptr, g.col_idx)
    _close(oracle.gcn_layer(120, 120, g.row_ptr, g.col_idx, X, W, act), dense.gcn_layer_dense(A, X, W, act), 1e-12)


def test_gcn_layer_rectangular_block_matches_dense():
    g = _rect_block(7, 20, 55, 4)
    X = synth.normal(7, 10, (55, 6))
    W = synth.glorot(7, 11, 6, 8)
    A = dense.dense_pattern(20, 55, g.row_ptr, g.col_idx)
    _close(oracle.gcn_layer(20, 55, g.row_ptr, g.col_idx, X, W, 1), dense.gcn_layer_dense(A, X, W, 1), 1e-12)


def test_gcn_self_loops_only_is_a_gemm():
    g = synth.self_loops_only(33)
    X = synth.uniform(8, 10, (33, 12))
    W = synth.glorot(8, 11, 12, 7)
    _close(oracle.gcn_layer(33, 33, g.row_ptr, g.col_idx, X, W), X.astype(np.float64) @ W.astype(np.float64), 1e-13)


def test_gcn_regular_ring_constant_columns_are_fixed():
    n, kh = 40, 3
    g = synth.ring_lattice(n, kh)
    assert np.all(np.diff(g.row_ptr) == 2 * kh + 1)
    v = synth.uniform(9, 10, (1, 6))
    X = np.repeat(v, n, axis=0)
    W = synth.glorot(9, 11, 6, 4)
    Y = oracle.gcn_layer(n, n, g.row_ptr, g.col_idx, X, W)
    _close(Y, np.repeat(v.astype(np.float64) @ W.astype(np.float64), n, axis=0), 1e-13)


def test_gcn_complete_graph_gives_column_mean():
    n = 25
    g = synth.complete(n)
    X = synth.uniform(10, 10, (n, 5))
    W = synth.glorot(10, 11, 5, 3)
    Y = oracle.gcn_layer(n, n, g.row_ptr, g.col_idx, X, W)
    mean = (X.astype(np.float64) @ W.astype(np.float64)).mean(axis=0)
    _close(Y, np.repeat(mean[None, :], n, axis=0), 1e-13)


def test_star_graph_normalised_weights_closed_form():
    n = 17
    g = synth.star(n)
    dr, dc = oracle.degrees(n, n, g.row_ptr, g.col_idx)
    assert dr[0] == n and np.all(dr[1:] == 2) and np.array_equal(dr, dc)
    nt = oracle.sddmm_mul(g.row_ptr, g.col_idx, None, oracle.inv_sqrt_deg(dr), oracle.inv_sqrt_deg(dc))
    for i in range(n):
        for k in range(g.row_ptr[i], g.row_ptr[i + 1]):
            j = g.col_idx[k]
            if i == 0 and j == 0:
                want = 1.0 / n
            elif i == j:
                want = 0.5
            else:
                want = 1.0 / np.sqrt(2.0 * n)
            assert abs(nt[k] - want) < 1e-15


def test_gcn_rows_entry_point_matches_full():
    g = _rand_graph(11, 500, 4000)
    X = synth.uniform(11, 10, (500, 20))
    W = synth.glorot(11, 11, 20, 9)
    full = oracle.gcn_layer(500, 500, g.row_ptr, g.col_idx, X, W, 1)
    rows = np.array([0, 3, 499, 250, 3], dtype=np.int32)
    _close(oracle.gcn_layer(500, 500, g.row_ptr, g.col_idx, X, W, 1, rows=rows), full[rows], 1e-12)
    _close(oracle.gcn_layer(500, 500, g.row_ptr, g.col_idx, X, W, 1, omp=True), full, 1e-15)


@pytest.mark.parametrize("shape", [(7, 19), (19, 7), (8, 8)])
@pytest.mark.parametrize("act", [0, 1])
def test_all_gcn_reassociations_agree(shape, act):
    f_in, f_out = shape
    g = _rand_graph(12, 90, 300)
    X = synth.uniform(12, 10, (90, f_in))
    W = synth.glorot(12, 11, f_in, f_out)
    ref = oracle.gcn_layer(90, 90, g.row_ptr, g.col_idx, X, W, act)
    for cid in range(len(oracle.GCN_COMPOSITIONS)):
        _close(oracle.gcn_composition(cid, 90, 90, g.row_ptr, g.col_idx, X, W, act), ref, 1e-11)


def test_gcn_reassociations_agree_on_rectangular_block():
    g = _rect_block(13, 16, 40, 5)
    X = synth.normal(13, 10, (40, 6))
    W = synth.glorot(13, 11, 6, 10)
    ref = dense.gcn_layer_dense(dense.dense_pattern(16, 40, g.row_ptr, g.col_idx), X, W, 1)
    for cid in range(6):
        _close(oracle.gcn_composition(cid, 16, 40, g.row_ptr, g.col_idx, X, W, 1), ref, 1e-11)


# ------------------------------------------------------------------ GAT layer

def _gat_inputs(seed, n, f_in, f_out):
    X = synth.uniform(seed, 10, (n, f_in))
    W = synth.glorot(seed, 11, f_in, f_out)
    a_l = synth.normal(seed, 12, (f_out,), 0.0, 0.1)
    a_r = synth.normal(seed, 13, (f_out,), 0.0, 0.1)
    return X, W, a_l, a_r


@pytest.mark.parametrize("act", [0, 1])
def test_gat_layer_matches_dense_brute_force(act):
    n = 80
    g = _rand_graph(14, n, 300)
    X, W, a_l, a_r = _gat_inputs(14, n, 9, 6)
    a_l, a_r = a_l * 30, a_r * 30  # make the logits spread so softmax and LeakyReLU both matter
    A = dense.dense_pattern(n, n, g.row_ptr, g.col_idx)
    want, _ = dense.gat_layer_dense(A, X, W, a_l, a_r, 0.2, act)
    _close(oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, act), want, 1e-12)


def test_gat_layer_rectangular_block_matches_dense():
    g = _rect_block(15, 12, 30, 4)
    X, W, a_l, a_r = _gat_inputs(15, 30, 5, 7)
    A = dense.dense_pattern(12, 30, g.row_ptr, g.col_idx)
    want, _ = dense.gat_layer_dense(A, X, W, a_l * 20, a_r * 20)
    _close(oracle.gat_layer(12, 30, g.row_ptr, g.col_idx, X, W, a_l * 20, a_r * 20), want, 1e-12)


def test_gat_zero_attention_vectors_is_mean_aggregation():
    n = 70
    g = _rand_graph(16, n, 250)
    X, W, a_l, a_r = _gat_inputs(16, n, 8, 5)
    theta = X.astype(np.float64) @ W.astype(np.float64)
    deg = np.diff(g.row_ptr).astype(np.float64)
    want = oracle.spmm(g.row_ptr, g.col_idx, None, theta) / deg[:, None]
    _close(oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W, 0 * a_l, 0 * a_r), want, 1e-13)


def test_gat_self_loops_only_is_a_gemm():
    g = synth.self_loops_only(21)
    X, W, a_l, a_r = _gat_inputs(17, 21, 6, 4)
    _close(oracle.gat_layer(21, 21, g.row_ptr, g.col_idx, X, W, a_l, a_r), X.astype(np.float64) @ W.astype(np.float64), 1e-13)


def test_edge_softmax_invariants():
    g = _rand_graph(18, 64, 200)
    rng = np.random.default_rng(4)
    e = rng.standard_normal(g.nnz) * 5
    alpha = oracle.edge_softmax(g.row_ptr, e)
    assert np.all(alpha > 0)
    sums = np.add.reduceat(alpha, g.row_ptr[:-1])
    assert np.max(np.abs(sums - 1.0)) < 1e-14
    shift = np.repeat(rng.standard_normal(64) * 100, np.diff(g.row_ptr))
    _close(oracle.edge_softmax(g.row_ptr, e + shift), alpha, 1e-11)
    # direct formula on one row
    lo, hi = g.row_ptr[5], g.row_ptr[6]
    _close(alpha[lo:hi], np.exp(e[lo:hi]) / np.exp(e[lo:hi]).sum(), 1e-13)
    # huge logits stay finite
    assert np.all(np.isfinite(oracle.edge_softmax(g.row_ptr, e * 1e4)))


def test_gat_scores_leaky_relu_and_orientation():
    # 2 destination rows over 3 sources; s_l indexes the row, s_r the column
    row_ptr = np.array([0, 2, 3], dtype=np.int32)
    col_idx = np.array([0, 2, 1], dtype=np.int32)
    s_l = np.array([1.0, -4.0])
    s_r = np.array([0.5, 1.0, -3.0])
    e = oracle.gat_scores(row_ptr, col_idx, s_l, s_r, 0.2)
    assert np.allclose(e, [1.5, 0.2 * (1.0 - 3.0), 0.2 * (-4.0 + 1.0)])


def test_gat_fold_identity_and_all_reassociations_agree():
    n = 75
    g = _rand_graph(19, n, 280)
    for f_in, f_out in [(6, 14), (14, 6)]:
        X, W, a_l, a_r = _gat_inputs(19, n, f_in, f_out)
        a_l, a_r = a_l * 25, a_r * 25
        ref = oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1)
        for cid in range(len(oracle.GAT_COMPOSITIONS)):
            _close(oracle.gat_composition(cid, n, n, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1), ref, 1e-11)


def test_gat_rows_entry_point_matches_full():
    n = 400
    g = _rand_graph(20, n, 3000)
    X, W, a_l, a_r = _gat_inputs(20, n, 12, 18)
    a_l, a_r = a_l * 20, a_r * 20
    full = oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1)
    rows = np.array([399, 0, 17, 200], dtype=np.int32)
    _close(oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 1, rows=rows), full[rows], 1e-11)


def test_gat_empty_row_gives_zeros():
    row_ptr = np.array([0, 0, 2], dtype=np.int32)
    col_idx = np.array([0, 1], dtype=np.int32)
    X, W, a_l, a_r = _gat_inputs(21, 2, 3, 4)
    Y = oracle.gat_layer(2, 2, row_ptr, col_idx, X, W, a_l, a_r)
    assert np.all(Y[0] == 0.0) and np.all(np.isfinite(Y))
    Yg = oracle.gcn_layer(2, 2, row_ptr, col_idx, X, W)
    assert np.all(Yg[0] == 0.0) and np.all(np.isfinite(Yg))


# ------------------------------------------------------------- selector pieces

def test_density_feature_matches_the_papers_printed_values(golden_dir):
    import os
    for line in open(os.path.join(golden_dir, "paper_density.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, nodes, edges, printed, digits = line.split()
        d = oracle.density(int(nodes), int(nodes), int(edges))
        assert float(f"{d:.{int(digits) - 1}e}") == float(printed), (name, d)


def test_embedding_size_rules(golden_dir):
    import os
    counts = dict(l.split() for l in open(os.path.join(golden_dir, "paper_counts.txt")) if l.strip() and not l.startswith("#"))
    # the promoted GCN compositions (dynamic, precompute) x (update first, update last) come in two
    # sets keyed on the embedding sizes, each holding both normalisation styles
    paper_ids = {"dynamic_agg": 0, "dynamic_upd": 1, "pre_agg": 4, "pre_upd": 5}
    assert len(paper_ids) == int(counts["gcn_trees_promoted"])
    small_in = set(oracle.select_rules("gcn", 32, 256)) & set(paper_ids.values())
    large_in = set(oracle.select_rules("gcn", 256, 32)) & set(paper_ids.values())
    assert small_in == {0, 4} and large_in == {1, 5}
    assert len({frozenset(small_in), frozenset(large_in)}) == int(counts["gcn_sets"])
    # GAT: the paper's two compositions are ids 0 (reuse) and 1 (recompute, one extra GEMM)
    assert oracle.select_rules("gat", 256, 64) == (0,)
    assert oracle.select_rules("gat", 64, 64) == (0,)
    assert {0, 1} <= set(oracle.select_rules("gat", 64, 256))


def test_multi_head_gat_is_head_wise_and_matches_the_dense_definition():
    g = _rand_graph(17, 40, 120)
    rng = np.random.default_rng(17)
    X = rng.standard_normal((40, 6)).astype(np.float32)
    W = rng.standard_normal((6, 12)).astype(np.float32)
    a_l, a_r = rng.standard_normal(12).astype(np.float32), rng.standard_normal(12).astype(np.float32)
    Y = oracle.gat_layer_heads(40, 40, g.row_ptr, g.col_idx, X, W, a_l, a_r, 3, 0.2, 1)
    A = dense.dense_pattern(40, 40, g.row_ptr, g.col_idx)
    for h in range(3):
        sl = slice(4 * h, 4 * h + 4)
        _close(Y[:, sl], dense.gat_layer_dense(A, X, W[:, sl], a_l[sl], a_r[sl], 0.2, 1)[0])
    _close(oracle.gat_layer_heads(40, 40, g.row_ptr, g.col_idx, X, W, a_l, a_r, 1), oracle.gat_layer(40, 40, g.row_ptr, g.col_idx, X, W, a_l, a_r))
    # heads do not see each other: changing head 2 leaves heads 0 and 1 alone
    W2 = W.copy(); W2[:, 8:] *= -3.0
    Y2 = oracle.gat_layer_heads(40, 40, g.row_ptr, g.col_idx, X, W2, a_l, a_r, 3, 0.2, 1)
    _close(Y2[:, :8], Y[:, :8])
    assert np.max(np.abs(Y2[:, 8:] - Y[:, 8:])) > 1e-3


# --------------------------------------------------------------- K-hop simplified graph convolution

def test_sgc_is_the_matrix_power_and_one_hop_is_the_gcn_layer():
    n = 60
    g = _rand_graph(21, n, 200)
    X = synth.uniform(21, 10, (n, 7))
    W = synth.glorot(21, 11, 7, 5)
    A = dense.dense_pattern(n, n, g.row_ptr, g.col_idx)
    d = A.sum(axis=1)
    dc = A.sum(axis=0)
    Ahat = A / np.sqrt(d)[:, None] / np.sqrt(dc)[None, :]
    XW = X.astype(np.float64) @ W.astype(np.float64)
    for k in (1, 2, 3, 5):
        ref = np.linalg.matrix_power(Ahat, k) @ XW
        _close(oracle.sgc_layer(n, g.row_ptr, g.col_idx, X, W, k), ref, 1e-12)
        _close(oracle.sgc_layer(n, g.row_ptr, g.col_idx, X, W, k, 1), np.maximum(ref, 0.0), 1e-12)
    _close(oracle.sgc_layer(n, g.row_ptr, g.col_idx, X, W, 1, 1), oracle.gcn_layer(n, n, g.row_ptr, g.col_idx, X, W, 1), 1e-13)
    rows = np.array([7, 0, 59, 7, 31])   # selected rows (unsorted, one repeated) against the dense power as well
    for k in (1, 3):
        _close(oracle.sgc_layer(n, g.row_ptr, g.col_idx, X, W, k, 0, rows=rows), (np.linalg.matrix_power(Ahat, k) @ XW)[rows], 1e-12)


def test_sgc_on_a_regular_ring_keeps_constant_columns_and_smooths_the_rest():
    n, kh = 48, 2
    g = synth.ring_lattice(n, kh)
    v = synth.uniform(22, 10, (1, 4))
    W = synth.glorot(22, 11, 4, 3)
    Y = oracle.sgc_layer(n, g.row_ptr, g.col_idx, np.repeat(v, n, axis=0), W, 4)
    _close(Y, np.repeat(v.astype(np.float64) @ W.astype(np.float64), n, axis=0), 1e-13)
    # the normalised ring operator is a circulant averaging filter: mode m is scaled by (1 + 2 sum_t cos(2 pi m t / n)) / (2 kh + 1) per hop
    m = 3
    x = np.cos(2 * np.pi * m * np.arange(n) / n)[:, None].astype(np.float32)
    lam = (1 + 2 * sum(np.cos(2 * np.pi * m * t / n) for t in range(1, kh + 1))) / (2 * kh + 1)
    Y = oracle.sgc_layer(n, g.row_ptr, g.col_idx, x, np.ones((1, 1), dtype=np.float32), 6)
    _close(Y, lam ** 6 * x.astype(np.float64), 1e-7)


def test_tagcn_is_the_matrix_polynomial():
    n, f_in, f_out = 50, 6, 4
    g = _rand_graph(23, n, 160)
    X = synth.uniform(23, 10, (n, f_in))
    A = dense.dense_pattern(n, n, g.row_ptr, g.col_idx)
    Ahat = A / np.sqrt(A.sum(axis=1))[:, None] / np.sqrt(A.sum(axis=0))[None, :]
    X64 = X.astype(np.float64)
    for K in (1, 2, 4):
        W = synth.glorot(23, 11 + K, (K + 1) * f_in, f_out)
        W64 = W.astype(np.float64)
        ref = sum(np.linalg.matrix_power(Ahat, k) @ X64 @ W64[k * f_in:(k + 1) * f_in] for k in range(K + 1))
        _close(oracle.tagcn_layer(n, g.row_ptr, g.col_idx, X, W, K), ref, 1e-12)
        _close(oracle.tagcn_layer(n, g.row_ptr, g.col_idx, X, W, K, 1), np.maximum(ref, 0.0), 1e-12)
    # only the one-hop block non-zero: the GCN layer; only the last block non-zero: the K-hop SGC layer
    W = np.zeros((3 * f_in, f_out), dtype=np.float32)
    W1 = synth.glorot(23, 20, f_in, f_out)
    W[f_in:2 * f_in] = W1
    _close(oracle.tagcn_layer(n, g.row_ptr, g.col_idx, X, W, 2, 1), oracle.gcn_layer(n, n, g.row_ptr, g.col_idx, X, W1, 1), 1e-13)
    W[:] = 0.0
    W[2 * f_in:] = W1
    _close(oracle.tagcn_layer(n, g.row_ptr, g.col_idx, X, W, 2), oracle.sgc_layer(n, g.row_ptr, g.col_idx, X, W1, 2), 1e-13)
    # self loops only: A^ = I, the layer is X (W_0 + .. + W_K)
    gs = synth.self_loops_only(n)
    W = synth.glorot(23, 21, 3 * f_in, f_out)
    Wsum = W.astype(np.float64).reshape(3, f_in, f_out).sum(axis=0)
    _close(oracle.tagcn_layer(n, gs.row_ptr, gs.col_idx, X, W, 2), X64 @ Wsum, 1e-13)


# --------------------------------------------------------------- GATv2

def _v2_inputs(seed, n_cols, f_in, d):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n_cols, f_in)).astype(np.float32)
    W_l = (0.5 * rng.standard_normal((f_in, d))).astype(np.float32)
    W_r = (0.5 * rng.standard_normal((f_in, d))).astype(np.float32)
    att = rng.standard_normal(d).astype(np.float32)
    return X, W_l, W_r, att


@pytest.mark.parametrize("act", [0, 1])
def test_gatv2_matches_dense_brute_force(act):
    g = _rand_graph(24, 45, 150)
    X, W_l, W_r, att = _v2_inputs(24, 45, 7, 5)
    A = dense.dense_pattern(45, 45, g.row_ptr, g.col_idx)
    _close(oracle.gatv2_layer(45, 45, g.row_ptr, g.col_idx, X, W_l, W_r, att, 0.2, act), dense.gatv2_layer_dense(A, X, W_l, W_r, att, 0.2, act)[0])
    rows = np.array([3, 44, 0, 17])
    _close(oracle.gatv2_layer(45, 45, g.row_ptr, g.col_idx, X, W_l, W_r, att, 0.2, act, rows=rows),
           dense.gatv2_layer_dense(A, X, W_l, W_r, att, 0.2, act)[0][rows])
    gr = _rect_block(25, 12, 30, 4)
    Xr = X[:30]
    Ar = dense.dense_pattern(12, 30, gr.row_ptr, gr.col_idx)
    _close(oracle.gatv2_layer(12, 30, gr.row_ptr, gr.col_idx, Xr, W_l, W_r, att, 0.2, act), dense.gatv2_layer_dense(Ar, Xr, W_l, W_r, att, 0.2, act)[0])


def test_gatv2_special_cases():
    n = 40
    g = _rand_graph(26, n, 130)
    X, W_l, W_r, att = _v2_inputs(26, n, 6, 8)
    A = dense.dense_pattern(n, n, g.row_ptr, g.col_idx)
    Th_r = X.astype(np.float64) @ W_r.astype(np.float64)
    # zero attention vector: all logits equal, the layer averages the projected neighbours
    _close(oracle.gatv2_layer(n, n, g.row_ptr, g.col_idx, X, W_l, W_r, np.zeros(8, dtype=np.float32)), (A / A.sum(axis=1, keepdims=True)) @ Th_r, 1e-12)
    # slope 1 makes the score linear: e_ij = att.Theta_l[i] + att.Theta_r[j], and the term of i cancels in the row softmax, so
    # the weights are those of the GAT layer of Eq. 5 with W = W_r, a_r = att, slope 1 and any a_l
    a_any = np.linspace(-1.0, 1.0, 8).astype(np.float32)
    _close(oracle.gatv2_layer(n, n, g.row_ptr, g.col_idx, X, W_l, W_r, att, 1.0), oracle.gat_layer(n, n, g.row_ptr, g.col_idx, X, W_r, a_any, att, 1.0), 1e-11)
    # self loops only: alpha = 1, the layer is X W_r
    gs = synth.self_loops_only(n)
    _close(oracle.gatv2_layer(n, n, gs.row_ptr, gs.col_idx, X, W_l, W_r, att), Th_r, 1e-13)
    # unlike the GAT layer the ranking of the neighbours depends on the destination: with slope 0.2 some row's weights differ
    # from the slope-1 (static) ones
    assert np.max(np.abs(oracle.gatv2_layer(n, n, g.row_ptr, g.col_idx, X, W_l, W_r, att, 0.2) -
                         oracle.gatv2_layer(n, n, g.row_ptr, g.col_idx, X, W_l, W_r, att, 1.0))) > 1e-3


# ------------------------------------------------------------- key-query attention layer

def _kq_inputs(seed, n, f_in, d_k, f_out):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, f_in)).astype(np.float32)
    W_q = (0.6 * rng.standard_normal((f_in, d_k))).astype(np.float32)
    W_k = (0.6 * rng.standard_normal((f_in, d_k))).astype(np.float32)
    W_v = (0.5 * rng.standard_normal((f_in, f_out))).astype(np.float32)
    return X, W_q, W_k, W_v


@pytest.mark.parametrize("act", [0, 1])
def test_key_query_attention_matches_dense_masked_attention(act):
    g = _rand_graph(31, 45, 150)
    X, W_q, W_k, W_v = _kq_inputs(31, 45, 7, 5, 6)
    A = dense.dense_pattern(45, 45, g.row_ptr, g.col_idx)
    want = dense.dotgat_layer_dense(A, X, W_q, W_k, W_v, 0.4, act)[0]
    _close(oracle.dotgat_layer(45, 45, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.4, act), want)
    rows = np.array([3, 44, 0, 17])
    _close(oracle.dotgat_layer(45, 45, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.4, act, rows=rows), want[rows])
    gr = _rect_block(32, 12, 30, 4)
    Ar = dense.dense_pattern(12, 30, gr.row_ptr, gr.col_idx)
    _close(oracle.dotgat_layer(12, 30, gr.row_ptr, gr.col_idx, X[:30], W_q, W_k, W_v, 0.4, act), dense.dotgat_layer_dense(Ar, X[:30], W_q, W_k, W_v, 0.4, act)[0])


def test_key_query_attention_special_cases():
    n = 40
    g = _rand_graph(33, n, 130)
    X, W_q, W_k, W_v = _kq_inputs(33, n, 6, 8, 5)
    A = dense.dense_pattern(n, n, g.row_ptr, g.col_idx)
    V = X.astype(np.float64) @ W_v.astype(np.float64)
    # zero queries (or zero scale): all logits equal, the layer averages the value projections of the neighbours
    _close(oracle.dotgat_layer(n, n, g.row_ptr, g.col_idx, X, np.zeros_like(W_q), W_k, W_v, 1.0), (A / A.sum(axis=1, keepdims=True)) @ V, 1e-12)
    _close(oracle.dotgat_layer(n, n, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.0), (A / A.sum(axis=1, keepdims=True)) @ V, 1e-12)
    # self loops only: alpha = 1, the layer is X W_v
    gs = synth.self_loops_only(n)
    _close(oracle.dotgat_layer(n, n, gs.row_ptr, gs.col_idx, X, W_q, W_k, W_v, 0.3), V, 1e-13)
    # queries and keys are not interchangeable: swapping them changes the weights on a non-symmetric score
    a = oracle.dotgat_layer(n, n, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.5)
    b = oracle.dotgat_layer(n, n, g.row_ptr, g.col_idx, X, W_k, W_q, W_v, 0.5)
    assert np.max(np.abs(a - b)) > 1e-3
    # a very large scale picks the neighbour with the largest score: the row becomes that neighbour's value projection
    Q, K = X.astype(np.float64) @ W_q.astype(np.float64), X.astype(np.float64) @ W_k.astype(np.float64)
    hard = oracle.dotgat_layer(n, n, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 1e4)
    for i in (0, 7, 21):
        cols = g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
        _close(hard[i], V[cols[np.argmax(K[cols] @ Q[i])]], 1e-9)
