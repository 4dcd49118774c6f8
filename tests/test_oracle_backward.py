"""Pins for the backward-pass oracle: the gradients are checked against central finite differences of the
forward oracle, against dense linear algebra written here from the chain rule, and against closed forms."""
import numpy as np
import pytest

import oracle
import synth
from oracle import dense


def _grid(rng, shape, step=2.0 ** -6, span=32):
    """fp32 values on a coarse binary grid, so that value +- h is exact in fp32 for h a power of two >= 2^-12."""
    return (rng.integers(-span, span + 1, size=shape) * step).astype(np.float32)


def _rect_block(seed, n_rows, n_cols, per_row):
    rng = np.random.default_rng(seed)
    u = np.repeat(np.arange(n_rows), per_row)
    v = rng.integers(0, n_cols, size=u.size)
    return synth.build_csr(n_rows, n_cols, u, v, False, True)


def _close(a, b, tol):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    err = np.max(np.abs(a - b) / (1.0 + np.abs(b)))
    assert err < tol, err


def _central(f, x, h):
    """d f / d x by central differences, x an fp32 array perturbed in place, f() -> float (fp64)."""
    g = np.zeros(x.shape, dtype=np.float64)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        keep = x[idx]
        x[idx] = keep + np.float32(h)
        up = f()
        x[idx] = keep - np.float32(h)
        dn = f()
        x[idx] = keep
        g[idx] = (up - dn) / (2.0 * h)
    return g


def _richardson(f, x, h):
    return (4.0 * _central(f, x, h / 2) - _central(f, x, h)) / 3.0


# ------------------------------------------------------------------ GCN

@pytest.mark.parametrize("shape", ["square", "rect"])
def test_gcn_backward_is_the_gradient_of_the_forward(shape):
    rng = np.random.default_rng(5)
    g = synth.erdos_renyi(5, 14, 30) if shape == "square" else _rect_block(6, 6, 15, 3)
    f_in, f_out = 5, 4
    X, W, dY = _grid(rng, (g.n_cols, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (g.n_rows, f_out))

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.gcn_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, 0)))

    dX, dW = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY)
    # the identity-activation layer is linear in X and in W: central differences are exact up to rounding
    _close(dX, _central(loss, X, 2.0 ** -4), 1e-10)
    _close(dW, _central(loss, W, 2.0 ** -4), 1e-10)


def test_gcn_backward_with_relu_mask_matches_finite_differences():
    rng = np.random.default_rng(8)
    g = synth.erdos_renyi(8, 12, 25)
    f_in, f_out = 4, 3
    X, W, dY = _grid(rng, (12, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (12, f_out))
    P = oracle.gcn_layer(12, 12, g.row_ptr, g.col_idx, X, W, 0)
    h = 2.0 ** -12
    ok = np.abs(P) > 64 * h  # pre-activations close enough to zero for a +-h step to cross the kink are left out of the loss
    assert ok.mean() > 0.5 and (P[ok] > 0).any() and (P[ok] < 0).any()
    dY = (dY * ok).astype(np.float32)
    Y = np.maximum(P, 0.0).astype(np.float32)

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.gcn_layer(12, 12, g.row_ptr, g.col_idx, X, W, 1)))

    dX, dW = oracle.gcn_backward(12, 12, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=1)
    _close(dX, _central(loss, X, h), 1e-9)
    _close(dW, _central(loss, W, h), 1e-9)
    # and the mask really matters
    dX0, _ = oracle.gcn_backward(12, 12, g.row_ptr, g.col_idx, X, W, dY)
    assert np.max(np.abs(dX0 - dX)) > 1e-3


@pytest.mark.parametrize("shape", ["square", "rect"])
def test_gcn_backward_matches_dense_chain_rule(shape):
    rng = np.random.default_rng(11)
    g = synth.rmat(11, 40, 120) if shape == "square" else _rect_block(12, 9, 30, 4)
    f_in, f_out = 6, 5
    X = rng.standard_normal((g.n_cols, f_in)).astype(np.float32)
    W = rng.standard_normal((f_in, f_out)).astype(np.float32)
    dY = rng.standard_normal((g.n_rows, f_out)).astype(np.float32)
    A = dense.dense_pattern(g.n_rows, g.n_cols, g.row_ptr, g.col_idx)
    r = 1.0 / np.sqrt(np.maximum(A.sum(axis=1), 1.0))
    c = 1.0 / np.sqrt(np.maximum(A.sum(axis=0), 1.0))
    Ahat = r[:, None] * A * c[None, :]
    Y = np.maximum(Ahat @ X.astype(np.float64) @ W.astype(np.float64), 0.0).astype(np.float32)
    dP = dY.astype(np.float64) * (Y > 0)
    dX, dW = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=1)
    _close(dX, Ahat.T @ dP @ W.astype(np.float64).T, 1e-11)
    _close(dW, (Ahat @ X.astype(np.float64)).T @ dP, 1e-11)
    dZ = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=1, with_dz=True)[2]
    _close(dZ, Ahat.T @ dP, 1e-11)  # the optional third result: gradient with respect to Z = X W
    # selected rows of dX, with and without the dW reduction
    rows = np.array([0, g.n_cols - 1, 3, 3], dtype=np.int32)
    dXs, dWs = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=1, rows=rows)
    _close(dXs, dX[rows], 1e-12)
    _close(dWs, dW, 1e-12)
    dXs2, none = oracle.gcn_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W, dY, Y=Y, act=1, rows=rows, want_dw=False)
    assert none is None
    _close(dXs2, dX[rows], 1e-12)


def test_gcn_backward_on_self_loops_is_a_dense_linear_layer():
    rng = np.random.default_rng(2)
    g = synth.self_loops_only(17)
    X, W, dY = (rng.standard_normal(s).astype(np.float32) for s in ((17, 6), (6, 3), (17, 3)))
    dX, dW = oracle.gcn_backward(17, 17, g.row_ptr, g.col_idx, X, W, dY)
    _close(dX, dY.astype(np.float64) @ W.astype(np.float64).T, 1e-12)
    _close(dW, X.astype(np.float64).T @ dY.astype(np.float64), 1e-12)


# ------------------------------------------------------------------ GAT

def test_gat_backward_is_the_gradient_of_the_forward():
    rng = np.random.default_rng(21)
    g = synth.erdos_renyi(21, 10, 18)
    f_in, f_out = 4, 3
    X, W, dY = _grid(rng, (10, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (10, f_out))
    a_l, a_r = _grid(rng, (f_out,)), _grid(rng, (f_out,))

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.gat_layer(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.2, 0)))

    # stay clear of the LeakyReLU kink: every t_ij = s_l[i] + s_r[j] well away from zero
    Th = X.astype(np.float64) @ W.astype(np.float64)
    sl, sr = Th @ a_l.astype(np.float64), Th @ a_r.astype(np.float64)
    t = np.concatenate([sl[i] + sr[g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]] for i in range(10)])
    h = 2.0 ** -11  # a step of h moves a logit by less than 3 h for these value ranges
    assert np.min(np.abs(t)) > 8 * h
    dX, dW, dal, dar = oracle.gat_backward(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY)
    _close(dX, _richardson(loss, X, h), 1e-7)
    _close(dW, _richardson(loss, W, h), 1e-7)
    _close(dal, _richardson(loss, a_l, h), 1e-7)
    _close(dar, _richardson(loss, a_r, h), 1e-7)
    assert np.max(np.abs(dal)) > 1e-3 and np.max(np.abs(dar)) > 1e-3  # the attention path carries gradient


def test_gat_backward_with_relu_and_other_slope():
    f_in, f_out = 3, 4
    h = 2.0 ** -11
    g = synth.rmat(22, 12, 30)
    for seed in range(22, 40):  # first seed whose logits all stay clear of the LeakyReLU kink
        rng = np.random.default_rng(seed)
        X, W, dY = _grid(rng, (12, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (12, f_out))
        a_l, a_r = _grid(rng, (f_out,)), _grid(rng, (f_out,))
        Th = X.astype(np.float64) @ W.astype(np.float64)
        sl, sr = Th @ a_l.astype(np.float64), Th @ a_r.astype(np.float64)
        t = np.concatenate([sl[i] + sr[g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]] for i in range(12)])
        if np.min(np.abs(t)) > 8 * h:
            break
    else:
        raise AssertionError("no seed keeps the logits away from zero")
    P = oracle.gat_layer(12, 12, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.05, 0)
    ok = np.abs(P) > 64 * h  # outputs near the ReLU kink are left out of the loss
    assert ok.mean() > 0.5 and (P[ok] > 0).any() and (P[ok] < 0).any()
    dYm = (dY * ok).astype(np.float32)
    Y = np.maximum(P, 0.0).astype(np.float32)

    def loss():
        return float(np.sum(dYm.astype(np.float64) * oracle.gat_layer(12, 12, g.row_ptr, g.col_idx, X, W, a_l, a_r, 0.05, 1)))

    dX, dW, dal, dar = oracle.gat_backward(12, 12, g.row_ptr, g.col_idx, X, W, a_l, a_r, dYm, Y=Y, slope=0.05, act=1)
    _close(dX, _richardson(loss, X, h), 1e-7)
    _close(dW, _richardson(loss, W, h), 1e-7)
    _close(dal, _richardson(loss, a_l, h), 1e-7)
    _close(dar, _richardson(loss, a_r, h), 1e-7)
    # the slope enters: the default slope gives another gradient
    dX2 = oracle.gat_backward(12, 12, g.row_ptr, g.col_idx, X, W, a_l, a_r, dYm, Y=Y, slope=0.2, act=1)[0]
    assert np.max(np.abs(dX2 - dX)) > 1e-6


def test_gat_backward_with_zero_attention_vectors_is_mean_aggregation():
    rng = np.random.default_rng(23)
    g = synth.erdos_renyi(23, 15, 30)
    f_in, f_out = 5, 4
    X = rng.standard_normal((15, f_in)).astype(np.float32)
    W = rng.standard_normal((f_in, f_out)).astype(np.float32)
    dY = rng.standard_normal((15, f_out)).astype(np.float32)
    z = np.zeros(f_out, dtype=np.float32)
    A = dense.dense_pattern(15, 15, g.row_ptr, g.col_idx)
    M = A / A.sum(axis=1, keepdims=True)
    dX, dW, dal, dar = oracle.gat_backward(15, 15, g.row_ptr, g.col_idx, X, W, z, z, dY)
    _close(dX, M.T @ dY.astype(np.float64) @ W.astype(np.float64).T, 1e-11)
    _close(dW, X.astype(np.float64).T @ M.T @ dY.astype(np.float64), 1e-11)
    dTh = oracle.gat_backward(15, 15, g.row_ptr, g.col_idx, X, W, z, z, dY, with_dtheta=True)[4]
    _close(dTh, M.T @ dY.astype(np.float64), 1e-11)  # the optional fifth result: gradient with respect to Theta = X W
    # d/da of the logits at a = 0: uniform alpha, softmax backward still active, LeakyReLU slope at t = 0 is `slope`
    Th = X.astype(np.float64) @ W.astype(np.float64)
    dalpha = dY.astype(np.float64) @ Th.T                       # <dP_i, Theta_j>
    de = M * (dalpha - np.sum(M * dalpha, axis=1, keepdims=True)) * (A != 0)
    dt = 0.2 * de
    _close(dal, Th.T @ dt.sum(axis=1), 1e-11)
    _close(dar, Th.T @ dt.sum(axis=0), 1e-11)
    ds_l, ds_r = oracle.gat_backward(15, 15, g.row_ptr, g.col_idx, X, W, z, z, dY, with_dtheta=True)[5:]
    _close(ds_l, dt.sum(axis=1), 1e-11)                          # sixth and seventh results: gradients of s_l and s_r
    _close(ds_r, dt.sum(axis=0), 1e-11)


def test_backward_is_linear_in_the_upstream_gradient():
    rng = np.random.default_rng(31)
    g = synth.rmat(31, 30, 90)
    X = rng.standard_normal((30, 5)).astype(np.float32)
    W = rng.standard_normal((5, 4)).astype(np.float32)
    a_l, a_r = rng.standard_normal(4).astype(np.float32), rng.standard_normal(4).astype(np.float32)
    d1, d2 = _grid(rng, (30, 4)), _grid(rng, (30, 4))
    for fn in (lambda d: oracle.gcn_backward(30, 30, g.row_ptr, g.col_idx, X, W, d),
               lambda d: oracle.gat_backward(30, 30, g.row_ptr, g.col_idx, X, W, a_l, a_r, d)):
        for a, b, s in zip(fn(d1), fn(d2), fn((d1 + d2).astype(np.float32))):
            _close(np.asarray(a) + np.asarray(b), s, 1e-11)


# ------------------------------------------------------------------ K-hop layer (SGC)

@pytest.mark.parametrize("k_hops", [1, 2, 3])
def test_sgc_backward_is_the_gradient_of_the_forward(k_hops):
    rng = np.random.default_rng(40 + k_hops)
    u = rng.integers(0, 12, size=26)
    v = rng.integers(0, 12, size=26)
    g = synth.build_csr(12, 12, u, v, False, True)      # not symmetric: the transposed operator really is another matrix
    f_in, f_out = 4, 3
    X, W, dY = _grid(rng, (12, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (12, f_out))

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.sgc_layer(12, g.row_ptr, g.col_idx, X, W, k_hops, 0)))

    dX, dW = oracle.sgc_backward(12, g.row_ptr, g.col_idx, X, W, k_hops, dY)
    _close(dX, _central(loss, X, 2.0 ** -8), 1e-9)      # the layer is linear in X and in W: central differences are exact
    _close(dW, _central(loss, W, 2.0 ** -8), 1e-9)
    rows = np.array([7, 0, 3])
    _close(oracle.sgc_backward(12, g.row_ptr, g.col_idx, X, W, k_hops, dY, rows=rows)[0], dX[rows], 1e-14)


def test_sgc_backward_special_cases():
    rng = np.random.default_rng(44)
    g = synth.erdos_renyi(9, 20, 45)
    X, W, dY = _grid(rng, (20, 5)), _grid(rng, (5, 6)), _grid(rng, (20, 6))
    # one hop is the GCN layer
    a = oracle.sgc_backward(20, g.row_ptr, g.col_idx, X, W, 1, dY)
    b = oracle.gcn_backward(20, 20, g.row_ptr, g.col_idx, X, W, dY)
    _close(a[0], b[0], 1e-13)
    _close(a[1], b[1], 1e-13)
    # dense algebra: dX = (A^^T)^k dP W^T, dW = X^T (A^^T)^k dP, with the ReLU mask of the forward output
    A = dense.dense_pattern(20, 20, g.row_ptr, g.col_idx)
    d = A.sum(axis=1)
    Ahat = A / np.sqrt(np.outer(d, A.sum(axis=0)))
    Y = oracle.sgc_layer(20, g.row_ptr, g.col_idx, X, W, 3, 1).astype(np.float32)
    assert (Y > 0).any() and (Y == 0).any()
    G = np.linalg.matrix_power(Ahat.T, 3) @ (dY.astype(np.float64) * (Y > 0))
    dX, dW = oracle.sgc_backward(20, g.row_ptr, g.col_idx, X, W, 3, dY, Y=Y, act=1)
    _close(dX, G @ W.astype(np.float64).T, 1e-12)
    _close(dW, X.astype(np.float64).T @ G, 1e-12)
    # self loops only: A^ = I, the layer is a GEMM whatever k
    gs = synth.self_loops_only(20)
    dXs, dWs = oracle.sgc_backward(20, gs.row_ptr, gs.col_idx, X, W, 4, dY)
    _close(dXs, dY.astype(np.float64) @ W.astype(np.float64).T, 1e-13)
    _close(dWs, X.astype(np.float64).T @ dY.astype(np.float64), 1e-13)


# ------------------------------------------------------------------ K-hop layer with a weight block per hop (TAGCN)

@pytest.mark.parametrize("k_hops", [0, 1, 2, 3])
def test_tagcn_backward_is_the_gradient_of_the_forward(k_hops):
    rng = np.random.default_rng(60 + k_hops)
    u = rng.integers(0, 12, size=26)
    v = rng.integers(0, 12, size=26)
    g = synth.build_csr(12, 12, u, v, False, True)      # not symmetric: the transposed operator really is another matrix
    f_in, f_out = 4, 3
    X, W, dY = _grid(rng, (12, f_in)), _grid(rng, ((k_hops + 1) * f_in, f_out)), _grid(rng, (12, f_out))

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.tagcn_layer(12, g.row_ptr, g.col_idx, X, W, k_hops, 0)))

    dX, dW = oracle.tagcn_backward(12, g.row_ptr, g.col_idx, X, W, k_hops, dY)
    _close(dX, _central(loss, X, 2.0 ** -8), 1e-9)      # the layer is linear in X and in W: central differences are exact
    _close(dW, _central(loss, W, 2.0 ** -8), 1e-9)
    rows = np.array([7, 0, 3])
    _close(oracle.tagcn_backward(12, g.row_ptr, g.col_idx, X, W, k_hops, dY, rows=rows)[0], dX[rows], 1e-14)


def test_tagcn_backward_special_cases():
    rng = np.random.default_rng(64)
    g = synth.build_csr(20, 20, rng.integers(0, 20, size=60), rng.integers(0, 20, size=60), False, True)   # not symmetric
    f_in, f_out, K = 5, 6, 3
    X, dY = _grid(rng, (20, f_in)), _grid(rng, (20, f_out))
    W = _grid(rng, ((K + 1) * f_in, f_out))
    X64, dY64 = X.astype(np.float64), dY.astype(np.float64)
    # no hops: a dense layer
    dX0, dW0 = oracle.tagcn_backward(20, g.row_ptr, g.col_idx, X, W[:f_in], 0, dY)
    _close(dX0, dY64 @ W[:f_in].astype(np.float64).T, 1e-13)
    _close(dW0, X64.T @ dY64, 1e-13)
    # only the last block non-zero: dX and that block's dW are those of the K-hop layer without per-hop weights
    Wl = np.zeros_like(W)
    Wl[K * f_in:] = W[K * f_in:]
    dXl, dWl = oracle.tagcn_backward(20, g.row_ptr, g.col_idx, X, Wl, K, dY)
    dXs, dWs = oracle.sgc_backward(20, g.row_ptr, g.col_idx, X, W[K * f_in:], K, dY)
    _close(dXl, dXs, 1e-13)
    _close(dWl[K * f_in:], dWs, 1e-13)
    # dense algebra with the ReLU mask of the forward output: dW_k = (A^^k X)^T dP, dX = sum_k (A^^T)^k dP W_k^T
    A = dense.dense_pattern(20, 20, g.row_ptr, g.col_idx)
    Ahat = A / np.sqrt(np.outer(A.sum(axis=1), A.sum(axis=0)))
    Y = oracle.tagcn_layer(20, g.row_ptr, g.col_idx, X, W, K, 1).astype(np.float32)
    assert (Y > 0).any() and (Y == 0).any()
    dP = dY64 * (Y > 0)
    dX, dW = oracle.tagcn_backward(20, g.row_ptr, g.col_idx, X, W, K, dY, Y=Y, act=1)
    want_dx = np.zeros((20, f_in))
    for k in range(K + 1):
        Wk = W[k * f_in:(k + 1) * f_in].astype(np.float64)
        _close(dW[k * f_in:(k + 1) * f_in], (np.linalg.matrix_power(Ahat, k) @ X64).T @ dP, 1e-12)
        want_dx += np.linalg.matrix_power(Ahat.T, k) @ dP @ Wk.T
    _close(dX, want_dx, 1e-12)
    assert np.abs(Ahat - Ahat.T).max() > 1e-3     # a transposed operand would show
    # self loops only: A^ = I, every hop sees X itself
    gs = synth.self_loops_only(20)
    dXi, dWi = oracle.tagcn_backward(20, gs.row_ptr, gs.col_idx, X, W, K, dY)
    Wsum = sum(W[k * f_in:(k + 1) * f_in].astype(np.float64) for k in range(K + 1))
    _close(dXi, dY64 @ Wsum.T, 1e-13)
    for k in range(K + 1):
        _close(dWi[k * f_in:(k + 1) * f_in], X64.T @ dY64, 1e-13)


# ------------------------------------------------------------------ GATv2

def _gatv2_case(seed0, g, f_in, f_out, slope, h):
    """First seed whose per-entry vectors U = Theta_l[i] + Theta_r[j] all stay clear of the LeakyReLU kink."""
    for seed in range(seed0, seed0 + 200):
        rng = np.random.default_rng(seed)
        X, dY = _grid(rng, (g.n_cols, f_in)), _grid(rng, (g.n_rows, f_out))
        W_l, W_r, att = _grid(rng, (f_in, f_out)), _grid(rng, (f_in, f_out)), _grid(rng, (f_out,))
        Tl = X[:g.n_rows].astype(np.float64) @ W_l.astype(np.float64)
        Tr = X.astype(np.float64) @ W_r.astype(np.float64)
        U = np.concatenate([Tl[i][None, :] + Tr[g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]] for i in range(g.n_rows)])
        if np.min(np.abs(U)) > 16 * h and np.min(np.abs(att)) > 0:
            return X, W_l, W_r, att, dY
    raise AssertionError("no seed keeps the score vectors away from zero")


@pytest.mark.parametrize("shape", ["square", "rect"])
def test_gatv2_backward_is_the_gradient_of_the_forward(shape):
    g = synth.rmat(71, 10, 22) if shape == "square" else _rect_block(72, 5, 11, 3)
    f_in, f_out, slope, h = 3, 3, 0.2, 2.0 ** -11
    X, W_l, W_r, att, dY = _gatv2_case(300, g, f_in, f_out, slope, h)

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.gatv2_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, slope, 0)))

    dX, dWl, dWr, da = oracle.gatv2_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_l, W_r, att, dY, slope=slope)
    _close(dX, _richardson(loss, X, h), 1e-7)
    _close(dWl, _richardson(loss, W_l, h), 1e-7)
    _close(dWr, _richardson(loss, W_r, h), 1e-7)
    _close(da, _richardson(loss, att, h), 1e-7)
    assert min(np.max(np.abs(dWl)), np.max(np.abs(da))) > 1e-4       # the score path carries gradient


def test_gatv2_backward_with_relu_and_other_slope():
    g = synth.rmat(73, 12, 30)
    f_in, f_out, slope, h = 3, 4, 0.05, 2.0 ** -11
    X, W_l, W_r, att, dY = _gatv2_case(400, g, f_in, f_out, slope, h)
    P = oracle.gatv2_layer(12, 12, g.row_ptr, g.col_idx, X, W_l, W_r, att, slope, 0)
    ok = np.abs(P) > 64 * h          # outputs near the ReLU kink are left out of the loss
    dYm = (dY * ok).astype(np.float32)
    Y = oracle.gatv2_layer(12, 12, g.row_ptr, g.col_idx, X, W_l, W_r, att, slope, 1).astype(np.float32)
    assert (Y > 0).any() and (Y == 0).any()

    def loss():
        return float(np.sum(dYm.astype(np.float64) * oracle.gatv2_layer(12, 12, g.row_ptr, g.col_idx, X, W_l, W_r, att, slope, 1)))

    got = oracle.gatv2_backward(12, 12, g.row_ptr, g.col_idx, X, W_l, W_r, att, dYm, Y=Y, slope=slope, act=1)
    for grad, x in zip(got, (X, W_l, W_r, att)):
        _close(grad, _richardson(loss, x, h), 1e-7)


def test_gatv2_backward_special_cases():
    rng = np.random.default_rng(75)
    g = synth.rmat(75, 16, 40)
    f_in, f_out = 4, 3
    X, dY = _grid(rng, (16, f_in)), _grid(rng, (16, f_out))
    W_l, W_r, att = _grid(rng, (f_in, f_out)), _grid(rng, (f_in, f_out)), _grid(rng, (f_out,))
    # slope 1: the score is att.Theta_l[i] + att.Theta_r[j], whose first term cancels in the softmax: the layer is the GAT layer with
    # W = W_r and a_r = att, nothing flows through W_l, and the gradients are those of that layer (its own oracle, written in C)
    dX, dWl, dWr, da = oracle.gatv2_backward(16, 16, g.row_ptr, g.col_idx, X, W_l, W_r, att, dY, slope=1.0)
    a_l = _grid(rng, (f_out,))
    wx, ww, _, war = oracle.gat_backward(16, 16, g.row_ptr, g.col_idx, X, W_r, a_l, att, dY, slope=1.0)
    _close(dWl, np.zeros_like(dWl), 1e-12)
    _close(dX, wx, 1e-11)
    _close(dWr, ww, 1e-11)
    _close(da, war, 1e-11)
    # att = 0: every row averages its neighbours and the score path is switched off: dTheta_r = M^T dP with M the row-normalised
    # pattern, dX = dTheta_r W_r^T, dW_r = X^T dTheta_r, dW_l = 0
    A = dense.dense_pattern(16, 16, g.row_ptr, g.col_idx)
    M = A / A.sum(axis=1, keepdims=True)
    zero = np.zeros(f_out, dtype=np.float32)
    dX0, dWl0, dWr0, da0 = oracle.gatv2_backward(16, 16, g.row_ptr, g.col_idx, X, W_l, W_r, zero, dY)
    dTr = M.T @ dY.astype(np.float64)
    _close(dX0, dTr @ W_r.astype(np.float64).T, 1e-12)
    _close(dWr0, X.astype(np.float64).T @ dTr, 1e-12)
    _close(dWl0, np.zeros_like(dWl0), 1e-12)
    # linear in dY
    d2 = _grid(rng, (16, f_out))
    a = oracle.gatv2_backward(16, 16, g.row_ptr, g.col_idx, X, W_l, W_r, att, dY)
    b = oracle.gatv2_backward(16, 16, g.row_ptr, g.col_idx, X, W_l, W_r, att, d2)
    c = oracle.gatv2_backward(16, 16, g.row_ptr, g.col_idx, X, W_l, W_r, att, (dY + d2).astype(np.float32))
    for x, y, z in zip(a, b, c):
        _close(np.asarray(x) + np.asarray(y), z, 1e-11)


# ------------------------------------------------------------------ key-query attention

@pytest.mark.parametrize("shape", ["square", "rect"])
def test_key_query_attention_backward_is_the_gradient_of_the_forward(shape):
    rng = np.random.default_rng(81)
    g = synth.rmat(81, 10, 22) if shape == "square" else _rect_block(82, 5, 11, 3)
    f_in, d_k, f_out, scale, h = 3, 2, 4, 0.7, 2.0 ** -11
    X, dY = _grid(rng, (g.n_cols, f_in)), _grid(rng, (g.n_rows, f_out))
    W_q, W_k, W_v = _grid(rng, (f_in, d_k)), _grid(rng, (f_in, d_k)), _grid(rng, (f_in, f_out))
    Y = oracle.dotgat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, 1).astype(np.float32)
    P = oracle.dotgat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, 0)
    for act in (0, 1):
        dYm = dY if act == 0 else (dY * (np.abs(P) > 64 * h)).astype(np.float32)   # outputs near the ReLU kink stay out of the loss

        def loss():
            return float(np.sum(dYm.astype(np.float64) * oracle.dotgat_layer(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, act)))

        got = oracle.dotgat_backward(g.n_rows, g.n_cols, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, dYm, Y=Y, act=act)
        for grad, x in zip(got, (X, W_q, W_k, W_v)):
            _close(grad, _richardson(loss, x, h), 1e-7)
        assert min(np.max(np.abs(got[1])), np.max(np.abs(got[2]))) > 1e-4      # the score path carries gradient


def test_key_query_attention_backward_special_cases():
    rng = np.random.default_rng(83)
    g = synth.build_csr(14, 14, rng.integers(0, 14, size=40), rng.integers(0, 14, size=40), False, True)   # not symmetric
    f_in, d_k, f_out, scale = 4, 3, 3, 0.5
    X, dY = _grid(rng, (14, f_in)), _grid(rng, (14, f_out))
    W_q, W_k, W_v = _grid(rng, (f_in, d_k)), _grid(rng, (f_in, d_k)), _grid(rng, (f_in, f_out))
    X64, d64 = X.astype(np.float64), dY.astype(np.float64)
    Wq, Wk, Wv = W_q.astype(np.float64), W_k.astype(np.float64), W_v.astype(np.float64)
    # the textbook gradient of dense masked attention softmax(scale Q K^T + mask) V, in matrices
    A = dense.dense_pattern(14, 14, g.row_ptr, g.col_idx)
    Q, K, V = X64 @ Wq, X64 @ Wk, X64 @ Wv
    S = np.where(A > 0, scale * Q @ K.T, -np.inf)
    Pm = np.exp(S - S.max(axis=1, keepdims=True))
    Pm /= Pm.sum(axis=1, keepdims=True)
    dPm = d64 @ V.T
    dS = Pm * (dPm - np.sum(Pm * dPm, axis=1, keepdims=True))
    dQ, dK, dV = scale * dS @ K, scale * dS.T @ Q, Pm.T @ d64
    got = oracle.dotgat_backward(14, 14, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, scale, dY)
    _close(got[0], dQ @ Wq.T + dK @ Wk.T + dV @ Wv.T, 1e-12)
    _close(got[1], X64.T @ dQ, 1e-12)
    _close(got[2], X64.T @ dK, 1e-12)
    _close(got[3], X64.T @ dV, 1e-12)
    assert np.abs(dS - dS.T).max() > 1e-4            # swapping the roles of rows and columns would show
    # scale 0: every row averages its neighbours, nothing flows through the queries and keys
    M = A / A.sum(axis=1, keepdims=True)
    z = oracle.dotgat_backward(14, 14, g.row_ptr, g.col_idx, X, W_q, W_k, W_v, 0.0, dY)
    _close(z[1], np.zeros_like(z[1]), 1e-13)
    _close(z[2], np.zeros_like(z[2]), 1e-13)
    _close(z[3], X64.T @ (M.T @ d64), 1e-12)
    _close(z[0], (M.T @ d64) @ Wv.T, 1e-12)


# ------------------------------------------------------------------ multi-head GAT

def test_multi_head_gat_backward_is_the_gradient_of_the_forward():
    g = synth.rmat(91, 10, 22)
    f_in, f_out, heads, h = 3, 4, 2, 2.0 ** -11
    for seed in range(91, 191):   # first seed whose logits, in every head, stay clear of the LeakyReLU kink
        rng = np.random.default_rng(seed)
        X, W, dY = _grid(rng, (10, f_in)), _grid(rng, (f_in, f_out)), _grid(rng, (10, f_out))
        a_l, a_r = _grid(rng, (f_out,)), _grid(rng, (f_out,))
        Th = X.astype(np.float64) @ W.astype(np.float64)
        d = f_out // heads
        t = []
        for k in range(heads):
            sl, sr = Th[:, k * d:(k + 1) * d] @ a_l[k * d:(k + 1) * d], Th[:, k * d:(k + 1) * d] @ a_r[k * d:(k + 1) * d]
            t += [sl[i] + sr[g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]] for i in range(10)]
        if np.min(np.abs(np.concatenate(t))) > 8 * h:
            break
    else:
        raise AssertionError("no seed keeps the logits away from zero")

    def loss():
        return float(np.sum(dY.astype(np.float64) * oracle.gat_layer_heads(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, heads, 0.2, 0)))

    got = oracle.gat_backward_heads(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, heads, dY)
    for grad, x in zip(got, (X, W, a_l, a_r)):
        _close(grad, _richardson(loss, x, h), 1e-7)
    # one head is the single-head layer
    one = oracle.gat_backward_heads(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, 1, dY)
    ref = oracle.gat_backward(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, dY)
    for a, b in zip(one, ref):
        _close(a, b, 1e-14)
    # a head's parameters do not feel the other head's output gradient
    dY2 = dY.copy()
    dY2[:, d:] = 0
    part = oracle.gat_backward_heads(10, 10, g.row_ptr, g.col_idx, X, W, a_l, a_r, heads, dY2)
    _close(part[1][:, :d], got[1][:, :d], 1e-14)
    _close(part[1][:, d:], np.zeros((f_in, d)), 1e-14)
