"""CPU oracle (fp64, plain definitions).  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product path never does.  It shares no code with the HIP
library: the C file ``sensei_oracle.c`` is compiled on its own with gcc.

Contents
  * thin ctypes wrappers over ``sensei_oracle.c`` (primitives, plain-definition
    GCN / GAT layers, row-sampled layers),
  * ``gcn_composition`` / ``gat_composition``: every re-association of a layer,
    each following its sequence of primitives literally in fp64 (used for the
    "all re-associations agree" invariant; Matrix representation section:
    adjacent operands may be re-associated freely),
  * ``dense``: brute force with dense matrices, independent of the CSR code,
  * ``select_rules``: the embedding-size conditions of the code-generation
    section (which compositions are candidates for in<out / in>out).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sensei_oracle.c")
_LIBS = {False: os.path.join(_HERE, "liboracle.so"), True: os.path.join(_HERE, "liboracle_omp.so")}
_loaded = {}


def build(force: bool = False) -> None:
    for omp, path in _LIBS.items():
        if force or not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
            cmd = ["gcc", "-O2", "-shared", "-fPIC", _SRC, "-o", path, "-lm"]
            if omp:
                cmd[1:1] = ["-fopenmp", "-DORC_OMP"]
            subprocess.check_call(cmd)


def _lib(omp: bool = False):
    if omp not in _loaded:
        if not os.path.exists(_LIBS[omp]):
            build()
        lib = ctypes.CDLL(_LIBS[omp])
        lib.orc_threads.restype = ctypes.c_int
        _loaded[omp] = lib
    return _loaded[omp]


def threads(omp: bool = False) -> int:
    return int(_lib(omp).orc_threads())


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    a = np.asarray(a)
    assert a.dtype == np.float32, "oracle layers take the fp32 input bits"
    return np.ascontiguousarray(a)


I32, I64, DBL = ctypes.c_int32, ctypes.c_int64, ctypes.c_double


# ------------------------------------------------------------------ primitives

def degrees(n_rows, n_cols, row_ptr, col_idx):
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    dr = np.empty(n_rows, dtype=np.int32)
    dc = np.empty(n_cols, dtype=np.int32)
    _lib().orc_degrees(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(dr), _p(dc))
    return dr, dc


def inv_sqrt_deg(deg):
    deg = _i32(deg)
    out = np.empty(deg.size, dtype=np.float64)
    _lib().orc_inv_sqrt_deg(_p(deg), I64(deg.size), _p(out))
    return out


def spmm(row_ptr, col_idx, val, B):
    row_ptr, col_idx, B = _i32(row_ptr), _i32(col_idx), _f64(B)
    val = None if val is None else _f64(val)
    n_rows, F = row_ptr.size - 1, B.shape[1]
    C = np.empty((n_rows, F), dtype=np.float64)
    _lib().orc_spmm(I32(n_rows), _p(row_ptr), _p(col_idx), _p(val), _p(B), I64(F), I32(F), _p(C), I64(F))
    return C


def sddmm_mul(row_ptr, col_idx, a, b, c):
    row_ptr, col_idx, b, c = _i32(row_ptr), _i32(col_idx), _f64(b), _f64(c)
    a = None if a is None else _f64(a)
    d = np.empty(col_idx.size, dtype=np.float64)
    _lib().orc_sddmm_mul(I32(row_ptr.size - 1), _p(row_ptr), _p(col_idx), _p(a), _p(b), _p(c), _p(d))
    return d


def gat_scores(row_ptr, col_idx, s_l, s_r, slope=0.2):
    row_ptr, col_idx, s_l, s_r = _i32(row_ptr), _i32(col_idx), _f64(s_l), _f64(s_r)
    e = np.empty(col_idx.size, dtype=np.float64)
    _lib().orc_gat_scores(I32(row_ptr.size - 1), _p(row_ptr), _p(col_idx), _p(s_l), _p(s_r), DBL(slope), _p(e))
    return e


def edge_softmax(row_ptr, e):
    row_ptr, e = _i32(row_ptr), _f64(e)
    alpha = np.zeros(e.size, dtype=np.float64)
    _lib().orc_edge_softmax(I32(row_ptr.size - 1), _p(row_ptr), _p(e), _p(alpha))
    return alpha


def row_broadcast(s, X):
    s, X = _f64(s), _f64(X)
    Y = np.empty_like(X)
    _lib().orc_row_broadcast(I64(X.shape[0]), I32(X.shape[1]), _p(s), _p(X), I64(X.shape[1]), _p(Y), I64(X.shape[1]))
    return Y


def gemm(A, W):
    A, W = _f64(A), _f64(W)
    assert A.shape[1] == W.shape[0]
    Y = np.empty((A.shape[0], W.shape[1]), dtype=np.float64)
    _lib().orc_gemm(I64(A.shape[0]), I32(A.shape[1]), I32(W.shape[1]), _p(A), I64(A.shape[1]), _p(W), I64(W.shape[1]),
                    _p(Y), I64(W.shape[1]))
    return Y


def gemv(A, v):
    A, v = _f64(A), _f64(v)
    y = np.empty(A.shape[0], dtype=np.float64)
    _lib().orc_gemv(I64(A.shape[0]), I32(A.shape[1]), _p(A), I64(A.shape[1]), _p(v), _p(y))
    return y


def activation(Y, act):
    Y = _f64(Y).copy()
    _lib().orc_activation(I64(Y.size), ctypes.c_int(act), _p(Y))
    return Y


# ------------------------------------------------------- plain-definition layers

def gcn_layer(n_rows, n_cols, row_ptr, col_idx, X, W, act=0, rows=None, omp=False):
    """Eq. 3 / Eq. 4 as one plain definition; ``rows`` selects output rows."""
    row_ptr, col_idx, X, W = _i32(row_ptr), _i32(col_idx), _f32(X), _f32(W)
    F_in, F_out = W.shape
    assert X.shape == (n_cols, F_in)
    lib = _lib(omp)
    if rows is None:
        Y = np.empty((n_rows, F_out), dtype=np.float64)
        rc = lib.orc_gcn_layer(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in),
                               _p(W), I64(F_out), I32(F_out), ctypes.c_int(act), _p(Y))
    else:
        rows = _i32(rows)
        Y = np.empty((rows.size, F_out), dtype=np.float64)
        rc = lib.orc_gcn_layer_rows(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in),
                                    _p(W), I64(F_out), I32(F_out), ctypes.c_int(act), _p(rows), I32(rows.size), _p(Y))
    if rc != 0:
        raise RuntimeError(f"oracle gcn_layer failed ({rc})")
    return Y


def gat_layer(n_rows, n_cols, row_ptr, col_idx, X, W, a_l, a_r, slope=0.2, act=0, rows=None, omp=False):
    """Eq. 5 / Eq. 6 as one plain definition; ``rows`` selects output rows."""
    row_ptr, col_idx, X, W, a_l, a_r = _i32(row_ptr), _i32(col_idx), _f32(X), _f32(W), _f32(a_l), _f32(a_r)
    F_in, F_out = W.shape
    assert X.shape == (n_cols, F_in) and a_l.size == F_out and a_r.size == F_out
    lib = _lib(omp)
    if rows is None:
        Y = np.empty((n_rows, F_out), dtype=np.float64)
        rc = lib.orc_gat_layer(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in),
                               _p(W), I64(F_out), I32(F_out), _p(a_l), _p(a_r), DBL(slope), ctypes.c_int(act), _p(Y))
    else:
        rows = _i32(rows)
        Y = np.empty((rows.size, F_out), dtype=np.float64)
        rc = lib.orc_gat_layer_rows(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in),
                                    _p(W), I64(F_out), I32(F_out), _p(a_l), _p(a_r), DBL(slope), ctypes.c_int(act),
                                    _p(rows), I32(rows.size), _p(Y))
    if rc != 0:
        raise RuntimeError(f"oracle gat_layer failed ({rc})")
    return Y


def sgc_layer(n, row_ptr, col_idx, X, W, k_hops, act=0, rows=None):
    """K-hop simplified graph convolution act(A^^k X W), A^ = D^-1/2 A~ D^-1/2 as in Eq. 3, on a square pattern:
    k propagations (column scaling, neighbour sum of Eq. 1, row scaling) followed by the update.

    ``rows`` selects output rows: hop by hop only the nodes those rows reach are kept (row i of a propagation needs
    the previous values at the neighbours of i and nowhere else), which is the same sum restricted to what it reads."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    dr, dc = degrees(n, n, row_ptr, col_idx)
    r, c = inv_sqrt_deg(dr), inv_sqrt_deg(dc)
    W64 = _f32(W).astype(np.float64)
    if rows is None:
        H = _f32(X).astype(np.float64)
        for _ in range(k_hops):
            H = row_broadcast(r, spmm(row_ptr, col_idx, None, row_broadcast(c, H)))
        return activation(gemm(H, W64), act)
    need = [np.unique(np.asarray(rows, dtype=np.int64))]
    for _ in range(k_hops):   # need[h + 1]: the nodes read by the rows need[h]
        seg = [col_idx[row_ptr[i]:row_ptr[i + 1]] for i in need[-1]]
        need.append(np.unique(np.concatenate(seg)) if seg else np.zeros(0, dtype=np.int64))
    H = _f32(X)[need[k_hops]].astype(np.float64)
    for h in range(k_hops - 1, -1, -1):
        dst, src = need[h], need[h + 1]
        seg = [np.searchsorted(src, col_idx[row_ptr[i]:row_ptr[i + 1]]) for i in dst]   # neighbours as positions in src
        sub_ptr = np.concatenate([[0], np.cumsum([x.size for x in seg])])
        sub_idx = np.concatenate(seg) if seg else np.zeros(0, dtype=np.int32)
        H = row_broadcast(r[dst], spmm(sub_ptr, sub_idx, None, row_broadcast(c[src], H)))
    pick = np.searchsorted(need[0], np.asarray(rows, dtype=np.int64))
    return activation(gemm(H[pick], W64), act)


def sgc_backward(n, row_ptr, col_idx, X, W, k_hops, dY, Y=None, act=0, rows=None):
    """Gradient of sum(dY * Y) for the K-hop layer Y = act(A^^k X W) (chain rule on the definition in sgc_layer) -> (dX, dW):
    dP = dY (.) [Y > 0] (the fp32 forward output ``Y`` supplies the ReLU mask), G = (A^^T)^k dP, dW = X^T G, dX = G W^T.
    A^^T is written out as the transposed pattern with the same entry weights r_i c_j.  ``rows`` selects rows of dX."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    dr, dc = degrees(n, n, row_ptr, col_idx)
    r, c = inv_sqrt_deg(dr), inv_sqrt_deg(dc)
    val = sddmm_mul(row_ptr, col_idx, None, r, c)                      # A^[i, j] = r_i c_j on the pattern
    src = np.repeat(np.arange(n, dtype=np.int32), np.diff(row_ptr))    # row of every stored entry
    order = np.lexsort((src, col_idx))                                 # the same entries by (column, row): rows of the transpose
    t_ptr = np.concatenate([[0], np.cumsum(np.bincount(col_idx, minlength=n))]).astype(np.int32)
    t_idx, t_val = src[order], val[order]
    G = _f32(dY).astype(np.float64)
    if act == 1:
        G = G * (_f32(Y) > 0)
    for _ in range(k_hops):
        G = spmm(t_ptr, t_idx, t_val, G)
    dW = gemm(np.ascontiguousarray(_f32(X).astype(np.float64).T), G)
    dX = gemm(G if rows is None else G[np.asarray(rows, dtype=np.int64)], np.ascontiguousarray(_f32(W).astype(np.float64).T))
    return dX, dW


def tagcn_layer(n, row_ptr, col_idx, X, W, k_hops, act=0):
    """TAGCN layer act(sum_{k=0..K} A^^k X W_k) with A^ the normalised operator of Eq. 3 on a square pattern and W the
    K + 1 weight blocks stacked by rows: the sum written out term by term, each hop one more propagation of the last."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    dr, dc = degrees(n, n, row_ptr, col_idx)
    r, c = inv_sqrt_deg(dr), inv_sqrt_deg(dc)
    H = _f32(X).astype(np.float64)
    W64 = _f32(W).astype(np.float64)
    f_in = H.shape[1]
    assert W64.shape[0] == (k_hops + 1) * f_in
    Y = gemm(H, W64[:f_in])
    for k in range(1, k_hops + 1):
        H = row_broadcast(r, spmm(row_ptr, col_idx, None, row_broadcast(c, H)))
        Y = Y + gemm(H, W64[k * f_in:(k + 1) * f_in])
    return activation(Y, act)


def tagcn_backward(n, row_ptr, col_idx, X, W, k_hops, dY, Y=None, act=0, rows=None):
    """Gradient of sum(dY * Y) for the TAGCN layer Y = act(sum_k A^^k X W_k) (chain rule on tagcn_layer, term by term) -> (dX, dW):
    dP = dY (.) [Y > 0] (the fp32 forward output ``Y`` supplies the ReLU mask); term k is H_k W_k with H_k = A^^k X, so
    dW_k = H_k^T dP (stacked by rows like W) and the term's share of dX is dP W_k^T carried back through its k propagations,
    (A^^T)^k (dP W_k^T).  A^^T is written out as the transposed pattern with the same entry weights r_i c_j.  ``rows`` selects
    rows of dX."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    dr, dc = degrees(n, n, row_ptr, col_idx)
    r, c = inv_sqrt_deg(dr), inv_sqrt_deg(dc)
    val = sddmm_mul(row_ptr, col_idx, None, r, c)                      # A^[i, j] = r_i c_j on the pattern
    src = np.repeat(np.arange(n, dtype=np.int32), np.diff(row_ptr))    # row of every stored entry
    order = np.lexsort((src, col_idx))                                 # the same entries by (column, row): rows of the transpose
    t_ptr = np.concatenate([[0], np.cumsum(np.bincount(col_idx, minlength=n))]).astype(np.int32)
    t_idx, t_val = src[order], val[order]
    W64 = _f32(W).astype(np.float64)
    H = _f32(X).astype(np.float64)
    f_in = H.shape[1]
    assert W64.shape[0] == (k_hops + 1) * f_in
    dP = _f32(dY).astype(np.float64)
    if act == 1:
        dP = dP * (_f32(Y) > 0)
    dW = np.zeros_like(W64)
    dX = np.zeros_like(H)
    for k in range(k_hops + 1):
        if k > 0:
            H = row_broadcast(r, spmm(row_ptr, col_idx, None, row_broadcast(c, H)))     # H_k = A^ H_(k-1)
        dW[k * f_in:(k + 1) * f_in] = gemm(np.ascontiguousarray(H.T), dP)
        M = gemm(dP, np.ascontiguousarray(W64[k * f_in:(k + 1) * f_in].T))
        for _ in range(k):
            M = spmm(t_ptr, t_idx, t_val, M)
        dX = dX + M
    return (dX if rows is None else dX[np.asarray(rows, dtype=np.int64)]), dW


def gatv2_layer(n_rows, n_cols, row_ptr, col_idx, X, W_l, W_r, att, slope=0.2, act=0, rows=None):
    """GATv2 layer: Theta_l = X W_l (destinations = the first n_rows sources), Theta_r = X W_r,
    e_ij = att . LeakyReLU(Theta_l[i] + Theta_r[j]) on the stored entries (Eq. 2 with a vector per entry), alpha = row
    softmax of e as in Eq. 5, Y = act(alpha Theta_r) as in Eq. 6.  ``rows`` selects output rows."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    X32 = _f32(X)
    Th_r = gemm(X32.astype(np.float64), _f32(W_r).astype(np.float64))
    a = _f32(att).astype(np.float64)
    sel = np.arange(n_rows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    Th_l = gemm(X32[sel].astype(np.float64), _f32(W_l).astype(np.float64))
    seg = [col_idx[row_ptr[i]:row_ptr[i + 1]] for i in sel]
    sub_ptr = np.concatenate([[0], np.cumsum([x.size for x in seg])]).astype(np.int32)
    sub_idx = (np.concatenate(seg) if seg else np.zeros(0)).astype(np.int32)
    e = np.empty(sub_idx.size, dtype=np.float64)
    for q in range(sel.size):
        lo, hi = sub_ptr[q], sub_ptr[q + 1]
        T = Th_l[q][None, :] + Th_r[sub_idx[lo:hi]]
        e[lo:hi] = np.where(T > 0.0, T, slope * T) @ a
    alpha = edge_softmax(sub_ptr, e)
    return activation(spmm(sub_ptr, sub_idx, alpha, Th_r), act)


def gatv2_backward(n_rows, n_cols, row_ptr, col_idx, X, W_l, W_r, att, dY, Y=None, slope=0.2, act=0):
    """Gradient of sum(dY * Y) for the GATv2 layer of gatv2_layer -> (dX, dW_l, dW_r, datt): the chain rule taken backwards through
    its steps, row by row.  dP = dY (.) [Y > 0] (the fp32 forward output ``Y`` supplies the ReLU mask).  For row i with
    neighbours j, U = Theta_l[i] + Theta_r[j] (one vector per entry), e = LeakyReLU(U) att, alpha = softmax(e):
      aggregation  Y_i = sum_j alpha_j Theta_r[j]:   dTheta_r[j] += alpha_j dP_i,  dalpha_j = <dP_i, Theta_r[j]>
      softmax:     de_j = alpha_j (dalpha_j - sum_k alpha_k dalpha_k)
      score:       datt += sum_j de_j LeakyReLU(U_j);   dU_j = de_j att (.) LeakyReLU'(U_j);   dTheta_l[i] += sum_j dU_j;
                   dTheta_r[j] += dU_j
    and then dW_l = X_dst^T dTheta_l, dW_r = X^T dTheta_r, dX = dTheta_r W_r^T with dTheta_l W_l^T added to the first n_rows rows."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    X64 = _f32(X).astype(np.float64)
    Wl, Wr = _f32(W_l).astype(np.float64), _f32(W_r).astype(np.float64)
    a = _f32(att).astype(np.float64)
    Th_l, Th_r = gemm(X64[:n_rows], Wl), gemm(X64, Wr)
    dP = _f32(dY).astype(np.float64)
    if act == 1:
        dP = dP * (_f32(Y) > 0)
    dTh_l, dTh_r = np.zeros_like(Th_l), np.zeros_like(Th_r)
    datt = np.zeros_like(a)
    for i in range(n_rows):
        nb = col_idx[row_ptr[i]:row_ptr[i + 1]]
        if nb.size == 0:
            continue
        U = Th_l[i][None, :] + Th_r[nb]
        L = np.where(U > 0.0, U, slope * U)
        e = L @ a
        p = np.exp(e - e.max())
        alpha = p / p.sum()
        dalpha = Th_r[nb] @ dP[i]
        de = alpha * (dalpha - float(alpha @ dalpha))
        datt += de @ L
        dU = de[:, None] * (a[None, :] * np.where(U > 0.0, 1.0, slope))
        dTh_l[i] += dU.sum(axis=0)
        np.add.at(dTh_r, nb, alpha[:, None] * dP[i][None, :] + dU)
    dW_l = gemm(np.ascontiguousarray(X64[:n_rows].T), dTh_l)
    dW_r = gemm(np.ascontiguousarray(X64.T), dTh_r)
    dX = gemm(dTh_r, np.ascontiguousarray(Wr.T))
    dX[:n_rows] += gemm(dTh_l, np.ascontiguousarray(Wl.T))
    return dX, dW_l, dW_r, datt


def dotgat_layer(n_rows, n_cols, row_ptr, col_idx, X, W_q, W_k, W_v, scale, act=0, rows=None):
    """Key-query attention layer (the score function of GaAN-style layers, which the paper's discussion of attention variants
    names): Q = X W_q over the destinations (= the first n_rows sources), K = X W_k and V = X W_v over the sources,
    e_ij = scale <Q[i], K[j]> on the stored entries (Eq. 2 with a dot product), alpha = row softmax of e as in Eq. 5,
    Y = act(alpha V) as in Eq. 6.  ``rows`` selects output rows."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    X32 = _f32(X)
    K = gemm(X32.astype(np.float64), _f32(W_k).astype(np.float64))
    V = gemm(X32.astype(np.float64), _f32(W_v).astype(np.float64))
    sel = np.arange(n_rows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    Q = gemm(X32[sel].astype(np.float64), _f32(W_q).astype(np.float64))
    seg = [col_idx[row_ptr[i]:row_ptr[i + 1]] for i in sel]
    sub_ptr = np.concatenate([[0], np.cumsum([x.size for x in seg])]).astype(np.int32)
    sub_idx = (np.concatenate(seg) if seg else np.zeros(0)).astype(np.int32)
    e = np.empty(sub_idx.size, dtype=np.float64)
    for q in range(sel.size):
        lo, hi = sub_ptr[q], sub_ptr[q + 1]
        e[lo:hi] = float(scale) * (K[sub_idx[lo:hi]] @ Q[q])
    alpha = edge_softmax(sub_ptr, e)
    return activation(spmm(sub_ptr, sub_idx, alpha, V), act)


def dotgat_backward(n_rows, n_cols, row_ptr, col_idx, X, W_q, W_k, W_v, scale, dY, Y=None, act=0):
    """Gradient of sum(dY * Y) for the key-query attention layer of dotgat_layer -> (dX, dW_q, dW_k, dW_v): the chain rule backwards
    through its steps, row by row.  dP = dY (.) [Y > 0] (the fp32 forward output ``Y`` supplies the ReLU mask).  For row i with
    neighbours j: e_j = scale <Q_i, K_j>, alpha = softmax(e), Y_i = sum_j alpha_j V_j, hence
      dV_j += alpha_j dP_i,   dalpha_j = <dP_i, V_j>,   de_j = alpha_j (dalpha_j - sum_k alpha_k dalpha_k),
      dQ_i = scale sum_j de_j K_j,   dK_j += scale de_j Q_i,
    and dW_q = X_dst^T dQ, dW_k = X^T dK, dW_v = X^T dV, dX = dK W_k^T + dV W_v^T with dQ W_q^T added to the first n_rows rows."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    X64 = _f32(X).astype(np.float64)
    Wq, Wk, Wv = (_f32(W).astype(np.float64) for W in (W_q, W_k, W_v))
    Q, K, V = gemm(X64[:n_rows], Wq), gemm(X64, Wk), gemm(X64, Wv)
    dP = _f32(dY).astype(np.float64)
    if act == 1:
        dP = dP * (_f32(Y) > 0)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    sc = float(scale)
    for i in range(n_rows):
        nb = col_idx[row_ptr[i]:row_ptr[i + 1]]
        if nb.size == 0:
            continue
        e = sc * (K[nb] @ Q[i])
        p = np.exp(e - e.max())
        alpha = p / p.sum()
        dalpha = V[nb] @ dP[i]
        de = alpha * (dalpha - float(alpha @ dalpha))
        dQ[i] = sc * (de @ K[nb])
        np.add.at(dK, nb, sc * de[:, None] * Q[i][None, :])
        np.add.at(dV, nb, alpha[:, None] * dP[i][None, :])
    dW_q = gemm(np.ascontiguousarray(X64[:n_rows].T), dQ)
    dW_k = gemm(np.ascontiguousarray(X64.T), dK)
    dW_v = gemm(np.ascontiguousarray(X64.T), dV)
    dX = gemm(dK, np.ascontiguousarray(Wk.T)) + gemm(dV, np.ascontiguousarray(Wv.T))
    dX[:n_rows] += gemm(dQ, np.ascontiguousarray(Wq.T))
    return dX, dW_q, dW_k, dW_v


def gat_layer_heads(n_rows, n_cols, row_ptr, col_idx, X, W, a_l, a_r, n_heads, slope=0.2, act=0, rows=None, omp=False):
    """Multi-head GAT with concatenated heads: head h is the single-head layer of Eq. 5 / 6 on columns
    [h d, (h + 1) d) of W, a_l, a_r (heads share nothing but the input)."""
    W, a_l, a_r = _f32(W), _f32(a_l), _f32(a_r)
    assert W.shape[1] % n_heads == 0
    d = W.shape[1] // n_heads
    return np.concatenate([gat_layer(n_rows, n_cols, row_ptr, col_idx, X, np.ascontiguousarray(W[:, h * d:(h + 1) * d]),
                                     a_l[h * d:(h + 1) * d], a_r[h * d:(h + 1) * d], slope, act, rows=rows, omp=omp)
                           for h in range(n_heads)], axis=1)


def gcn_backward(n_rows, n_cols, row_ptr, col_idx, X, W, dY, Y=None, act=0, rows=None, want_dw=True, omp=False, with_dz=False):
    """Gradient of sum(dY * Y) for the GCN layer (chain rule on Eq. 3) -> (dX, dW).

    ``Y`` (the fp32 forward output) supplies the ReLU mask when ``act`` == 1; ``rows`` selects rows of dX;
    ``with_dz`` appends dZ = d(X W) (n_cols x F_out) to the result."""
    row_ptr, col_idx, X, W, dY = _i32(row_ptr), _i32(col_idx), _f32(X), _f32(W), _f32(dY)
    F_in, F_out = W.shape
    assert X.shape == (n_cols, F_in) and dY.shape == (n_rows, F_out)
    if act == 1:
        Y = _f32(Y)
        assert Y.shape == dY.shape
    sel = None if rows is None else _i32(rows)
    n_out = n_cols if sel is None else sel.size
    dX = np.empty((n_out, F_in), dtype=np.float64)
    dW = np.empty((F_in, F_out), dtype=np.float64) if (want_dw or sel is None) else None
    dZ = np.empty((n_cols, F_out), dtype=np.float64) if (with_dz and dW is not None) else None
    rc = _lib(omp).orc_gcn_backward(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in), _p(W), I64(F_out),
                                   I32(F_out), _p(Y) if act == 1 else None, I64(F_out), _p(dY), I64(F_out), ctypes.c_int(act),
                                   None if sel is None else _p(sel), I32(0 if sel is None else sel.size),
                                   ctypes.c_int(1 if dW is not None else 0), _p(dX), None if dW is None else _p(dW),
                                   None if dZ is None else _p(dZ))
    if rc != 0:
        raise RuntimeError(f"oracle gcn_backward failed ({rc})")
    return (dX, dW, dZ) if with_dz else (dX, dW)


def gat_backward(n_rows, n_cols, row_ptr, col_idx, X, W, a_l, a_r, dY, Y=None, slope=0.2, act=0, omp=False, with_dtheta=False):
    """Gradient of sum(dY * Y) for the GAT layer (chain rule on Eq. 5 / 6) -> (dX, dW, da_l, da_r[, dTheta, ds_l, ds_r])."""
    row_ptr, col_idx, X, W, a_l, a_r, dY = _i32(row_ptr), _i32(col_idx), _f32(X), _f32(W), _f32(a_l), _f32(a_r), _f32(dY)
    F_in, F_out = W.shape
    assert X.shape == (n_cols, F_in) and dY.shape == (n_rows, F_out)
    if act == 1:
        Y = _f32(Y)
        assert Y.shape == dY.shape
    dX = np.empty((n_cols, F_in), dtype=np.float64)
    dW = np.empty((F_in, F_out), dtype=np.float64)
    dal, dar = np.empty(F_out, dtype=np.float64), np.empty(F_out, dtype=np.float64)
    dTh = np.empty((n_cols, F_out), dtype=np.float64) if with_dtheta else None
    ds = np.empty(2 * n_cols, dtype=np.float64) if with_dtheta else None
    rc = _lib(omp).orc_gat_backward(I32(n_rows), I32(n_cols), _p(row_ptr), _p(col_idx), _p(X), I64(F_in), I32(F_in), _p(W), I64(F_out),
                                   I32(F_out), _p(a_l), _p(a_r), DBL(slope), _p(Y) if act == 1 else None, I64(F_out), _p(dY),
                                   I64(F_out), ctypes.c_int(act), _p(dX), _p(dW), _p(dal), _p(dar), None if dTh is None else _p(dTh),
                                   None if ds is None else _p(ds))
    if rc != 0:
        raise RuntimeError(f"oracle gat_backward failed ({rc})")
    return (dX, dW, dal, dar, dTh, ds[:n_cols], ds[n_cols:]) if with_dtheta else (dX, dW, dal, dar)


def gat_backward_heads(n_rows, n_cols, row_ptr, col_idx, X, W, a_l, a_r, n_heads, dY, Y=None, slope=0.2, act=0, omp=False):
    """Gradient of sum(dY * Y) for the multi-head layer of gat_layer_heads -> (dX, dW, da_l, da_r).  The heads share only the input:
    head h is the single-head layer on columns [h d, (h + 1) d), so its gradients with respect to its own columns of W, a_l, a_r
    are those of that layer for its columns of dY, and dX is the sum of the heads' input gradients."""
    W, a_l, a_r, dY = _f32(W), _f32(a_l), _f32(a_r), _f32(dY)
    assert W.shape[1] % n_heads == 0
    d = W.shape[1] // n_heads
    dX = np.zeros((n_cols, W.shape[0]), dtype=np.float64)
    dW = np.empty(W.shape, dtype=np.float64)
    dal, dar = np.empty(W.shape[1], dtype=np.float64), np.empty(W.shape[1], dtype=np.float64)
    for h in range(n_heads):
        c = slice(h * d, (h + 1) * d)
        Yh = None if Y is None else np.ascontiguousarray(_f32(Y)[:, c])
        gx, gw, gl, gr = gat_backward(n_rows, n_cols, row_ptr, col_idx, X, np.ascontiguousarray(W[:, c]), a_l[c], a_r[c],
                                      np.ascontiguousarray(dY[:, c]), Y=Yh, slope=slope, act=act, omp=omp)
        dX += gx
        dW[:, c], dal[c], dar[c] = gw, gl, gr
    return dX, dW, dal, dar


# ------------------------------------------------------------- re-associations

GCN_COMPOSITIONS = ("DYN_AGG", "DYN_UPD", "DYNF_AGG", "DYNF_UPD", "PRE_AGG", "PRE_UPD")
GAT_COMPOSITIONS = ("REUSE", "RECOMP", "RECOMP_FOLD", "REUSE_FOLD")


def gcn_composition(comp_id, n_rows, n_cols, row_ptr, col_idx, X, W, act=0):
    """One GCN layer following composition ``comp_id`` step by step in fp64.

    0 DYN_AGG   row-broadcast(c,X) -> pattern SpMM -> row-broadcast(r) -> GEMM    (Eq. 3, update last)
    1 DYN_UPD   GEMM -> row-broadcast(c) -> pattern SpMM -> row-broadcast(r)      (Eq. 3, update first)
    2 DYNF_AGG  SpMM with both scalings applied inside the sum -> GEMM
    3 DYNF_UPD  GEMM -> SpMM with both scalings applied inside the sum
    4 PRE_AGG   N~ by SDDMM (Eq. 4) -> weighted SpMM -> GEMM
    5 PRE_UPD   N~ by SDDMM (Eq. 4) -> GEMM -> weighted SpMM
    """
    dr, dc = degrees(n_rows, n_cols, row_ptr, col_idx)
    r, c = inv_sqrt_deg(dr), inv_sqrt_deg(dc)
    X64, W64 = _f64(X), _f64(W)
    if comp_id == 0:
        out = gemm(row_broadcast(r, spmm(row_ptr, col_idx, None, row_broadcast(c, X64))), W64)
    elif comp_id == 1:
        out = row_broadcast(r, spmm(row_ptr, col_idx, None, row_broadcast(c, gemm(X64, W64))))
    elif comp_id == 2:
        out = gemm(_spmm_scaled(row_ptr, col_idx, r, c, X64), W64)
    elif comp_id == 3:
        out = _spmm_scaled(row_ptr, col_idx, r, c, gemm(X64, W64))
    elif comp_id == 4:
        nt = sddmm_mul(row_ptr, col_idx, None, r, c)
        out = gemm(spmm(row_ptr, col_idx, nt, X64), W64)
    elif comp_id == 5:
        nt = sddmm_mul(row_ptr, col_idx, None, r, c)
        out = spmm(row_ptr, col_idx, nt, gemm(X64, W64))
    else:
        raise ValueError("bad GCN composition id")
    return activation(out, act)


def _spmm_scaled(row_ptr, col_idx, r, c, B):
    """U[i,:] = r_i * sum_j c_j B[j,:] (pure-Python loop over rows; small inputs only)."""
    n_rows = len(row_ptr) - 1
    U = np.zeros((n_rows, B.shape[1]), dtype=np.float64)
    for i in range(n_rows):
        acc = np.zeros(B.shape[1], dtype=np.float64)
        for k in range(row_ptr[i], row_ptr[i + 1]):
            acc += c[col_idx[k]] * B[col_idx[k]]
        U[i] = r[i] * acc
    return U


def gat_composition(comp_id, n_rows, n_cols, row_ptr, col_idx, X, W, a_l, a_r, slope=0.2, act=0):
    """One GAT layer following composition ``comp_id`` step by step in fp64.

    0 REUSE        Theta=XW; s=Theta.a; scores; softmax; alpha.Theta                  (Eq. 5-6)
    1 RECOMP       Theta=XW; s=Theta.a; scores; softmax; (alpha.X).W                  (Eq. 7)
    2 RECOMP_FOLD  s=X.(W.a); scores; softmax; (alpha.X).W
    3 REUSE_FOLD   s=X.(W.a); scores; softmax; alpha.(XW)
    """
    X64, W64, al, ar = _f64(X), _f64(W), _f64(a_l), _f64(a_r)
    theta = None
    if comp_id in (0, 1):
        theta = gemm(X64, W64)
        s_l, s_r = gemv(theta, al), gemv(theta, ar)
    elif comp_id in (2, 3):
        s_l, s_r = gemv(X64, gemv(W64, al)), gemv(X64, gemv(W64, ar))
    else:
        raise ValueError("bad GAT composition id")
    alpha = edge_softmax(row_ptr, gat_scores(row_ptr, col_idx, s_l[:n_rows], s_r, slope))
    if comp_id == 0:
        out = spmm(row_ptr, col_idx, alpha, theta)
    elif comp_id == 3:
        out = spmm(row_ptr, col_idx, alpha, gemm(X64, W64))
    else:
        out = gemm(spmm(row_ptr, col_idx, alpha, X64), W64)
    return activation(out, act)


# -------------------------------------------------------------- selector rules

def select_rules(kind, f_in, f_out):
    """Composition ids left after the embedding-size conditions (code generation section;
    GAT: recomputation is a candidate only when the input size is smaller than the output)."""
    if kind == "gcn":
        agg, upd = (0, 2, 4), (1, 3, 5)
        if f_in < f_out:
            return agg
        if f_in > f_out:
            return upd
        return tuple(sorted(agg + upd))
    if kind == "gat":
        return (0, 1, 2, 3) if f_in < f_out else (0,)
    raise ValueError(kind)


def density(n_rows, n_cols, nnz):
    """Graph feature used by the cost models: non-zeros over matrix area."""
    return nnz / (float(n_rows) * float(n_cols))
