"""Dense brute force for tiny graphs.  TEST INFRASTRUCTURE ONLY.

Materialises the adjacency (with self edges, as stored), the degree matrices
and the attention matrix as dense fp64 arrays and evaluates the layer formulas
as written (Case study GCN Eq. 3-4; Case study GAT Eq. 5-6).  It shares
nothing with the CSR code in ``sensei_oracle.c``: the only sparse step is
scattering the pattern into a dense 0/1 matrix.
"""
from __future__ import annotations

import numpy as np


def dense_pattern(n_rows, n_cols, row_ptr, col_idx):
    A = np.zeros((n_rows, n_cols), dtype=np.float64)
    for i in range(n_rows):
        for k in range(row_ptr[i], row_ptr[i + 1]):
            A[i, col_idx[k]] = 1.0
    return A


def gcn_layer_dense(A, X, W, act=0):
    """sigma( D_r^-1/2 . A~ . D_c^-1/2 . X . W ) with dense matrices."""
    deg_r = np.maximum(A.sum(axis=1), 1.0)
    deg_c = np.maximum(A.sum(axis=0), 1.0)
    Dr = np.diag(1.0 / np.sqrt(deg_r))
    Dc = np.diag(1.0 / np.sqrt(deg_c))
    Y = Dr @ A @ Dc @ X.astype(np.float64) @ W.astype(np.float64)
    return np.maximum(Y, 0.0) if act == 1 else Y


def gat_layer_dense(A, X, W, a_l, a_r, slope=0.2, act=0):
    """Dense masked softmax attention: alpha = softmax_row(mask(LeakyReLU(s_l 1^T + 1 s_r^T)))."""
    n_rows, n_cols = A.shape
    theta = X.astype(np.float64) @ W.astype(np.float64)
    s_l = theta @ a_l.astype(np.float64)
    s_r = theta @ a_r.astype(np.float64)
    T = s_l[:n_rows, None] + s_r[None, :]
    E = np.where(T > 0.0, T, slope * T)
    alpha = np.zeros_like(E)
    for i in range(n_rows):
        mask = A[i] != 0.0
        if not mask.any():
            continue
        ex = np.exp(E[i, mask] - E[i, mask].max())
        alpha[i, mask] = ex / ex.sum()
    Y = alpha @ theta
    return (np.maximum(Y, 0.0) if act == 1 else Y), alpha


def gatv2_layer_dense(A, X, W_l, W_r, att, slope=0.2, act=0):
    """Dense GATv2: every pair (i, j) gets att . LeakyReLU(Theta_l[i] + Theta_r[j]); the pattern masks the softmax."""
    n_rows, n_cols = A.shape
    th_r = X.astype(np.float64) @ W_r.astype(np.float64)
    th_l = X[:n_rows].astype(np.float64) @ W_l.astype(np.float64)
    T = th_l[:, None, :] + th_r[None, :, :]
    E = np.where(T > 0.0, T, slope * T) @ att.astype(np.float64)
    alpha = np.zeros_like(E)
    for i in range(n_rows):
        mask = A[i] != 0.0
        if not mask.any():
            continue
        ex = np.exp(E[i, mask] - E[i, mask].max())
        alpha[i, mask] = ex / ex.sum()
    Y = alpha @ th_r
    return (np.maximum(Y, 0.0) if act == 1 else Y), alpha


def dotgat_layer_dense(A, X, W_q, W_k, W_v, scale, act=0):
    """Dense key-query attention: softmax over the pattern of scale * Q K^T, times V (the textbook masked attention)."""
    n_rows, _ = A.shape
    Xd = X.astype(np.float64)
    E = float(scale) * ((Xd[:n_rows] @ W_q.astype(np.float64)) @ (Xd @ W_k.astype(np.float64)).T)
    E = np.where(A != 0.0, E, -np.inf)
    alpha = np.zeros_like(E)
    for i in range(n_rows):
        if np.isfinite(E[i]).any():
            ex = np.exp(E[i] - E[i][np.isfinite(E[i])].max())
            alpha[i] = ex / ex.sum()
    Y = alpha @ (Xd @ W_v.astype(np.float64))
    return (np.maximum(Y, 0.0) if act == 1 else Y), alpha


def spmm_dense(A_val, B):
    """Eq. 1 over every (i,j), zeros included: plain GEMM on the densified matrix."""
    n, m = A_val.shape
    C = np.zeros((n, B.shape[1]), dtype=np.float64)
    for i in range(n):
        for j in range(m):
            C[i] += A_val[i, j] * B[j]
    return C


def sddmm_dense(A, Bm, Cm):
    """Eq. 2 with (+,x): D = A o (Bm . Cm^T), evaluated densely then masked."""
    return A * (Bm.astype(np.float64) @ Cm.astype(np.float64).T)
