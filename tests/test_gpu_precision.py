"""The kernels that run on the bf16 matrix instruction claim fp32 accuracy: every fp32 operand element is cut exactly into three
bf16 pieces (8 + 8 + 8 significand bits) and only piece products below 2^-23 of a term are left out.  These tests hold them to
that claim on operands whose low significand bits matter (full 24-bit significands, exponents spread over many binades): the
error against the fp64 oracle must be a small multiple of fp32 rounding, and several times smaller than the error that dropping
the third piece (a 16-bit significand) would cause on the same operands, which the test works out on the CPU."""
import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2306_15155_amd import ACT_NONE, GCN_BWD_AGG, SPMM_PATTERN, Context, Tiles, binding, csr_struct

from gpu_util import DeviceCSR, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = Context(0)
    yield c
    c.close()


def _wide(seed, stream, shape, binades):
    """fp32 values with random 24-bit significands, random signs and exponents spread over `binades` binades."""
    m = synth.uniform(seed, stream, shape, 1.0, 2.0).astype(np.float64)
    e = np.floor(synth.uniform(seed, stream + 1, shape, -binades / 2.0, binades / 2.0))
    s = np.where(synth.uniform(seed, stream + 2, shape, -1.0, 1.0) < 0, -1.0, 1.0)
    return (s * m * np.exp2(e)).astype(np.float32)


def _cut16(x):
    """x with its significand truncated to 16 bits: what two bf16 pieces keep."""
    return (x.view(np.uint32) & np.uint32(0xFFFFFF00)).view(np.float32)


@pytest.mark.parametrize("shape", [(70_000, 602, 256), (140_000, 100, 64), (300_000, 48, 24), (90_000, 101, 96)])   # 8-, 16-, 16- and 4-byte aligned rows
def test_gemm_on_bf16_pieces_is_as_accurate_as_fp32(ctx, shape):
    n, k, m = shape
    assert binding.gemm_kernel(n, k, m) == binding.GEMM_BF16_PIECES
    A, W = _wide(11, 10, (n, k), 12), _wide(11, 20, (k, m), 12)
    rows = np.random.default_rng(3).choice(n, 400, replace=False)
    rows[0], rows[1] = 0, n - 1
    A64, W64 = A[rows].astype(np.float64), W.astype(np.float64)
    ref = A64 @ W64
    terms = np.abs(A64) @ np.abs(W64)                      # sum of |a w| per output: what rounding errors scale with
    got = ctx.gemm(dev(A), dev(W), ACT_NONE)[torch.from_numpy(rows).to("cuda:0")].double().cpu().numpy()
    err = np.abs(got - ref) / terms
    # fp32 accumulation of k products: a few units of 2^-24 relative to the sum of the terms' magnitudes
    assert err.max() < 2.0e-6, err.max()
    # two pieces per operand would lose the low 8 bits of every operand: that error, on the same data
    two_piece = np.abs(_cut16(A[rows]).astype(np.float64) @ _cut16(W).astype(np.float64) - ref) / terms
    assert np.median(err) < 0.2 * np.median(two_piece), (np.median(err), np.median(two_piece))
    # and the same rows through the fp32 instruction (a small product takes that kernel): errors of the same size
    assert binding.gemm_kernel(len(rows), k, m) == binding.GEMM_FP32
    small = ctx.gemm(dev(A[rows]), dev(W), ACT_NONE).double().cpu().numpy()
    err32 = np.abs(small - ref) / terms
    assert np.median(err) < 3.0 * np.median(err32) + 1e-9, (np.median(err), np.median(err32))


def test_value_less_tiles_on_bf16_pieces_are_as_accurate_as_fp32(ctx):
    g = synth.rmat(52, 6000, 400_000)
    f = 96
    B = _wide(12, 30, (g.n_cols, f), 10)
    ref = oracle.spmm(g.row_ptr, g.col_idx, None, B)
    terms = oracle.spmm(g.row_ptr, g.col_idx, None, np.abs(B))
    two_piece = np.abs(oracle.spmm(g.row_ptr, g.col_idx, None, _cut16(B)) - ref)
    A = DeviceCSR(g)
    T = Tiles(ctx, A.s, 0.05, 128, min_width=32)
    assert T.n_tiles > 0 and T.nnz_dense > 0.3 * g.row_ptr[-1]
    At = csr_struct(g.n_rows, g.n_cols, A.row_ptr, A.col_idx, None, None, T)
    dr, dc = ctx.degrees(A.s)
    ones = torch.ones(g.n_rows, device="cuda:0")
    # the layer path (slice-major operand) is what takes the split: an identity update, unit scalings
    X = dev(B)
    W = torch.eye(f, device="cuda:0")
    Y = ctx.gcn_layer(At, ones, ones, X, W, 3, ACT_NONE).double().cpu().numpy()
    Yp = ctx.gcn_layer(A.s, ones, ones, X, W, 3, ACT_NONE).double().cpu().numpy()
    scale = np.maximum(terms, 1e-30)
    err, err_plain = np.abs(Y - ref) / scale, np.abs(Yp - ref) / scale
    hub = np.argsort(-np.diff(g.row_ptr))[:512]          # the rows whose sums come mostly from the tiles
    assert err.max() < 2.0e-6, err.max()
    assert np.median(err[hub]) < 3.0 * np.median(err_plain[hub]) + 1e-9
    assert np.median(err[hub]) < 0.2 * np.median((two_piece / scale)[hub]), (np.median(err[hub]), np.median((two_piece / scale)[hub]))
    T.close()


def test_long_transposed_product_has_no_systematic_error(ctx):
    """dW = X^T dP over 200,000 rows on the bf16 instruction.  The instruction's own summation loses low bits of its smaller addends
    downwards whatever their sign; summed over that many rows this showed as an offset of every element by several units of fp32
    rounding of the root-sum-square of its terms (8 units at 233,000 rows).  The kernel multiplies -A in every other group of steps and
    subtracts, so the offset cancels: the mean error over the elements must stay within a fraction of a unit, and the spread within the
    few units that fp32 accumulation inside a group of 32 rows and the final rounding explain."""
    n, f_in, f_out = 200_000, 96, 64
    g = synth.self_loops_only(n)                       # A^ = I: the layer without hops is a dense layer, dW = X^T dY
    A = DeviceCSR(g)
    ones = torch.ones(n, device="cuda:0")
    X, dY = synth.uniform(13, 10, (n, f_in)), synth.normal(13, 11, (n, f_out), 0.0, 1.0)
    W = synth.glorot(13, 12, f_in, f_out)
    _, dW = ctx.tagcn_backward(A.s, A.s, ones, ones, dev(X), dev(W), 0, dev(dY), GCN_BWD_AGG, want_dx=False)
    X64, d64 = X.astype(np.float64), dY.astype(np.float64)
    ref = X64.T @ d64
    rss = np.sqrt((X64 ** 2).T @ (d64 ** 2))
    e = (dW.double().cpu().numpy() - ref) / rss * 2.0 ** 24
    assert abs(e.mean()) < 0.5, e.mean()
    assert np.sqrt((e ** 2).mean()) < 2.5 and np.abs(e).max() < 12.0, (np.sqrt((e ** 2).mean()), np.abs(e).max())
