"""sensei_spmm_static, the entry point that allocates nothing: its output against sensei_spmm's (the existing entry point with a
caller-provided workspace) and against the fp64 oracle, on two calls in a row that share the GPU's static scratch array, the
second on a smaller input; and the rejection of inputs beyond the array's size."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import synth
from paper_2306_15155_amd import ACT_NONE, ACT_RELU, SPMM_PATTERN, SPMM_SCALED, SPMM_WEIGHTED, Context, binding

from gpu_util import DEV, DeviceCSR, assert_close, dev, hub_and_empty_graph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def _one_call(ctx, g, f, mode, act, seed):
    """Runs both entry points on the same inputs; returns nothing, asserts parity with each other and with the oracle."""
    rng = np.random.default_rng(seed)
    val = rng.uniform(-1.0, 1.0, g.nnz).astype(np.float32) if mode == SPMM_WEIGHTED else None
    A = DeviceCSR(g, val)
    B = synth.uniform(seed, 10, (g.n_cols, f))
    r = c = None
    if mode == SPMM_SCALED:
        r, c = rng.uniform(0.1, 1.0, g.n_rows).astype(np.float32), rng.uniform(0.1, 1.0, g.n_cols).astype(np.float32)
    Bd = dev(B)
    rd, cd = (None, None) if r is None else (dev(r), dev(c))
    want = ctx.spmm(A.s, mode, Bd, r=rd, c=cd, activation=act)                    # existing entry point, workspace from the caller
    out = torch.full((g.n_rows, f), float("nan"), device=DEV)                      # every element must be written
    got = ctx.spmm_static(A.s, mode, Bd, out, r=rd, c=cd, activation=act)          # static scratch, nothing allocated
    torch.cuda.synchronize()
    assert_close(got, want.cpu().numpy(), what="static vs workspace entry point")
    # the plain definition (Eq. 1) in fp64: weights val, 1 or c_j per entry, then the row factor and the activation
    w = val if mode == SPMM_WEIGHTED else (c[g.col_idx] if mode == SPMM_SCALED else None)
    ref = oracle.spmm(g.row_ptr, g.col_idx, w, B)
    if mode == SPMM_SCALED:
        ref = oracle.row_broadcast(r, ref)
    assert_close(got, oracle.activation(ref, act), what="static entry point vs oracle")


def test_two_calls_in_a_row_second_one_smaller(ctx):
    # first call: several chunks, a hub row that spans chunk boundaries (carry slots in use), empty rows, ragged width
    big = hub_and_empty_graph(21, 12_000, 150_000, 9000, 40)
    _one_call(ctx, big, 100, SPMM_WEIGHTED, ACT_RELU, 5)
    # second call, smaller input: the array still holds the first call's plan and carry slots
    small = hub_and_empty_graph(22, 700, 4_000, 600, 5)
    _one_call(ctx, small, 33, SPMM_PATTERN, ACT_NONE, 6)
    # and a third in the scaled flavour on a rectangular block
    rect = synth.build_csr(300, 900, np.repeat(np.arange(300), 7), np.random.default_rng(3).integers(0, 900, 2100), False, True)
    _one_call(ctx, rect, 64, SPMM_SCALED, ACT_NONE, 7)


def test_input_beyond_the_static_scratch_is_rejected_before_any_launch(ctx):
    L = binding.lib()
    # 50 M stored entries at 256 columns need ~200 MB of carry slots: more than the 32 MiB array.  The check is host
    # arithmetic on the sizes, nothing is dereferenced or launched, so the pointers only have to be non-null.
    A = binding.CsrStruct(100_000, 100_000, 50_000_000, 0x1000, 0x2000, None)
    B = binding.MatStruct(0x10000000000, 100_000, 256, 256)
    st = L.sensei_spmm_static(ctx._h, ctypes.byref(A), SPMM_PATTERN, None, None, B, ctypes.c_void_p(0x20000000000), 256, ACT_NONE, None)
    assert st == 6 and "static scratch" in binding.status_string(st)
    torch.cuda.synchronize()
