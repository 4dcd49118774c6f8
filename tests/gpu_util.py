"""Helpers for the GPU parity tests: upload seeded inputs, compare with the fp64 oracle."""
import numpy as np
import torch

import synth
from paper_2306_15155_amd import csr_struct

DEV = "cuda:0"
TOL = 1e-4  # |gpu - ref| <= TOL * (1 + |ref|) per element, fp32 path against the fp64 oracle


class DeviceCSR:
    def __init__(self, g: synth.CSR, val=None):
        self.g = g
        self.row_ptr = torch.from_numpy(g.row_ptr).to(DEV)
        self.col_idx = torch.from_numpy(np.ascontiguousarray(g.col_idx)).to(DEV)
        self.val = None if val is None else torch.from_numpy(np.ascontiguousarray(val, dtype=np.float32)).to(DEV)
        self.s = csr_struct(g.n_rows, g.n_cols, self.row_ptr, self.col_idx, self.val)

    def with_val(self, val_t):
        out = DeviceCSR.__new__(DeviceCSR)
        out.g, out.row_ptr, out.col_idx, out.val = self.g, self.row_ptr, self.col_idx, val_t
        out.s = csr_struct(self.g.n_rows, self.g.n_cols, self.row_ptr, self.col_idx, val_t)
        return out


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def assert_close(gpu, ref, tol=TOL, what=""):
    got = gpu.detach().cpu().numpy().astype(np.float64) if isinstance(gpu, torch.Tensor) else np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref) / (1.0 + np.abs(ref))
    worst = float(err.max()) if err.size else 0.0
    assert worst <= tol, f"{what}: max scaled error {worst:.3e} > {tol}"
    return worst


def assert_close_reduced(gpu, ref, terms_rss, tol=TOL, what="", max_share=0.01):
    """For a gradient that is a sum over all nodes (dW = X^T G): |gpu - ref| <= tol (1 + |ref|) + 2^-16 rss, where rss is the
    root-sum-square of the terms of that sum.  The terms are products with G (or dTheta), itself an fp32 sum over up to 1e5
    neighbours and so carrying a relative rounding error of the order of sqrt(degree) 2^-24 per node; these errors are
    independent across nodes, so what reaches the sum scales with the root-sum-square of its terms, not with its value, and
    entries that cancel to nearly zero cannot be held to tol (1 + |ref|).  The second term is an allowance for those entries
    only: at most `max_share` of the elements may need it (the others meet the plain bound), and the share is returned."""
    got = gpu.detach().cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    plain = tol * (1.0 + np.abs(ref))
    bound = plain + 2.0 ** -16 * np.asarray(terms_rss, dtype=np.float64)
    worst = float(np.max(err / bound))
    share = float(np.mean(err > plain))
    print(f"{what}: worst {worst:.3f} of the bound; {share:.4%} of {err.size} elements are beyond the plain bound "
          f"(largest plain-scaled error {float(np.max(err / (1.0 + np.abs(ref)))):.2e})")
    assert worst <= 1.0, f"{what}: error reaches {worst:.3f} of its bound"
    assert share <= max_share, f"{what}: {share:.4%} of the elements need the allowance for cancelled sums (ceiling {max_share:.2%})"
    return worst, share


def hub_and_empty_graph(seed, n, pairs, hub_deg, n_empty):
    """Random graph with one hub row of about hub_deg entries and n_empty all-zero rows (no self loop)."""
    rng = np.random.default_rng(seed)
    u = rng.integers(n_empty, n, size=pairs).astype(np.int32)
    v = rng.integers(0, n, size=pairs).astype(np.int32)
    hub = n // 2
    hv = rng.choice(n, size=hub_deg, replace=False).astype(np.int32)
    u = np.concatenate([u, np.full(hub_deg, hub, dtype=np.int32)])
    v = np.concatenate([v, hv])
    return synth.build_csr(n, n, u, v, False, False)


def rect_block(seed, n_rows, n_cols, per_row):
    rng = np.random.default_rng(seed)
    u = np.repeat(np.arange(n_rows), per_row)
    v = rng.integers(0, n_cols, size=u.size)
    return synth.build_csr(n_rows, n_cols, u, v, False, True)
