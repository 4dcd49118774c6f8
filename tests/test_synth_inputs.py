"""Checks of the seeded input generators and of the canonical CSR form (integer work: exact)."""
import numpy as np

import oracle
import synth


def _reference_csr(n_rows, n_cols, u, v, symmetrize, self_loops):
    """Independent construction with numpy: unique sorted (row, col) keys."""
    u, v = np.asarray(u, dtype=np.int64), np.asarray(v, dtype=np.int64)
    ok = (u >= 0) & (v >= 0)
    u, v = u[ok], v[ok]
    rows, cols = [u], [v]
    if symmetrize:
        rows.append(v)
        cols.append(u)
    if self_loops:
        d = np.arange(min(n_rows, n_cols), dtype=np.int64)
        rows.append(d)
        cols.append(d)
    r, c = np.concatenate(rows), np.concatenate(cols)
    keep = (r < n_rows) & (c < n_cols)
    keys = np.unique(r[keep] * n_cols + c[keep])
    r, c = keys // n_cols, keys % n_cols
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.add.at(row_ptr, r + 1, 1)
    return np.cumsum(row_ptr).astype(np.int32), c.astype(np.int32)


def _check_canonical(g, symmetric):
    deg = np.diff(g.row_ptr)
    assert g.row_ptr[0] == 0 and np.all(deg >= 0) and g.row_ptr[-1] == g.col_idx.size
    for i in range(g.n_rows):
        cols = g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
        if i < g.n_cols:
            assert np.count_nonzero(cols == i) == 1
    dr, dc = oracle.degrees(g.n_rows, g.n_cols, g.row_ptr, g.col_idx)
    assert dr.sum() == g.nnz and dc.sum() == g.nnz
    if symmetric:
        assert np.array_equal(dr, dc)


def test_config1_graph_has_exact_size():
    g = synth.erdos_renyi(1, 10_000, 50_000)
    assert g.nnz == 110_000
    _check_canonical(g, True)


def test_csr_builder_matches_independent_construction():
    rng = np.random.default_rng(0)
    u = rng.integers(-1, 300, size=5000).astype(np.int32)
    v = rng.integers(-1, 300, size=5000).astype(np.int32)
    for sym, loops, nr, nc in [(True, True, 300, 300), (False, True, 120, 300), (False, False, 300, 200)]:
        g = synth.build_csr(nr, nc, u, v, sym, loops)
        rp, ci = _reference_csr(nr, nc, u, v, sym, loops)
        assert g.row_ptr.tobytes() == rp.tobytes() and g.col_idx.tobytes() == ci.tobytes()


def test_rmat_is_skewed_symmetric_and_reproducible():
    g = synth.rmat(5, 3000, 40_000)
    _check_canonical(g, True)
    deg = np.diff(g.row_ptr)
    assert deg.max() > 8 * deg.mean()
    g2 = synth.rmat(5, 3000, 40_000)
    assert g.col_idx.tobytes() == g2.col_idx.tobytes()
    assert synth.rmat(6, 3000, 40_000).nnz != g.nnz or synth.rmat(6, 3000, 40_000).col_idx.tobytes() != g.col_idx.tobytes()


def test_dense_fills_have_the_stated_distributions():
    x = synth.uniform(1, 3, (200_000,))
    assert x.min() >= -1.0 and x.max() <= 1.0
    assert abs(x.mean()) < 5 * np.sqrt(1 / 3 / x.size) and abs(x.var() - 1 / 3) < 5e-3
    z = synth.normal(1, 4, (200_000,))
    assert abs(z.mean()) < 5 / np.sqrt(z.size) and abs(z.std() - 1.0) < 1e-2
    a = synth.normal(1, 5, (100_000,), 0.0, 0.1)
    assert abs(a.std() - 0.1) < 2e-3
    w = synth.glorot(1, 6, 602, 256)
    b = np.sqrt(6.0 / (602 + 256))
    assert w.shape == (602, 256) and np.abs(w).max() <= b and np.abs(w).max() > 0.99 * b
    assert np.array_equal(synth.uniform(1, 3, (1000,)), x[:1000])  # counter based: prefix stable


def test_normal_rows_addresses_a_virtual_matrix():
    full = synth.normal(9, 7, (50, 6))
    ids = np.array([49, 0, 13], dtype=np.int32)
    assert np.array_equal(synth.normal_rows(9, 7, ids, 6), full[ids])


def test_fanout_blocks():
    g = synth.rmat(8, 5000, 60_000)
    seeds = synth.distinct_nodes(8, 20, 5000, 64)
    assert len(set(seeds.tolist())) == 64
    b2, ids1 = synth.sample_block(8, 21, g, seeds, 10)
    b1, ids0 = synth.sample_block(8, 22, g, ids1, 25)
    for blk, dst, ids, fan in [(b2, seeds, ids1, 10), (b1, ids1, ids0, 25)]:
        assert blk.n_rows == dst.size and blk.n_cols == ids.size
        assert np.array_equal(ids[:dst.size], dst) and len(set(ids.tolist())) == ids.size
        _check_canonical(blk, False)
        for t in range(blk.n_rows):
            cols = blk.col_idx[blk.row_ptr[t]:blk.row_ptr[t + 1]]
            nbrs = set(g.col_idx[g.row_ptr[dst[t]]:g.row_ptr[dst[t] + 1]].tolist())
            full_deg = len(nbrs - {int(dst[t])})
            assert cols.size == 1 + min(fan, full_deg)
            assert set(ids[cols].tolist()) <= nbrs | {int(dst[t])}
