"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP library.

Graphs (Erdos-Renyi G(n,M), R-MAT, fan-out sampled blocks) as canonical CSR,
and dense fills (uniform, normal, Glorot-uniform).  Nothing here computes any
part of a GNN layer; the module only produces inputs.  The work is done by
``gen.c`` (counter-based PRNG, OpenMP), loaded through ctypes.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.c into libsynth.so (host code only)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        u64, i64, i32, dbl, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.synth_hash.restype = u64
        lib.synth_hash.argtypes = [u64, u64, u64]
        lib.synth_fill_uniform.argtypes = [u64, u64, i64, dbl, dbl, vp]
        lib.synth_fill_normal.argtypes = [u64, u64, i64, dbl, dbl, vp]
        lib.synth_fill_normal_rows.argtypes = [u64, u64, vp, i64, i32, dbl, dbl, vp]
        lib.synth_rmat_pairs.argtypes = [u64, u64, i32, i32, dbl, dbl, dbl, i64, vp, vp]
        lib.synth_gnm_pairs.restype = i64
        lib.synth_gnm_pairs.argtypes = [u64, u64, i32, i64, vp, vp]
        lib.synth_build_csr.restype = i64
        lib.synth_build_csr.argtypes = [i32, i32, vp, vp, i64, ctypes.c_int, ctypes.c_int, vp, vp]
        lib.synth_sample_block.restype = i64
        lib.synth_sample_block.argtypes = [u64, u64, i32, vp, vp, vp, i32, i32, vp, vp, vp]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


@dataclass
class CSR:
    """Sparsity pattern in canonical CSR (int32, columns strictly ascending per row)."""
    n_rows: int
    n_cols: int
    row_ptr: np.ndarray
    col_idx: np.ndarray

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


# ------------------------------------------------------------------ dense fills

def uniform(seed: int, stream: int, shape, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_uniform(seed, stream, out.size, lo, hi, _p(out))
    return out


def normal(seed: int, stream: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_normal(seed, stream, out.size, mean, std, _p(out))
    return out


def normal_rows(seed: int, stream: int, ids: np.ndarray, f: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """Rows ``ids`` of a virtual (n x f) normal matrix (row id -> fixed values)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty((ids.size, f), dtype=np.float32)
    _load().synth_fill_normal_rows(seed, stream, _p(ids), ids.size, f, mean, std, _p(out))
    return out


def glorot(seed: int, stream: int, fan_in: int, fan_out: int) -> np.ndarray:
    """Glorot-uniform weights, U(-b, b) with b = sqrt(6 / (fan_in + fan_out))."""
    b = math.sqrt(6.0 / (fan_in + fan_out))
    return uniform(seed, stream, (fan_in, fan_out), -b, b)


# ---------------------------------------------------------------------- graphs

def build_csr(n_rows: int, n_cols: int, u: np.ndarray, v: np.ndarray, symmetrize: bool, self_loops: bool) -> CSR:
    u = np.ascontiguousarray(u, dtype=np.int32)
    v = np.ascontiguousarray(v, dtype=np.int32)
    assert u.shape == v.shape and u.ndim == 1
    lib = _load()
    row_ptr = np.empty(n_rows + 1, dtype=np.int32)
    nnz = lib.synth_build_csr(n_rows, n_cols, _p(u), _p(v), u.size, int(symmetrize), int(self_loops), _p(row_ptr), None)
    if nnz < 0:
        raise RuntimeError(f"synth_build_csr failed ({nnz})")
    col_idx = np.empty(max(nnz, 1), dtype=np.int32)
    nnz2 = lib.synth_build_csr(n_rows, n_cols, _p(u), _p(v), u.size, int(symmetrize), int(self_loops), _p(row_ptr), _p(col_idx))
    assert nnz2 == nnz
    return CSR(n_rows, n_cols, row_ptr, col_idx[:nnz])


def erdos_renyi(seed: int, n: int, n_pairs: int, self_loops: bool = True) -> CSR:
    """G(n, M): exactly ``n_pairs`` distinct undirected non-loop pairs, mirrored."""
    u = np.empty(n_pairs, dtype=np.int32)
    v = np.empty(n_pairs, dtype=np.int32)
    got = _load().synth_gnm_pairs(seed, 1, n, n_pairs, _p(u), _p(v))
    if got < 0:
        raise RuntimeError("synth_gnm_pairs failed")
    return build_csr(n, n, u[:got], v[:got], True, self_loops)


def rmat(seed: int, n: int, n_draws: int, a: float = 0.57, b: float = 0.19, c: float = 0.19,
         self_loops: bool = True) -> CSR:
    """R-MAT on ceil(log2 n) levels; out-of-range and loop draws rejected; mirrored; deduplicated."""
    scale = max(1, int(math.ceil(math.log2(n))))
    u = np.empty(n_draws, dtype=np.int32)
    v = np.empty(n_draws, dtype=np.int32)
    _load().synth_rmat_pairs(seed, 2, scale, n, a, b, c, n_draws, _p(u), _p(v))
    return build_csr(n, n, u, v, True, self_loops)


def ring_lattice(n: int, k_half: int, self_loops: bool = True) -> CSR:
    """Each node joined to its k_half nearest neighbours on each side (2*k_half-regular)."""
    i = np.repeat(np.arange(n, dtype=np.int64), k_half)
    d = np.tile(np.arange(1, k_half + 1, dtype=np.int64), n)
    return build_csr(n, n, i.astype(np.int32), ((i + d) % n).astype(np.int32), True, self_loops)


def thinned_grid(seed: int, side: int, keep: float, self_loops: bool = True) -> CSR:
    """side x side square grid whose right/down links are each kept with probability ``keep``: a planar,
    near-constant-degree pattern with the shape of a road network (row-major node numbering)."""
    n = side * side
    idx = np.arange(n, dtype=np.int64)
    right = idx[(idx % side) != side - 1]
    down = idx[idx < n - side]
    u = np.concatenate([right, down])
    v = np.concatenate([right + 1, down + side])
    m = uniform(seed, 3, (u.size,), 0.0, 1.0) < keep
    return build_csr(n, n, u[m].astype(np.int32), v[m].astype(np.int32), True, self_loops)


def complete(n: int) -> CSR:
    i, j = np.triu_indices(n, 1)
    return build_csr(n, n, i.astype(np.int32), j.astype(np.int32), True, True)


def star(n: int) -> CSR:
    """Hub 0 joined to leaves 1..n-1, plus self loops."""
    return build_csr(n, n, np.zeros(n - 1, dtype=np.int32), np.arange(1, n, dtype=np.int32), True, True)


def self_loops_only(n: int) -> CSR:
    e = np.empty(0, dtype=np.int32)
    return build_csr(n, n, e, e, False, True)


def transpose(g: CSR) -> CSR:
    """The transposed pattern (n_cols x n_rows), columns ascending within a row."""
    rows = np.repeat(np.arange(g.n_rows, dtype=np.int32), np.diff(g.row_ptr))
    return build_csr(g.n_cols, g.n_rows, g.col_idx, rows, False, False)


def sample_block(seed: int, stream: int, g: CSR, dst: np.ndarray, fanout: int):
    """One hop of fan-out sampling -> (block CSR with local columns, global ids of its columns)."""
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    n_dst = dst.size
    cap = n_dst * (fanout + 1)
    src_ids = np.empty(cap, dtype=np.int32)
    row_ptr = np.empty(n_dst + 1, dtype=np.int32)
    col_idx = np.empty(cap, dtype=np.int32)
    n_src = _load().synth_sample_block(seed, stream, g.n_rows, _p(g.row_ptr), _p(g.col_idx), _p(dst), n_dst, fanout,
                                       _p(src_ids), _p(row_ptr), _p(col_idx))
    if n_src < 0:
        raise RuntimeError("synth_sample_block failed")
    nnz = int(row_ptr[-1])
    return CSR(n_dst, int(n_src), row_ptr, col_idx[:nnz].copy()), src_ids[:n_src].copy()


def distinct_nodes(seed: int, stream: int, n: int, k: int) -> np.ndarray:
    """k distinct node ids in [0,n), in draw order, from the counter stream."""
    lib = _load()
    seen, out, t = set(), [], 0
    while len(out) < k:
        x = int((int(lib.synth_hash(seed, stream, t)) >> 32) * n >> 32)
        t += 1
        if x not in seen:
            seen.add(x)
            out.append(x)
    return np.asarray(out, dtype=np.int32)
