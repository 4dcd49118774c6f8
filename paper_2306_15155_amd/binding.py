"""ctypes binding of libsensei_hip.so: argument marshalling only.

Every function mirrors the C entry point of the same name in ``include/sensei.h``.
Tensors are PyTorch ROCm tensors used as device buffers (``data_ptr()``); the
stream is PyTorch's current HIP stream.  There is no fallback: if the library
has not been built the import of :func:`lib` raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsensei_hip.so")

ACT_NONE, ACT_RELU = 0, 1
KIND_GCN, KIND_GAT = 0, 1
SPMM_PATTERN, SPMM_WEIGHTED, SPMM_SCALED = 0, 1, 2
GCN_BWD_AGG, GCN_BWD_UPD = 0, 1
SELECT_MODEL, SELECT_TIMED, SELECT_LEARNED, SELECT_AUTO = 0, 1, 2, 3
GCN_NAMES = ("DYN_AGG", "DYN_UPD", "DYNF_AGG", "DYNF_UPD", "PRE_AGG", "PRE_UPD")
GAT_NAMES = ("REUSE", "RECOMP", "RECOMP_FOLD", "REUSE_FOLD")

EXPORTS = (
    "sensei_create", "sensei_destroy", "sensei_calibrate", "sensei_num_compositions", "sensei_composition_name",
    "sensei_status_string", "sensei_degrees", "sensei_norm_vectors", "sensei_sparse_workspace", "sensei_chunk_nnz", "sensei_gemm_kernel", "sensei_gcn_precompute",
    "sensei_row_broadcast", "sensei_spmm", "sensei_spmm_static", "sensei_gemm", "sensei_gemv2", "sensei_sddmm_score", "sensei_edge_softmax",
    "sensei_gcn_workspace", "sensei_gcn_layer", "sensei_gat_workspace", "sensei_gat_attention_path", "sensei_gat_layer", "sensei_select_workspace",
    "sensei_select", "sensei_profile_enable", "sensei_profile_read", "sensei_panels_bytes", "sensei_panels_create",
    "sensei_panels_count", "sensei_panels_destroy", "sensei_panels_set_min_width", "sensei_panels_tune_bytes",
    "sensei_panels_tune", "sensei_gcn_backward_workspace", "sensei_gcn_backward", "sensei_select_gcn_backward", "sensei_select_khop_backward", "sensei_transpose_positions",
    "sensei_gat_backward_workspace", "sensei_gat_backward", "sensei_gat_backward_heads_workspace", "sensei_gat_backward_heads", "sensei_gat_layer_heads", "sensei_sgc_workspace", "sensei_sgc_layer", "sensei_sgc_backward_workspace", "sensei_sgc_backward", "sensei_tagcn_workspace", "sensei_tagcn_layer", "sensei_tagcn_backward_workspace", "sensei_tagcn_backward", "sensei_gatv2_workspace", "sensei_gatv2_layer", "sensei_gatv2_backward_workspace", "sensei_gatv2_backward", "sensei_dotgat_workspace", "sensei_dotgat_layer", "sensei_dotgat_backward_workspace", "sensei_dotgat_backward", "sensei_tiles_remainder_panels", "sensei_tiles_bytes", "sensei_tiles_create", "sensei_tiles_info",
           "sensei_tiles_set_min_width", "sensei_tiles_destroy",
)


class SenseiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class CsrStruct(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("val", ctypes.c_void_p), ("panels", ctypes.c_void_p),
                ("tiles", ctypes.c_void_p)]


class MatStruct(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("ld", ctypes.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_15155_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
        P = ctypes.POINTER
        L.sensei_create.argtypes = [P(vp), i32]
        L.sensei_destroy.argtypes = [vp]
        L.sensei_calibrate.argtypes = [vp, vp, sz, vp]
        L.sensei_num_compositions.argtypes = [i32]
        L.sensei_composition_name.argtypes = [i32, i32]
        L.sensei_composition_name.restype = ctypes.c_char_p
        L.sensei_status_string.argtypes = [i32]
        L.sensei_status_string.restype = ctypes.c_char_p
        L.sensei_degrees.argtypes = [vp, P(CsrStruct), vp, vp, vp]
        L.sensei_norm_vectors.argtypes = [vp, vp, i64, vp, vp]
        L.sensei_sparse_workspace.argtypes = [P(CsrStruct), i32, P(sz)]
        L.sensei_chunk_nnz.argtypes = [i64]
        L.sensei_gemm_kernel.argtypes = [i64, i32, i32]
        L.sensei_gcn_precompute.argtypes = [vp, P(CsrStruct), vp, vp, vp, vp, sz, vp]
        L.sensei_row_broadcast.argtypes = [vp, vp, MatStruct, vp, i64, vp]
        L.sensei_spmm.argtypes = [vp, P(CsrStruct), i32, vp, vp, MatStruct, vp, i64, i32, vp, sz, vp]
        L.sensei_spmm_static.argtypes = [vp, P(CsrStruct), i32, vp, vp, MatStruct, vp, i64, i32, vp]
        L.sensei_gemm.argtypes = [vp, MatStruct, MatStruct, vp, i64, i32, vp]
        L.sensei_gemv2.argtypes = [vp, MatStruct, vp, vp, vp, vp, vp]
        L.sensei_sddmm_score.argtypes = [vp, P(CsrStruct), vp, vp, f32, vp, vp, sz, vp]
        L.sensei_edge_softmax.argtypes = [vp, P(CsrStruct), vp, vp, vp, sz, vp]
        L.sensei_gcn_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_gcn_layer.argtypes = [vp, P(CsrStruct), vp, vp, MatStruct, MatStruct, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_gcn_backward_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_gcn_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, vp, MatStruct, MatStruct, vp, i64, MatStruct, i32, vp, i64,
                                          vp, i64, vp, i64, i32, vp, sz, vp]
        L.sensei_select_gcn_backward.argtypes = [vp, P(CsrStruct), i32, i32, i32, i32, P(ctypes.c_int), P(f32)]
        L.sensei_select_khop_backward.argtypes = [vp, P(CsrStruct), i32, i32, i32, i32, i32, P(ctypes.c_int), P(f32)]
        L.sensei_transpose_positions.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, vp, sz, vp]
        L.sensei_gat_backward_workspace.argtypes = [P(CsrStruct), P(CsrStruct), i32, i32, P(sz)]
        L.sensei_gat_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, MatStruct, MatStruct, vp, vp, f32, vp, i64, MatStruct, i32,
                                          vp, i64, vp, i64, vp, vp, vp, sz, vp]
        L.sensei_gatv2_backward_workspace.argtypes = [P(CsrStruct), i32, i32, P(sz)]
        L.sensei_gatv2_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, MatStruct, MatStruct, MatStruct, vp, f32, vp, i64, MatStruct, i32,
                                            vp, i64, vp, i64, vp, i64, vp, vp, sz, vp]
        L.sensei_dotgat_backward_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_dotgat_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, MatStruct, MatStruct, MatStruct, MatStruct, f32, vp, i64, MatStruct, i32,
                                             vp, i64, vp, i64, vp, i64, vp, i64, vp, sz, vp]
        L.sensei_gat_backward_heads_workspace.argtypes = [P(CsrStruct), P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_gat_backward_heads.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, MatStruct, MatStruct, vp, vp, i32, f32, vp, i64, MatStruct, i32,
                                                vp, i64, vp, i64, vp, vp, vp, sz, vp]
        L.sensei_gat_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_gat_attention_path.argtypes = [P(CsrStruct), i32, i32, i32, i32]
        L.sensei_gat_layer.argtypes = [vp, P(CsrStruct), MatStruct, MatStruct, vp, vp, f32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_gat_layer_heads.argtypes = [vp, P(CsrStruct), MatStruct, MatStruct, vp, vp, i32, f32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_sgc_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_sgc_layer.argtypes = [vp, P(CsrStruct), vp, vp, MatStruct, MatStruct, i32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_sgc_backward_workspace.argtypes = [P(CsrStruct), i32, i32, i32, i32, P(sz)]
        L.sensei_sgc_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, vp, MatStruct, MatStruct, i32, vp, i64, MatStruct, i32, vp, i64, vp, i64,
                                          i32, vp, sz, vp]
        L.sensei_tagcn_workspace.argtypes = [P(CsrStruct), i32, i32, i32, i32, P(sz)]
        L.sensei_tagcn_backward_workspace.argtypes = [P(CsrStruct), i32, i32, i32, i32, P(sz)]
        L.sensei_tagcn_backward.argtypes = [vp, P(CsrStruct), P(CsrStruct), vp, vp, MatStruct, MatStruct, i32, vp, i64, MatStruct, i32, vp, i64, vp, i64,
                                            i32, vp, sz, vp]
        L.sensei_tagcn_layer.argtypes = [vp, P(CsrStruct), vp, vp, MatStruct, MatStruct, i32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_gatv2_workspace.argtypes = [P(CsrStruct), i32, i32, i32, P(sz)]
        L.sensei_gatv2_layer.argtypes = [vp, P(CsrStruct), MatStruct, MatStruct, MatStruct, vp, f32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_dotgat_workspace.argtypes = [P(CsrStruct), i32, i32, i32, i32, P(sz)]
        L.sensei_dotgat_layer.argtypes = [vp, P(CsrStruct), MatStruct, MatStruct, MatStruct, MatStruct, f32, vp, i64, i32, i32, vp, sz, vp]
        L.sensei_tiles_remainder_panels.argtypes = [i32]
        L.sensei_tiles_bytes.argtypes = [P(CsrStruct), f32, i32, P(sz)]
        L.sensei_tiles_create.argtypes = [vp, P(CsrStruct), f32, i32, vp, sz, vp, P(vp)]
        L.sensei_tiles_info.argtypes = [vp, P(i32), P(i64), P(i64)]
        L.sensei_tiles_set_min_width.argtypes = [vp, i32]
        L.sensei_tiles_destroy.argtypes = [vp]
        L.sensei_select_workspace.argtypes = [i32, P(CsrStruct), i32, i32, P(sz)]
        L.sensei_select.argtypes = [vp, i32, P(CsrStruct), i32, i32, i32, P(ctypes.c_int), P(f32), vp, sz, vp]
        L.sensei_panels_bytes.argtypes = [P(CsrStruct), i32, P(sz)]
        L.sensei_panels_create.argtypes = [vp, P(CsrStruct), i32, vp, sz, vp, P(vp)]
        L.sensei_panels_count.argtypes = [vp]
        L.sensei_panels_destroy.argtypes = [vp]
        L.sensei_panels_set_min_width.argtypes = [vp, i32]
        L.sensei_panels_tune_bytes.argtypes = [P(CsrStruct), P(sz)]
        L.sensei_panels_tune.argtypes = [vp, P(CsrStruct), vp, sz, vp, P(ctypes.c_int), P(ctypes.c_int), P(f32)]
        L.sensei_profile_enable.argtypes = [vp, i32]
        L.sensei_profile_read.argtypes = [vp, i32, P(f32), i32, P(ctypes.c_int)]
        for name in EXPORTS:
            if name not in ("sensei_composition_name", "sensei_status_string"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().sensei_status_string(status).decode()


def composition_name(kind: int, comp_id: int) -> str:
    return lib().sensei_composition_name(kind, comp_id).decode()


def chunk_nnz(nnz: int) -> int:
    return lib().sensei_chunk_nnz(nnz)


GEMM_FP32, GEMM_BF16_PIECES = 0, 1


def gemm_kernel(n: int, k: int, m: int) -> int:
    return lib().sensei_gemm_kernel(n, k, m)


GAT_PATH_TWO_PASS, GAT_PATH_ONE_WALK, GAT_PATH_TILES, GAT_PATH_PANELS = 0, 1, 2, 3


def gat_attention_path(A: "CsrStruct", f_in: int, f_out: int, comp_id: int, n_heads: int = 1) -> int:
    return lib().sensei_gat_attention_path(ctypes.byref(A), f_in, f_out, n_heads, comp_id)


def num_compositions(kind: int) -> int:
    return lib().sensei_num_compositions(kind)


def _check(status: int, where: str):
    if status != 0:
        raise SenseiError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def csr_struct(n_rows, n_cols, row_ptr, col_idx, val=None, panels=None, tiles=None) -> CsrStruct:
    assert row_ptr.dtype == torch.int32 and col_idx.dtype == torch.int32
    assert val is None or val.dtype == torch.float32
    A = CsrStruct(n_rows, n_cols, int(col_idx.numel()), row_ptr.data_ptr(), col_idx.data_ptr() if col_idx.numel() else None,
                  None if val is None else val.data_ptr(), None if panels is None else panels.handle,
                  None if tiles is None else tiles.handle)
    # the struct holds raw addresses: keep what they point into alive for as long as the struct is (the tensors, and the
    # Panels / Tiles objects, whose host handle and device buffer would otherwise go with their last Python reference)
    A._keep = (row_ptr, col_idx, val, panels, tiles)
    return A


class Panels:
    """Column-panel copy of a pattern (sensei_panels_create); owns the device buffer it lives in."""

    def __init__(self, ctx: "Context", A: CsrStruct, n_panels: int = 0, tune: bool = False):
        """n_panels 1..8 forces a count, 0 lets the library guess from the graph features; tune=True measures instead."""
        self.tune_ms = None
        min_width = None
        if tune:
            n_panels, min_width, self.tune_ms = self.measure(ctx, A)
        need = ctypes.c_size_t()
        _check(lib().sensei_panels_bytes(ctypes.byref(A), n_panels, ctypes.byref(need)), "sensei_panels_bytes")
        self.buf = torch.empty(need.value + 256, dtype=torch.uint8, device=ctx.device)
        p = (self.buf.data_ptr() + 255) // 256 * 256
        self._h = ctypes.c_void_p()
        _check(lib().sensei_panels_create(ctx._h, ctypes.byref(A), n_panels, ctypes.c_void_p(p), need.value, _stream(),
                                          ctypes.byref(self._h)), "sensei_panels_create")
        self.count = lib().sensei_panels_count(self._h)
        if min_width is not None:
            _check(lib().sensei_panels_set_min_width(self._h, min_width), "sensei_panels_set_min_width")
        self.min_width = 128 if min_width is None else min_width

    @staticmethod
    def measure(ctx: "Context", A: CsrStruct):
        """sensei_panels_tune on a scratch buffer that is released afterwards -> (count, min_width, trial times:
        [q] at width 256 and [9 + q] at width 64, -1 where not tried)."""
        need = ctypes.c_size_t()
        _check(lib().sensei_panels_tune_bytes(ctypes.byref(A), ctypes.byref(need)), "sensei_panels_tune_bytes")
        buf = torch.empty(need.value + 256, dtype=torch.uint8, device=ctx.device)
        p = (buf.data_ptr() + 255) // 256 * 256
        count, width = ctypes.c_int(), ctypes.c_int()
        ms = (ctypes.c_float * 18)()
        _check(lib().sensei_panels_tune(ctx._h, ctypes.byref(A), ctypes.c_void_p(p), need.value, _stream(), ctypes.byref(count),
                                        ctypes.byref(width), ms), "sensei_panels_tune")
        del buf
        return count.value, width.value, [float(x) for x in ms]

    @property
    def handle(self):
        return self._h.value

    def close(self):
        if self._h:
            lib().sensei_panels_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Tiles:
    """Dense-tile split of a pattern (sensei_tiles_create); owns the device buffer it lives in."""

    def __init__(self, ctx: "Context", A: CsrStruct, min_density: float = 0.07, max_width: int = 1024, min_width: int = 64, remainder_panels: int = 0):
        """remainder_panels: 0 lets the library decide whether the remainder is also kept panel-major, 1 never, 2..8 forces that many panels."""
        prev = lib().sensei_tiles_remainder_panels(remainder_panels)
        try:
            self._build(ctx, A, min_density, max_width, min_width)
        finally:
            lib().sensei_tiles_remainder_panels(prev)

    def _build(self, ctx, A, min_density, max_width, min_width):
        need = ctypes.c_size_t()
        _check(lib().sensei_tiles_bytes(ctypes.byref(A), min_density, max_width, ctypes.byref(need)), "sensei_tiles_bytes")
        self.buf = torch.empty(need.value + 256, dtype=torch.uint8, device=ctx.device)
        p = (self.buf.data_ptr() + 255) // 256 * 256
        self._h = ctypes.c_void_p()
        _check(lib().sensei_tiles_create(ctx._h, ctypes.byref(A), min_density, max_width, ctypes.c_void_p(p), need.value, _stream(),
                                         ctypes.byref(self._h)), "sensei_tiles_create")
        kept, dense, sparse = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
        _check(lib().sensei_tiles_info(self._h, ctypes.byref(kept), ctypes.byref(dense), ctypes.byref(sparse)), "sensei_tiles_info")
        self.n_tiles, self.nnz_dense, self.nnz_sparse = kept.value, dense.value, sparse.value
        _check(lib().sensei_tiles_set_min_width(self._h, min_width), "sensei_tiles_set_min_width")

    @property
    def handle(self):
        return self._h.value

    def close(self):
        if self._h:
            lib().sensei_tiles_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mat_struct(t: torch.Tensor) -> MatStruct:
    assert t.dtype == torch.float32 and t.dim() == 2 and (t.stride(1) == 1 or t.size(1) <= 1)
    return MatStruct(t.data_ptr(), t.size(0), t.size(1), t.stride(0) if t.size(0) > 1 else max(t.stride(0), t.size(1)))


class Workspace:
    """A grow-only device byte buffer (PyTorch owns the memory)."""

    def __init__(self, device="cuda:0"):
        self.device = torch.device(device)
        self.buf = torch.empty(0, dtype=torch.uint8, device=self.device)

    def ensure(self, nbytes: int):
        if self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=self.device)
        return self

    @property
    def ptr(self):
        p = self.buf.data_ptr()
        return ctypes.c_void_p((p + 255) // 256 * 256)

    @property
    def nbytes(self):
        p = self.buf.data_ptr()
        return max(0, self.buf.numel() - ((p + 255) // 256 * 256 - p))


class Context:
    def __init__(self, device: int = 0):
        self._h = ctypes.c_void_p()
        _check(lib().sensei_create(ctypes.byref(self._h), device), "sensei_create")
        self.device = torch.device(f"cuda:{device}")
        self.ws = Workspace(self.device)

    def close(self):
        if self._h:
            lib().sensei_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- primitives
    def degrees(self, A: CsrStruct):
        dr = torch.empty(A.n_rows, dtype=torch.int32, device=self.device)
        dc = torch.empty(A.n_cols, dtype=torch.int32, device=self.device)
        _check(lib().sensei_degrees(self._h, ctypes.byref(A), _ptr(dr), _ptr(dc), _stream()), "sensei_degrees")
        return dr, dc

    def norm_vectors(self, deg: torch.Tensor):
        out = torch.empty(deg.numel(), dtype=torch.float32, device=self.device)
        _check(lib().sensei_norm_vectors(self._h, _ptr(deg), deg.numel(), _ptr(out), _stream()), "sensei_norm_vectors")
        return out

    def sparse_workspace(self, A: CsrStruct, f: int) -> int:
        n = ctypes.c_size_t()
        _check(lib().sensei_sparse_workspace(ctypes.byref(A), f, ctypes.byref(n)), "sensei_sparse_workspace")
        return n.value

    def gcn_precompute(self, A: CsrStruct, r, c):
        val = torch.empty(max(A.nnz, 1), dtype=torch.float32, device=self.device)[:A.nnz]
        self.ws.ensure(self.sparse_workspace(A, 1))
        _check(lib().sensei_gcn_precompute(self._h, ctypes.byref(A), _ptr(r), _ptr(c), _ptr(val), self.ws.ptr, self.ws.nbytes,
                                           _stream()), "sensei_gcn_precompute")
        return val

    def row_broadcast(self, s, X, out=None):
        Y = torch.empty_like(X) if out is None else out
        _check(lib().sensei_row_broadcast(self._h, _ptr(s), mat_struct(X), _ptr(Y), mat_struct(Y).ld, _stream()), "sensei_row_broadcast")
        return Y

    def spmm(self, A: CsrStruct, mode, B, r=None, c=None, activation=ACT_NONE, out=None):
        C = torch.empty((A.n_rows, B.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        self.ws.ensure(self.sparse_workspace(A, B.size(1)))
        _check(lib().sensei_spmm(self._h, ctypes.byref(A), mode, _ptr(r), _ptr(c), mat_struct(B), _ptr(C), mat_struct(C).ld,
                                 activation, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_spmm")
        return C

    def spmm_static(self, A: CsrStruct, mode, B, out, r=None, c=None, activation=ACT_NONE):
        """sensei_spmm_static: the caller passes the output; nothing is allocated on either side of the boundary."""
        _check(lib().sensei_spmm_static(self._h, ctypes.byref(A), mode, _ptr(r), _ptr(c), mat_struct(B), _ptr(out), mat_struct(out).ld,
                                        activation, _stream()), "sensei_spmm_static")
        return out

    def gemm(self, A, W, activation=ACT_NONE, out=None):
        Y = torch.empty((A.size(0), W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        _check(lib().sensei_gemm(self._h, mat_struct(A), mat_struct(W), _ptr(Y), mat_struct(Y).ld, activation, _stream()), "sensei_gemm")
        return Y

    def gemv2(self, A, v1, v2):
        y1 = torch.empty(A.size(0), dtype=torch.float32, device=self.device)
        y2 = torch.empty(A.size(0), dtype=torch.float32, device=self.device)
        _check(lib().sensei_gemv2(self._h, mat_struct(A), _ptr(v1), _ptr(v2), _ptr(y1), _ptr(y2), _stream()), "sensei_gemv2")
        return y1, y2

    def sddmm_score(self, A: CsrStruct, s_l, s_r, neg_slope=0.2):
        e = torch.empty(max(A.nnz, 1), dtype=torch.float32, device=self.device)[:A.nnz]
        self.ws.ensure(self.sparse_workspace(A, 1))
        _check(lib().sensei_sddmm_score(self._h, ctypes.byref(A), _ptr(s_l), _ptr(s_r), neg_slope, _ptr(e), self.ws.ptr,
                                        self.ws.nbytes, _stream()), "sensei_sddmm_score")
        return e

    def edge_softmax(self, A: CsrStruct, e, out=None):
        alpha = torch.empty_like(e) if out is None else out
        self.ws.ensure(self.sparse_workspace(A, 1))
        _check(lib().sensei_edge_softmax(self._h, ctypes.byref(A), _ptr(e), _ptr(alpha), self.ws.ptr, self.ws.nbytes, _stream()),
               "sensei_edge_softmax")
        return alpha

    # ---- layers
    def gcn_workspace(self, A: CsrStruct, f_in, f_out, comp_id) -> int:
        n = ctypes.c_size_t()
        _check(lib().sensei_gcn_workspace(ctypes.byref(A), f_in, f_out, comp_id, ctypes.byref(n)), "sensei_gcn_workspace")
        return n.value

    def gcn_layer(self, A: CsrStruct, r, c, X, W, comp_id, activation=ACT_NONE, out=None):
        Y = torch.empty((A.n_rows, W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        self.ws.ensure(self.gcn_workspace(A, X.size(1), W.size(1), comp_id))
        _check(lib().sensei_gcn_layer(self._h, ctypes.byref(A), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), _ptr(Y),
                                      mat_struct(Y).ld, activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_gcn_layer")
        return Y

    def gat_workspace(self, A: CsrStruct, f_in, f_out, comp_id) -> int:
        n = ctypes.c_size_t()
        _check(lib().sensei_gat_workspace(ctypes.byref(A), f_in, f_out, comp_id, ctypes.byref(n)), "sensei_gat_workspace")
        return n.value

    def gcn_backward(self, A: CsrStruct, At: CsrStruct, r, c, X, W, dY, bwd_id, Y=None, activation=ACT_NONE, U_saved=None, want_dx=True):
        """Backward of gcn_layer -> (dX or None, dW); ``At`` is the transposed pattern (A itself when symmetric)."""
        f_in, f_out = W.size(0), W.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dW = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_gcn_backward_workspace(ctypes.byref(A), f_in, f_out, bwd_id, ctypes.byref(need)), "sensei_gcn_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_gcn_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), _ptr(Y),
                                         mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation, _ptr(U_saved),
                                         mat_struct(U_saved).ld if U_saved is not None else 0, _ptr(dX),
                                         mat_struct(dX).ld if dX is not None else 0, _ptr(dW), mat_struct(dW).ld, bwd_id, self.ws.ptr,
                                         self.ws.nbytes, _stream()), "sensei_gcn_backward")
        return dX, dW

    def transpose_positions(self, A: CsrStruct, At: CsrStruct):
        """int32 tensor: place of every stored entry of A in the transposed pattern At."""
        pos = torch.empty(max(A.nnz, 1), dtype=torch.int32, device=self.device)
        self.ws.ensure(self.sparse_workspace(A, 1) + 1024)
        _check(lib().sensei_transpose_positions(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(pos), self.ws.ptr, self.ws.nbytes, _stream()),
               "sensei_transpose_positions")
        return pos

    def gat_backward(self, A: CsrStruct, At: CsrStruct, t_pos, X, W, a_l, a_r, dY, Y=None, neg_slope=0.2, activation=ACT_NONE, want_dx=True):
        """Backward of gat_layer -> (dX or None, dW, da_l, da_r)."""
        f_in, f_out = W.size(0), W.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dW = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        dal = torch.empty(f_out, dtype=torch.float32, device=self.device)
        dar = torch.empty(f_out, dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_gat_backward_workspace(ctypes.byref(A), ctypes.byref(At), f_in, f_out, ctypes.byref(need)), "sensei_gat_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_gat_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(t_pos), mat_struct(X), mat_struct(W), _ptr(a_l),
                                         _ptr(a_r), neg_slope, _ptr(Y), mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation,
                                         _ptr(dX), mat_struct(dX).ld if dX is not None else 0, _ptr(dW), mat_struct(dW).ld, _ptr(dal),
                                         _ptr(dar), self.ws.ptr, self.ws.nbytes, _stream()), "sensei_gat_backward")
        return dX, dW, dal, dar

    def gat_backward_heads(self, A: CsrStruct, At: CsrStruct, t_pos, X, W, a_l, a_r, n_heads, dY, Y=None, neg_slope=0.2, activation=ACT_NONE,
                           want_dx=True):
        """Backward of gat_layer_heads -> (dX or None, dW, da_l, da_r)."""
        f_in, f_out = W.size(0), W.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dW = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        dal = torch.empty(f_out, dtype=torch.float32, device=self.device)
        dar = torch.empty(f_out, dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_gat_backward_heads_workspace(ctypes.byref(A), ctypes.byref(At), f_in, f_out, n_heads, ctypes.byref(need)),
               "sensei_gat_backward_heads_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_gat_backward_heads(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(t_pos), mat_struct(X), mat_struct(W), _ptr(a_l),
                                               _ptr(a_r), n_heads, neg_slope, _ptr(Y), mat_struct(Y).ld if Y is not None else 0, mat_struct(dY),
                                               activation, _ptr(dX), mat_struct(dX).ld if dX is not None else 0, _ptr(dW), mat_struct(dW).ld,
                                               _ptr(dal), _ptr(dar), self.ws.ptr, self.ws.nbytes, _stream()), "sensei_gat_backward_heads")
        return dX, dW, dal, dar

    def gatv2_backward(self, A: CsrStruct, At: CsrStruct, t_pos, X, W_l, W_r, att, dY, Y=None, neg_slope=0.2, activation=ACT_NONE, want_dx=True):
        """Backward of gatv2_layer -> (dX or None, dW_l, dW_r, datt)."""
        f_in, f_out = W_r.size(0), W_r.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dWl = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        dWr = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        da = torch.empty(f_out, dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_gatv2_backward_workspace(ctypes.byref(A), f_in, f_out, ctypes.byref(need)), "sensei_gatv2_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_gatv2_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(t_pos), mat_struct(X), mat_struct(W_l), mat_struct(W_r),
                                           _ptr(att), neg_slope, _ptr(Y), mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation,
                                           _ptr(dX), mat_struct(dX).ld if dX is not None else 0, _ptr(dWl), mat_struct(dWl).ld, _ptr(dWr),
                                           mat_struct(dWr).ld, _ptr(da), self.ws.ptr, self.ws.nbytes, _stream()), "sensei_gatv2_backward")
        return dX, dWl, dWr, da

    def dotgat_backward(self, A: CsrStruct, At: CsrStruct, t_pos, X, W_q, W_k, W_v, scale, dY, Y=None, activation=ACT_NONE, want_dx=True):
        """Backward of dotgat_layer -> (dX or None, dW_q, dW_k, dW_v)."""
        f_in, d_k, f_out = W_q.size(0), W_q.size(1), W_v.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dWq = torch.empty((f_in, d_k), dtype=torch.float32, device=self.device)
        dWk = torch.empty((f_in, d_k), dtype=torch.float32, device=self.device)
        dWv = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_dotgat_backward_workspace(ctypes.byref(A), f_in, d_k, f_out, ctypes.byref(need)), "sensei_dotgat_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_dotgat_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(t_pos), mat_struct(X), mat_struct(W_q), mat_struct(W_k),
                                            mat_struct(W_v), scale, _ptr(Y), mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation,
                                            _ptr(dX), mat_struct(dX).ld if dX is not None else 0, _ptr(dWq), mat_struct(dWq).ld, _ptr(dWk),
                                            mat_struct(dWk).ld, _ptr(dWv), mat_struct(dWv).ld, self.ws.ptr, self.ws.nbytes, _stream()),
               "sensei_dotgat_backward")
        return dX, dWq, dWk, dWv

    def select_khop_backward(self, A: CsrStruct, f_in, f_out, k_hops, per_hop_weights, want_dx=True):
        """Predicted faster association of sgc_backward (per_hop_weights False) or tagcn_backward (True) -> (bwd_id, [ms AGG, ms UPD])."""
        pick = ctypes.c_int()
        est = (ctypes.c_float * 2)()
        _check(lib().sensei_select_khop_backward(self._h, ctypes.byref(A), f_in, f_out, k_hops, int(per_hop_weights), int(want_dx), ctypes.byref(pick),
                                                 est), "sensei_select_khop_backward")
        return pick.value, [float(x) for x in est]

    def select_gcn_backward(self, A: CsrStruct, f_in, f_out, have_saved_u=False, want_dx=True):
        pick = ctypes.c_int()
        est = (ctypes.c_float * 2)()
        _check(lib().sensei_select_gcn_backward(self._h, ctypes.byref(A), f_in, f_out, int(have_saved_u), int(want_dx), ctypes.byref(pick), est),
               "sensei_select_gcn_backward")
        return pick.value, [float(x) for x in est]

    def gat_layer(self, A: CsrStruct, X, W, a_l, a_r, comp_id, neg_slope=0.2, activation=ACT_NONE, out=None):
        Y = torch.empty((A.n_rows, W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        self.ws.ensure(self.gat_workspace(A, X.size(1), W.size(1), comp_id))
        _check(lib().sensei_gat_layer(self._h, ctypes.byref(A), mat_struct(X), mat_struct(W), _ptr(a_l), _ptr(a_r), neg_slope,
                                      _ptr(Y), mat_struct(Y).ld, activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()),
               "sensei_gat_layer")
        return Y

    def sgc_layer(self, A: CsrStruct, r, c, X, W, k_hops, comp_id, activation=ACT_NONE, out=None):
        """K-hop simplified graph convolution act(A^^k X W); comp_id 0 aggregates first, 1 updates first."""
        Y = torch.empty((A.n_rows, W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        need = ctypes.c_size_t()
        _check(lib().sensei_sgc_workspace(ctypes.byref(A), X.size(1), W.size(1), comp_id, ctypes.byref(need)), "sensei_sgc_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_sgc_layer(self._h, ctypes.byref(A), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), k_hops, _ptr(Y), mat_struct(Y).ld,
                                      activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_sgc_layer")
        return Y

    def sgc_backward(self, A: CsrStruct, At: CsrStruct, r, c, X, W, k_hops, dY, bwd_id, Y=None, activation=ACT_NONE, want_dx=True):
        """Backward of sgc_layer -> (dX or None, dW); ``At`` is the transposed pattern (A itself when symmetric)."""
        f_in, f_out = W.size(0), W.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dW = torch.empty((f_in, f_out), dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_sgc_backward_workspace(ctypes.byref(A), f_in, f_out, k_hops, bwd_id, ctypes.byref(need)), "sensei_sgc_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_sgc_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), k_hops, _ptr(Y),
                                         mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation, _ptr(dX),
                                         mat_struct(dX).ld if dX is not None else 0, _ptr(dW), mat_struct(dW).ld, bwd_id, self.ws.ptr,
                                         self.ws.nbytes, _stream()), "sensei_sgc_backward")
        return dX, dW

    def tagcn_backward(self, A: CsrStruct, At: CsrStruct, r, c, X, W, k_hops, dY, bwd_id, Y=None, activation=ACT_NONE, want_dx=True):
        """Backward of tagcn_layer -> (dX or None, dW); W and dW stack the k_hops + 1 blocks by rows; ``At`` is the transposed pattern."""
        f_in, f_out = X.size(1), W.size(1)
        dX = torch.empty((A.n_cols, f_in), dtype=torch.float32, device=self.device) if want_dx else None
        dW = torch.empty((W.size(0), f_out), dtype=torch.float32, device=self.device)
        need = ctypes.c_size_t()
        _check(lib().sensei_tagcn_backward_workspace(ctypes.byref(A), f_in, f_out, k_hops, bwd_id, ctypes.byref(need)),
               "sensei_tagcn_backward_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_tagcn_backward(self._h, ctypes.byref(A), ctypes.byref(At), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), k_hops, _ptr(Y),
                                           mat_struct(Y).ld if Y is not None else 0, mat_struct(dY), activation, _ptr(dX),
                                           mat_struct(dX).ld if dX is not None else 0, _ptr(dW), mat_struct(dW).ld, bwd_id, self.ws.ptr,
                                           self.ws.nbytes, _stream()), "sensei_tagcn_backward")
        return dX, dW

    def tagcn_layer(self, A: CsrStruct, r, c, X, W, k_hops, comp_id, activation=ACT_NONE, out=None):
        """TAGCN layer act(sum_k A^^k X W_k); W stacks W_0 .. W_k_hops by rows; comp_id 0 aggregates first, 1 updates first."""
        Y = torch.empty((A.n_rows, W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        need = ctypes.c_size_t()
        _check(lib().sensei_tagcn_workspace(ctypes.byref(A), X.size(1), W.size(1), k_hops, comp_id, ctypes.byref(need)), "sensei_tagcn_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_tagcn_layer(self._h, ctypes.byref(A), _ptr(r), _ptr(c), mat_struct(X), mat_struct(W), k_hops, _ptr(Y), mat_struct(Y).ld,
                                        activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_tagcn_layer")
        return Y

    def gatv2_layer(self, A: CsrStruct, X, W_l, W_r, att, comp_id, neg_slope=0.2, activation=ACT_NONE, out=None):
        """GATv2 layer; pass the same tensor as W_l and W_r to share the weights; comp_id 0 reuses Theta_r, 1 recomputes."""
        Y = torch.empty((A.n_rows, W_r.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        need = ctypes.c_size_t()
        _check(lib().sensei_gatv2_workspace(ctypes.byref(A), X.size(1), W_r.size(1), comp_id, ctypes.byref(need)), "sensei_gatv2_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_gatv2_layer(self._h, ctypes.byref(A), mat_struct(X), mat_struct(W_l), mat_struct(W_r), _ptr(att), neg_slope, _ptr(Y),
                                        mat_struct(Y).ld, activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_gatv2_layer")
        return Y

    def dotgat_layer(self, A: CsrStruct, X, W_q, W_k, W_v, scale, comp_id, activation=ACT_NONE, out=None):
        """Key-query attention layer: e_ij = scale <x_i W_q, x_j W_k>; comp_id 0 aggregates X W_v, 1 aggregates X and projects afterwards."""
        Y = torch.empty((A.n_rows, W_v.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        need = ctypes.c_size_t()
        _check(lib().sensei_dotgat_workspace(ctypes.byref(A), X.size(1), W_q.size(1), W_v.size(1), comp_id, ctypes.byref(need)), "sensei_dotgat_workspace")
        self.ws.ensure(need.value)
        _check(lib().sensei_dotgat_layer(self._h, ctypes.byref(A), mat_struct(X), mat_struct(W_q), mat_struct(W_k), mat_struct(W_v), scale, _ptr(Y),
                                         mat_struct(Y).ld, activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_dotgat_layer")
        return Y

    def gat_layer_heads(self, A: CsrStruct, X, W, a_l, a_r, n_heads, comp_id, neg_slope=0.2, activation=ACT_NONE, out=None):
        """Multi-head GAT layer, heads concatenated: W is f_in x (n_heads * d), a_l / a_r hold n_heads * d entries."""
        Y = torch.empty((A.n_rows, W.size(1)), dtype=torch.float32, device=self.device) if out is None else out
        self.ws.ensure(self.gat_workspace(A, X.size(1), W.size(1), comp_id))
        _check(lib().sensei_gat_layer_heads(self._h, ctypes.byref(A), mat_struct(X), mat_struct(W), _ptr(a_l), _ptr(a_r), n_heads, neg_slope,
                                            _ptr(Y), mat_struct(Y).ld, activation, comp_id, self.ws.ptr, self.ws.nbytes, _stream()),
               "sensei_gat_layer_heads")
        return Y

    # ---- selector
    def select(self, kind, A: CsrStruct, f_in, f_out, mode=SELECT_MODEL):
        n = num_compositions(kind)
        est = (ctypes.c_float * n)()
        cid = ctypes.c_int(-1)
        ws_ptr, ws_bytes = None, 0
        if mode == SELECT_LEARNED:
            self.ws.ensure(256)
            ws_ptr, ws_bytes = self.ws.ptr, self.ws.nbytes
        if mode in (SELECT_TIMED, SELECT_AUTO):
            need = ctypes.c_size_t()
            _check(lib().sensei_select_workspace(kind, ctypes.byref(A), f_in, f_out, ctypes.byref(need)), "sensei_select_workspace")
            self.ws.ensure(need.value)
            ws_ptr, ws_bytes = self.ws.ptr, self.ws.nbytes
        _check(lib().sensei_select(self._h, kind, ctypes.byref(A), f_in, f_out, mode, ctypes.byref(cid), est, ws_ptr, ws_bytes,
                                   _stream()), "sensei_select")
        return cid.value, [float(x) for x in est]

    def profile_enable(self, enable: bool):
        _check(lib().sensei_profile_enable(self._h, int(enable)), "sensei_profile_enable")

    def profile_read(self, kernel: int = 0):
        """Elapsed ms of every launch of the SpMM (kernel=0) or GEMM (kernel=1) kernel recorded since
        profile_enable(True), in launch order."""
        n = ctypes.c_int(0)
        _check(lib().sensei_profile_read(self._h, kernel, None, 0, ctypes.byref(n)), "sensei_profile_read")
        buf = (ctypes.c_float * max(n.value, 1))()
        _check(lib().sensei_profile_read(self._h, kernel, buf, n.value, ctypes.byref(n)), "sensei_profile_read")
        return [float(buf[i]) for i in range(n.value)]

    def calibrate(self):
        self.ws.ensure(64 << 20)
        _check(lib().sensei_calibrate(self._h, self.ws.ptr, self.ws.nbytes, _stream()), "sensei_calibrate")
