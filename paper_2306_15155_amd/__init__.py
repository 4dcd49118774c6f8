"""MI355X-native hot path of input-sensitive GNN execution (SENSEi, arXiv 2306.15155).

The work is done by ``libsensei_hip.so`` (hand-written HIP for gfx950, C ABI in
``include/sensei.h``); :mod:`paper_2306_15155_amd.binding` marshals arguments.
"""
from .binding import (ACT_NONE, ACT_RELU, GAT_NAMES, GCN_BWD_AGG, GCN_BWD_UPD, GCN_NAMES, KIND_GAT, KIND_GCN, SELECT_AUTO, SELECT_LEARNED, SELECT_MODEL, SELECT_TIMED, SPMM_PATTERN,
                      SPMM_SCALED, SPMM_WEIGHTED, Context, Panels, SenseiError, Tiles, csr_struct, lib)

__all__ = ["ACT_NONE", "ACT_RELU", "GAT_NAMES", "GCN_BWD_AGG", "GCN_BWD_UPD", "GCN_NAMES", "KIND_GAT", "KIND_GCN", "SELECT_AUTO", "SELECT_LEARNED", "SELECT_MODEL", "SELECT_TIMED",
           "SPMM_PATTERN", "SPMM_SCALED", "SPMM_WEIGHTED", "Context", "Panels", "SenseiError", "Tiles", "csr_struct", "lib"]
