"""ctypes binding of libaffmae.so.  Argument marshalling only.

torch is used for device memory (outputs and workspaces are torch tensors) and
for the current HIP stream; every step of the computation runs inside the
library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaffmae.so")
_LIB_TIMED_PATH = os.path.join(_HERE, "libaffmae_timed.so")  # instrumented twin (include/affmae_timing.h), benchmarks only
_lib = None        # the library every call goes through
_libs = {}         # path -> loaded library

AFFMAE_F32 = 0
AFFMAE_BF16 = 1

_c_int = ctypes.c_int
_c_void_p = ctypes.c_void_p
_c_size_t = ctypes.c_size_t
_c_float = ctypes.c_float


class AffmaeError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} returned {status}: {status_string(status)}")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """The library in use: libaffmae.so unless use_timed_library(True) switched to the instrumented build
    (built first only if it does not exist)."""
    global _lib
    if _lib is None:
        _lib = _load(_LIB_PATH)
    return _lib


def use_timed_library(on: bool) -> None:
    """Route every call through libaffmae_timed.so (per-kernel event timing compiled in) or back through
    libaffmae.so.  For benchmarks."""
    global _lib
    _lib = _load(_LIB_TIMED_PATH if on else _LIB_PATH)


def _load(path: str):
    if path in _libs:
        return _libs[path]
    if not os.path.exists(path):
        from .build import build_library  # needs hipcc
        build_library()
    lib = ctypes.CDLL(path)
    lib.affmae_status_string.restype = ctypes.c_char_p
    lib.affmae_status_string.argtypes = [_c_int]
    lib.affmae_version.restype = _c_int
    lib.affmae_build_id.restype = ctypes.c_char_p
    lib.affmae_cluster_workspace_bytes.restype = _c_size_t
    lib.affmae_cluster_workspace_bytes.argtypes = [_c_int] * 2
    lib.affmae_cluster.restype = _c_int
    lib.affmae_cluster.argtypes = ([_c_void_p] + [_c_int] * 3 + [ctypes.c_double] * 4
                                   + [_c_void_p, _c_void_p, _c_void_p, _c_size_t, _c_void_p])
    lib.affmae_vts_table.restype = _c_int
    lib.affmae_vts_table.argtypes = [_c_void_p] + [_c_int] * 4 + [_c_float] * 3 + [_c_int, _c_void_p, _c_void_p]
    lib.affmae_vts_fwd.restype = _c_int
    lib.affmae_vts_fwd.argtypes = ([_c_void_p] * 4 + [_c_int] * 6 + [_c_float] * 3 + [_c_int] + [_c_float] * 2 + [_c_int]
                                   + [_c_void_p, _c_void_p])
    lib.affmae_vts_bwd_workspace_bytes.restype = _c_size_t
    lib.affmae_vts_bwd_workspace_bytes.argtypes = [_c_int] * 4
    lib.affmae_vts_bwd.restype = _c_int
    lib.affmae_vts_bwd.argtypes = ([_c_void_p] * 5 + [_c_int] * 6 + [_c_float] * 3 + [_c_int] + [_c_float] * 2 + [_c_int]
                                   + [_c_void_p] * 4 + [_c_size_t, _c_void_p])
    lib.affmae_merge_select.restype = _c_int
    lib.affmae_merge_select.argtypes = [_c_void_p, _c_void_p] + [_c_int] * 3 + [_c_void_p] * 3
    lib.affmae_merge_fwd.restype = _c_int
    lib.affmae_merge_fwd.argtypes = [_c_void_p] * 5 + [_c_int] * 5 + [_c_float, _c_int, _c_void_p, _c_void_p]
    lib.affmae_merge_bwd_workspace_bytes.restype = _c_size_t
    lib.affmae_merge_bwd_workspace_bytes.argtypes = [_c_int] * 4
    lib.affmae_merge_bwd.restype = _c_int
    lib.affmae_merge_bwd.argtypes = ([_c_void_p] * 6 + [_c_int] * 5 + [_c_float, _c_int] + [_c_void_p] * 4
                                     + [_c_size_t, _c_void_p])
    lib.affmae_knn_workspace_bytes.restype = _c_size_t
    lib.affmae_knn_workspace_bytes.argtypes = [_c_int] * 5
    lib.affmae_knn.restype = _c_int
    lib.affmae_knn.argtypes = [_c_void_p, _c_void_p] + [_c_int] * 5 + [_c_void_p, _c_void_p, _c_void_p, _c_size_t,
                                                                      _c_void_p]
    lib.affmae_knn_static.restype = _c_int
    lib.affmae_knn_static.argtypes = [_c_void_p, _c_void_p] + [_c_int] * 5 + [_c_void_p, _c_void_p, _c_void_p]
    for name in ("affmae_pla_fwd_workspace_bytes", "affmae_pla_bwd_workspace_bytes"):
        f = getattr(lib, name)
        f.restype = _c_size_t
        f.argtypes = [_c_int] * 9
    lib.affmae_pla_fwd.restype = _c_int
    lib.affmae_pla_fwd.argtypes = ([_c_void_p] * 9 + [_c_int] * 7 + [_c_float, _c_int] + [_c_void_p, _c_void_p]
                                   + [_c_void_p, _c_size_t, _c_void_p])
    lib.affmae_pla_bwd.restype = _c_int
    lib.affmae_pla_bwd.argtypes = ([_c_void_p] * 12 + [_c_int] * 7 + [_c_float, _c_int] + [_c_void_p] * 6
                                   + [_c_void_p, _c_size_t, _c_void_p])
    lib.affmae_pla_fwd_relpos_workspace_bytes.restype = _c_size_t
    lib.affmae_pla_fwd_relpos_workspace_bytes.argtypes = [_c_int] * 9
    lib.affmae_pla_bwd_relpos_workspace_bytes.restype = _c_size_t
    lib.affmae_pla_bwd_relpos_workspace_bytes.argtypes = [_c_int] * 10
    lib.affmae_pla_fwd_relpos.restype = _c_int
    lib.affmae_pla_fwd_relpos.argtypes = ([_c_void_p] * 10 + [_c_int] * 7 + [_c_float, _c_int, _c_float, _c_int]
                                          + [_c_void_p, _c_void_p] + [_c_void_p, _c_size_t, _c_void_p])
    lib.affmae_pla_bwd_relpos.restype = _c_int
    lib.affmae_pla_bwd_relpos.argtypes = ([_c_void_p] * 13 + [_c_int] * 7 + [_c_float, _c_int, _c_float, _c_int]
                                          + [_c_void_p] * 6 + [_c_void_p, _c_size_t, _c_void_p])
    lib.affmae_pla_plan_bytes.restype = _c_size_t
    lib.affmae_pla_plan_bytes.argtypes = [_c_int] * 5
    lib.affmae_pla_plan.restype = _c_int
    lib.affmae_pla_plan.argtypes = [_c_void_p, _c_void_p] + [_c_int] * 5 + [_c_void_p, _c_size_t, _c_void_p]
    _libs[path] = lib
    return lib


def build_id() -> str:
    """Digest of the sources the loaded library was built from."""
    return load_library().affmae_build_id().decode()


def status_string(status: int) -> str:
    return load_library().affmae_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, name: str, dtype=None, shape=None) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return AFFMAE_F32
    if t.dtype == torch.bfloat16:
        return AFFMAE_BF16
    raise ValueError(f"unsupported storage dtype {t.dtype}")


def affmae_cluster(coords: torch.Tensor, S: int, frame: Tuple[float, float, float, float],
                   order: Optional[torch.Tensor] = None, cluster_id: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """coords [B,N,2] fp32, frame (x0, y0, w, h) -> (order [B,N]: token at each place of the Z-order curve,
    cluster_id [B,N]: place // S of every token)."""
    lib = load_library()
    _dev(coords, "coords", torch.float32)
    B, N, two = coords.shape
    if two != 2:
        raise ValueError("coords must be [B,N,2]")
    if order is None:
        order = torch.empty((B, N), dtype=torch.int32, device=coords.device)
    if cluster_id is None:
        cluster_id = torch.empty((B, N), dtype=torch.int32, device=coords.device)
    _dev(order, "order", torch.int32, (B, N))
    _dev(cluster_id, "cluster_id", torch.int32, (B, N))
    need = lib.affmae_cluster_workspace_bytes(B, N)
    if workspace is None:
        workspace = _workspace(max(need, 256), coords.device)
    x0, y0, w, h = (float(t) for t in frame)
    rc = lib.affmae_cluster(_ptr(coords), B, N, int(S), x0, y0, w, h, _ptr(order), _ptr(cluster_id),
                            _ptr(workspace), workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_cluster", rc)
    return order, cluster_id


def _grid(grid):
    Hg, Wg, x0, y0, cell = grid
    return int(Hg), int(Wg), float(x0), float(y0), float(cell)


def affmae_vts_table(vis_xy: torch.Tensor, grid, Kt: int, table: Optional[torch.Tensor] = None) -> torch.Tensor:
    """vis_xy [B,Nv,2] fp32, grid (Hg, Wg, x0, y0, cell) -> table [B,Hg,Wg,Kt] int32: nearest visible tokens of
    every patch centre."""
    lib = load_library()
    _dev(vis_xy, "vis_xy", torch.float32)
    B, Nv, two = vis_xy.shape
    if two != 2:
        raise ValueError("vis_xy must be [B,Nv,2]")
    Hg, Wg, x0, y0, cell = _grid(grid)
    if table is None:
        table = torch.empty((B, Hg, Wg, int(Kt)), dtype=torch.int32, device=vis_xy.device)
    _dev(table, "table", torch.int32, (B, Hg, Wg, int(Kt)))
    rc = lib.affmae_vts_table(_ptr(vis_xy), B, Nv, Hg, Wg, x0, y0, cell, int(Kt), _ptr(table), _stream())
    if rc != 0:
        raise AffmaeError("affmae_vts_table", rc)
    return table


def affmae_vts_fwd(query_xy: torch.Tensor, vis_xy: torch.Tensor, feat: torch.Tensor, table: torch.Tensor, grid,
                   p: float, eps: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Virtual sampled tokens: query_xy [B,Mq,2] fp32, feat [B,Nv,C] -> out [B,Mq,C] in feat's dtype."""
    lib = load_library()
    _dev(query_xy, "query_xy", torch.float32)
    B, Mq, _ = query_xy.shape
    _dev(feat, "feat")
    _, Nv, C = feat.shape
    _dev(vis_xy, "vis_xy", torch.float32, (B, Nv, 2))
    Hg, Wg, x0, y0, cell = _grid(grid)
    _dev(table, "table", torch.int32)
    Kt = table.shape[-1]
    if tuple(table.shape) != (B, Hg, Wg, Kt):
        raise ValueError("table must be [B,Hg,Wg,Kt]")
    if out is None:
        out = torch.empty((B, Mq, C), dtype=feat.dtype, device=feat.device)
    _dev(out, "out", feat.dtype, (B, Mq, C))
    rc = lib.affmae_vts_fwd(_ptr(query_xy), _ptr(vis_xy), _ptr(feat), _ptr(table), B, Mq, Nv, C, Hg, Wg, x0, y0, cell,
                            Kt, float(p), float(eps), _dtype_code(feat), _ptr(out), _stream())
    if rc != 0:
        raise AffmaeError("affmae_vts_fwd", rc)
    return out


def affmae_vts_bwd(query_xy: torch.Tensor, vis_xy: torch.Tensor, feat: torch.Tensor, table: torch.Tensor,
                   dout: torch.Tensor, grid, p: float, eps: float, want_dp: bool = True,
                   workspace: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """Backward of affmae_vts_fwd -> dict(dfeat [B,Nv,C], dquery [B,Mq,2] fp32, dp [1] fp32 when asked for)."""
    lib = load_library()
    _dev(query_xy, "query_xy", torch.float32)
    B, Mq, _ = query_xy.shape
    _dev(feat, "feat")
    _, Nv, C = feat.shape
    _dev(vis_xy, "vis_xy", torch.float32, (B, Nv, 2))
    _dev(dout, "dout", feat.dtype, (B, Mq, C))
    Hg, Wg, x0, y0, cell = _grid(grid)
    _dev(table, "table", torch.int32)
    Kt = table.shape[-1]
    code = _dtype_code(feat)
    dfeat = torch.empty_like(feat)
    dquery = torch.empty((B, Mq, 2), dtype=torch.float32, device=feat.device)
    dp = torch.empty((1,), dtype=torch.float32, device=feat.device) if want_dp else None
    need = lib.affmae_vts_bwd_workspace_bytes(B, Mq, Nv, Kt)
    if workspace is None:
        workspace = _workspace(need, feat.device)
    rc = lib.affmae_vts_bwd(_ptr(query_xy), _ptr(vis_xy), _ptr(feat), _ptr(table), _ptr(dout), B, Mq, Nv, C, Hg, Wg,
                            x0, y0, cell, Kt, float(p), float(eps), code, _ptr(dfeat), _ptr(dquery), _ptr(dp),
                            _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_vts_bwd", rc)
    g = {"dfeat": dfeat, "dquery": dquery}
    if want_dp:
        g["dp"] = dp
    return g


def affmae_merge_select(score: torch.Tensor, n_keep: int, coords: Optional[torch.Tensor] = None,
                        anchor_idx: Optional[torch.Tensor] = None, anchor_xy: Optional[torch.Tensor] = None
                        ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """score [B,N] fp32 -> (anchor_idx [B,n_keep] int32, anchor_xy [B,n_keep,2] fp32 or None without coords)."""
    lib = load_library()
    _dev(score, "score", torch.float32)
    B, N = score.shape
    if coords is not None:
        _dev(coords, "coords", torch.float32, (B, N, 2))
    if anchor_idx is None:
        anchor_idx = torch.empty((B, n_keep), dtype=torch.int32, device=score.device)
    _dev(anchor_idx, "anchor_idx", torch.int32, (B, n_keep))
    if anchor_xy is None and coords is not None:
        anchor_xy = torch.empty((B, n_keep, 2), dtype=torch.float32, device=score.device)
    if anchor_xy is not None:
        _dev(anchor_xy, "anchor_xy", torch.float32, (B, n_keep, 2))
    rc = lib.affmae_merge_select(_ptr(score), _ptr(coords), B, N, n_keep, _ptr(anchor_idx), _ptr(anchor_xy), _stream())
    if rc != 0:
        raise AffmaeError("affmae_merge_select", rc)
    return anchor_idx, anchor_xy


def affmae_merge_fwd(feat: torch.Tensor, coords: torch.Tensor, score: torch.Tensor, nbr_idx: torch.Tensor,
                     anchor_idx: torch.Tensor, p: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Merged features [B,n_keep,C] in feat's dtype."""
    lib = load_library()
    code = _dtype_code(feat)
    _dev(feat, "feat")
    B, N, C = feat.shape
    _dev(coords, "coords", torch.float32, (B, N, 2))
    _dev(score, "score", torch.float32, (B, N))
    _dev(nbr_idx, "nbr_idx", torch.int32)
    K = nbr_idx.shape[2]
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    _dev(anchor_idx, "anchor_idx", torch.int32)
    n_keep = anchor_idx.shape[1]
    _dev(anchor_idx, "anchor_idx", torch.int32, (B, n_keep))
    if out is None:
        out = torch.empty((B, n_keep, C), dtype=feat.dtype, device=feat.device)
    _dev(out, "out", feat.dtype, (B, n_keep, C))
    rc = lib.affmae_merge_fwd(_ptr(feat), _ptr(coords), _ptr(score), _ptr(nbr_idx), _ptr(anchor_idx), B, N, C, K, n_keep,
                              float(p), code, _ptr(out), _stream())
    if rc != 0:
        raise AffmaeError("affmae_merge_fwd", rc)
    return out


def affmae_merge_bwd(feat: torch.Tensor, coords: torch.Tensor, score: torch.Tensor, nbr_idx: torch.Tensor,
                     anchor_idx: torch.Tensor, dout: torch.Tensor, p: float, want_dp: bool = True,
                     grads: Optional[Dict[str, torch.Tensor]] = None, workspace: Optional[torch.Tensor] = None
                     ) -> Dict[str, torch.Tensor]:
    """Gradients of the merging -> dict(dfeat [B,N,C], dscore [B,N] fp32[, dp scalar fp32])."""
    lib = load_library()
    code = _dtype_code(feat)
    _dev(feat, "feat")
    B, N, C = feat.shape
    K = nbr_idx.shape[2]
    n_keep = anchor_idx.shape[1]
    _dev(coords, "coords", torch.float32, (B, N, 2))
    _dev(score, "score", torch.float32, (B, N))
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    _dev(anchor_idx, "anchor_idx", torch.int32, (B, n_keep))
    _dev(dout, "dout", feat.dtype, (B, n_keep, C))
    g = grads if grads is not None else {}
    if "dfeat" not in g:
        g["dfeat"] = torch.empty_like(feat)
    if "dscore" not in g:
        g["dscore"] = torch.empty((B, N), dtype=torch.float32, device=feat.device)
    if want_dp and "dp" not in g:
        g["dp"] = torch.empty((), dtype=torch.float32, device=feat.device)
    _dev(g["dfeat"], "dfeat", feat.dtype, (B, N, C))
    _dev(g["dscore"], "dscore", torch.float32, (B, N))
    need = lib.affmae_merge_bwd_workspace_bytes(B, N, K, n_keep)
    if workspace is None:
        workspace = _workspace(max(need, 256), feat.device)
    rc = lib.affmae_merge_bwd(_ptr(feat), _ptr(coords), _ptr(score), _ptr(nbr_idx), _ptr(anchor_idx), _ptr(dout), B, N, C,
                              K, n_keep, float(p), code, _ptr(g["dfeat"]), _ptr(g["dscore"]),
                              _ptr(g["dp"]) if want_dp else None, _ptr(workspace), workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_merge_bwd", rc)
    return g


def affmae_knn(coords: torch.Tensor, cluster_id: Optional[torch.Tensor], S: int, M: int, K: int,
               nbr_idx: Optional[torch.Tensor] = None, near_clusters: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """coords [B,N,2] fp32, cluster_id [B,N] int32 or None -> (nbr_idx [B,N,K], near_clusters [B,G,M])."""
    lib = load_library()
    _dev(coords, "coords", torch.float32)
    B, N, two = coords.shape
    if two != 2:
        raise ValueError("coords must be [B,N,2]")
    if cluster_id is not None:
        _dev(cluster_id, "cluster_id", torch.int32, (B, N))
    G = -(-N // S) if S > 0 else 0  # the last cluster is short when S does not divide N
    if nbr_idx is None:
        nbr_idx = torch.empty((B, N, K), dtype=torch.int32, device=coords.device)
    if near_clusters is None:
        near_clusters = torch.empty((B, max(G, 0), M), dtype=torch.int32, device=coords.device)
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    _dev(near_clusters, "near_clusters", torch.int32, (B, G, M))
    need = lib.affmae_knn_workspace_bytes(B, N, S, M, K)
    if workspace is None:
        workspace = _workspace(max(need, 256), coords.device)
    rc = lib.affmae_knn(_ptr(coords), _ptr(cluster_id), B, N, S, M, K, _ptr(nbr_idx), _ptr(near_clusters),
                        _ptr(workspace), workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_knn", rc)
    return nbr_idx, near_clusters


def affmae_knn_static(coords: torch.Tensor, cluster_id: Optional[torch.Tensor], S: int, M: int, K: int,
                      nbr_idx: torch.Tensor, near_clusters: Optional[torch.Tensor] = None) -> None:
    """affmae_knn into caller-given outputs with the library's fixed scratch: no allocation anywhere."""
    lib = load_library()
    B, N, _ = coords.shape
    rc = lib.affmae_knn_static(_ptr(coords), _ptr(cluster_id), B, N, S, M, K, _ptr(nbr_idx), _ptr(near_clusters),
                               _stream())
    if rc != 0:
        raise AffmaeError("affmae_knn_static", rc)


def affmae_pla_plan(nbr_idx: torch.Tensor, near_clusters: torch.Tensor, S: int, M: int,
                    plan: Optional[torch.Tensor] = None) -> Optional[torch.Tensor]:
    """Re-tile a clustered neighbour table for the tiled attention kernels.  Returns the opaque
    plan buffer, or None when the shapes are outside what those kernels take."""
    lib = load_library()
    _dev(nbr_idx, "nbr_idx", torch.int32)
    B, N, K = nbr_idx.shape
    _dev(near_clusters, "near_clusters", torch.int32, (B, -(-N // S), M))
    need = lib.affmae_pla_plan_bytes(B, N, K, S, M)
    if need == 0:
        return None
    if plan is None:
        plan = torch.empty(need, dtype=torch.uint8, device=nbr_idx.device)
    rc = lib.affmae_pla_plan(_ptr(nbr_idx), _ptr(near_clusters), B, N, K, S, M, _ptr(plan), plan.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_pla_plan", rc)
    return plan


def affmae_pla_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, bias: Optional[torch.Tensor],
                   nbr_idx: torch.Tensor, scale: float, near_clusters: Optional[torch.Tensor] = None,
                   S: int = 0, M: int = 0, k_blank: Optional[torch.Tensor] = None,
                   v_blank: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                   lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                   plan: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Local attention forward -> (out [B,N,H,d] in q's dtype, lse [B,N,H] fp32)."""
    lib = load_library()
    code = _dtype_code(q)
    _dev(q, "q")
    B, N, H, d = q.shape
    _dev(k, "k", q.dtype, q.shape)
    _dev(v, "v", q.dtype, q.shape)
    _dev(nbr_idx, "nbr_idx", torch.int32)
    K = nbr_idx.shape[2]
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    if bias is not None:
        _dev(bias, "bias", q.dtype, (B, N, H, K))
    if near_clusters is not None:
        _dev(near_clusters, "near_clusters", torch.int32, (B, -(-N // S), M))
    if k_blank is not None:
        _dev(k_blank, "k_blank", q.dtype, (H, d))
        _dev(v_blank, "v_blank", q.dtype, (H, d))
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, N, H), dtype=torch.float32, device=q.device)
    _dev(out, "out", q.dtype, q.shape)
    _dev(lse, "lse", torch.float32, (B, N, H))
    need = lib.affmae_pla_fwd_workspace_bytes(B, N, H, d, K, S, M, code, int(near_clusters is not None))
    if workspace is None:
        workspace = _workspace(need, q.device)
    rc = lib.affmae_pla_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(bias), _ptr(nbr_idx), _ptr(near_clusters), _ptr(plan),
                            _ptr(k_blank), _ptr(v_blank), B, N, H, d, K, S, M, float(scale), code, _ptr(out),
                            _ptr(lse), _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_pla_fwd", rc)
    return out, lse


def affmae_pla_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, bias: Optional[torch.Tensor],
                   nbr_idx: torch.Tensor, out: Optional[torch.Tensor], lse: torch.Tensor, dout: torch.Tensor,
                   scale: float, near_clusters: Optional[torch.Tensor] = None, S: int = 0, M: int = 0,
                   k_blank: Optional[torch.Tensor] = None, v_blank: Optional[torch.Tensor] = None,
                   want_dbias: bool = True, grads: Optional[Dict[str, torch.Tensor]] = None,
                   workspace: Optional[torch.Tensor] = None, plan: Optional[torch.Tensor] = None
                   ) -> Dict[str, torch.Tensor]:
    """Local attention backward -> dict(dq, dk, dv[, dbias][, dk_blank, dv_blank])."""
    lib = load_library()
    code = _dtype_code(q)
    _dev(q, "q")
    B, N, H, d = q.shape
    _dev(k, "k", q.dtype, q.shape)
    _dev(v, "v", q.dtype, q.shape)
    _dev(dout, "dout", q.dtype, q.shape)
    if out is not None:
        _dev(out, "out", q.dtype, q.shape)
    K = nbr_idx.shape[2]
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    _dev(lse, "lse", torch.float32, (B, N, H))
    if bias is not None:
        _dev(bias, "bias", q.dtype, (B, N, H, K))
    if near_clusters is not None:
        _dev(near_clusters, "near_clusters", torch.int32, (B, -(-N // S), M))
    if k_blank is not None:
        _dev(k_blank, "k_blank", q.dtype, (H, d))
        _dev(v_blank, "v_blank", q.dtype, (H, d))
    g = dict(grads) if grads else {}
    for name in ("dq", "dk", "dv"):
        if name not in g:
            g[name] = torch.empty_like(q)
        _dev(g[name], name, q.dtype, q.shape)
    if want_dbias:
        if "dbias" not in g:
            g["dbias"] = torch.empty((B, N, H, K), dtype=q.dtype, device=q.device)
        _dev(g["dbias"], "dbias", q.dtype, (B, N, H, K))
    if k_blank is not None:
        for name in ("dk_blank", "dv_blank"):
            if name not in g:
                g[name] = torch.empty((H, d), dtype=torch.float32, device=q.device)
            _dev(g[name], name, torch.float32, (H, d))
    need = lib.affmae_pla_bwd_workspace_bytes(B, N, H, d, K, S, M, code, int(near_clusters is not None))
    if workspace is None:
        workspace = _workspace(need, q.device)
    rc = lib.affmae_pla_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(bias), _ptr(nbr_idx), _ptr(near_clusters), _ptr(plan),
                            _ptr(k_blank), _ptr(v_blank), _ptr(out), _ptr(lse), _ptr(dout), B, N, H, d, K, S, M,
                            float(scale), code, _ptr(g["dq"]), _ptr(g["dk"]), _ptr(g["dv"]), _ptr(g.get("dbias")),
                            _ptr(g.get("dk_blank")), _ptr(g.get("dv_blank")), _ptr(workspace),
                            0 if workspace is None else workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_pla_bwd", rc)
    return g


def affmae_pla_fwd_relpos(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, coords: torch.Tensor,
                          rel_table: torch.Tensor, nbr_idx: torch.Tensor, scale: float, rate: float,
                          near_clusters: Optional[torch.Tensor] = None, S: int = 0, M: int = 0,
                          k_blank: Optional[torch.Tensor] = None, v_blank: Optional[torch.Tensor] = None,
                          out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, plan: Optional[torch.Tensor] = None
                          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Local attention forward with the bias taken from rel_table [H, 2R+1, 2R+1] at the quantised offset of
    every (token, neighbour) pair -> (out [B,N,H,d], lse [B,N,H])."""
    lib = load_library()
    code = _dtype_code(q)
    _dev(q, "q")
    B, N, H, d = q.shape
    _dev(k, "k", q.dtype, q.shape)
    _dev(v, "v", q.dtype, q.shape)
    _dev(coords, "coords", torch.float32, (B, N, 2))
    W = rel_table.shape[-1]
    _dev(rel_table, "rel_table", q.dtype, (H, W, W))
    R = (W - 1) // 2
    K = nbr_idx.shape[2]
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    if near_clusters is not None:
        _dev(near_clusters, "near_clusters", torch.int32, (B, -(-N // S), M))
    if k_blank is not None:
        _dev(k_blank, "k_blank", q.dtype, (H, d))
        _dev(v_blank, "v_blank", q.dtype, (H, d))
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, N, H), dtype=torch.float32, device=q.device)
    need = lib.affmae_pla_fwd_relpos_workspace_bytes(B, N, H, d, K, S, M, code, int(near_clusters is not None))
    if workspace is None:
        workspace = _workspace(need, q.device)
    rc = lib.affmae_pla_fwd_relpos(_ptr(q), _ptr(k), _ptr(v), _ptr(coords), _ptr(rel_table), _ptr(nbr_idx),
                                   _ptr(near_clusters), _ptr(plan), _ptr(k_blank), _ptr(v_blank), B, N, H, d, K, S, M,
                                   float(scale), R, float(rate), code, _ptr(out), _ptr(lse), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_pla_fwd_relpos", rc)
    return out, lse


def affmae_pla_bwd_relpos(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, coords: torch.Tensor,
                          rel_table: torch.Tensor, nbr_idx: torch.Tensor, out: torch.Tensor, lse: torch.Tensor,
                          dout: torch.Tensor, scale: float, rate: float,
                          near_clusters: Optional[torch.Tensor] = None, S: int = 0, M: int = 0,
                          k_blank: Optional[torch.Tensor] = None, v_blank: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, plan: Optional[torch.Tensor] = None
                          ) -> Dict[str, torch.Tensor]:
    """Backward of affmae_pla_fwd_relpos -> dict(dq, dk, dv, drel_table [H,2R+1,2R+1] fp32[, dk_blank, dv_blank])."""
    lib = load_library()
    code = _dtype_code(q)
    _dev(q, "q")
    B, N, H, d = q.shape
    for name, t in (("k", k), ("v", v), ("dout", dout), ("out", out)):
        _dev(t, name, q.dtype, q.shape)
    _dev(coords, "coords", torch.float32, (B, N, 2))
    W = rel_table.shape[-1]
    _dev(rel_table, "rel_table", q.dtype, (H, W, W))
    R = (W - 1) // 2
    K = nbr_idx.shape[2]
    _dev(nbr_idx, "nbr_idx", torch.int32, (B, N, K))
    _dev(lse, "lse", torch.float32, (B, N, H))
    if near_clusters is not None:
        _dev(near_clusters, "near_clusters", torch.int32, (B, -(-N // S), M))
    g = {name: torch.empty_like(q) for name in ("dq", "dk", "dv")}
    g["drel_table"] = torch.empty((H, W, W), dtype=torch.float32, device=q.device)
    if k_blank is not None:
        _dev(k_blank, "k_blank", q.dtype, (H, d))
        _dev(v_blank, "v_blank", q.dtype, (H, d))
        g["dk_blank"] = torch.empty((H, d), dtype=torch.float32, device=q.device)
        g["dv_blank"] = torch.empty((H, d), dtype=torch.float32, device=q.device)
    need = lib.affmae_pla_bwd_relpos_workspace_bytes(B, N, H, d, K, S, M, R, code, int(near_clusters is not None))
    if workspace is None:
        workspace = _workspace(need, q.device)
    rc = lib.affmae_pla_bwd_relpos(_ptr(q), _ptr(k), _ptr(v), _ptr(coords), _ptr(rel_table), _ptr(nbr_idx),
                                   _ptr(near_clusters), _ptr(plan), _ptr(k_blank), _ptr(v_blank), _ptr(out), _ptr(lse),
                                   _ptr(dout), B, N, H, d, K, S, M, float(scale), R, float(rate), code, _ptr(g["dq"]),
                                   _ptr(g["dk"]), _ptr(g["dv"]), _ptr(g["drel_table"]), _ptr(g.get("dk_blank")),
                                   _ptr(g.get("dv_blank")), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream())
    if rc != 0:
        raise AffmaeError("affmae_pla_bwd_relpos", rc)
    return g


def timing_enable(on: bool) -> None:
    """Bracket every kernel launch of the instrumented library with HIP events (benchmarks only; the calls must
    go through it: use_timed_library(True))."""
    _load(_LIB_TIMED_PATH).affmae_timing_enable(int(bool(on)))


def timing_reset() -> None:
    _load(_LIB_TIMED_PATH).affmae_timing_reset()


def timing_read() -> Dict[str, Tuple[float, int]]:
    """Per kernel name: (total milliseconds, launches) since the last reset."""
    lib = _load(_LIB_TIMED_PATH)
    lib.affmae_timing_read.restype = _c_int
    out = {}
    n = lib.affmae_timing_read(-1, None, 0, None, None)
    for i in range(n):
        name = ctypes.create_string_buffer(128)
        ms = ctypes.c_double(0.0)
        cnt = ctypes.c_int(0)
        lib.affmae_timing_read(i, name, 128, ctypes.byref(ms), ctypes.byref(cnt))
        out[name.value.decode()] = (ms.value, cnt.value)
    return out
