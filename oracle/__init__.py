"""ctypes front end of the CPU oracle (oracle/affmae_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu-baseline leg.  The product package never imports this module,
and this module never imports the product package.

All floating-point tensors cross as float64 numpy arrays (callers convert the
stored fp32 / bf16 values exactly); indices are int32; coordinates are fp32
because the neighbour search is defined on fp32 arithmetic.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "affmae_oracle.c")
_LIB = os.path.join(_HERE, "libaffmae_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for name in ("oracle_centroids", "oracle_knn", "oracle_knn_bruteforce", "oracle_cluster", "oracle_vts_table", "oracle_vts_fwd", "oracle_vts_bwd",
                     "oracle_merge_select", "oracle_merge_fwd", "oracle_merge_bwd",
                     "oracle_pla_fwd", "oracle_pla_bwd", "oracle_relpos_bias", "oracle_relpos_dtable", "oracle_num_threads"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.oracle_set_num_threads.restype = None
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f64(a, shape=None) -> Optional[np.ndarray]:
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"shape {a.shape} != expected {shape}")
    return a


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle status {rc}")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(ctypes.c_int(int(n)))


def cluster(coords: np.ndarray, S: int, frame: Tuple[float, float, float, float]) -> Tuple[np.ndarray, np.ndarray]:
    """Balanced clustering along the Z-order curve of `frame` = (x0, y0, w, h)
    -> (order [B,N]: token at each place of the curve, cluster_id [B,N]: place // S per token)."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    B, N, two = coords.shape
    assert two == 2
    x0, y0, w, h = (float(t) for t in frame)
    order = np.empty((B, N), dtype=np.int32)
    cid = np.empty((B, N), dtype=np.int32)
    _check(_load().oracle_cluster(_p(coords), B, N, int(S), ctypes.c_double(x0), ctypes.c_double(y0),
                                  ctypes.c_double(w), ctypes.c_double(h), _p(order), _p(cid)), "oracle_cluster")
    return order, cid


def _grid_args(grid):
    Hg, Wg, x0, y0, cell = grid
    return int(Hg), int(Wg), ctypes.c_float(x0), ctypes.c_float(y0), ctypes.c_float(cell)


def vts_table(vis_xy: np.ndarray, grid, Kt: int) -> np.ndarray:
    """Nearest-visible-token table of the patch grid `grid` = (Hg, Wg, x0, y0, cell) -> [B,Hg,Wg,Kt] int32."""
    vis_xy = np.ascontiguousarray(vis_xy, dtype=np.float32)
    B, Nv, _ = vis_xy.shape
    Hg, Wg, x0, y0, cell = _grid_args(grid)
    table = np.empty((B, Hg, Wg, Kt), dtype=np.int32)
    _check(_load().oracle_vts_table(_p(vis_xy), B, Nv, Hg, Wg, x0, y0, cell, int(Kt), _p(table)), "oracle_vts_table")
    return table


def vts_fwd(query_xy, vis_xy, feat, table, grid, p: float, eps: float, want_weights: bool = False):
    """Virtual sampled tokens -> out [B,Mq,C] (and the weights [B,Mq,Kt])."""
    query_xy = np.ascontiguousarray(query_xy, dtype=np.float32)
    vis_xy = np.ascontiguousarray(vis_xy, dtype=np.float32)
    feat = _f64(feat)
    table = np.ascontiguousarray(table, dtype=np.int32)
    B, Mq, _ = query_xy.shape
    _, Nv, C = feat.shape
    Kt = table.shape[-1]
    Hg, Wg, x0, y0, cell = _grid_args(grid)
    out = np.empty((B, Mq, C), dtype=np.float64)
    w = np.empty((B, Mq, Kt), dtype=np.float64) if want_weights else None
    _check(_load().oracle_vts_fwd(_p(query_xy), _p(vis_xy), _p(feat), _p(table), B, Mq, Nv, C, Hg, Wg, x0, y0, cell,
                                  Kt, ctypes.c_double(p), ctypes.c_double(eps), _p(out), _p(w)), "oracle_vts_fwd")
    return (out, w) if want_weights else out


def vts_bwd(query_xy, vis_xy, feat, table, dout, grid, p: float, eps: float):
    """Backward of vts_fwd -> dict(dfeat [B,Nv,C], dquery [B,Mq,2], dp float, dp_abs float = the sum of the
    absolute per-query contributions to dp, a scale for judging errors of dp)."""
    query_xy = np.ascontiguousarray(query_xy, dtype=np.float32)
    vis_xy = np.ascontiguousarray(vis_xy, dtype=np.float32)
    feat = _f64(feat)
    dout = _f64(dout)
    table = np.ascontiguousarray(table, dtype=np.int32)
    B, Mq, _ = query_xy.shape
    _, Nv, C = feat.shape
    Kt = table.shape[-1]
    Hg, Wg, x0, y0, cell = _grid_args(grid)
    dfeat = np.empty((B, Nv, C), dtype=np.float64)
    dq = np.empty((B, Mq, 2), dtype=np.float64)
    dp = ctypes.c_double(0.0)
    dp_abs = ctypes.c_double(0.0)
    _check(_load().oracle_vts_bwd(_p(query_xy), _p(vis_xy), _p(feat), _p(table), _p(dout), B, Mq, Nv, C, Hg, Wg, x0, y0,
                                  cell, Kt, ctypes.c_double(p), ctypes.c_double(eps), _p(dfeat), _p(dq),
                                  ctypes.byref(dp), ctypes.byref(dp_abs)), "oracle_vts_bwd")
    return {"dfeat": dfeat, "dquery": dq, "dp": float(dp.value), "dp_abs": float(dp_abs.value)}


def merge_select(score: np.ndarray, n_keep: int) -> np.ndarray:
    """Anchors of the neighbourhood merging: score [B,N] fp32 -> anchor_idx [B,n_keep] int32, the n_keep tokens
    with the largest score (equal scores: lower index first), in ascending token index."""
    score = np.ascontiguousarray(score, dtype=np.float32)
    B, N = score.shape
    out = np.empty((B, n_keep), dtype=np.int32)
    _check(_load().oracle_merge_select(_p(score), B, N, n_keep, _p(out)), "oracle_merge_select")
    return out


def merge_fwd(coords, feat, score, nbr_idx, anchor_idx, p: float, want_weights: bool = False):
    """Merged features [B,n_keep,C] (and the aggregation weights [B,n_keep,K] on request)."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    feat = _f64(feat)
    score = np.ascontiguousarray(score, dtype=np.float32)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    anchor_idx = np.ascontiguousarray(anchor_idx, dtype=np.int32)
    B, N, C = feat.shape
    K = nbr_idx.shape[2]
    n_keep = anchor_idx.shape[1]
    out = np.empty((B, n_keep, C), dtype=np.float64)
    w = np.empty((B, n_keep, K), dtype=np.float64) if want_weights else None
    _check(_load().oracle_merge_fwd(_p(coords), _p(feat), _p(score), _p(nbr_idx), _p(anchor_idx), B, N, C, K, n_keep,
                                    ctypes.c_double(p), _p(out), _p(w)), "oracle_merge_fwd")
    return (out, w) if want_weights else out


def merge_bwd(coords, feat, score, nbr_idx, anchor_idx, dout, p: float):
    """Backward of merge_fwd -> dict(dfeat [B,N,C], dscore [B,N], dp float, dp_abs float)."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    feat = _f64(feat)
    dout = _f64(dout)
    score = np.ascontiguousarray(score, dtype=np.float32)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    anchor_idx = np.ascontiguousarray(anchor_idx, dtype=np.int32)
    B, N, C = feat.shape
    K = nbr_idx.shape[2]
    n_keep = anchor_idx.shape[1]
    dfeat = np.empty((B, N, C), dtype=np.float64)
    dscore = np.empty((B, N), dtype=np.float64)
    dp = ctypes.c_double(0.0)
    dp_abs = ctypes.c_double(0.0)
    _check(_load().oracle_merge_bwd(_p(coords), _p(feat), _p(score), _p(nbr_idx), _p(anchor_idx), _p(dout), B, N, C, K,
                                    n_keep, ctypes.c_double(p), _p(dfeat), _p(dscore), ctypes.byref(dp),
                                    ctypes.byref(dp_abs)), "oracle_merge_bwd")
    return {"dfeat": dfeat, "dscore": dscore, "dp": float(dp.value), "dp_abs": float(dp_abs.value)}


def centroids(coords: np.ndarray, cluster_id: Optional[np.ndarray], S: int) -> np.ndarray:
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    B, N, _ = coords.shape
    if cluster_id is not None:
        cluster_id = np.ascontiguousarray(cluster_id, dtype=np.int32)
    out = np.empty((B, -(-N // S), 2), dtype=np.float32)
    _check(_load().oracle_centroids(_p(coords), _p(cluster_id), B, N, S, _p(out)), "oracle_centroids")
    return out


def knn(coords: np.ndarray, cluster_id: Optional[np.ndarray], S: int, M: int, K: int
        ) -> Tuple[np.ndarray, np.ndarray]:
    """Clustered neighbour search -> (nbr_idx [B,N,K], near_clusters [B,G,M])."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    B, N, two = coords.shape
    assert two == 2
    if cluster_id is not None:
        cluster_id = np.ascontiguousarray(cluster_id, dtype=np.int32)
        assert cluster_id.shape == (B, N)
    if S <= 0:
        raise ValueError("S must be positive")
    nbr = np.empty((B, N, K), dtype=np.int32)
    near = np.empty((B, -(-N // S), M), dtype=np.int32)  # the last cluster is short when S does not divide N
    _check(_load().oracle_knn(_p(coords), _p(cluster_id), B, N, S, M, K, _p(nbr), _p(near)), "oracle_knn")
    return nbr, near


def knn_bruteforce(coords: np.ndarray, K: int) -> np.ndarray:
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    B, N, _ = coords.shape
    nbr = np.empty((B, N, K), dtype=np.int32)
    _check(_load().oracle_knn_bruteforce(_p(coords), B, N, K, _p(nbr)), "oracle_knn_bruteforce")
    return nbr


def pla_fwd(q, k, v, bias, nbr_idx, scale: float, k_blank=None, v_blank=None, want_prob: bool = False):
    """Local attention forward -> (out [B,N,H,d], lse [B,N,H][, prob [B,N,H,K+1]])."""
    q = _f64(q)
    B, N, H, d = q.shape
    k = _f64(k, q.shape)
    v = _f64(v, q.shape)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    K = nbr_idx.shape[2]
    assert nbr_idx.shape == (B, N, K)
    bias = _f64(bias, (B, N, H, K))
    k_blank = _f64(k_blank, (H, d))
    v_blank = _f64(v_blank, (H, d))
    out = np.empty((B, N, H, d), dtype=np.float64)
    lse = np.empty((B, N, H), dtype=np.float64)
    prob = np.empty((B, N, H, K + 1), dtype=np.float64) if want_prob else None
    _check(_load().oracle_pla_fwd(_p(q), _p(k), _p(v), _p(bias), _p(nbr_idx), _p(k_blank), _p(v_blank),
                                  B, N, H, d, K, ctypes.c_double(scale), _p(out), _p(lse), _p(prob)),
           "oracle_pla_fwd")
    return (out, lse, prob) if want_prob else (out, lse)


def pla_bwd(q, k, v, bias, nbr_idx, dout, scale: float, k_blank=None, v_blank=None):
    """Local attention backward -> dict(dq, dk, dv, dbias[, dk_blank, dv_blank])."""
    q = _f64(q)
    B, N, H, d = q.shape
    k = _f64(k, q.shape)
    v = _f64(v, q.shape)
    dout = _f64(dout, q.shape)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    K = nbr_idx.shape[2]
    bias = _f64(bias, (B, N, H, K))
    k_blank = _f64(k_blank, (H, d))
    v_blank = _f64(v_blank, (H, d))
    dq = np.empty_like(q)
    dk = np.empty_like(q)
    dv = np.empty_like(q)
    dbias = np.empty((B, N, H, K), dtype=np.float64)
    dkb = np.empty((H, d), dtype=np.float64) if k_blank is not None else None
    dvb = np.empty((H, d), dtype=np.float64) if k_blank is not None else None
    _check(_load().oracle_pla_bwd(_p(q), _p(k), _p(v), _p(bias), _p(nbr_idx), _p(k_blank), _p(v_blank),
                                  _p(dout), B, N, H, d, K, ctypes.c_double(scale), _p(dq), _p(dk), _p(dv),
                                  _p(dbias), _p(dkb), _p(dvb)), "oracle_pla_bwd")
    res = {"dq": dq, "dk": dk, "dv": dv, "dbias": dbias}
    if dkb is not None:
        res["dk_blank"] = dkb
        res["dv_blank"] = dvb
    return res


def relpos_bias(coords, nbr_idx, table, R: int, rate: float) -> np.ndarray:
    """Relative-position bias from a per-head table [H, 2R+1, 2R+1] over quantised offsets -> [B,N,H,K]."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    B, N, K = nbr_idx.shape
    W = 2 * int(R) + 1
    table = _f64(table)
    H = table.shape[0]
    assert table.shape == (H, W, W) and coords.shape == (B, N, 2)
    bias = np.empty((B, N, H, K), dtype=np.float64)
    _check(_load().oracle_relpos_bias(_p(coords), _p(nbr_idx), _p(table), B, N, H, K, int(R), ctypes.c_float(rate),
                                      _p(bias)), "oracle_relpos_bias")
    return bias


def relpos_dtable(coords, nbr_idx, dbias, R: int, rate: float) -> np.ndarray:
    """Gradient of the table: the bias gradients [B,N,H,K] added up per bin -> [H, 2R+1, 2R+1]."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    nbr_idx = np.ascontiguousarray(nbr_idx, dtype=np.int32)
    B, N, K = nbr_idx.shape
    dbias = _f64(dbias)
    H = dbias.shape[2]
    assert dbias.shape == (B, N, H, K)
    W = 2 * int(R) + 1
    dtable = np.empty((H, W, W), dtype=np.float64)
    _check(_load().oracle_relpos_dtable(_p(coords), _p(nbr_idx), _p(dbias), B, N, H, K, int(R), ctypes.c_float(rate),
                                        _p(dtable)), "oracle_relpos_dtable")
    return dtable


def pla_fwd_relpos(q, k, v, coords, table, nbr_idx, scale: float, R: int, rate: float, k_blank=None, v_blank=None):
    """Local attention with the bias taken from the relative-position table -> (out, lse)."""
    return pla_fwd(q, k, v, relpos_bias(coords, nbr_idx, table, R, rate), nbr_idx, scale, k_blank, v_blank)


def pla_bwd_relpos(q, k, v, coords, table, nbr_idx, dout, scale: float, R: int, rate: float, k_blank=None,
                   v_blank=None):
    """Backward of pla_fwd_relpos -> dict(dq, dk, dv, dtable[, dk_blank, dv_blank])."""
    g = pla_bwd(q, k, v, relpos_bias(coords, nbr_idx, table, R, rate), nbr_idx, dout, scale, k_blank, v_blank)
    g["dtable"] = relpos_dtable(coords, nbr_idx, g.pop("dbias"), R, rate)
    return g
