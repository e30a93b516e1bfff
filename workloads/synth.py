"""Seeded input generators shaped like the paper's microscopy token sets.

The paper trains on a private archive of electron-microscopy images (Sec.
"Experiments"); the cost of the neighbourhood-attention path depends only on
token geometry and tensor shapes, so synthetic token sets stand in for it:

* stage-1 tokens sit at the centres of 8-pixel patches (Supp. "AFF
  architecture": patch size 8), i.e. a 128x128 grid for a 1024px image;
* MAE pre-training keeps a random 25 % of them (Sec. "AFFMAE": the encoder sees
  visible tokens only);
* deeper stages hold fewer, off-grid tokens produced by adaptive merging
  (Sec. "AutoFocusFormer"), concentrated on structures (Sec. "Discussion").

Tokens are put into equal-size clusters along a space-filling curve (Sec.
"AutoFocusFormer").  The curve is not named by the paper; Z-order (Morton) on
coordinates quantised to 16 bits per axis is used here, ties by original index.

Nothing in this file computes neighbourhoods or attention.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

BASE_SEED = 2602016249


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int          # position in the benchmark's config list (seed offset)
    B: int              # images
    N: int              # tokens per image
    C: int              # channels = H * d
    H: int              # heads
    K: int              # neighbours per token
    S: int              # cluster size
    M: int              # nearest clusters searched
    dtype: str          # "f32" or "bf16": storage type of q/k/v/bias/out
    coords: str         # coordinate recipe, see make_coords
    frame: float        # side of the square frame in pixels

    @property
    def d(self) -> int:
        return self.C // self.H

    @property
    def G(self) -> int:
        return -(-self.N // self.S)  # the last cluster is short when S does not divide N

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "WorkloadConfig":
        """Same recipe at other sizes (used by tests for small parity cases)."""
        d = dict(self.__dict__)
        d.update(kw)
        return WorkloadConfig(**d)


CONFIGS: Dict[str, WorkloadConfig] = {
    c.name: c
    for c in [
        # exact kNN: one cluster holding the whole image
        WorkloadConfig("tiny_f32", 0, 1, 256, 64, 2, 16, 256, 1, "f32", "uniform", 64.0),
        WorkloadConfig("mae_pt_s1_1024", 1, 16, 4096, 64, 2, 48, 64, 8, "bf16", "masked_grid", 1024.0),
        WorkloadConfig("ft_s1_1024", 2, 8, 16384, 64, 2, 48, 64, 8, "bf16", "jitter_grid", 1024.0),
        WorkloadConfig("merged_stage", 3, 64, 1024, 256, 8, 48, 32, 8, "bf16", "uniform", 1024.0),
        WorkloadConfig("knn_scale", 4, 16, 16384, 128, 4, 48, 64, 8, "bf16", "blobs", 1024.0),
    ]
}


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); returns fp32
    holding exactly representable values.  Storage-format conversion only."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


def _morton_key(qx: np.ndarray, qy: np.ndarray) -> np.ndarray:
    """Interleave two 16-bit integers (x in even bits, y in odd bits)."""
    def spread(v):
        v = v.astype(np.uint64) & np.uint64(0xFFFF)
        v = (v | (v << np.uint64(8))) & np.uint64(0x00FF00FF)
        v = (v | (v << np.uint64(4))) & np.uint64(0x0F0F0F0F)
        v = (v | (v << np.uint64(2))) & np.uint64(0x33333333)
        v = (v | (v << np.uint64(1))) & np.uint64(0x55555555)
        return v
    return spread(qx) | (spread(qy) << np.uint64(1))


def morton_cluster_order(coords: np.ndarray, frame: float) -> np.ndarray:
    """Permutation [B,N] that sorts each image's tokens along a Z-order curve.

    Consecutive chunks of S tokens of the permuted array are the equal-size
    clusters.  Stable sort: equal keys keep their original order."""
    B, N, _ = coords.shape
    q = np.floor(coords.astype(np.float64) / frame * 65536.0)
    q = np.clip(q, 0, 65535).astype(np.uint32)
    key = _morton_key(q[..., 0], q[..., 1])
    return np.argsort(key, axis=1, kind="stable")


def make_coords(recipe: str, B: int, N: int, frame: float, rng: np.random.Generator) -> np.ndarray:
    """fp32 [B,N,2] (x,y) pixel coordinates, before cluster ordering."""
    if recipe == "uniform":
        return rng.uniform(0.0, frame, size=(B, N, 2)).astype(np.float32)
    if recipe in ("masked_grid", "jitter_grid"):
        side = int(round(frame / 8.0))
        ix, iy = np.meshgrid(np.arange(side), np.arange(side), indexing="xy")
        grid = np.stack([8.0 * ix.ravel() + 4.0, 8.0 * iy.ravel() + 4.0], axis=-1).astype(np.float32)
        out = np.empty((B, N, 2), dtype=np.float32)
        if recipe == "masked_grid":
            if N > side * side:
                raise ValueError("more visible tokens than grid cells")
            for b in range(B):
                keep = np.sort(rng.permutation(side * side)[:N])
                out[b] = grid[keep]
        else:
            if N != side * side:
                raise ValueError("jitter_grid needs N == (frame/8)^2")
            jit = rng.uniform(-2.0, 2.0, size=(B, N, 2)).astype(np.float32)
            out[:] = grid[None] + jit
        return out
    if recipe == "blobs":
        out = np.empty((B, N, 2), dtype=np.float32)
        for b in range(B):
            centres = rng.uniform(0.0, frame, size=(64, 2))
            pts = np.empty((N, 2), dtype=np.float64)
            todo = np.arange(N)
            while todo.size:
                which = rng.integers(0, 64, size=todo.size)
                cand = centres[which] + rng.normal(0.0, 20.0, size=(todo.size, 2))
                ok = np.all((cand >= 0.0) & (cand < frame), axis=1)
                pts[todo[ok]] = cand[ok]
                todo = todo[~ok]
            out[b] = pts.astype(np.float32)
        return out
    raise ValueError(f"unknown coordinate recipe {recipe!r}")


def make_features(B: int, N: int, H: int, d: int, K: int, dtype: str,
                  rng: np.random.Generator, blank: bool = False) -> Dict[str, np.ndarray]:
    """q,k,v,dout ~ N(0,1) [B,N,H,d]; bias ~ N(0, 0.1) [B,N,H,K]; all returned as
    fp32 arrays whose values are exactly representable in `dtype`."""
    cast = bf16_round if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    out = {}
    for name in ("q", "k", "v", "dout"):
        out[name] = cast(rng.standard_normal((B, N, H, d), dtype=np.float32))
    out["bias"] = cast((0.1 * rng.standard_normal((B, N, H, K), dtype=np.float32)).astype(np.float32))
    if blank:
        out["k_blank"] = cast(rng.standard_normal((H, d), dtype=np.float32))
        out["v_blank"] = cast(rng.standard_normal((H, d), dtype=np.float32))
    return out


def random_neighbours(B: int, N: int, K: int, rng: np.random.Generator,
                      distinct: bool = True) -> np.ndarray:
    """Arbitrary neighbour lists int32 [B,N,K] with values in [0,N) (the
    attention entry points accept any such table).  `distinct=False` allows a
    token to list the same neighbour more than once."""
    if not distinct:
        return rng.integers(0, N, size=(B, N, K)).astype(np.int32)
    if K > N:
        raise ValueError("K > N with distinct neighbours")
    out = np.empty((B, N, K), dtype=np.int32)
    for b in range(B):
        for i in range(N):
            out[b, i] = rng.choice(N, size=K, replace=False)
    return out


def make_workload(cfg: WorkloadConfig, seed: Optional[int] = None, blank: bool = False,
                  features: bool = True) -> Dict[str, np.ndarray]:
    """Coordinates in cluster order, cluster ids, and (optionally) features."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    coords = make_coords(cfg.coords, cfg.B, cfg.N, cfg.frame, rng)
    perm = morton_cluster_order(coords, cfg.frame)
    coords = np.ascontiguousarray(np.take_along_axis(coords, perm[..., None], axis=1))
    cluster_id = np.broadcast_to((np.arange(cfg.N, dtype=np.int32) // cfg.S)[None], (cfg.B, cfg.N))
    w = {"coords": coords, "cluster_id": np.ascontiguousarray(cluster_id, dtype=np.int32)}
    if features:
        w.update(make_features(cfg.B, cfg.N, cfg.H, cfg.d, cfg.K, cfg.dtype, rng, blank=blank))
    return w
