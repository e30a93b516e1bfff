"""GPU parity: affmae_knn against the CPU oracle, bit-exact on every index."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_16249_amd as aff
from workloads import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _gpu_knn(coords, cluster_id, S, M, K):
    c = torch.from_numpy(coords).cuda()
    cid = torch.from_numpy(cluster_id).cuda() if cluster_id is not None else None
    nbr, near = aff.affmae_knn(c, cid, S, M, K)
    torch.cuda.synchronize()
    return nbr.cpu().numpy(), near.cpu().numpy()


SMALL = [
    # name, B, N, S, M, K
    ("tiny_f32", 1, 256, 256, 1, 16),          # the exact-kNN configuration as specified
    ("tiny_f32", 2, 256, 32, 8, 16),           # M == G: exact through the clustered path
    ("mae_pt_s1_1024", 3, 1024, 64, 8, 48),    # on-grid, ties everywhere
    ("mae_pt_s1_1024", 2, 960, 48, 5, 33),     # ragged sizes: S, M*S, K not multiples of 64
    ("ft_s1_1024", 1, 16384, 64, 8, 48),       # one full 1024px image
    ("merged_stage", 4, 1024, 32, 8, 48),
    ("knn_scale", 2, 2048, 64, 8, 48),
    ("knn_scale", 2, 2048, 64, 8, 64),         # K at the limit
    ("knn_scale", 2, 512, 8, 3, 1),            # K = 1: every token is its own nearest
    ("knn_scale", 1, 640, 10, 64, 64),         # M at the limit, odd S
    ("knn_scale", 1, 4096, 64, 64, 64),        # the most candidates the library takes (4096)
    ("tiny_f32", 2, 1024, 128, 8, 48),         # 1024 candidates: the general kernel
]


@pytest.mark.parametrize("name,B,N,S,M,K", SMALL)
def test_knn_matches_oracle(name, B, N, S, M, K):
    cfg = CONFIGS[name].scaled(B=B, N=N, S=S, M=M, K=K)
    if cfg.coords == "jitter_grid" and N != 16384:
        cfg = cfg.scaled(frame=8.0 * int(round(N ** 0.5)))
    print(f"case {name} B={B} N={N} S={S} M={M} K={K}", flush=True)
    w = make_workload(cfg, features=False)
    nbr, near = _gpu_knn(w["coords"], None, S, M, K)
    rnbr, rnear = oracle.knn(w["coords"], None, S, M, K)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)


def test_knn_with_scattered_cluster_ids():
    rng = np.random.default_rng(5)
    B, N, S, M, K = 2, 768, 24, 6, 40
    coords = rng.uniform(0, 300, size=(B, N, 2)).astype(np.float32)
    cid = np.stack([rng.permutation(np.repeat(np.arange(N // S), S)) for _ in range(B)]).astype(np.int32)
    nbr, near = _gpu_knn(coords, cid, S, M, K)
    rnbr, rnear = oracle.knn(coords, cid, S, M, K)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)


def test_knn_coincident_points_and_integer_grid():
    """All distances tie in groups: order is decided by the index alone."""
    rng = np.random.default_rng(6)
    B, N, S, M, K = 1, 512, 32, 16, 48
    coords = rng.integers(0, 5, size=(B, N, 2)).astype(np.float32)
    nbr, near = _gpu_knn(coords, None, S, M, K)
    rnbr, rnear = oracle.knn(coords, None, S, M, K)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)


@pytest.mark.parametrize("S,M,K", [(64, 8, 48), (64, 8, 64), (16, 4, 1), (128, 8, 48)])
def test_knn_all_points_identical(S, M, K):
    """Every distance is 0: no distance threshold separates K candidates, the index decides everything."""
    B, N = 2, 1024
    coords = np.full((B, N, 2), 3.25, dtype=np.float32)
    nbr, near = _gpu_knn(coords, None, S, M, K)
    rnbr, rnear = oracle.knn(coords, None, S, M, K)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)


@pytest.mark.parametrize("name", ["mae_pt_s1_1024", "ft_s1_1024", "merged_stage", "knn_scale"])
def test_knn_full_size_configs(name):
    """The benchmark's configurations at full size, every index compared."""
    cfg = CONFIGS[name]
    print(f"case {name} full size", flush=True)
    w = make_workload(cfg, features=False)
    nbr, near = _gpu_knn(w["coords"], w["cluster_id"], cfg.S, cfg.M, cfg.K)
    rnbr, rnear = oracle.knn(w["coords"], w["cluster_id"], cfg.S, cfg.M, cfg.K)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)
    # the table produced without an explicit assignment (tokens are in cluster order) is the same
    nbr2, near2 = _gpu_knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    assert np.array_equal(nbr2, rnbr) and np.array_equal(near2, rnear)


RAGGED = [
    # name, B, N, S, M, K: the last cluster holds N - (G - 1) S tokens
    ("mae_pt_s1_1024", 2, 4000, 64, 8, 48),    # 62 clusters of 64 and one of 32
    ("knn_scale", 2, 481, 32, 3, 20),          # a last cluster of one token
    ("knn_scale", 3, 33, 32, 2, 1),            # two clusters, the second a single token
    ("merged_stage", 2, 1001, 32, 8, 48),      # N odd: nothing is a whole tile
    ("tiny_f32", 2, 1000, 128, 8, 48),         # 1024 candidate places (general kernel), 104 tokens in the last cluster
    ("knn_scale", 1, 100, 64, 2, 100),         # M == G: exact search over 100 tokens, K = all of them... capped below
]


@pytest.mark.parametrize("name,B,N,S,M,K", RAGGED)
def test_knn_short_last_cluster(name, B, N, S, M, K):
    K = min(K, 64)
    cfg = CONFIGS[name].scaled(B=B, N=N, S=S, M=M, K=K)
    print(f"case ragged {name} B={B} N={N} S={S} M={M} K={K}", flush=True)
    w = make_workload(cfg, features=False)
    nbr, near = _gpu_knn(w["coords"], None, S, M, K)
    rnbr, rnear = oracle.knn(w["coords"], None, S, M, K)
    assert near.shape == rnear.shape == (B, -(-N // S), M)
    assert np.array_equal(near, rnear)
    assert np.array_equal(nbr, rnbr)
    # the same clusters given as an explicit (scattered) assignment
    rng = np.random.default_rng(N)
    perm = np.stack([rng.permutation(N) for _ in range(B)])
    coords = np.ascontiguousarray(np.take_along_axis(w["coords"], perm[..., None], axis=1))
    cid = (perm // S).astype(np.int32)
    nbr_s, near_s = _gpu_knn(coords, cid, S, M, K)
    rnbr_s, rnear_s = oracle.knn(coords, cid, S, M, K)
    assert np.array_equal(near_s, rnear_s)
    assert np.array_equal(nbr_s, rnbr_s)
