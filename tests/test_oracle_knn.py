"""Pins for the oracle's neighbour search (CPU only).

Each test checks oracle/affmae_oracle.c against something that is not itself:
hand-derived fixtures, exact integer arithmetic, a library sort over all pairs,
closed-form centroids, and the invariants a nearest-neighbour list must have.
"""
import os

import numpy as np
import pytest

import oracle
from workloads import CONFIGS, make_workload


def _read_lists(path, prefix=None):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, tail = line.split(":")
            head = head.split()
            if prefix is None:
                key = int(head[0])
            elif head[0] == prefix:
                key = int(head[1])
            else:
                continue
            out[key] = [int(t) for t in tail.split()]
    return out


def _numpy_bruteforce(coords, K):
    """All-pairs search with numpy's fp32 elementwise ops and a library sort."""
    B, N, _ = coords.shape
    res = np.empty((B, N, K), dtype=np.int32)
    for b in range(B):
        x = coords[b, :, 0].astype(np.float32)
        y = coords[b, :, 1].astype(np.float32)
        dx = (x[:, None] - x[None, :]).astype(np.float32)
        dy = (y[:, None] - y[None, :]).astype(np.float32)
        d2 = (dx * dx).astype(np.float32) + (dy * dy).astype(np.float32)
        assert d2.dtype == np.float32
        idx = np.broadcast_to(np.arange(N)[None, :], (N, N))
        order = np.lexsort((idx, d2), axis=1)  # last key is primary
        res[b] = order[:, :K]
    return res


def test_grid4x4_hand_derived(golden_dir):
    want = _read_lists(os.path.join(golden_dir, "knn_grid4x4.txt"))
    xs, ys = np.meshgrid(np.arange(4), np.arange(4), indexing="xy")
    coords = np.stack([xs.ravel(), ys.ravel()], -1).astype(np.float32)[None]
    got = oracle.knn_bruteforce(coords, 9)
    for tok, lst in want.items():
        assert got[0, tok].tolist() == lst
    # the same lists from the clustered search when every cluster is searched
    got2, _ = oracle.knn(coords, None, S=4, M=4, K=9)
    for tok, lst in want.items():
        assert got2[0, tok].tolist() == lst


def test_line_clustered_hand_derived(golden_dir):
    path = os.path.join(golden_dir, "knn_line_clustered.txt")
    near_want = _read_lists(path, "near")
    nbr_want = _read_lists(path, "nbr")
    coords = np.stack([np.arange(16), np.zeros(16)], -1).astype(np.float32)[None]
    nbr, near = oracle.knn(coords, None, S=4, M=2, K=6)
    for c, lst in near_want.items():
        assert near[0, c].tolist() == lst
    for tok, lst in nbr_want.items():
        assert nbr[0, tok].tolist() == lst


def test_near_clusters_blocks_hand_derived(golden_dir):
    want = _read_lists(os.path.join(golden_dir, "near_clusters_blocks.txt"))
    xs, ys = np.meshgrid(np.arange(8), np.arange(8), indexing="xy")
    coords = np.stack([xs.ravel(), ys.ravel()], -1).astype(np.float32)[None]
    cid = (4 * (ys.ravel() // 2) + (xs.ravel() // 2)).astype(np.int32)[None]
    cen = oracle.centroids(coords, cid, S=4)
    bx, by = np.meshgrid(np.arange(4), np.arange(4), indexing="xy")
    closed = np.stack([2 * bx.ravel() + 0.5, 2 * by.ravel() + 0.5], -1).astype(np.float32)
    assert np.array_equal(cen[0], closed)
    _, near = oracle.knn(coords, cid, S=4, M=9, K=4)
    for c, lst in want.items():
        assert near[0, c].tolist() == lst


def test_scattered_cluster_ids_match_reordered_contiguous():
    """A scattered cluster assignment must give the lists of the same token set
    stored in cluster order, mapped back through the permutation."""
    rng = np.random.default_rng(11)
    N, S, M, K = 96, 8, 3, 10
    coords = rng.uniform(0, 50, size=(1, N, 2)).astype(np.float32)
    cid = rng.permutation(np.repeat(np.arange(N // S), S)).astype(np.int32)[None]
    nbr, near = oracle.knn(coords, cid, S, M, K)
    order = np.argsort(cid[0], kind="stable")          # new position -> old token
    inv = np.empty(N, dtype=np.int64)
    inv[order] = np.arange(N)
    nbr2, near2 = oracle.knn(coords[:, order], None, S, M, K)
    assert np.array_equal(near, near2)
    # As sets: the index tie-break may differ between the two numberings, but
    # random real coordinates have no equal distances.
    back = order[nbr2[0]]                              # lists of new tokens in old numbering
    assert np.array_equal(nbr[0][order], back)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_integer_coordinates_exact_arithmetic(seed):
    """On small integer coordinates fp32 distances are exact, so plain Python
    integer arithmetic and tuple sorting decide the answer."""
    rng = np.random.default_rng(seed)
    N, K = 60, 12
    pts = rng.integers(0, 6, size=(N, 2))  # many coincident points and ties
    coords = pts.astype(np.float32)[None]
    got = oracle.knn_bruteforce(coords, K)[0]
    for i in range(N):
        keyed = sorted(((int(pts[i, 0] - pts[j, 0]) ** 2 + int(pts[i, 1] - pts[j, 1]) ** 2, j) for j in range(N)))
        assert got[i].tolist() == [j for _, j in keyed[:K]]


@pytest.mark.parametrize("recipe_cfg", ["tiny_f32", "mae_pt_s1_1024", "ft_s1_1024", "knn_scale"])
def test_bruteforce_matches_library_sort(recipe_cfg):
    cfg = CONFIGS[recipe_cfg].scaled(B=2, N=512, S=32, M=4, K=20)
    # masked_grid keeps 512 of the 16384 cells: sparse but on-grid, ties everywhere
    if cfg.coords == "jitter_grid":
        cfg = cfg.scaled(N=256, frame=128.0)
    w = make_workload(cfg, features=False)
    got = oracle.knn_bruteforce(w["coords"], cfg.K)
    assert np.array_equal(got, _numpy_bruteforce(w["coords"], cfg.K))


def test_clustered_search_over_all_clusters_is_exact():
    cfg = CONFIGS["mae_pt_s1_1024"].scaled(B=2, N=256, S=16, M=16, K=24)
    w = make_workload(cfg, features=False)
    nbr, near = oracle.knn(w["coords"], w["cluster_id"], cfg.S, cfg.M, cfg.K)
    assert np.array_equal(nbr, oracle.knn_bruteforce(w["coords"], cfg.K))
    # near lists are permutations of all clusters starting with the cluster itself
    assert np.array_equal(np.sort(near, axis=2), np.broadcast_to(np.arange(16), near.shape))
    assert np.array_equal(near[:, :, 0], np.broadcast_to(np.arange(16), near.shape[:2]))


def test_clustered_search_is_bruteforce_restricted_to_candidates():
    """With M < G the list must equal a library-sorted search over exactly the
    members of the near clusters (and the near clusters must be the library-
    sorted nearest centroids)."""
    cfg = CONFIGS["knn_scale"].scaled(B=2, N=512, S=32, M=4, K=40)
    w = make_workload(cfg, features=False)
    coords = w["coords"]
    nbr, near = oracle.knn(coords, w["cluster_id"], cfg.S, cfg.M, cfg.K)
    G = cfg.G
    for b in range(cfg.B):
        cen = coords[b].reshape(G, cfg.S, 2).astype(np.float64).mean(axis=1).astype(np.float32)
        want_near = _numpy_bruteforce(cen[None], cfg.M)[0]
        assert np.array_equal(near[b], want_near)
        for c in range(G):
            cand = np.concatenate([np.arange(e * cfg.S, (e + 1) * cfg.S) for e in want_near[c]])
            cand.sort()
            sub = _numpy_bruteforce(coords[b, cand][None], len(cand))[0]  # local indices, full order
            for r in range(cfg.S):
                i = c * cfg.S + r
                li = int(np.searchsorted(cand, i))
                assert np.array_equal(nbr[b, i], cand[sub[li, :cfg.K]])


def test_invariants_on_distinct_coordinates():
    cfg = CONFIGS["merged_stage"].scaled(B=3, N=256, S=32, M=4, K=48)
    w = make_workload(cfg, features=False)
    coords = w["coords"]
    nbr, _ = oracle.knn(coords, w["cluster_id"], cfg.S, cfg.M, cfg.K)
    assert nbr.min() >= 0 and nbr.max() < cfg.N
    assert np.array_equal(nbr[:, :, 0], np.broadcast_to(np.arange(cfg.N), (cfg.B, cfg.N)))
    for b in range(cfg.B):
        p = coords[b].astype(np.float64)
        d = ((p[:, None, :] - p[nbr[b]]) ** 2).sum(-1)
        assert np.all(np.diff(d, axis=1) >= -1e-9)
        assert all(len(set(row)) == cfg.K for row in nbr[b].tolist())


def test_argument_errors():
    coords = np.zeros((1, 16, 2), dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.knn(coords, None, S=4, M=5, K=4)       # M > G
    with pytest.raises(RuntimeError):
        oracle.knn(coords, None, S=4, M=2, K=9)       # K > M*S
    bad = np.zeros((1, 16), dtype=np.int32)            # all tokens in cluster 0
    with pytest.raises(RuntimeError):
        oracle.knn(coords, bad, S=4, M=2, K=4)


def test_short_last_cluster_hand_derived(golden_dir):
    path = os.path.join(golden_dir, "knn_line_short_last_cluster.txt")
    near_want = _read_lists(path, "near")
    nbr_want = _read_lists(path, "nbr")
    coords = np.stack([np.arange(14), np.zeros(14)], -1).astype(np.float32)[None]
    cen = oracle.centroids(coords, None, S=4)
    assert cen[0, :, 0].tolist() == [1.5, 5.5, 9.5, 12.5]
    nbr, near = oracle.knn(coords, None, S=4, M=2, K=5)
    assert near.shape == (1, 4, 2)
    for c, lst in near_want.items():
        assert near[0, c].tolist() == lst
    for tok, lst in nbr_want.items():
        assert nbr[0, tok].tolist() == lst
    with pytest.raises(RuntimeError):
        oracle.knn(coords, None, S=4, M=2, K=7)       # clusters 2 and 3 offer six candidates only


@pytest.mark.parametrize("N", [500, 481, 33])
def test_short_last_cluster_is_bruteforce_restricted_to_candidates(N):
    """The library-sorted search over exactly the members of the near clusters, with a last cluster of
    N - (G - 1) S tokens; with M = G the search is exact; scattered cluster ids equal the re-ordered case."""
    S, M, K = 32, 3, 20
    rng = np.random.default_rng(N)
    coords = rng.uniform(0, 100, size=(2, N, 2)).astype(np.float32)
    G = -(-N // S)
    M = min(M, G)
    if G == 2:
        K = 1  # the smallest candidate set is the short cluster plus one full one
    nbr, near = oracle.knn(coords, None, S, M, K)
    for b in range(2):
        members = [np.arange(c * S, min((c + 1) * S, N)) for c in range(G)]
        cen = np.stack([coords[b, m].astype(np.float64).mean(axis=0) for m in members]).astype(np.float32)
        want_near = _numpy_bruteforce(cen[None], M)[0]
        assert np.array_equal(near[b], want_near)
        for c in range(G):
            cand = np.sort(np.concatenate([members[e] for e in want_near[c]]))
            sub = _numpy_bruteforce(coords[b, cand][None], len(cand))[0]
            for i in members[c]:
                li = int(np.searchsorted(cand, i))
                assert np.array_equal(nbr[b, i], cand[sub[li, :K]])
    exact, _ = oracle.knn(coords, None, S, G, K)
    assert np.array_equal(exact, oracle.knn_bruteforce(coords, K))
    # scattered ids: the short cluster must be the last one
    sizes = [len(m) for m in members]
    cid = rng.permutation(np.repeat(np.arange(G), sizes)).astype(np.int32)
    nbr_s, near_s = oracle.knn(coords[:1], cid[None], S, M, K)
    order = np.argsort(cid, kind="stable")
    nbr_o, near_o = oracle.knn(coords[:1, order], None, S, M, K)
    assert np.array_equal(near_s, near_o)
    assert np.array_equal(nbr_s[0][order], order[nbr_o[0]])
