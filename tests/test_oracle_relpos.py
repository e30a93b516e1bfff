"""Pins of the relative-position bias oracle (oracle_relpos_bias, oracle_relpos_dtable): a fixture written out by
hand, the rounding and clamping rules one case at a time, the same quantities from numpy library routines, the
conservation of the gradient, and finite differences of the whole attention with respect to the table."""
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _index_table(H, R):
    """A table whose entries name their own (head, row, column)."""
    W = 2 * R + 1
    return (np.arange(H)[:, None, None] * 10000 + np.arange(W)[None, :, None] * 100 + np.arange(W)[None, None, :]).astype(np.float64)


def test_fixture_written_by_hand():
    coords = np.array([[[0, 0], [1, 0], [0, 2], [2.5, 0], [-1.5, 3]]], dtype=np.float32)
    nbr = np.tile(np.arange(5, dtype=np.int32), (1, 5, 1))
    want = {}
    for line in open(os.path.join(HERE, "golden", "relpos_5tokens.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        want[int(parts[0])] = [tuple(int(t) for t in p.split(",")) for p in parts[1:]]
    bias = oracle.relpos_bias(coords, nbr, _index_table(2, 1), 1, 1.0)
    for q in range(5):
        for j, (by, bx) in enumerate(want[q]):
            assert bias[0, q, 0, j] == by * 100 + bx, (q, j)
            assert bias[0, q, 1, j] == 10000 + by * 100 + bx, (q, j)


@pytest.mark.parametrize("offset,rate,R,want", [
    (0.5, 1.0, 3, 0), (1.5, 1.0, 3, 2), (2.5, 1.0, 3, 2), (-0.5, 1.0, 3, 0), (-1.5, 1.0, 3, -2),   # ties go to even
    (0.49, 1.0, 3, 0), (0.51, 1.0, 3, 1), (7.0, 1.0, 3, 3), (-7.0, 1.0, 3, -3),                      # clamping
    (12.0, 0.125, 4, 2), (-20.0, 0.125, 4, -2), (3.0, 0.125, 4, 0), (4.0, 0.125, 4, 0), (4.1, 0.125, 4, 1),  # bins of 8 px
    (5.0, 1.0, 0, 0),                                                                                  # a single bin
])
def test_one_offset_at_a_time(offset, rate, R, want):
    coords = np.array([[[10.0, 20.0], [10.0 + offset, 20.0]]], dtype=np.float32)
    nbr = np.array([[[1], [0]]], dtype=np.int32)
    T = _index_table(1, R)
    bias = oracle.relpos_bias(coords, nbr, T, R, rate)
    assert bias[0, 0, 0, 0] == R * 100 + (want + R)          # neighbour to the right of the query by `offset`
    assert bias[0, 1, 0, 0] == R * 100 + (-want + R)         # and the mirror image
    # the same offset along y selects the row
    coords_y = coords[..., ::-1].copy()
    bias_y = oracle.relpos_bias(coords_y, nbr, T, R, rate)
    assert bias_y[0, 0, 0, 0] == (want + R) * 100 + R


def _numpy_bins(coords, nbr, R, rate):
    B, N, K = nbr.shape
    b = np.arange(B)[:, None, None]
    off = coords[b, nbr] - coords[:, :, None, :]                       # fp32, neighbour minus query
    t = (off * np.float32(rate)).astype(np.float32)
    return (np.clip(np.rint(t), -R, R).astype(np.int64) + R)           # [..., 0] = bx, [..., 1] = by


@pytest.mark.parametrize("seed,R,rate", [(0, 2, 0.5), (1, 7, 0.125), (2, 0, 1.0), (3, 5, 0.37)])
def test_against_numpy_indexing(seed, R, rate):
    rng = np.random.default_rng(seed)
    B, N, K, H = 2, 40, 9, 3
    coords = rng.uniform(0, 64, size=(B, N, 2)).astype(np.float32)
    if seed == 1:
        coords = np.round(coords / 4) * 4        # on a lattice: offsets sit exactly on bin edges and ties
    nbr = rng.integers(0, N, size=(B, N, K)).astype(np.int32)
    W = 2 * R + 1
    T = rng.normal(size=(H, W, W))
    bins = _numpy_bins(coords, nbr, R, rate)
    want = np.transpose(T[:, bins[..., 1], bins[..., 0]], (1, 2, 0, 3))        # [H,B,N,K] -> [B,N,H,K]
    assert np.array_equal(oracle.relpos_bias(coords, nbr, T, R, rate), want)
    # gradient of the table: a histogram of the bias gradients
    dbias = rng.normal(size=(B, N, H, K))
    want_dt = np.zeros((H, W, W))
    for h in range(H):
        np.add.at(want_dt[h], (bins[..., 1].ravel(), bins[..., 0].ravel()), dbias[:, :, h, :].ravel())
    got = oracle.relpos_dtable(coords, nbr, dbias, R, rate)
    assert np.allclose(got, want_dt, rtol=0, atol=1e-12)
    assert np.allclose(got.sum(axis=(1, 2)), dbias.sum(axis=(0, 1, 3)), rtol=0, atol=1e-10)   # nothing lost


def test_table_gradient_by_finite_differences():
    rng = np.random.default_rng(5)
    B, N, K, H, d, R, rate = 1, 24, 6, 2, 8, 2, 0.25
    coords = rng.uniform(0, 20, size=(B, N, 2)).astype(np.float32)
    nbr = np.stack([np.stack([rng.permutation(N)[:K] for _ in range(N)]) for _ in range(B)]).astype(np.int32)
    q, k, v, dout = (rng.normal(size=(B, N, H, d)) for _ in range(4))
    kb, vb = rng.normal(size=(H, d)), rng.normal(size=(H, d))
    W = 2 * R + 1
    T = rng.normal(size=(H, W, W))
    scale = 0.3
    g = oracle.pla_bwd_relpos(q, k, v, coords, T, nbr, dout, scale, R, rate, kb, vb)

    def loss(table):
        out, _ = oracle.pla_fwd_relpos(q, k, v, coords, table, nbr, scale, R, rate, kb, vb)
        return float((out * dout).sum())

    eps = 1e-6
    for h in range(H):
        for by in range(W):
            for bx in range(W):
                tp, tm = T.copy(), T.copy()
                tp[h, by, bx] += eps
                tm[h, by, bx] -= eps
                fd = (loss(tp) - loss(tm)) / (2 * eps)
                assert abs(fd - g["dtable"][h, by, bx]) <= 1e-6 * max(1.0, abs(fd)), (h, by, bx)
    # the other gradients are those of attention with the materialised bias
    ref = oracle.pla_bwd(q, k, v, oracle.relpos_bias(coords, nbr, T, R, rate), nbr, dout, scale, kb, vb)
    for name in ("dq", "dk", "dv", "dk_blank", "dv_blank"):
        assert np.array_equal(g[name], ref[name])
