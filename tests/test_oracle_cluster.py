"""Pins of the oracle's balanced clustering (Z-order curve, chunks of S): values fixed by the
definition of the curve, a second independent implementation, and invariants."""
import os

import numpy as np
import pytest

import oracle
from workloads.synth import morton_cluster_order

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_curve_visits_a_4x4_grid_in_z_order():
    cells = np.loadtxt(os.path.join(GOLDEN, "zorder_4x4.txt"), dtype=np.int64)  # curve order of (ix, iy)
    assert cells.shape == (16, 2)
    # tokens stored row by row (index = iy * 4 + ix), at the cell centres of the frame [0, 4)^2
    ix, iy = np.meshgrid(np.arange(4), np.arange(4), indexing="xy")
    coords = np.stack([ix.ravel() + 0.5, iy.ravel() + 0.5], axis=-1)[None].astype(np.float32)
    order, cid = oracle.cluster(coords, 4, (0.0, 0.0, 4.0, 4.0))
    want = cells[:, 1] * 4 + cells[:, 0]
    assert np.array_equal(order[0], want)
    # chunks of 4 along the curve are the four 2 x 2 blocks
    block = (iy.ravel() // 2) * 2 + (ix.ravel() // 2)
    assert np.array_equal(cid[0], block)


def test_coincident_points_keep_index_order_and_ragged_tail():
    coords = np.full((2, 11, 2), 7.25, dtype=np.float32)
    order, cid = oracle.cluster(coords, 4, (0.0, 0.0, 16.0, 16.0))
    assert np.array_equal(order, np.tile(np.arange(11), (2, 1)))
    assert np.array_equal(cid[0], np.arange(11) // 4)  # clusters of 4, 4, 3


def test_quadrants_come_in_z_order():
    """Whatever the points, everything in the lower-left quadrant of the frame precedes the lower-right
    quadrant, then upper-left, then upper-right (x owns the lower bit of every bit pair)."""
    rng = np.random.default_rng(3)
    coords = rng.uniform(0, 100, size=(3, 500, 2)).astype(np.float32)
    order, _ = oracle.cluster(coords, 16, (0.0, 0.0, 100.0, 100.0))
    for b in range(3):
        xy = coords[b][order[b]]
        quad = (xy[:, 1] >= 50).astype(int) * 2 + (xy[:, 0] >= 50).astype(int)
        assert np.all(np.diff(quad) >= 0)
        # and again inside the first quadrant
        sub = xy[quad == 0]
        q2 = (sub[:, 1] >= 25).astype(int) * 2 + (sub[:, 0] >= 25).astype(int)
        assert np.all(np.diff(q2) >= 0)


def test_matches_the_generator_ordering():
    """The workload generator orders tokens with its own numpy implementation of the same reading."""
    rng = np.random.default_rng(4)
    coords = rng.uniform(0, 1024, size=(2, 3000, 2)).astype(np.float32)
    coords[0, 100:140] = coords[0, 5]  # ties
    order, cid = oracle.cluster(coords, 64, (0.0, 0.0, 1024.0, 1024.0))
    assert np.array_equal(order, morton_cluster_order(coords, 1024.0).astype(np.int32))
    # cluster_id is the place along the curve divided by S
    place = np.empty_like(order)
    for b in range(2):
        place[b, order[b]] = np.arange(3000)
    assert np.array_equal(cid, place // 64)


def test_keys_do_not_decrease_along_the_curve_and_order_is_a_permutation():
    rng = np.random.default_rng(5)
    coords = rng.normal(30.0, 40.0, size=(1, 777, 2)).astype(np.float32)  # many points outside the frame
    x0, y0, w, h = -10.0, 5.0, 90.0, 60.0
    order, _ = oracle.cluster(coords, 10, (x0, y0, w, h))
    assert sorted(order[0].tolist()) == list(range(777))

    def key(x, y):  # bit by bit with python integers
        qx = min(max(int(np.floor((float(x) - x0) / w * 65536.0)), 0), 65535)
        qy = min(max(int(np.floor((float(y) - y0) / h * 65536.0)), 0), 65535)
        return int("".join(f"{(qy >> i) & 1}{(qx >> i) & 1}" for i in reversed(range(16))), 2)

    keys = [key(*coords[0, i]) for i in order[0]]
    assert all(a <= b for a, b in zip(keys, keys[1:]))
    for (ka, ia), (kb, ib) in zip(zip(keys, order[0]), zip(keys[1:], order[0][1:])):
        if ka == kb:
            assert ia < ib


def test_points_outside_the_frame_clamp_to_its_border_cells():
    coords = np.array([[[-5.0, -5.0], [1e9, 1e9], [0.25, 0.25], [-1.0, 0.9]]], dtype=np.float32)
    order, _ = oracle.cluster(coords, 2, (0.0, 0.0, 1.0, 1.0))
    # token 0 clamps to cell (0, 0): first; token 1 to (65535, 65535): last; token 2 lies in the lower-left
    # quadrant; token 3 clamps to x = 0 with y in the upper half: the upper-left quadrant, after token 2
    assert order[0].tolist() == [0, 2, 3, 1]


def test_bad_arguments_are_refused():
    coords = np.zeros((1, 4, 2), dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.cluster(coords, 2, (0.0, 0.0, 0.0, 1.0))
    with pytest.raises(RuntimeError):
        oracle.cluster(coords, 0, (0.0, 0.0, 1.0, 1.0))
