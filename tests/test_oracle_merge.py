"""Pins of the merging oracle (oracle_merge_select / _fwd / _bwd) against things other than itself: a hand-derived
fixture, a library sort, library gather / softmax / autograd in fp64, central finite differences, and the
identities that the definition implies."""
import os

import numpy as np
import pytest
import torch

import oracle


def _read(path):
    rows = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, vals = line.split(":")
        rows[tuple(head.split())] = [float(v) for v in vals.split()]
    return rows


def test_hand_derived_six_tokens(golden_dir):
    rows = _read(os.path.join(golden_dir, "merge_6tokens.txt"))
    score = np.array([rows[("score",)]], dtype=np.float32)
    for n_keep in range(1, 7):
        assert oracle.merge_select(score, n_keep)[0].tolist() == [int(v) for v in rows[("keep", str(n_keep))]]
    coords = np.stack([np.arange(6), np.zeros(6)], -1).astype(np.float32)[None]
    ln2 = np.log(2.0)
    sc = np.array([[ln2, 2 * ln2, ln2, 0.0, 0.0, 0.0]], dtype=np.float32)
    nbr = np.array([[[0, 1], [1, 2], [2, 2], [3, 1], [4, 4], [5, 5]]], dtype=np.int32)
    feat = np.array([[[2, 2], [10, 0], [0, 5], [4, 6], [0, 0], [0, 0]]], dtype=np.float64)
    anchors = np.array([[0, 1, 3]], dtype=np.int32)
    out, w = oracle.merge_fwd(coords, feat, sc, nbr, anchors, float(np.float32(ln2)), want_weights=True)
    for a, t in enumerate((0, 1, 3)):
        assert np.allclose(w[0, a], rows[("weights", str(t))], atol=1e-7)     # fp32 scores: ln 2 is rounded
        assert np.allclose(out[0, a], rows[("out", str(t))], atol=1e-6)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_selection_equals_library_sort(seed):
    rng = np.random.default_rng(seed)
    B, N = 3, 500
    # few distinct values: ties everywhere, both zeros among them
    score = rng.choice(np.array([-1.5, -0.0, 0.0, 0.25, 3.0], dtype=np.float32), size=(B, N))
    for n_keep in (1, 37, 250, 499, 500):
        got = oracle.merge_select(score, n_keep)
        for b in range(B):
            order = np.lexsort((np.arange(N), -score[b].astype(np.float64)))   # score descending, then index
            assert got[b].tolist() == sorted(order[:n_keep].tolist())


def _case(seed, B=2, N=40, C=5, K=7, n_keep=11):
    rng = np.random.default_rng(seed)
    coords = rng.uniform(0, 10, size=(B, N, 2)).astype(np.float32)
    feat = rng.normal(size=(B, N, C))
    score = rng.normal(size=(B, N)).astype(np.float32)
    nbr = np.stack([np.stack([rng.permutation(N)[:K] for _ in range(N)]) for _ in range(B)]).astype(np.int32)
    nbr[:, :, 0] = np.arange(N)          # the token itself leads its neighbourhood, as in a kNN table
    nbr[:, 3, 2] = nbr[:, 3, 1]          # a repeated neighbour
    anchors = oracle.merge_select(score, n_keep)
    dout = rng.normal(size=(B, n_keep, C))
    return coords, feat, score, nbr, anchors, dout


def _torch_merge(coords, feat, score, nbr, anchors, p):
    """The same quantity from library routines: index arithmetic, gather, softmax (all fp64)."""
    B, N, C = feat.shape
    idx = torch.from_numpy(nbr.astype(np.int64))
    anc = torch.from_numpy(anchors.astype(np.int64))
    xy = torch.from_numpy(coords.astype(np.float64))
    rows = torch.gather(idx, 1, anc[:, :, None].expand(-1, -1, idx.shape[2]))            # [B,A,K]
    ax = torch.gather(xy, 1, anc[:, :, None].expand(-1, -1, 2))                            # [B,A,2]
    nx = torch.gather(xy, 1, rows.reshape(B, -1, 1).expand(-1, -1, 2)).reshape(*rows.shape, 2)
    dist = (nx - ax[:, :, None, :]).norm(dim=-1)
    z = torch.gather(score, 1, rows.reshape(B, -1)).reshape(rows.shape) - p * dist
    w = torch.softmax(z, dim=-1)
    f = torch.gather(feat, 1, rows.reshape(B, -1, 1).expand(-1, -1, C)).reshape(*rows.shape, C)
    return (w[..., None] * f).sum(dim=2), w


@pytest.mark.parametrize("seed", [0, 1])
def test_forward_and_backward_equal_library_autograd(seed):
    coords, feat, score, nbr, anchors, dout = _case(seed)
    p = 0.7
    tf = torch.from_numpy(feat).requires_grad_(True)
    ts = torch.from_numpy(score.astype(np.float64)).requires_grad_(True)
    tp = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    out_t, w_t = _torch_merge(coords, tf, ts, nbr, anchors, tp)
    out, w = oracle.merge_fwd(coords, feat, score, nbr, anchors, p, want_weights=True)
    assert np.allclose(out, out_t.detach().numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(w, w_t.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(w.sum(-1), 1.0, atol=1e-14)
    (out_t * torch.from_numpy(dout)).sum().backward()
    g = oracle.merge_bwd(coords, feat, score, nbr, anchors, dout, p)
    assert np.allclose(g["dfeat"], tf.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(g["dscore"], ts.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.isclose(g["dp"], float(tp.grad), rtol=1e-10, atol=1e-12)
    assert g["dp_abs"] >= abs(g["dp"])


def test_backward_equals_central_differences():
    coords, feat, score, nbr, anchors, dout = _case(5, B=1, N=12, C=3, K=4, n_keep=5)
    p, h = 0.9, 1e-6
    score64 = score.astype(np.float64)

    def loss(f=feat, s=score64, pp=p):
        out, _ = _torch_merge(coords, torch.from_numpy(f), torch.from_numpy(s), nbr, anchors, pp)
        return float((out.numpy() * dout).sum())

    g = oracle.merge_bwd(coords, feat, score, nbr, anchors, dout, p)
    rng = np.random.default_rng(0)
    for _ in range(12):
        i, c = int(rng.integers(12)), int(rng.integers(3))
        fp, fm = feat.copy(), feat.copy()
        fp[0, i, c] += h; fm[0, i, c] -= h
        assert np.isclose((loss(f=fp) - loss(f=fm)) / (2 * h), g["dfeat"][0, i, c], rtol=1e-6, atol=1e-8)
    for i in range(12):
        sp, sm = score64.copy(), score64.copy()
        sp[0, i] += h; sm[0, i] -= h
        assert np.isclose((loss(s=sp) - loss(s=sm)) / (2 * h), g["dscore"][0, i], rtol=1e-6, atol=1e-8)
    assert np.isclose((loss(pp=p + h) - loss(pp=p - h)) / (2 * h), g["dp"], rtol=1e-6, atol=1e-8)


def test_identities():
    coords, feat, score, nbr, anchors, dout = _case(9)
    B, N, C = feat.shape
    g = oracle.merge_bwd(coords, feat, score, nbr, anchors, dout, 0.4)
    # the weights of an anchor sum to 1: the score gradients of its neighbourhood cancel, and every unit of dout
    # arrives somewhere in dfeat
    assert np.allclose(g["dscore"].sum(axis=1), 0.0, atol=1e-12)
    assert np.allclose(g["dfeat"].sum(axis=1), dout.sum(axis=1), atol=1e-12)
    # equal features everywhere: the merged feature is that feature, whatever the weights
    same = np.broadcast_to(feat[:, :1], feat.shape).copy()
    out = oracle.merge_fwd(coords, same, score, nbr, anchors, 0.4)
    assert np.allclose(out, same[:, : anchors.shape[1]], atol=1e-12)
    # p = 0 and equal scores: the plain mean of the neighbourhood
    flat = np.zeros_like(score)
    out = oracle.merge_fwd(coords, feat, flat, nbr, anchors, 0.0)
    for b in range(B):
        want = feat[b][nbr[b][anchors[b]]].mean(axis=1)
        assert np.allclose(out[b], want, atol=1e-12)
    # a very large p: only the neighbours at distance 0 (the anchor itself) count
    nbr2 = nbr.copy()
    nbr2[:, 3, 2] = (nbr2[:, 3, 0] + 1) % N   # undo the repeated neighbour of the fixture
    out = oracle.merge_fwd(coords, feat, flat, nbr2, anchors, 1e6)
    for b in range(B):
        assert np.allclose(out[b], feat[b][anchors[b]], atol=1e-9)
    # adding a constant to every score changes nothing (softmax), and n_keep = N keeps every token in order
    out_a = oracle.merge_fwd(coords, feat, score, nbr, anchors, 0.4)
    out_b = oracle.merge_fwd(coords, feat, score + np.float32(2.0), nbr, anchors, 0.4)
    assert np.allclose(out_a, out_b, atol=1e-6)   # fp32 scores: the shifted ones are rounded again
    assert np.array_equal(oracle.merge_select(score, N), np.broadcast_to(np.arange(N), (B, N)))


def test_argument_errors():
    score = np.zeros((1, 8), dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.merge_select(score, 0)
    with pytest.raises(RuntimeError):
        oracle.merge_select(score, 9)
    bad = score.copy(); bad[0, 3] = np.nan
    with pytest.raises(RuntimeError):
        oracle.merge_select(bad, 2)
