"""Pins of the oracle's virtual sampled tokens (point decoder): hand-derived tables and weights, a second
formulation built from library routines (torch gather / softmax / autograd), finite differences."""
import numpy as np
import pytest
import torch

import oracle


def _lattice(n, cell):
    ix, iy = np.meshgrid(np.arange(n), np.arange(n), indexing="xy")
    return np.stack([(ix.ravel() + 0.5) * cell, (iy.ravel() + 0.5) * cell], axis=-1)[None].astype(np.float32)


def test_table_on_a_fully_visible_lattice():
    """Every patch centre is a visible token (index = iy * n + ix): a grid point's nearest token is itself,
    then its four lattice neighbours at one cell's distance, lower index first."""
    n, cell = 6, 8.0
    table = oracle.vts_table(_lattice(n, cell), (n, n, 0.0, 0.0, cell), 5)
    assert table.shape == (1, n, n, 5)
    for iy in range(1, n - 1):
        for ix in range(1, n - 1):
            me = iy * n + ix
            assert table[0, iy, ix].tolist() == [me, me - n, me - 1, me + 1, me + n]
    # a corner has only two such neighbours; the next ring is the diagonal one
    assert table[0, 0, 0, :3].tolist() == [0, 1, n]
    assert table[0, 0, 0, 3] == n + 1


def test_table_matches_exhaustive_search_on_tiny_inputs():
    rng = np.random.default_rng(1)
    vis = rng.uniform(0, 32, size=(2, 9, 2)).astype(np.float32)
    vis[1, 4] = vis[1, 2]  # coincident tokens: lower index first
    Hg, Wg, x0, y0, cell = 3, 5, 1.5, -2.0, 7.0
    table = oracle.vts_table(vis, (Hg, Wg, x0, y0, cell), 4)
    for b in range(2):
        for iy in range(Hg):
            for ix in range(Wg):
                gx = np.float32(x0) + np.float32(ix + 0.5) * np.float32(cell)
                gy = np.float32(y0) + np.float32(iy + 0.5) * np.float32(cell)
                keyed = []
                for i in range(9):
                    dx, dy = np.float32(gx - vis[b, i, 0]), np.float32(gy - vis[b, i, 1])
                    keyed.append((float(np.float32(np.float32(dx * dx) + np.float32(dy * dy))), i))
                assert table[b, iy, ix].tolist() == [i for _, i in sorted(keyed)[:4]]


def test_query_cell_and_clamping():
    """A table whose entry for cell c is [c] and features feat[i] = i make the output name the cell used."""
    Hg, Wg, cell, x0, y0 = 3, 4, 2.0, 10.0, 20.0
    table = np.arange(Hg * Wg, dtype=np.int32).reshape(1, Hg, Wg, 1)
    vis = np.zeros((1, Hg * Wg, 2), dtype=np.float32)
    feat = np.arange(Hg * Wg, dtype=np.float64).reshape(1, Hg * Wg, 1)
    q = np.array([[[10.0, 20.0], [11.99, 20.0], [12.0, 20.0], [17.9, 25.9], [-5.0, 21.0], [100.0, 100.0],
                   [13.0, 23.0]]], dtype=np.float32)
    out = oracle.vts_fwd(q, vis, feat, table, (Hg, Wg, x0, y0, cell), 1.0, 1e-6)
    #            cell (0,0)  (0,0)   (1,0)  (3,2)        (0,0) clamp x  (3,2) clamp   (1,1)
    assert out[0, :, 0].tolist() == [0.0, 0.0, 1.0, 11.0, 0.0, 11.0, 5.0]


def test_equidistant_tokens_get_equal_weights_and_special_values_of_p():
    vis = np.array([[[0.0, 0.0], [2.0, 0.0], [0.0, 2.0], [2.0, 2.0], [9.0, 9.0]]], dtype=np.float32)
    feat = np.random.default_rng(2).normal(size=(1, 5, 3))
    table = np.array([0, 1, 2, 3], dtype=np.int32).reshape(1, 1, 1, 4)
    grid = (1, 1, 0.0, 0.0, 2.0)
    q = np.array([[[1.0, 1.0]]], dtype=np.float32)
    out, w = oracle.vts_fwd(q, vis, feat, table, grid, 3.0, 1e-6, want_weights=True)
    assert np.allclose(w, 0.25, atol=1e-15) and np.allclose(out[0, 0], feat[0, :4].mean(0), atol=1e-15)
    # p = 0: plain mean whatever the distances; large p: the nearest token alone
    q2 = np.array([[[0.25, 0.5]]], dtype=np.float32)
    out0 = oracle.vts_fwd(q2, vis, feat, table, grid, 0.0, 1e-6)
    assert np.allclose(out0[0, 0], feat[0, :4].mean(0), atol=1e-15)
    outbig = oracle.vts_fwd(q2, vis, feat, table, grid, 500.0, 1e-6)
    assert np.allclose(outbig[0, 0], feat[0, 0], atol=1e-12)
    # a single candidate: a copy
    t1 = np.array([3], dtype=np.int32).reshape(1, 1, 1, 1)
    assert np.array_equal(oracle.vts_fwd(q2, vis, feat, t1, grid, 2.0, 1e-6)[0, 0], feat[0, 3])
    # two candidates at distances 1 and 3 with p = ln 2 / 2: weights 2/3 and 1/3 (ratio exp(p * 2) = 2)
    vis2 = np.array([[[1.0, 0.0], [0.0, 3.0]]], dtype=np.float32)
    t2 = np.array([0, 1], dtype=np.int32).reshape(1, 1, 1, 2)
    q3 = np.zeros((1, 1, 2), dtype=np.float32)
    _, w2 = oracle.vts_fwd(q3, vis2, np.zeros((1, 2, 1)), t2, (1, 1, -1.0, -1.0, 8.0), np.log(2.0) / 2, 0.0,
                           want_weights=True)
    assert np.allclose(w2[0, 0], [2 / 3, 1 / 3], atol=1e-15)


def _torch_form(q, vis, feat, table, grid, p, eps):
    """The same quantities from library routines: index arithmetic, gather, softmax."""
    Hg, Wg, x0, y0, cell = grid
    B, Mq, _ = q.shape
    qd = q.detach()
    ix = torch.clamp(torch.floor((qd[..., 0].float() - np.float32(x0)) / np.float32(cell)), 0, Wg - 1).long()
    iy = torch.clamp(torch.floor((qd[..., 1].float() - np.float32(y0)) / np.float32(cell)), 0, Hg - 1).long()
    rows = table[torch.arange(B)[:, None], iy, ix].long()                      # [B,Mq,Kt]
    xs = vis[torch.arange(B)[:, None, None], rows]                             # [B,Mq,Kt,2]
    d = torch.linalg.vector_norm(q[:, :, None, :] - xs, dim=-1) + eps
    w = torch.softmax(-p * d, dim=-1)
    f = feat[torch.arange(B)[:, None, None], rows]                             # [B,Mq,Kt,C]
    return torch.einsum("bmk,bmkc->bmc", w, f), w


@pytest.fixture
def problem():
    rng = np.random.default_rng(7)
    B, Nv, Mq, C, Kt = 2, 40, 33, 5, 4
    grid = (8, 8, 0.0, 0.0, 8.0)
    vis = rng.uniform(0, 64, size=(B, Nv, 2)).astype(np.float32)
    q = rng.uniform(-4, 68, size=(B, Mq, 2)).astype(np.float32)
    feat = rng.normal(size=(B, Nv, C))
    dout = rng.normal(size=(B, Mq, C))
    table = oracle.vts_table(vis, grid, Kt)
    return q, vis, feat, dout, table, grid


def test_forward_and_backward_match_the_library_formulation(problem):
    q, vis, feat, dout, table, grid = problem
    p, eps = 0.7, 1e-6
    out, w = oracle.vts_fwd(q, vis, feat, table, grid, p, eps, want_weights=True)
    g = oracle.vts_bwd(q, vis, feat, table, dout, grid, p, eps)
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tf = torch.tensor(feat, requires_grad=True)
    tp = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    tout, tw = _torch_form(tq, torch.tensor(vis, dtype=torch.float64), tf, torch.tensor(table), grid, tp, eps)
    assert np.allclose(out, tout.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(w, tw.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(w.sum(-1), 1.0, atol=1e-14)
    (tout * torch.tensor(dout)).sum().backward()
    assert np.allclose(g["dfeat"], tf.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(g["dquery"], tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.isclose(g["dp"], float(tp.grad), rtol=1e-10, atol=1e-12)


def test_backward_matches_finite_differences(problem):
    q, vis, feat, dout, table, grid = problem
    p, eps = 0.4, 1e-6
    g = oracle.vts_bwd(q, vis, feat, table, dout, grid, p, eps)

    def loss(qq=q, ff=feat, pp=p):
        return float((oracle.vts_fwd(qq, vis, ff, table, grid, pp, eps) * dout).sum())

    h = 1e-5
    assert np.isclose((loss(pp=p + h) - loss(pp=p - h)) / (2 * h), g["dp"], rtol=1e-6, atol=1e-8)
    rng = np.random.default_rng(8)
    for _ in range(6):
        b, i, c = rng.integers(2), rng.integers(40), rng.integers(5)
        fp, fm = feat.copy(), feat.copy()
        fp[b, i, c] += h
        fm[b, i, c] -= h
        assert np.isclose((loss(ff=fp) - loss(ff=fm)) / (2 * h), g["dfeat"][b, i, c], rtol=1e-6, atol=1e-8)
    # query coordinates are fp32 and decide the cell: step with exactly representable offsets inside the cell
    hq = np.float32(2.0 ** -7)
    for _ in range(6):
        b, m, a = rng.integers(2), rng.integers(33), rng.integers(2)
        base = q.copy()
        base[b, m, a] = np.float32(np.floor(base[b, m, a] / 8.0) * 8.0 + 3.0)  # well inside its cell
        gb = oracle.vts_bwd(base, vis, feat, table, dout, grid, p, eps)
        qp, qm = base.copy(), base.copy()
        qp[b, m, a] += hq
        qm[b, m, a] -= hq
        fd = (loss(qq=qp) - loss(qq=qm)) / (2 * float(hq))
        assert np.isclose(fd, gb["dquery"][b, m, a], rtol=2e-4, atol=1e-7)


def test_query_on_a_token_has_zero_direction_term():
    vis = np.array([[[1.0, 1.0], [3.0, 1.0]]], dtype=np.float32)
    table = np.array([0, 1], dtype=np.int32).reshape(1, 1, 1, 2)
    q = np.array([[[1.0, 1.0]]], dtype=np.float32)
    feat = np.array([[[1.0], [2.0]]])
    g = oracle.vts_bwd(q, vis, feat, table, np.ones((1, 1, 1)), (1, 1, 0.0, 0.0, 4.0), 1.0, 1e-6)
    assert np.all(np.isfinite(g["dquery"]))
    # only the second token pulls: dz_1 * (-p) * (q - x_1)/|q - x_1| with (q - x_1) = (-2, 0)
    assert g["dquery"][0, 0, 1] == 0.0 and g["dquery"][0, 0, 0] > 0.0
