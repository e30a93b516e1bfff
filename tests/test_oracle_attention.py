"""Pins for the oracle's local attention, forward and backward (CPU only).

The forward is pinned to dense softmax attention restricted by a mask to the
neighbour set (library matmuls), to special cases with closed forms, and to the
invariants of softmax.  The backward is pinned to reverse-mode autodiff of that
dense form (torch, fp64), to central finite differences, and to identities the
gradients must satisfy.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import CONFIGS, make_features, make_workload, random_neighbours

SCALE = 1.0 / np.sqrt(32.0)


def _case(B=2, N=40, H=2, d=8, K=6, seed=0, blank=False, distinct=True):
    rng = np.random.default_rng(seed)
    f = make_features(B, N, H, d, K, "f32", rng, blank=blank)
    f = {k: v.astype(np.float64) for k, v in f.items()}
    f["nbr"] = random_neighbours(B, N, K, rng, distinct=distinct)
    return f


def _dense_masked_attention_torch(q, k, v, bias, nbr, scale, k_blank=None, v_blank=None):
    """softmax(scale * Q K^T + Bias + Mask) V over all N x N pairs per (b,h); Mask
    is -inf outside the neighbour set.  The blank token is one more column."""
    B, N, H, d = q.shape
    K = nbr.shape[2]
    logits = scale * torch.einsum("bihd,bjhd->bhij", q, k)
    mask = torch.full((B, H, N, N), float("-inf"), dtype=q.dtype)
    bi = torch.arange(B)[:, None, None].expand(B, N, K)
    ii = torch.arange(N)[None, :, None].expand(B, N, K)
    nn = torch.as_tensor(nbr, dtype=torch.long)
    dense_bias = torch.zeros((B, H, N, N), dtype=q.dtype)
    for h in range(H):
        mask[bi, h, ii, nn] = 0.0
        dense_bias = dense_bias.index_put((bi, torch.full_like(bi, h), ii, nn), bias[:, :, h, :])
    logits = logits + dense_bias + mask
    vals = v.permute(0, 2, 1, 3)  # [B,H,N,d]
    if k_blank is not None:
        blank_logit = scale * torch.einsum("bihd,hd->bhi", q, k_blank)[..., None]
        logits = torch.cat([logits, blank_logit], dim=-1)
        vals = torch.cat([vals, v_blank[None, :, None, :].expand(B, H, 1, d)], dim=2)
    lse = torch.logsumexp(logits, dim=-1)
    p = torch.softmax(logits, dim=-1)
    out = torch.einsum("bhij,bhjd->bihd", p, vals)
    return out, lse.permute(0, 2, 1)


def _t(x, grad=False):
    return torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=grad)


@pytest.mark.parametrize("blank", [False, True])
def test_forward_equals_dense_masked_softmax_attention(blank):
    c = _case(blank=blank, seed=3)
    out, lse = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE,
                              c.get("k_blank"), c.get("v_blank"))
    kb = _t(c["k_blank"]) if blank else None
    vb = _t(c["v_blank"]) if blank else None
    want, want_lse = _dense_masked_attention_torch(_t(c["q"]), _t(c["k"]), _t(c["v"]), _t(c["bias"]),
                                                   c["nbr"], SCALE, kb, vb)
    np.testing.assert_allclose(out, want.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse.numpy(), rtol=0, atol=1e-12)


def test_forward_on_knn_neighbourhoods_equals_dense_form():
    """Same pin on a real (small) clustered token set with kNN tables."""
    cfg = CONFIGS["merged_stage"].scaled(B=2, N=128, C=32, H=4, K=12, S=16, M=4)
    w = make_workload(cfg)
    nbr, _ = oracle.knn(w["coords"], w["cluster_id"], cfg.S, cfg.M, cfg.K)
    scale = 1.0 / np.sqrt(cfg.d)
    out, lse = oracle.pla_fwd(w["q"], w["k"], w["v"], w["bias"], nbr, scale)
    want, want_lse = _dense_masked_attention_torch(_t(w["q"]), _t(w["k"]), _t(w["v"]), _t(w["bias"]), nbr, scale)
    np.testing.assert_allclose(out, want.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("blank", [False, True])
def test_backward_equals_autodiff_of_dense_form(blank):
    c = _case(blank=blank, seed=5)
    q, k, v, bias = (_t(c[n], True) for n in ("q", "k", "v", "bias"))
    kb = _t(c["k_blank"], True) if blank else None
    vb = _t(c["v_blank"], True) if blank else None
    out, _ = _dense_masked_attention_torch(q, k, v, bias, c["nbr"], SCALE, kb, vb)
    (out * _t(c["dout"])).sum().backward()
    g = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE,
                       c.get("k_blank"), c.get("v_blank"))
    np.testing.assert_allclose(g["dq"], q.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(g["dk"], k.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(g["dv"], v.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(g["dbias"], bias.grad.numpy(), rtol=0, atol=1e-12)
    if blank:
        np.testing.assert_allclose(g["dk_blank"], kb.grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(g["dv_blank"], vb.grad.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("blank", [False, True])
def test_backward_matches_central_finite_differences(blank):
    c = _case(B=1, N=12, H=2, d=4, K=5, seed=7, blank=blank, distinct=False)  # repeats allowed
    names = ["q", "k", "v", "bias"] + (["k_blank", "v_blank"] if blank else [])
    gname = {"q": "dq", "k": "dk", "v": "dv", "bias": "dbias", "k_blank": "dk_blank", "v_blank": "dv_blank"}

    def loss(x):
        out, _ = oracle.pla_fwd(x["q"], x["k"], x["v"], x["bias"], c["nbr"], SCALE,
                                x.get("k_blank"), x.get("v_blank"))
        return float((out * c["dout"]).sum())

    g = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE,
                       c.get("k_blank"), c.get("v_blank"))
    eps = 1e-5
    for n in names:
        flat_g = g[gname[n]].ravel()
        fd = np.empty_like(flat_g)
        for e in range(flat_g.size):
            xp = {m: c[m].copy() for m in names}
            xm = {m: c[m].copy() for m in names}
            xp[n].ravel()[e] += eps
            xm[n].ravel()[e] -= eps
            fd[e] = (loss(xp) - loss(xm)) / (2 * eps)
        err = np.abs(fd - flat_g).max() / max(np.abs(flat_g).max(), 1e-30)
        assert err < 1e-6, (n, err)


def test_probabilities_sum_to_one_and_identities():
    c = _case(seed=9)
    out, lse, prob = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE, want_prob=True)
    np.testing.assert_allclose(prob.sum(-1), 1.0, atol=1e-14)
    assert np.all(prob[..., -1] == 0.0)  # no blank column
    g = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE)
    # softmax rows sum to one => bias gradients of a row sum to zero
    np.testing.assert_allclose(g["dbias"].sum(axis=3), 0.0, atol=1e-13)
    # every probability row sums to one => the v-gradient conserves dout per head
    np.testing.assert_allclose(g["dv"].sum(axis=1), c["dout"].sum(axis=1), atol=1e-11)


def test_single_neighbour_copies_value_row():
    c = _case(K=1, seed=1)
    out, lse = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE)
    B, N = c["nbr"].shape[:2]
    want = np.stack([c["v"][b, c["nbr"][b, :, 0]] for b in range(B)])
    np.testing.assert_allclose(out, want, atol=1e-15)
    # lse of a single logit is the logit itself
    s = SCALE * np.einsum("bihd,bihd->bih", c["q"], np.stack([c["k"][b, c["nbr"][b, :, 0]] for b in range(B)]))
    np.testing.assert_allclose(lse, s + c["bias"][:, :, :, 0], atol=1e-13)


def test_zero_query_zero_bias_gives_mean_of_value_rows():
    c = _case(seed=2)
    out, lse = oracle.pla_fwd(np.zeros_like(c["q"]), c["k"], c["v"], None, c["nbr"], SCALE)
    B, N, K = c["nbr"].shape
    want = np.stack([c["v"][b, c["nbr"][b]].mean(axis=1) for b in range(B)])
    np.testing.assert_allclose(out, want, atol=1e-14)
    np.testing.assert_allclose(lse, np.log(K), atol=1e-14)


def test_row_shift_of_bias_changes_nothing_but_lse():
    """softmax(z) = softmax(z - const): the max-subtraction identity."""
    c = _case(seed=4)
    shift = np.random.default_rng(0).normal(size=(2, 40, 2, 1)) * 3.0
    o1, l1 = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE)
    o2, l2 = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"] + shift, c["nbr"], SCALE)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l2 - l1, shift[:, :, :, 0], atol=1e-13)
    g1 = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE)
    g2 = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"] + shift, c["nbr"], c["dout"], SCALE)
    for n in g1:
        np.testing.assert_allclose(g1[n], g2[n], atol=1e-12)


def test_permuting_neighbour_order_permutes_only_dbias():
    c = _case(seed=6)
    rng = np.random.default_rng(1)
    B, N, K = c["nbr"].shape
    perm = np.stack([[rng.permutation(K) for _ in range(N)] for _ in range(B)])
    nbr2 = np.take_along_axis(c["nbr"], perm, axis=2)
    bias2 = np.take_along_axis(c["bias"], perm[:, :, None, :], axis=3)
    o1, l1 = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE)
    o2, l2 = oracle.pla_fwd(c["q"], c["k"], c["v"], bias2, nbr2, SCALE)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l1, l2, atol=1e-13)
    g1 = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE)
    g2 = oracle.pla_bwd(c["q"], c["k"], c["v"], bias2, nbr2, c["dout"], SCALE)
    for n in ("dq", "dk", "dv"):
        np.testing.assert_allclose(g1[n], g2[n], atol=1e-12)
    np.testing.assert_allclose(np.take_along_axis(g1["dbias"], perm[:, :, None, :], axis=3), g2["dbias"], atol=1e-13)


def test_blank_token_is_one_more_shared_neighbour():
    """Appending the blank row to every image as token N and listing it as a
    (K+1)-th neighbour with zero bias must give the same numbers."""
    c = _case(seed=8, blank=True)
    B, N, H, d = c["q"].shape
    K = c["nbr"].shape[2]

    def ext(x, row):
        return np.concatenate([x, np.broadcast_to(row[None, None], (B, 1, H, d))], axis=1)

    q2 = ext(c["q"], np.zeros((H, d)))
    k2 = ext(c["k"], c["k_blank"])
    v2 = ext(c["v"], c["v_blank"])
    dout2 = ext(c["dout"], np.zeros((H, d)))  # the extra token's own output carries no loss
    nbr2 = np.concatenate([np.concatenate([c["nbr"], np.full((B, N, 1), N, np.int32)], axis=2),
                           np.full((B, 1, K + 1), N, np.int32)], axis=1)
    bias2 = np.zeros((B, N + 1, H, K + 1))
    bias2[:, :N, :, :K] = c["bias"]
    o1, l1 = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], SCALE, c["k_blank"], c["v_blank"])
    o2, l2 = oracle.pla_fwd(q2, k2, v2, bias2, nbr2, SCALE)
    np.testing.assert_allclose(o1, o2[:, :N], atol=1e-13)
    np.testing.assert_allclose(l1, l2[:, :N], atol=1e-13)
    g1 = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], c["nbr"], c["dout"], SCALE, c["k_blank"], c["v_blank"])
    g2 = oracle.pla_bwd(q2, k2, v2, bias2, nbr2, dout2, SCALE)
    for n in ("dq", "dk", "dv"):
        np.testing.assert_allclose(g1[n], g2[n][:, :N], atol=1e-12)
    np.testing.assert_allclose(g1["dbias"], g2["dbias"][:, :N, :, :K], atol=1e-13)
    # with q = 0 and dout = 0 for the extra token, its row collects exactly the blank gradients
    np.testing.assert_allclose(g1["dk_blank"], g2["dk"][:, N].sum(axis=0), atol=1e-12)
    np.testing.assert_allclose(g1["dv_blank"], g2["dv"][:, N].sum(axis=0), atol=1e-12)


def test_repeated_neighbour_is_a_cloned_row():
    """A neighbour listed twice acts like two identical rows, each with its own
    bias entry; its gradient is the sum over the clones."""
    c = _case(B=1, N=10, H=1, d=4, K=4, seed=10)
    nbr = c["nbr"].copy()
    nbr[0, :, 3] = nbr[0, :, 0]          # slot 3 repeats slot 0
    N = 10
    # clone set: token N+i is a copy of token nbr[i,0]
    src = nbr[0, :, 0]
    k2 = np.concatenate([c["k"], c["k"][:, src]], axis=1)
    v2 = np.concatenate([c["v"], c["v"][:, src]], axis=1)
    q2 = np.concatenate([c["q"], np.zeros_like(c["q"])], axis=1)
    dout2 = np.concatenate([c["dout"], np.zeros_like(c["dout"])], axis=1)
    nbr2 = np.zeros((1, 2 * N, 4), np.int32)
    nbr2[0, :N] = nbr[0]
    nbr2[0, :N, 3] = N + np.arange(N)
    bias2 = np.concatenate([c["bias"], np.zeros_like(c["bias"])], axis=1)
    o1, _ = oracle.pla_fwd(c["q"], c["k"], c["v"], c["bias"], nbr, SCALE)
    o2, _ = oracle.pla_fwd(q2, k2, v2, bias2, nbr2, SCALE)
    np.testing.assert_allclose(o1, o2[:, :N], atol=1e-14)
    g1 = oracle.pla_bwd(c["q"], c["k"], c["v"], c["bias"], nbr, c["dout"], SCALE)
    g2 = oracle.pla_bwd(q2, k2, v2, bias2, nbr2, dout2, SCALE)
    fold_k = g2["dk"][:, :N].copy()
    fold_v = g2["dv"][:, :N].copy()
    for i in range(N):
        fold_k[0, src[i]] += g2["dk"][0, N + i]
        fold_v[0, src[i]] += g2["dv"][0, N + i]
    np.testing.assert_allclose(g1["dk"], fold_k, atol=1e-13)
    np.testing.assert_allclose(g1["dv"], fold_v, atol=1e-13)
    np.testing.assert_allclose(g1["dbias"], g2["dbias"][:, :N], atol=1e-14)
