"""GPU parity: affmae_merge_select / affmae_merge_fwd / affmae_merge_bwd against the CPU oracle.  Anchor indices
bit-exact; floats at max|gpu - ref| / max|ref| <= 1e-5 (fp32 storage) and 2e-2 (bf16 storage); dp, one scalar, is
judged against the sum of the absolute per-anchor contributions (returned by the oracle)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_16249_amd as aff
from workloads import CONFIGS, bf16_round, make_workload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.mark.parametrize("B,N,n_keep,kind", [
    (3, 1000, 250, "normal"), (2, 16384, 4096, "normal"), (2, 5000, 1, "ties"), (4, 777, 777, "ties"),
    (2, 4096, 1638, "ties"), (1, 100000, 40000, "ties"), (2, 64, 33, "equal"), (1, 2049, 1024, "normal"),
    # each size class of the selection: keys in registers (4, 16, 32 per thread), sizes that are not whole pieces
    (2, 4097, 1000, "ties"), (2, 16383, 16383, "normal"), (2, 20000, 5000, "ties"), (1, 32768, 1, "normal"),
    (1, 32769, 8192, "ties"), (3, 5, 5, "equal"), (2, 16384, 16384, "equal"),
])
def test_select_matches_oracle(B, N, n_keep, kind):
    print(f"case select B={B} N={N} n_keep={n_keep} {kind}", flush=True)
    rng = np.random.default_rng(N + n_keep)
    if kind == "normal":
        score = rng.normal(size=(B, N)).astype(np.float32)
    elif kind == "ties":  # few distinct values, both zeros, extremes of the fp32 range
        score = rng.choice(np.array([-3e38, -1.5, -0.0, 0.0, 1e-45, 0.25, 3.0, 3e38], dtype=np.float32), size=(B, N))
    else:
        score = np.full((B, N), 0.75, dtype=np.float32)
    coords = rng.uniform(0, 100, size=(B, N, 2)).astype(np.float32)
    idx, xy = aff.affmae_merge_select(torch.from_numpy(score).cuda(), n_keep, torch.from_numpy(coords).cuda())
    torch.cuda.synchronize()
    ref = oracle.merge_select(score, n_keep)
    assert np.array_equal(idx.cpu().numpy(), ref)
    assert np.array_equal(xy.cpu().numpy(), np.take_along_axis(coords, ref[..., None].astype(np.int64), axis=1))


CASES = [
    # dtype, B, N, C, K, S, M, n_keep, p
    ("f32", 2, 512, 64, 16, 32, 4, 128, 0.5),
    ("f32", 1, 256, 20, 7, 32, 2, 100, 1.3),      # rows of whole pieces (5), K odd
    ("f32", 2, 256, 6, 5, 16, 4, 64, 0.0),        # rows that are not whole 16-byte pieces: lanes are channels
    ("bf16", 2, 1024, 64, 48, 64, 8, 256, 0.25),  # the stage-1 shape: 8 pieces per row, 8 rows per trip
    ("bf16", 2, 512, 256, 48, 32, 8, 205, 0.7),   # 32 pieces per row
    ("bf16", 1, 512, 1032, 33, 64, 4, 77, 0.1),   # more than 64 pieces per row: several trips over the pieces
    ("bf16", 3, 300, 6, 64, 50, 6, 299, 2.0),     # K at the limit, odd rows, nearly every token an anchor
    ("bf16", 1, 128, 8, 1, 16, 2, 64, 1.0),       # K = 1: the merged token is the anchor itself
    ("f32", 2, 512, 64, 16, 32, 4, 128, 3.0),     # weights close to saturated on the anchor itself: gradients are small differences
    ("f32", 1, 256, 32, 12, 32, 2, 64, 8.0),
]


@pytest.mark.parametrize("dtype,B,N,C,K,S,M,n_keep,p", CASES)
def test_merge_forward_backward_match_oracle(dtype, B, N, C, K, S, M, n_keep, p):
    print(f"case merge {dtype} B={B} N={N} C={C} K={K} n_keep={n_keep} p={p}", flush=True)
    cfg = CONFIGS["knn_scale"].scaled(B=B, N=N, S=S, M=M, K=K)
    w = make_workload(cfg, features=False)
    coords = w["coords"]
    nbr, _ = oracle.knn(coords, None, S, M, K)
    rng = np.random.default_rng(N + C + K)
    feat = rng.normal(size=(B, N, C)).astype(np.float32)
    dout = rng.normal(size=(B, n_keep, C)).astype(np.float32)
    score = rng.normal(size=(B, N)).astype(np.float32)
    tdt = torch.float32
    if dtype == "bf16":
        feat, dout, tdt = bf16_round(feat), bf16_round(dout), torch.bfloat16
    d_coords, d_score = torch.from_numpy(coords).cuda(), torch.from_numpy(score).cuda()
    d_feat, d_dout = torch.from_numpy(feat).cuda().to(tdt), torch.from_numpy(dout).cuda().to(tdt)
    d_nbr = torch.from_numpy(nbr).cuda()
    anchors, _ = aff.affmae_merge_select(d_score, n_keep)
    out = aff.affmae_merge_fwd(d_feat, d_coords, d_score, d_nbr, anchors, p)
    g = aff.affmae_merge_bwd(d_feat, d_coords, d_score, d_nbr, anchors, d_dout, p)
    torch.cuda.synchronize()
    r_anchors = oracle.merge_select(score, n_keep)
    assert np.array_equal(anchors.cpu().numpy(), r_anchors)
    r_out = oracle.merge_fwd(coords, feat, score, nbr, r_anchors, p)
    rg = oracle.merge_bwd(coords, feat, score, nbr, r_anchors, dout, p)

    def err(a, ref):
        a = a.float().cpu().numpy().astype(np.float64)
        return float(np.abs(a - ref).max() / max(np.abs(ref).max(), 1e-30))

    tol = TOL[dtype]
    assert err(out, r_out) <= tol
    assert err(g["dfeat"], rg["dfeat"]) <= tol
    if K > 1:  # with one neighbour the weight is 1 whatever the score: dscore and dp are exactly 0
        assert err(g["dscore"], rg["dscore"]) <= tol
        assert abs(float(g["dp"].cpu()) - rg["dp"]) <= tol * rg["dp_abs"]
    else:
        assert float(g["dscore"].abs().max().cpu()) == 0.0 and float(g["dp"].cpu()) == 0.0


def test_merge_at_the_stage1_shape():
    """One step of the 1024px fine-tuning configuration going from stage 1 to stage 2 at d_s = 0.25: 8 images of
    16384 tokens, C = 64, K = 48, 4096 anchors each; the first two images against the oracle."""
    cfg = CONFIGS["ft_s1_1024"]
    w = make_workload(cfg, features=False)
    rng = np.random.default_rng(7)
    B, N, C, K, n_keep, p = cfg.B, cfg.N, cfg.C, cfg.K, cfg.N // 4, 0.25
    nbr_d, _ = aff.affmae_knn(torch.from_numpy(w["coords"]).cuda(), None, cfg.S, cfg.M, K)
    feat = bf16_round(rng.normal(size=(B, N, C)).astype(np.float32))
    dout = bf16_round(rng.normal(size=(B, n_keep, C)).astype(np.float32))
    score = rng.normal(size=(B, N)).astype(np.float32)
    d_coords, d_score = torch.from_numpy(w["coords"]).cuda(), torch.from_numpy(score).cuda()
    d_feat, d_dout = torch.from_numpy(feat).cuda().bfloat16(), torch.from_numpy(dout).cuda().bfloat16()
    anchors, _ = aff.affmae_merge_select(d_score, n_keep)
    out = aff.affmae_merge_fwd(d_feat, d_coords, d_score, nbr_d, anchors, p)
    g = aff.affmae_merge_bwd(d_feat, d_coords, d_score, nbr_d, anchors, d_dout, p, want_dp=False)
    torch.cuda.synchronize()
    nb = 2
    nbr = nbr_d[:nb].cpu().numpy()
    r_anchors = oracle.merge_select(score[:nb], n_keep)
    assert np.array_equal(anchors[:nb].cpu().numpy(), r_anchors)
    r_out = oracle.merge_fwd(w["coords"][:nb], feat[:nb], score[:nb], nbr, r_anchors, p)
    rg = oracle.merge_bwd(w["coords"][:nb], feat[:nb], score[:nb], nbr, r_anchors, dout[:nb], p)
    for a, ref in ((out[:nb], r_out), (g["dfeat"][:nb], rg["dfeat"]), (g["dscore"][:nb], rg["dscore"])):
        a = a.float().cpu().numpy().astype(np.float64)
        assert np.abs(a - ref).max() / np.abs(ref).max() <= 2e-2
