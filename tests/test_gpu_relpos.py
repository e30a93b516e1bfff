"""GPU parity: attention with the bias taken from a relative-position table (affmae_pla_fwd_relpos,
affmae_pla_bwd_relpos) against the CPU oracle: outputs, every gradient and the gradient of the table."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_16249_amd as aff
from helpers import LSE_TOL, TOL, rel_err, to_dev
from workloads import CONFIGS, bf16_round, make_workload, random_neighbours

pytestmark = pytest.mark.gpu


def _check(w, coords, nbr, table, R, rate, dtype, scale, near=None, S=0, M=0, blank=False, use_plan=False):
    q, k, v, dout = (to_dev(w[n], dtype) for n in ("q", "k", "v", "dout"))
    c_d = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.float32)).cuda()
    t_d = to_dev(table.astype(np.float32), dtype)
    nbr_d = torch.from_numpy(np.ascontiguousarray(nbr, dtype=np.int32)).cuda()
    near_d = torch.from_numpy(np.ascontiguousarray(near, dtype=np.int32)).cuda() if near is not None else None
    kb = to_dev(w["k_blank"], dtype) if blank else None
    vb = to_dev(w["v_blank"], dtype) if blank else None
    plan = aff.affmae_pla_plan(nbr_d, near_d, S, M) if (use_plan and near_d is not None) else None
    out, lse = aff.affmae_pla_fwd_relpos(q, k, v, c_d, t_d, nbr_d, scale, rate, near_d, S, M, kb, vb, plan=plan)
    g = aff.affmae_pla_bwd_relpos(q, k, v, c_d, t_d, nbr_d, out, lse, dout, scale, rate, near_d, S, M, kb, vb,
                                  plan=plan)
    torch.cuda.synchronize()
    kbo = w["k_blank"] if blank else None
    vbo = w["v_blank"] if blank else None
    rout, rlse = oracle.pla_fwd_relpos(w["q"], w["k"], w["v"], coords, table, nbr, scale, R, rate, kbo, vbo)
    rg = oracle.pla_bwd_relpos(w["q"], w["k"], w["v"], coords, table, nbr, w["dout"], scale, R, rate, kbo, vbo)
    tol = TOL[dtype]
    errs = {"out": rel_err(out, rout), "lse": rel_err(lse, rlse)}
    for name in rg:
        errs[name] = rel_err(g["drel_table" if name == "dtable" else name], rg[name])
    bad = {n: e for n, e in errs.items() if not (e <= (LSE_TOL if n == "lse" else tol))}
    assert not bad, f"errors above tolerance {tol}: {bad} (all: {errs})"


def _table(rng, H, R, dtype):
    t = rng.normal(0, 0.5, size=(H, 2 * R + 1, 2 * R + 1)).astype(np.float32)
    return bf16_round(t).astype(np.float64) if dtype == "bf16" else t.astype(np.float64)


@pytest.mark.parametrize("dtype,B,N,H,d,K,R,rate,blank", [
    ("f32", 1, 256, 2, 32, 16, 3, 0.125, False),   # the tiny fp32 configuration, any neighbour table
    ("f32", 2, 150, 3, 16, 9, 0, 1.0, True),       # a single bin: one bias value per head
    ("bf16", 2, 200, 2, 32, 24, 5, 0.2, True),
    ("f32", 1, 100, 8, 16, 7, 15, 0.5, False),     # 8 heads x 31 x 31 bins
])
def test_relpos_any_neighbour_table(dtype, B, N, H, d, K, R, rate, blank):
    print(f"case relpos gather {dtype} B={B} N={N} H={H} d={d} K={K} R={R}", flush=True)
    rng = np.random.default_rng(N + K)
    cfg = CONFIGS["tiny_f32"].scaled(B=B, N=N, C=H * d, H=H, K=K, S=N, M=1, dtype=dtype)
    w = make_workload(cfg, blank=blank)
    nbr = random_neighbours(B, N, K, rng, distinct=True)
    _check(w, w["coords"], nbr, _table(rng, H, R, dtype), R, rate, dtype, 1.0 / np.sqrt(d), blank=blank)


@pytest.mark.parametrize("name,B,N,S,M,K,H,R,rate,blank,use_plan", [
    ("ft_s1_1024", 1, 16384, 64, 8, 48, 2, 4, 0.125, False, True),   # one full image, bins of one patch
    ("mae_pt_s1_1024", 2, 1024, 64, 8, 48, 2, 6, 0.125, True, False),  # on-grid: offsets on bin centres
    ("knn_scale", 2, 2048, 32, 8, 40, 4, 3, 0.05, False, True),
    ("merged_stage", 1, 1024, 64, 4, 20, 8, 2, 0.01, True, True),     # K not a multiple of 8
    ("knn_scale", 1, 1024, 16, 16, 64, 2, 4, 0.1, True, False),       # strips that touch more tiles than one pass holds
    ("ft_s1_1024", 3, 1024, 32, 4, 8, 1, 31, 2.0, False, True),        # the largest table, one head
    ("knn_scale", 2, 1001, 64, 8, 48, 2, 4, 0.05, True, True),        # a last strip / token tile of 9 tokens
    ("mae_pt_s1_1024", 2, 1000, 32, 4, 24, 2, 6, 0.125, False, False),  # ... of 8, table too large for the in-kernel sums
])
def test_relpos_clustered(name, B, N, S, M, K, H, R, rate, blank, use_plan):
    print(f"case relpos tiled {name} B={B} N={N} S={S} M={M} K={K} H={H} R={R}", flush=True)
    rng = np.random.default_rng(N + K + H)
    cfg = CONFIGS[name].scaled(B=B, N=N, S=S, M=M, K=K, C=32 * H, H=H, dtype="bf16")
    if cfg.coords == "jitter_grid" and N != 16384:
        cfg = cfg.scaled(frame=8.0 * int(round(N ** 0.5)))
    w = make_workload(cfg, blank=blank)
    nbr, near = oracle.knn(w["coords"], None, S, M, K)
    _check(w, w["coords"], nbr, _table(rng, H, R, "bf16"), R, rate, "bf16", 1.0 / np.sqrt(32.0), near, S, M, blank,
           use_plan)
