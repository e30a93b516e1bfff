"""Shared helpers of the GPU parity tests: upload a seeded workload, run the
library through its C ABI (via the thin binding), run the CPU oracle on the same
stored values, and compare with the benchmark's error metric."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2602_16249_amd as aff

TOL = {"f32": 1e-5, "bf16": 2e-2}   # max|gpu - ref| / max|ref| per tensor (forward and gradients)
LSE_TOL = 1e-5                      # lse is fp32 whatever the storage type; bf16 inputs are exact in both paths


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    if x.dtype == np.float32 and dtype == "bf16":
        t = t.to(torch.bfloat16)   # exact: the generators return bf16-representable values
    return t


def rel_err(got, ref: np.ndarray) -> float:
    if isinstance(got, torch.Tensor):
        got = got.detach().float().cpu().numpy()
    got = got.astype(np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def run_gpu_attention(w, nbr, dtype, scale, near=None, S=0, M=0, blank=False, use_plan=False):
    q, k, v, dout = (to_dev(w[n], dtype) for n in ("q", "k", "v", "dout"))
    bias = to_dev(w["bias"], dtype) if w.get("bias") is not None else None
    nbr_d = torch.from_numpy(np.ascontiguousarray(nbr, dtype=np.int32)).cuda()
    near_d = torch.from_numpy(np.ascontiguousarray(near, dtype=np.int32)).cuda() if near is not None else None
    kb = to_dev(w["k_blank"], dtype) if blank else None
    vb = to_dev(w["v_blank"], dtype) if blank else None
    plan = aff.affmae_pla_plan(nbr_d, near_d, S, M) if (use_plan and near_d is not None) else None
    out, lse = aff.affmae_pla_fwd(q, k, v, bias, nbr_d, scale, near_d, S, M, kb, vb, plan=plan)
    g = aff.affmae_pla_bwd(q, k, v, bias, nbr_d, out, lse, dout, scale, near_d, S, M, kb, vb, plan=plan)
    torch.cuda.synchronize()
    return out, lse, g


def run_oracle_attention(w, nbr, scale, blank=False):
    kb = w["k_blank"] if blank else None
    vb = w["v_blank"] if blank else None
    out, lse = oracle.pla_fwd(w["q"], w["k"], w["v"], w.get("bias"), nbr, scale, kb, vb)
    g = oracle.pla_bwd(w["q"], w["k"], w["v"], w.get("bias"), nbr, w["dout"], scale, kb, vb)
    return out, lse, g


def check_attention(w, nbr, dtype, scale, near=None, S=0, M=0, blank=False, tol=None, use_plan=False):
    tol = TOL[dtype] if tol is None else tol
    out, lse, g = run_gpu_attention(w, nbr, dtype, scale, near, S, M, blank, use_plan)
    rout, rlse, rg = run_oracle_attention(w, nbr, scale, blank)
    errs = {"out": rel_err(out, rout), "lse": rel_err(lse, rlse)}
    for name in rg:
        errs[name] = rel_err(g[name], rg[name])
    bad = {n: e for n, e in errs.items() if not (e <= (LSE_TOL if n == "lse" else tol))}
    assert not bad, f"errors above tolerance {tol}: {bad} (all: {errs})"
    return errs
