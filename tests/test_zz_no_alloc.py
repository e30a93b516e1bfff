"""The allocation-free entry point affmae_knn_static against affmae_knn (same kernels, the scratch in the
library's fixed device array instead of a caller workspace): bit-equal outputs through the raw C ABI, on two
calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import paper_2602_16249_amd as aff
from workloads import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _knn_both(lib, coords, cid, S, M, K, with_near):
    B, N, _ = coords.shape
    G = N // S
    dev = coords.device
    ref_nbr = torch.full((B, N, K), -1, dtype=torch.int32, device=dev)
    ref_near = torch.full((B, G, M), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(lib.affmae_knn_workspace_bytes(B, N, S, M, K), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    cid_p = None if cid is None else cid.data_ptr()
    rc = lib.affmae_knn(coords.data_ptr(), cid_p, B, N, S, M, K, ref_nbr.data_ptr(), ref_near.data_ptr(), ws.data_ptr(),
                        ws.numel(), stream)
    assert rc == 0
    nbr = torch.full((B, N, K), -2, dtype=torch.int32, device=dev)
    near = torch.full((B, G, M), -2, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = lib.affmae_knn_static(coords.data_ptr(), cid_p, B, N, S, M, K, nbr.data_ptr(),
                               near.data_ptr() if with_near else None, stream)
    assert rc == 0, aff.status_string(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(nbr, ref_nbr)
    if with_near:
        assert torch.equal(near, ref_near)
    return nbr


def test_knn_static_matches_knn_twice():
    lib = aff.load_library()
    # first call: a full configuration (16 images of 4096 masked-grid tokens), explicit scattered cluster ids
    cfg = CONFIGS["mae_pt_s1_1024"]
    w = make_workload(cfg, features=False)
    rng = np.random.default_rng(5)
    perm = np.stack([rng.permutation(cfg.N) for _ in range(cfg.B)])
    coords = np.ascontiguousarray(np.take_along_axis(w["coords"], perm[..., None], axis=1))
    cid = (perm // cfg.S).astype(np.int32)  # the token now at place p sat at place perm[b, p] of the cluster order
    _knn_both(lib, torch.from_numpy(coords).cuda(), torch.from_numpy(np.ascontiguousarray(cid)).cuda(), cfg.S, cfg.M,
              cfg.K, with_near=True)
    # second call, smaller, tokens in cluster order, near-cluster table kept in the scratch
    small = CONFIGS["mae_pt_s1_1024"].scaled(B=2, N=1024)
    w2 = make_workload(small, features=False)
    _knn_both(lib, torch.from_numpy(w2["coords"]).cuda(), None, small.S, small.M, small.K, with_near=False)
