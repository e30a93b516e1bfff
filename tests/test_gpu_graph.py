"""GPU: the library's calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a caller can record them into a HIP graph.  A graph holding the neighbour search, the
plan, the forward and the backward is replayed several times, with eager work and synchronisations between the
replays and new inputs each time; every replay must reproduce the eager results bit for bit (the tiled kernels
sum in a fixed order)."""
import numpy as np
import pytest
import torch

import paper_2602_16249_amd as aff
from helpers import to_dev
from workloads import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _eager(coords, q, k, v, bias, dout, S, M, K, scale):
    nbr, near = aff.affmae_knn(coords, None, S, M, K)
    plan = aff.affmae_pla_plan(nbr, near, S, M)
    out, lse = aff.affmae_pla_fwd(q, k, v, bias, nbr, scale, near, S, M, plan=plan)
    g = aff.affmae_pla_bwd(q, k, v, bias, nbr, out, lse, dout, scale, near, S, M, plan=plan)
    torch.cuda.synchronize()
    return {"nbr": nbr, "out": out, "lse": lse, **g}


def test_search_plan_forward_backward_replayed_from_a_graph():
    cfg = CONFIGS["merged_stage"].scaled(B=2, N=2048, C=64, H=2, K=48, S=64, M=8, dtype="bf16")
    S, M, K, scale = cfg.S, cfg.M, cfg.K, 1.0 / np.sqrt(32.0)
    w = make_workload(cfg)
    coords = torch.from_numpy(w["coords"]).cuda()
    q, k, v, dout, bias = (to_dev(w[n], "bf16") for n in ("q", "k", "v", "dout", "bias"))
    B, N, H, d = q.shape

    # static buffers of the graph: inputs are copied in before a replay, outputs read after it
    s_coords, s_q, s_dout = coords.clone(), q.clone(), dout.clone()
    lib = aff.load_library()
    nbr = torch.empty((B, N, K), dtype=torch.int32, device="cuda")
    near = torch.empty((B, N // S, M), dtype=torch.int32, device="cuda")
    plan = torch.empty((lib.affmae_pla_plan_bytes(B, N, K, S, M),), dtype=torch.uint8, device="cuda")
    out, lse = torch.empty_like(q), torch.empty((B, N, H), dtype=torch.float32, device="cuda")
    grads = {n: torch.empty_like(q) for n in ("dq", "dk", "dv")}
    grads["dbias"] = torch.empty_like(bias)
    ws_knn = torch.empty((lib.affmae_knn_workspace_bytes(B, N, S, M, K),), dtype=torch.uint8, device="cuda")
    ws_fwd = torch.empty((max(lib.affmae_pla_fwd_workspace_bytes(B, N, H, d, K, S, M, 1, 1), 256),), dtype=torch.uint8,
                         device="cuda")
    ws_bwd = torch.empty((lib.affmae_pla_bwd_workspace_bytes(B, N, H, d, K, S, M, 1, 1),), dtype=torch.uint8,
                         device="cuda")

    def enqueue():
        aff.affmae_knn(s_coords, None, S, M, K, nbr_idx=nbr, near_clusters=near, workspace=ws_knn)
        aff.affmae_pla_plan(nbr, near, S, M, plan=plan)
        aff.affmae_pla_fwd(s_q, k, v, bias, nbr, scale, near, S, M, out=out, lse=lse, workspace=ws_fwd, plan=plan)
        aff.affmae_pla_bwd(s_q, k, v, bias, nbr, out, lse, s_dout, scale, near, S, M, grads=grads,
                           workspace=ws_bwd, plan=plan)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue()

    for rep in range(4):
        # new inputs: shifted coordinates (another neighbour table), rescaled q, permuted dout rows
        c_new = coords + float(rep) * 0.37
        q_new = (q.float() * (1.0 + 0.25 * rep)).to(torch.bfloat16)
        d_new = dout.roll(rep, dims=1).contiguous()
        ref = _eager(c_new, q_new, k, v, bias, d_new, S, M, K, scale)   # eager work between the replays
        s_coords.copy_(c_new); s_q.copy_(q_new); s_dout.copy_(d_new)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = {"nbr": nbr, "out": out, "lse": lse, **grads}
        for name, t in ref.items():
            assert torch.equal(got[name], t), f"replay {rep}: {name} differs from the eager result"


def test_clustering_and_sampling_replayed_from_a_graph():
    """Curve order, sampling table, sampling forward and backward in one graph.  Everything is deterministic
    except the order of the additions inside a token's dfeat list, so dfeat is compared with the bf16 bound."""
    rng = np.random.default_rng(11)
    B, Nv, Mq, C, Hg, Wg, Kt, cell, p, eps, S = 3, 600, 4000, 64, 40, 40, 4, 8.0, 0.7, 1e-6, 32
    grid = (Hg, Wg, 0.0, 0.0, cell)
    frame = (0.0, 0.0, Wg * cell, Hg * cell)

    def inputs(rep):
        vis = rng.uniform(0, Wg * cell, size=(B, Nv, 2)).astype(np.float32)
        qxy = rng.uniform(-3, Wg * cell + 3, size=(B, Mq, 2)).astype(np.float32)
        feat = torch.from_numpy(rng.normal(size=(B, Nv, C)).astype(np.float32)).cuda().to(torch.bfloat16)
        dout = torch.from_numpy(rng.normal(size=(B, Mq, C)).astype(np.float32)).cuda().to(torch.bfloat16)
        return torch.from_numpy(vis).cuda(), torch.from_numpy(qxy).cuda(), feat, dout

    def run(vis, qxy, feat, dout):
        order, cid = aff.affmae_cluster(vis, S, frame)
        table = aff.affmae_vts_table(vis, grid, Kt)
        out = aff.affmae_vts_fwd(qxy, vis, feat, table, grid, p, eps)
        g = aff.affmae_vts_bwd(qxy, vis, feat, table, dout, grid, p, eps)
        return {"order": order, "cluster_id": cid, "table": table, "out": out, **g}

    s_vis, s_q, s_feat, s_dout = inputs(-1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(s_vis, s_q, s_feat, s_dout)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        got = run(s_vis, s_q, s_feat, s_dout)  # outputs live in the graph's memory pool

    for rep in range(4):
        vis, qxy, feat, dout = inputs(rep)
        ref = run(vis, qxy, feat, dout)  # eager work between the replays
        torch.cuda.synchronize()
        s_vis.copy_(vis); s_q.copy_(qxy); s_feat.copy_(feat); s_dout.copy_(dout)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        # (dp is the sum of the waves' parts in a fixed order: bit-equal like everything but dfeat)
        for name in ("order", "cluster_id", "table", "out", "dquery", "dp"):
            assert torch.equal(got[name], ref[name]), f"replay {rep}: {name} differs from the eager result"
        a, b = got["dfeat"].float(), ref["dfeat"].float()
        assert float((a - b).abs().max()) <= 2e-2 * float(b.abs().max()), f"replay {rep}: dfeat"


def test_relative_position_attention_replayed_from_a_graph():
    """Forward and backward with the bias from a relative-position table, recorded once and replayed with new
    coordinates, tables and gradients.  The table's gradient is summed with LDS atomics whose order may vary, in
    fp64, so it is compared to 1e-6 of its largest entry; everything else bit for bit."""
    cfg = CONFIGS["ft_s1_1024"].scaled(B=2, N=4096, C=64, H=2, K=48, S=64, M=8, dtype="bf16", frame=512.0)
    S, M, K, scale, rate = cfg.S, cfg.M, cfg.K, 1.0 / np.sqrt(32.0), 0.125
    w = make_workload(cfg)
    coords = torch.from_numpy(w["coords"]).cuda()
    q, k, v, dout = (to_dev(w[n], "bf16") for n in ("q", "k", "v", "dout"))
    nbr, near = aff.affmae_knn(coords, None, S, M, K)
    plan = aff.affmae_pla_plan(nbr, near, S, M)
    gen = torch.Generator(device="cuda").manual_seed(3)

    def run(c, table, g):
        out, lse = aff.affmae_pla_fwd_relpos(q, k, v, c, table, nbr, scale, rate, near, S, M, plan=plan)
        grads = aff.affmae_pla_bwd_relpos(q, k, v, c, table, nbr, out, lse, g, scale, rate, near, S, M, plan=plan)
        return {"out": out, "lse": lse, **grads}

    for R in (4, 7):   # the table's gradient summed inside the backward kernel / by the kernel of its own
        s_c = coords.clone()
        s_t = (0.3 * torch.randn((cfg.H, 2 * R + 1, 2 * R + 1), device="cuda", generator=gen)).to(torch.bfloat16)
        s_g = dout.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run(s_c, s_t, s_g)  # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            got = run(s_c, s_t, s_g)
        for rep in range(3):
            # jittered coordinates (same neighbour table: any table is a valid input), a new table, rolled gradients
            c_new = coords + 0.9 * torch.rand(coords.shape, device="cuda", generator=gen)
            t_new = (0.3 * torch.randn(s_t.shape, device="cuda", generator=gen)).to(torch.bfloat16)
            g_new = dout.roll(rep + 1, dims=1).contiguous()
            ref = run(c_new, t_new, g_new)  # eager work between the replays
            torch.cuda.synchronize()
            s_c.copy_(c_new); s_t.copy_(t_new); s_g.copy_(g_new)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name, t in ref.items():
                if name == "drel_table":
                    assert float((got[name] - t).abs().max()) <= 1e-6 * float(t.abs().max()), f"R={R} replay {rep}"
                else:
                    assert torch.equal(got[name], t), f"R={R} replay {rep}: {name} differs from the eager result"


def test_neighbour_search_and_merging_replayed_from_a_graph():
    """Neighbour table, anchor selection, merging forward and backward in one graph, replayed with new coordinates,
    scores, features and gradients.  Indices, merged features and dp are deterministic (bit-equal to the eager
    results); dfeat and dscore are sums over per-token lists whose order may vary, compared with the bf16 bound."""
    rng = np.random.default_rng(12)
    B, N, C, K, S, M, n_keep, p = 2, 2048, 64, 48, 64, 8, 512, 0.3

    def inputs(rep):
        cfg = CONFIGS["knn_scale"].scaled(B=B, N=N, S=S, M=M, K=K)
        w = make_workload(cfg, seed=100 + rep, features=False)
        feat = torch.from_numpy(rng.normal(size=(B, N, C)).astype(np.float32)).cuda().to(torch.bfloat16)
        dout = torch.from_numpy(rng.normal(size=(B, n_keep, C)).astype(np.float32)).cuda().to(torch.bfloat16)
        score = torch.from_numpy(rng.normal(size=(B, N)).astype(np.float32)).cuda()
        return torch.from_numpy(w["coords"]).cuda(), score, feat, dout

    def run(coords, score, feat, dout):
        nbr, _ = aff.affmae_knn(coords, None, S, M, K)
        anchors, axy = aff.affmae_merge_select(score, n_keep, coords)
        out = aff.affmae_merge_fwd(feat, coords, score, nbr, anchors, p)
        g = aff.affmae_merge_bwd(feat, coords, score, nbr, anchors, dout, p)
        return {"nbr": nbr, "anchors": anchors, "anchor_xy": axy, "out": out, **g}

    s_in = inputs(-1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(*s_in)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        got = run(*s_in)

    for rep in range(3):
        new = inputs(rep)
        ref = run(*new)  # eager work between the replays
        torch.cuda.synchronize()
        for dst, src in zip(s_in, new):
            dst.copy_(src)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("nbr", "anchors", "anchor_xy", "out", "dp"):
            assert torch.equal(got[name], ref[name]), f"replay {rep}: {name} differs from the eager result"
        for name in ("dfeat", "dscore"):
            a, b = got[name].float(), ref[name].float()
            assert float((a - b).abs().max()) <= 2e-2 * float(b.abs().max()), f"replay {rep}: {name}"
