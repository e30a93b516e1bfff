"""GPU parity: affmae_pla_fwd / affmae_pla_bwd against the CPU oracle.

Tolerance (per tensor, forward and every gradient): max|gpu - ref| / max|ref|
<= 1e-5 for fp32 storage and <= 2e-2 for bf16 storage; the oracle runs in
double precision on the same stored (already rounded) inputs."""
import numpy as np
import pytest

import oracle
from helpers import check_attention
from workloads import CONFIGS, make_features, make_workload, random_neighbours

pytestmark = pytest.mark.gpu


def test_tiny_fp32_config():
    """B=1, N=256, C=64, 2 heads, K=16 exact neighbours, fp32."""
    cfg = CONFIGS["tiny_f32"]
    w = make_workload(cfg)
    nbr = oracle.knn_bruteforce(w["coords"], cfg.K)
    errs = check_attention(w, nbr, "f32", 1.0 / np.sqrt(cfg.d))
    print(errs)


GATHER_CASES = [
    # dtype, B, N, H, d, K, blank, distinct
    ("f32", 2, 200, 2, 32, 16, False, True),
    ("f32", 1, 130, 3, 16, 7, True, False),    # repeats, odd sizes, blank token
    ("f32", 1, 96, 1, 64, 64, True, True),     # K at the limit
    ("f32", 2, 64, 4, 32, 1, False, True),     # K = 1: out = v[nbr]
    ("bf16", 2, 200, 2, 32, 48, False, True),
    ("bf16", 1, 130, 8, 32, 48, True, False),
    ("bf16", 1, 77, 2, 64, 33, True, True),
    ("bf16", 1, 300, 4, 16, 5, False, False),
    ("bf16", 2, 150, 2, 16, 64, True, False),  # two pieces per row, both trips full; tokens that nobody lists
    ("f32", 1, 90, 2, 16, 64, False, True),
    ("bf16", 1, 70, 1, 64, 64, False, True),
]


@pytest.mark.parametrize("dtype,B,N,H,d,K,blank,distinct", GATHER_CASES)
def test_arbitrary_neighbour_tables(dtype, B, N, H, d, K, blank, distinct):
    """No cluster promise: any indices, repeats allowed (gather kernels)."""
    print(f"case {dtype} B={B} N={N} H={H} d={d} K={K} blank={blank} distinct={distinct}", flush=True)
    rng = np.random.default_rng(100 + N + K)
    w = make_features(B, N, H, d, K, dtype, rng, blank=blank)
    nbr = random_neighbours(B, N, K, rng, distinct=distinct)
    check_attention(w, nbr, dtype, 1.0 / np.sqrt(d), blank=blank)


def test_no_bias_argument():
    rng = np.random.default_rng(3)
    w = make_features(1, 128, 2, 32, 12, "bf16", rng)
    w["bias"] = None
    nbr = random_neighbours(1, 128, 12, rng)
    check_attention(w, nbr, "bf16", 0.2)


CLUSTER_CASES = [
    # name, B, N, C, H, K, S, M, blank
    ("mae_pt_s1_1024", 2, 1024, 64, 2, 48, 64, 8, False),
    ("mae_pt_s1_1024", 1, 1024, 64, 2, 48, 64, 8, True),
    ("merged_stage", 3, 512, 256, 8, 48, 32, 8, False),
    ("knn_scale", 2, 1024, 128, 4, 48, 64, 8, False),
    ("knn_scale", 1, 960, 96, 3, 20, 48, 5, True),     # ragged: S=48, M=5, H=3
    ("merged_stage", 2, 512, 64, 2, 64, 16, 32, False),  # 32 candidate tiles per strip: two passes of the bias tile
    ("tiny_f32", 1, 256, 64, 2, 16, 256, 1, False),    # one cluster per image (exact kNN), bf16 storage here
    ("merged_stage", 2, 224, 96, 3, 8, 32, 3, True),   # K = 8: one 16-byte chunk of slots per query
    ("merged_stage", 2, 64, 64, 2, 1, 16, 2, False),   # K = 1: every token attends to itself only
    ("mae_pt_s1_1024", 2, 1000, 64, 2, 48, 64, 8, True),   # N % 16 = 8: short last strip and token tile, blank sums
    ("merged_stage", 3, 250, 256, 8, 16, 32, 4, False),    # N % 16 = 10, eight heads (four head groups per tile)
    ("knn_scale", 1, 33, 64, 2, 12, 16, 2, True),          # three strips, the last of one query
    ("merged_stage", 2, 250, 96, 3, 7, 32, 4, True),       # short last strip with single-entry items and one head per sweep
]


@pytest.mark.parametrize("name,B,N,C,H,K,S,M,blank", CLUSTER_CASES)
@pytest.mark.parametrize("promise", ["none", "promise", "plan"])
def test_clustered_tables(name, B, N, C, H, K, S, M, blank, promise):
    """kNN tables of small clustered token sets: without the cluster promise
    (gather kernels), with it (near_clusters; tiled kernels, plan rebuilt inside
    the call) and with a plan built once by affmae_pla_plan."""
    print(f"case {name} B={B} N={N} C={C} H={H} K={K} S={S} M={M} blank={blank} promise={promise}", flush=True)
    cfg = CONFIGS[name].scaled(B=B, N=N, C=C, H=H, K=K, S=S, M=M, dtype="bf16")
    w = make_workload(cfg, blank=blank)
    nbr, near = oracle.knn(w["coords"], None, S, M, K)
    check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), near=near if promise != "none" else None, S=S, M=M,
                    blank=blank, use_plan=promise == "plan")


@pytest.mark.parametrize("scale", [1.5, 4.0])
@pytest.mark.parametrize("blank", [False, True])
def test_wide_range_of_scores(scale, blank):
    """Logits with a standard deviation of 8 to 20: the running maximum of the streaming softmax rises many
    times along the tiles and most probabilities underflow next to the largest ones."""
    print(f"case wide scores scale={scale} blank={blank}", flush=True)
    cfg = CONFIGS["mae_pt_s1_1024"].scaled(B=2, N=1024, dtype="bf16")
    w = make_workload(cfg, blank=blank)
    nbr, near = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    check_attention(w, nbr, cfg.dtype, scale, near=near, S=cfg.S, M=cfg.M, blank=blank, use_plan=True)


@pytest.mark.parametrize("name", ["mae_pt_s1_1024", "ft_s1_1024", "merged_stage", "knn_scale"])
def test_full_size_configs(name):
    """The benchmark's configurations at full size in the launch configuration
    the benchmark times (cluster promise given), every element compared."""
    cfg = CONFIGS[name]
    print(f"case {name} full size", flush=True)
    w = make_workload(cfg)
    nbr, near = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    errs = check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), near=near, S=cfg.S, M=cfg.M, use_plan=True)
    print(errs)


def test_full_image_with_blank_tokens():
    """Two full 1024px images with blank tokens: the blank column in the tiled forward and backward, and
    the sums for dk_blank / dv_blank over 2048 strips."""
    cfg = CONFIGS["ft_s1_1024"].scaled(B=2)
    print("case ft_s1_1024 B=2 blank", flush=True)
    w = make_workload(cfg, blank=True)
    nbr, near = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    errs = check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), near=near, S=cfg.S, M=cfg.M, blank=True,
                           use_plan=True)
    print(errs)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_through_the_tiled_kernels(seed):
    """Seeded random N (mostly not a multiple of 16 or of S), S, M, K, H, batch and blank tokens: neighbour table by
    the oracle's clustered search, tiled kernels with the plan rebuilt inside the call and with a plan built once."""
    rng = np.random.default_rng(9000 + seed)
    while True:
        S = int(rng.choice([16, 32, 48, 64]))
        N = int(rng.integers(1, 70 if seed % 4 == 0 else 1500))
        G = (N + S - 1) // S
        M = int(rng.integers(1, min(G, 8) + 1))
        kmax = min(64, (M - 1) * S + N - (G - 1) * S)
        if M * S <= 1024 and kmax >= 1:
            break
    K, H, B = int(rng.integers(1, kmax + 1)), int(rng.choice([1, 2, 3, 4, 8])), int(rng.integers(1, 4))
    blank = bool(rng.integers(0, 2))
    name = ["mae_pt_s1_1024", "merged_stage", "knn_scale"][int(rng.integers(0, 3))]
    print(f"case {name} B={B} N={N} S={S} M={M} K={K} H={H} blank={blank}", flush=True)
    cfg = CONFIGS[name].scaled(B=B, N=N, C=32 * H, H=H, K=K, S=S, M=M, dtype="bf16")
    w = make_workload(cfg, blank=blank)
    nbr, near = oracle.knn(w["coords"], None, S, M, K)
    for use_plan in (False, True):
        check_attention(w, nbr, "bf16", 1.0 / np.sqrt(32), near=near, S=S, M=M, blank=blank, use_plan=use_plan)


def test_instrumented_library_gives_the_same_bits():
    """The bench takes its per-kernel times in the instrumented twin library (the same sources with events around
    every launch): its tiled forward and backward results are bit-equal to the product library's."""
    import paper_2602_16249_amd as aff
    from helpers import run_gpu_attention
    cfg = CONFIGS["ft_s1_1024"].scaled(B=1)
    print("case ft_s1_1024 B=1 product against instrumented library", flush=True)
    w = make_workload(cfg)
    nbr, near = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    scale = 1.0 / np.sqrt(cfg.d)
    out, lse, g = run_gpu_attention(w, nbr, cfg.dtype, scale, near, cfg.S, cfg.M, use_plan=True)
    aff.use_timed_library(True)
    try:
        tout, tlse, tg = run_gpu_attention(w, nbr, cfg.dtype, scale, near, cfg.S, cfg.M, use_plan=True)
    finally:
        aff.use_timed_library(False)
    assert torch_equal(out, tout) and torch_equal(lse, tlse)
    for name in g:
        assert torch_equal(g[name], tg[name]), name


def torch_equal(a, b):
    import torch
    return a is None and b is None or torch.equal(a, b)


def test_gather_kernels_on_full_images():
    """Two full 1024px images without the cluster promise: the gather kernels at the benchmark's shape (16384
    queries per image: the list builder of the backward takes them in two sweeps), every element compared; the
    same with a table whose neighbours are drawn from the whole image (no locality: every token range of the list
    builder has to walk every query)."""
    cfg = CONFIGS["ft_s1_1024"].scaled(B=2)
    print("case ft_s1_1024 B=2 gather kernels", flush=True)
    w = make_workload(cfg, blank=True)
    nbr, _ = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    print(check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), blank=True))
    print("case ft_s1_1024 B=2 gather kernels, neighbours without locality", flush=True)
    rng = np.random.default_rng(77)
    nbr = random_neighbours(cfg.B, cfg.N, cfg.K, rng, distinct=False)
    print(check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), blank=True))


@pytest.mark.parametrize("use_plan", [False, True])
@pytest.mark.parametrize("bias", [True, False])
def test_promise_with_permuted_neighbour_lists(use_plan, bias):
    """The cluster promise asks for distinct neighbours inside the near clusters, not for distance order: every
    token's list is shuffled (the oracle's results are invariant to that order up to the slot each bias value
    belongs to, and it gets the same shuffled table).  Also the tiled kernels without a bias tensor."""
    print(f"case permuted lists plan={use_plan} bias={bias}", flush=True)
    cfg = CONFIGS["knn_scale"].scaled(B=2, N=1024, C=64, H=2, dtype="bf16")
    w = make_workload(cfg, blank=True)
    nbr, near = oracle.knn(w["coords"], None, cfg.S, cfg.M, cfg.K)
    rng = np.random.default_rng(17)
    nbr = np.ascontiguousarray(rng.permuted(nbr, axis=2))
    if not bias:
        w["bias"] = None
    check_attention(w, nbr, cfg.dtype, 1.0 / np.sqrt(cfg.d), near=near, S=cfg.S, M=cfg.M, blank=True, use_plan=use_plan)


@pytest.mark.parametrize("N,tiled", [(4000, True), (4001, True), (3983, True)])
def test_short_last_cluster_end_to_end(N, tiled):
    """coords -> affmae_cluster -> affmae_knn -> affmae_pla_fwd / affmae_pla_bwd with N not a multiple of the
    cluster size (a masked batch keeps whatever number of tokens the mask leaves): curve order, neighbour table
    and near clusters bit-equal to the oracle, attention within the bf16 bound, in the tiled kernels: N = 4000
    (whole 16-token tiles, short last cluster), N = 4001 (a last strip and token tile of one token, which is also
    the whole last cluster), N = 3983 (fifteen tokens in the last tile)."""
    import torch
    import paper_2602_16249_amd as aff
    print(f"case end to end N={N}", flush=True)
    S, M, K, H, d = 64, 8, 48, 2, 32
    cfg = CONFIGS["mae_pt_s1_1024"].scaled(B=2, N=N, C=H * d, H=H, K=K, S=S, M=M, dtype="bf16")
    w = make_workload(cfg)
    rng = np.random.default_rng(N)
    perm = np.stack([rng.permutation(N) for _ in range(cfg.B)])
    shuffled = np.ascontiguousarray(np.take_along_axis(w["coords"], perm[..., None], axis=1))
    frame = (0.0, 0.0, float(cfg.frame), float(cfg.frame))
    order, cid = aff.affmae_cluster(torch.from_numpy(shuffled).cuda(), S, frame)
    rorder, rcid = oracle.cluster(shuffled, S, frame)
    assert np.array_equal(order.cpu().numpy(), rorder) and np.array_equal(cid.cpu().numpy(), rcid)
    coords = np.ascontiguousarray(np.take_along_axis(shuffled, rorder[..., None].astype(np.int64), axis=1))
    nbr_d, near_d = aff.affmae_knn(torch.from_numpy(coords).cuda(), None, S, M, K)
    nbr, near = oracle.knn(coords, None, S, M, K)
    assert np.array_equal(nbr_d.cpu().numpy(), nbr) and np.array_equal(near_d.cpu().numpy(), near)
    assert (aff.load_library().affmae_pla_plan_bytes(cfg.B, N, K, S, M) > 0) == tiled
    check_attention(w, nbr, "bf16", 1.0 / np.sqrt(d), near=near, S=S, M=M, use_plan=tiled)
