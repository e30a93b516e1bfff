"""Statistic, not a parity item: how many of a token's exact K nearest neighbours (search over the whole image)
the clustered search (the method: candidates = members of the M nearest clusters) returns, on the synthetic
workloads.  Both searches are the oracle's; run as `python -m oracle.knn_recall [images per workload]`."""
import sys
import time

import numpy as np

import oracle
from workloads import CONFIGS, make_workload


def recall(name: str, images: int = 1):
    cfg = CONFIGS[name]
    w = make_workload(cfg, features=False)
    coords = w["coords"][:images]
    t = time.time()
    clustered, _ = oracle.knn(coords, None, cfg.S, cfg.M, cfg.K)
    exact, _ = oracle.knn(coords, None, cfg.S, cfg.G, cfg.K)  # every cluster is near: the whole image
    hit, same_rows = 0, 0
    for b in range(images):
        for i in range(cfg.N):
            hit += np.intersect1d(clustered[b, i], exact[b, i], assume_unique=True).size
            same_rows += bool(np.array_equal(clustered[b, i], exact[b, i]))
    total = images * cfg.N
    return hit / (total * cfg.K), same_rows / total, time.time() - t


if __name__ == "__main__":
    n = int(sys.argv[1]) if len(sys.argv) > 1 else 1
    for name in ("mae_pt_s1_1024", "ft_s1_1024", "merged_stage", "knn_scale"):
        r, rows, sec = recall(name, n)
        print(f"{name}: recall of the exact K nearest {r:.5f}, tokens with the identical list {rows:.5f} "
              f"({n} image(s), {sec:.1f} s)", flush=True)
