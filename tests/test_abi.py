"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2602_16249_amd as aff

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header="affmae.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(affmae_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = aff.load_library()
    names = _declared_symbols()
    assert {"affmae_knn", "affmae_pla_fwd", "affmae_pla_bwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_product_library_has_no_timing_registry():
    """The per-kernel timing lives in the instrumented twin only (include/affmae_timing.h)."""
    lib = aff.load_library()
    timed = ctypes.CDLL(os.path.join(os.path.dirname(aff.library_path()), "libaffmae_timed.so"))
    names = _declared_symbols("affmae_timing.h")
    assert names == ["affmae_timing_enable", "affmae_timing_read", "affmae_timing_reset"]
    for n in names:
        assert hasattr(timed, n), n
        assert not hasattr(lib, n), n
    for n in _declared_symbols():
        assert hasattr(timed, n), n


def test_status_strings():
    assert aff.status_string(0) == "ok"
    for code in range(-6, 0):
        assert aff.status_string(code) not in ("ok", "unknown status")
    assert aff.status_string(-99) == "unknown status"


def test_knn_rejects_bad_arguments_on_host():
    lib = aff.load_library()
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert lib.affmae_knn(None, None, 1, 64, 8, 2, 4, one, None, one, 1 << 20, None) == -1
    assert lib.affmae_knn(one, None, 1, 65, 8, 2, 10, one, None, one, 1 << 20, None) == -2    # a last cluster of one token: 9 candidates
    assert lib.affmae_knn(one, None, 1, 64, 8, 9, 4, one, None, one, 1 << 20, None) == -2     # M > G
    assert lib.affmae_knn(one, None, 1, 64, 8, 2, 17, one, None, one, 1 << 20, None) == -2    # K > M*S
    assert lib.affmae_knn(one, None, 1, 1024, 16, 8, 64 + 1, one, None, one, 1 << 20, None) == -5
    assert lib.affmae_knn(one, None, 1, 64, 8, 2, 4, one, None, None, 0, None) == -4          # no workspace
    assert lib.affmae_knn(one, None, 1, 64, 8, 2, 4, one, None, one, 16, None) == -4          # too small
    assert lib.affmae_knn_workspace_bytes(1, 64, 8, 2, 4) > 0
    assert lib.affmae_knn_workspace_bytes(1, 65, 8, 2, 4) > 0
    assert lib.affmae_knn_workspace_bytes(1, 65, 8, 2, 10) == 0


def test_cluster_rejects_bad_arguments_on_host():
    lib = aff.load_library()
    lib.affmae_cluster.argtypes = ([ctypes.c_void_p] + [ctypes.c_int] * 3 + [ctypes.c_double] * 4 +
                                   [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p])
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    big = 1 << 20
    assert lib.affmae_cluster(None, 1, 64, 8, 0.0, 0.0, 1.0, 1.0, one, None, one, big, None) == -1
    assert lib.affmae_cluster(one, 1, 64, 8, 0.0, 0.0, 1.0, 1.0, None, None, one, big, None) == -1
    assert lib.affmae_cluster(one, 1, 0, 8, 0.0, 0.0, 1.0, 1.0, one, None, one, big, None) == -2
    assert lib.affmae_cluster(one, 1, 64, 0, 0.0, 0.0, 1.0, 1.0, one, None, one, big, None) == -2
    assert lib.affmae_cluster(one, 1, 64, 8, 0.0, 0.0, 0.0, 1.0, one, None, one, big, None) == -2     # empty frame
    assert lib.affmae_cluster(one, 1, 64, 8, 0.0, 0.0, 1.0, float("nan"), one, None, one, big, None) == -2
    assert lib.affmae_cluster(one, 1, 64, 8, float("inf"), 0.0, 1.0, 1.0, one, None, one, big, None) == -2
    assert lib.affmae_cluster(one, 1, (1 << 24) + 1, 8, 0.0, 0.0, 1.0, 1.0, one, None, one, big, None) == -5
    assert lib.affmae_cluster(one, 1, 64, 8, 0.0, 0.0, 1.0, 1.0, one, None, None, 0, None) == -4
    assert lib.affmae_cluster(one, 1, 64, 8, 0.0, 0.0, 1.0, 1.0, one, None, one, 16, None) == -4
    assert lib.affmae_cluster_workspace_bytes(2, 100) == 2 * 128 * 8
    assert lib.affmae_cluster_workspace_bytes(0, 100) == 0


def test_virtual_tokens_reject_bad_arguments_on_host():
    lib = aff.load_library()
    f, i, v = ctypes.c_float, ctypes.c_int, ctypes.c_void_p
    lib.affmae_vts_table.argtypes = [v] + [i] * 4 + [f] * 3 + [i, v, v]
    lib.affmae_vts_fwd.argtypes = [v] * 4 + [i] * 6 + [f] * 3 + [i] + [f] * 2 + [i] + [v, v]
    lib.affmae_vts_bwd.argtypes = [v] * 5 + [i] * 6 + [f] * 3 + [i] + [f] * 2 + [i] + [v] * 4 + [ctypes.c_size_t, v]
    p = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    assert lib.affmae_vts_table(None, 1, 16, 4, 4, 0.0, 0.0, 8.0, 4, p, None) == -1
    assert lib.affmae_vts_table(p, 1, 16, 4, 4, 0.0, 0.0, 8.0, 17, p, None) == -2          # Kt > Nv
    assert lib.affmae_vts_table(p, 1, 16, 0, 4, 0.0, 0.0, 8.0, 4, p, None) == -2
    assert lib.affmae_vts_table(p, 1, 16, 4, 4, 0.0, 0.0, 0.0, 4, p, None) == -2           # empty cell
    assert lib.affmae_vts_table(p, 1, 100, 4, 4, 0.0, 0.0, 8.0, 65, p, None) == -5         # Kt beyond the limit

    def fwd(q=p, feat=p, out=p, C=8, dtype=1, Kt=4):
        return lib.affmae_vts_fwd(q, p, feat, p, 1, 10, 16, C, 4, 4, 0.0, 0.0, 8.0, Kt, 0.5, 1e-6, dtype, out, None)

    assert fwd(q=None) == -1 and fwd(out=None) == -1
    assert fwd(dtype=7) == -3
    assert fwd(C=7) == -5                                                                 # odd channel count
    assert fwd(feat=ctypes.c_void_p(4098)) == -2                                          # misaligned rows
    assert fwd(Kt=17) == -2

    def bwd(ws=p, nbytes=1 << 20, dq=p):
        return lib.affmae_vts_bwd(p, p, p, p, p, 1, 10, 16, 8, 4, 4, 0.0, 0.0, 8.0, 4, 0.5, 1e-6, 1, p, dq, None, ws,
                                  nbytes, None)

    assert bwd(dq=None) == -1
    assert bwd(ws=None, nbytes=0) == -4 and bwd(nbytes=16) == -4
    assert lib.affmae_vts_bwd_workspace_bytes(1, 10, 16, 4) > 0
    assert lib.affmae_vts_bwd_workspace_bytes(1, 10, 16, 65) == 0


def test_attention_rejects_bad_arguments_on_host():
    lib = aff.load_library()
    p = ctypes.c_void_p(4096)
    args = dict(B=1, N=64, H=2, d=32, K=8, S=8, M=2)

    def fwd(q=p, k=p, v=p, nbr=p, out=p, lse=p, dtype=1, kb=None, vb=None, near=None, **kw):
        a = dict(args)
        a.update(kw)
        return lib.affmae_pla_fwd(q, k, v, None, nbr, near, None, kb, vb, a["B"], a["N"], a["H"], a["d"], a["K"], a["S"],
                                  a["M"], 1.0, dtype, out, lse, None, 0, None)

    assert fwd(q=None) == -1
    assert fwd(kb=p) == -1            # blank key without blank value
    assert fwd(dtype=7) == -3
    assert fwd(d=24) == -5
    assert fwd(K=65) == -5
    assert fwd(B=0) == -2
    assert fwd(near=p, S=64, M=2) == -2   # more near clusters than clusters, with a cluster promise
    assert fwd(q=ctypes.c_void_p(4098)) == -2   # misaligned rows

    def bwd(ws=None, ws_bytes=0, dq=p, **kw):
        a = dict(args)
        a.update(kw)
        return lib.affmae_pla_bwd(p, p, p, None, p, None, None, None, None, None, p, p, a["B"], a["N"], a["H"], a["d"],
                                  a["K"], a["S"], a["M"], 1.0, 1, dq, p, p, None, None, None, ws, ws_bytes, None)

    assert bwd(dq=None) == -1
    assert bwd() == -4                # the backward keeps p and dS of every pair and the per-token pair lists
    pairs = 64 * 8
    for dtype in (0, 1):              # p, dS (fp32 per head), pair tokens, lists
        assert lib.affmae_pla_bwd_workspace_bytes(1, 64, 2, 32, 8, 8, 2, dtype, 0) >= (2 * 2 * 4 + 4 + 4) * pairs
    assert bwd(B=1 << 15, N=1 << 15, K=8) == -5   # pairs are numbered in 32 bits


def test_merging_rejects_bad_arguments_on_host():
    lib = aff.load_library()
    p = ctypes.c_void_p(4096)  # never dereferenced: validation fails first

    def select(score=p, idx=p, xy=None, coords=None, B=2, N=100, n_keep=25):
        return lib.affmae_merge_select(score, coords, B, N, n_keep, idx, xy, None)

    assert select(score=None) == -1 and select(idx=None) == -1
    assert select(xy=p) == -1                     # coordinates wanted but none given
    assert select(n_keep=0) == -2 and select(n_keep=101) == -2 and select(B=0) == -2
    assert select(xy=ctypes.c_void_p(4100), coords=p) == -2   # pairs are moved 8 bytes at a time
    assert select(N=(1 << 24) + 1, n_keep=5) == -5

    def fwd(feat=p, out=p, K=8, n_keep=25, pw=0.5, dtype=1, coords=p):
        return lib.affmae_merge_fwd(feat, coords, p, p, p, 2, 100, 64, K, n_keep, ctypes.c_float(pw), dtype, out, None)

    assert fwd(feat=None) == -1 and fwd(out=None) == -1
    assert fwd(dtype=5) == -3
    assert fwd(K=65) == -5 and fwd(K=0) == -2 and fwd(n_keep=101) == -2
    assert fwd(pw=-1.0) == -2 and fwd(pw=float("nan")) == -2   # p >= 0, finite
    assert fwd(coords=ctypes.c_void_p(4100)) == -2

    def bwd(ws=p, nbytes=1 << 30, dscore=p, K=8):
        return lib.affmae_merge_bwd(p, p, p, p, p, p, 2, 100, 64, K, 25, ctypes.c_float(0.5), 1, p, dscore, None, ws,
                                    nbytes, None)

    assert bwd(dscore=None) == -1
    assert bwd(ws=None, nbytes=0) == -4 and bwd(nbytes=64) == -4 and bwd(ws=ctypes.c_void_p(4100)) == -4
    need = lib.affmae_merge_bwd_workspace_bytes(2, 100, 8, 25)
    assert need >= 2 * 25 * 8 * (4 + 4 + 4 + 4) + 2 * 100 * 4   # w, dz, token and list place of every pair; offsets
    assert lib.affmae_merge_bwd_workspace_bytes(2, 100, 65, 25) == 0
    assert bwd(nbytes=need - 1) == -4


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        aff.affmae_knn(torch.zeros(1, 64, 2), None, 8, 2, 4)


def test_relpos_rejects_bad_arguments_on_host():
    lib = aff.load_library()
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    f = ctypes.c_float

    def fwd(coords=one, table=one, R=2, rate=0.125, ws=one, ws_bytes=1 << 30, H=2):
        return lib.affmae_pla_fwd_relpos(one, one, one, coords, table, one, None, None, None, None, 1, 64, H, 32, 8, 0, 0,
                                         f(0.2), R, f(rate), 0, one, one, ws, ws_bytes, None)

    assert fwd(coords=None) == -1 and fwd(table=None) == -1
    assert fwd(R=-1) == -2 and fwd(rate=0.0) == -2 and fwd(rate=float("inf")) == -2
    assert fwd(R=32) == -5 and fwd(R=31, H=8) == -5          # beyond the table limits
    assert fwd(ws=None) == -4 and fwd(ws_bytes=16) == -4
    assert fwd(coords=ctypes.c_void_p(260)) == -2             # coordinates are read as 8-byte pairs
    assert lib.affmae_pla_fwd_relpos_workspace_bytes(1, 64, 2, 32, 8, 0, 0, 0, 0) >= 64 * 2 * 8 * 4
    assert lib.affmae_pla_bwd_relpos_workspace_bytes(1, 64, 2, 32, 8, 0, 0, 2, 0, 0) >= 2 * 64 * 2 * 8 * 4
    assert lib.affmae_pla_bwd_relpos_workspace_bytes(1, 64, 2, 32, 8, 0, 0, 32, 0, 0) == 0


def test_relpos_validates_the_attention_call_before_its_first_launch():
    """The composed relative-position paths put a kernel of their own (the bias) in front of the attention call.
    Arguments that the attention call rejects must be rejected before that kernel: on this GPU-less host a launch
    attempt would surface as AFFMAE_ERR_DEVICE (-6) instead of the validation status."""
    lib = aff.load_library()
    one = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4098)
    f = ctypes.c_float
    big = 1 << 30

    def fwd(q=one, kb=None, vb=None, near=None, S=0, M=0):
        return lib.affmae_pla_fwd_relpos(q, one, one, one, one, one, near, None, kb, vb, 1, 64, 2, 32, 8, S, M, f(0.2), 2,
                                         f(0.125), 0, one, one, one, big, None)

    assert fwd(q=odd) == -2            # misaligned rows: found by the attention call's own checks
    assert fwd(kb=one) == -1           # blank key without blank value
    assert fwd(near=one, S=64, M=2) == -2   # more near clusters than clusters

    def bwd(q=one, kb=None, vb=None, dkb=None, dvb=None, dq=one):
        return lib.affmae_pla_bwd_relpos(q, one, one, one, one, one, None, None, kb, vb, one, one, one, 1, 64, 2, 32, 8, 0,
                                         0, f(0.2), 2, f(0.125), 0, dq, one, one, one, dkb, dvb, one, big, None)

    assert bwd(q=odd) == -2
    assert bwd(kb=one) == -1
    assert bwd(dkb=one) == -1          # dk_blank without dv_blank
    assert bwd(dq=odd) == -2


def test_knn_static_rejects_on_host():
    lib = aff.load_library()
    one = ctypes.c_void_p(256)
    B, N, S, M, K = 64, 32768, 64, 8, 48
    assert lib.affmae_knn_workspace_bytes(B, N, S, M, K) > (4 << 20)
    assert lib.affmae_knn_static(one, None, B, N, S, M, K, one, None, None) == -4   # beyond the fixed scratch
    assert lib.affmae_knn_static(None, None, 1, 64, 8, 2, 4, one, None, None) == -1
    assert lib.affmae_knn_static(one, None, 1, 65, 8, 2, 10, one, None, None) == -2
