"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before enqueuing
anything (so these calls are safe without a device)."""
import ctypes
import os
import re

import pytest

import paper_2412_03213_amd as ck
from paper_2412_03213_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "clusterkv.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ck_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ck.load_library()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert ck.ck_version() == 100


def test_header_constants_match_binding():
    text = open(HEADER).read()
    consts = dict(re.findall(r"#define\s+(CK_[A-Z0-9_]+)\s+\(?(-?\d+)u?\)?", text))
    assert int(consts["CK_BF16"]) == ck.CK_BF16 and int(consts["CK_F32"]) == ck.CK_F32
    assert int(consts["CK_SEL_WHOLE"]) == ck.CK_SEL_WHOLE
    assert int(consts["CK_SEL_TRIM_LAST"]) == ck.CK_SEL_TRIM_LAST
    assert int(consts["CK_MAX_CLUSTERS"]) == ck.CK_MAX_CLUSTERS
    assert int(consts["CK_METRIC_COSINE"]) == ck.CK_METRIC_COSINE
    assert int(consts["CK_METRIC_L2"]) == ck.CK_METRIC_L2
    assert int(consts["CK_METRIC_IP"]) == ck.CK_METRIC_IP
    assert int(consts["CK_KM_UNTIL_CONVERGED"]) == ck.CK_KM_UNTIL_CONVERGED
    assert ctypes.sizeof(binding._CkShape) == 32


def test_strerror_and_workspace_sizes():
    lib = ck.load_library()
    assert lib.ck_strerror(0) == b"success"
    for code in (-1, -2, -3, -4, -5):
        assert lib.ck_strerror(code) not in (b"success", b"unknown error code")
    sh = ck.Shape(1, 32, 8, 32768, 400)
    assert ck.ck_workspace_bytes(sh, binding.CK_WS_CLUSTER_KEYS, 32768, 400) > 8 * 400 * 256
    assert ck.ck_workspace_bytes(sh, binding.CK_WS_SPARSE_ATTN, 1024) > 0
    assert ck.ck_workspace_bytes(sh, 99, 1024) == 0
    assert ck.ck_workspace_bytes(ck.Shape(1, 32, 8, 32768, 400, d=64), 0, 100, 4) == 0


A = 0x1000  # a 16-byte aligned fake device address: validation never dereferences it


def expect(code, fn, *args, **kw):
    with pytest.raises(ck.ClusterKVError) as e:
        fn(*args, **kw)
    assert e.value.code == code, str(e.value)


def test_argument_validation_without_a_device():
    sh = ck.Shape(1, 32, 8, 1000, 40)
    ws = A
    lib = ck.load_library()

    def cluster(sh=sh, K=A, tb=0, tc=1000, cb=0, cc=40, it=10, init=A, cent=A, lab=A, sz=A, off=A,
                sidx=A, ws=A, wsb=1 << 30):
        s = sh.c()
        rc = lib.ck_cluster_keys(ctypes.byref(s), K, tb, tc, cb, cc, it, init, cent, lab, sz, off,
                                 sidx, ws, wsb, None)
        if rc:
            raise ck.ClusterKVError(rc, lib.ck_strerror(rc).decode(),
                                    lib.ck_last_error_detail().decode())

    expect(-1, cluster, K=None)
    expect(-1, cluster, tb=500, tc=501)
    expect(-1, cluster, cb=30, cc=11)
    expect(-1, cluster, tc=30, cc=40)
    expect(-1, cluster, it=0)
    expect(-2, cluster, sh=ck.Shape(1, 32, 8, 1000, 40, d=64))
    expect(-2, cluster, sh=ck.Shape(1, 24, 8, 1000, 40))            # group of 3
    expect(-2, cluster, sh=ck.Shape(1, 32, 8, 1000, 40, dtype=ck.CK_F32))
    expect(-2, cluster, sh=ck.Shape(1, 32, 8, 5000, 4000), tc=5000, cc=2049)
    expect(-3, cluster, ws=None)
    expect(-3, cluster, wsb=16)
    expect(-4, cluster, lab=A + 4)
    expect(-1, cluster, sh=ck.Shape(1, 30, 8, 1000, 40))            # Hq not a multiple of Hkv

    def cluster_opt(flags=0, it=10, iters=None, lab=A):
        s = sh.c()
        rc = lib.ck_cluster_keys_opt(ctypes.byref(s), A, 0, 1000, 0, 40, it, flags, A, A, lab, A, A,
                                     A, iters, A, 1 << 30, None)
        if rc:
            raise ck.ClusterKVError(rc, lib.ck_strerror(rc).decode(),
                                    lib.ck_last_error_detail().decode())

    expect(-1, cluster_opt, flags=3)                                # no such metric
    expect(-1, cluster_opt, flags=8)                                # unknown bit
    expect(-1, cluster_opt, it=0)
    expect(-2, cluster_opt, flags=ck.CK_KM_UNTIL_CONVERGED, it=257)
    expect(-4, cluster_opt, iters=A + 4)
    expect(-4, cluster_opt, flags=ck.CK_METRIC_L2 | ck.CK_KM_UNTIL_CONVERGED, lab=A + 8)

    expect(-1, ck.ck_select_clusters, sh, A, A, A, 0, 10, 0, A, A, A, A)
    expect(-1, ck.ck_select_clusters, sh, A, A, A, 41, 10, 0, A, A, A, A)
    expect(-1, ck.ck_select_clusters, sh, A, A, A, 40, 0, 0, A, A, A, A)
    expect(-1, ck.ck_select_clusters, sh, A, A, A, 40, 10, 7, A, A, A, A)
    expect(-1, ck.ck_select_clusters, sh, None, A, A, 40, 10, 0, A, A, A, A)
    expect(-1, ck.ck_select_clusters, sh, A, A, A, 40, 10, 0, A, A, A, None)
    expect(-4, ck.ck_select_clusters, sh, A, A + 8, A, 40, 10, 0, A, A, A, A)

    def fused(**kw):
        args = dict(q=A, K=A, V=A, cent=A, sizes=A, offs=A, sidx=A, nc=40, B=16, flags=0,
                    scores=A, sel=A, nsel=A, ntok=A, idx=A, n=A, out=A, workspace=A)
        args.update(kw)
        ck.ck_decode_step(sh, args["q"], args["K"], args["V"], args["cent"], args["sizes"],
                          args["offs"], args["sidx"], args["nc"], args["B"], args["flags"],
                          args["scores"], args["sel"], args["nsel"], args["ntok"], args["idx"],
                          args["n"], args["out"], workspace=args["workspace"])

    expect(-1, fused, sidx=None)
    expect(-1, fused, nc=41)
    expect(-1, fused, B=0)
    expect(-1, fused, flags=2)
    expect(-3, fused, workspace=0)
    expect(-4, fused, scores=A + 4)

    expect(-1, ck.ck_gather_indices, sh, A, A, A, A, 0, 0, A, A)
    expect(-1, ck.ck_gather_indices, sh, A, None, A, A, 16, 0, A, A)

    expect(-1, ck.ck_kmeans_assign, sh, A, 0, 1001, A, 0, 40, A)
    expect(-1, ck.ck_kmeans_assign, sh, A, 0, 1000, None, 0, 40, A)
    expect(-3, ck.ck_build_metadata, sh, A, 0, 1000, 0, 40, A, A, A, workspace=0)
    expect(-1, ck.ck_kmeans_objective, sh, A, 0, 1001, A, 0, 40, A, A, A, workspace=A)
    expect(-1, ck.ck_kmeans_objective, sh, A, 0, 1000, A, 0, 40, A, None, A, workspace=A)
    expect(-3, ck.ck_kmeans_objective, sh, A, 0, 1000, A, 0, 40, A, A, A, workspace=0)
    assert ck.ck_workspace_bytes(sh, binding.CK_WS_OBJECTIVE, 1000) >= 8 * 2 * 8
    expect(-1, ck.ck_kmeans_update, sh, A, A, A, A, 0, 41, A, A)

    def attn(**kw):
        args = dict(sh=sh, q=A, K=A, V=A, idx=A, n=A, stride=1024, mx=1024, sink=0, rb=0, re=0,
                    scale=0.088, out=A, ws=A, wsb=1 << 30)
        args.update(kw)
        s = args["sh"].c()
        rc = lib.ck_sparse_decode_attn(ctypes.byref(s), args["q"], args["K"], args["V"],
                                       args["idx"], args["n"], args["stride"], args["mx"],
                                       args["sink"], args["rb"], args["re"], args["scale"],
                                       args["out"], args["ws"], args["wsb"], None)
        if rc:
            raise ck.ClusterKVError(rc, lib.ck_strerror(rc).decode(),
                                    lib.ck_last_error_detail().decode())

    expect(-1, attn, out=None)
    expect(-1, attn, sink=1001)
    expect(-1, attn, rb=0, re=1001)
    expect(-1, attn, stride=512)
    expect(-1, attn, scale=0.0)
    expect(-1, attn, idx=None)
    expect(-3, attn, wsb=8)
    expect(-3, attn, ws=None)
    expect(-4, attn, V=A + 2)

    # the same call on the built-in scratch buffer: same validation, and shapes whose
    # partials exceed the buffer are rejected before anything touches a device
    def attn_static(**kw):
        args = dict(sh=sh, q=A, K=A, V=A, idx=A, n=A, stride=1024, mx=1024, sink=0, rb=0, re=0,
                    scale=0.088, out=A)
        args.update(kw)
        s = args["sh"].c()
        rc = lib.ck_sparse_decode_attn_static(ctypes.byref(s), args["q"], args["K"], args["V"],
                                              args["idx"], args["n"], args["stride"], args["mx"],
                                              args["sink"], args["rb"], args["re"],
                                              args["scale"], args["out"], None)
        if rc:
            raise ck.ClusterKVError(rc, lib.ck_strerror(rc).decode(),
                                    lib.ck_last_error_detail().decode())

    expect(-1, attn_static, out=None)
    expect(-1, attn_static, sink=1001)
    expect(-1, attn_static, stride=512)
    expect(-4, attn_static, V=A + 2)
    big = ck.Shape(512, 32, 8, 4096, 40)                            # 4096 head-problems x 4 heads
    assert ck.ck_workspace_bytes(big, binding.CK_WS_SPARSE_ATTN, 1024) > (4 << 20)
    expect(-3, attn_static, sh=big)

    # evaluation entry points
    expect(-1, ck.ck_full_decode_attn, sh, A, A, A, 0, A, workspace=A)
    expect(-1, ck.ck_full_decode_attn, sh, A, A, A, 1001, A, workspace=A)
    expect(-1, ck.ck_full_decode_attn, sh, A, A, None, 1000, A, workspace=A)
    expect(-3, ck.ck_full_decode_attn, sh, A, A, A, 1000, A, workspace=0)
    expect(-1, ck.ck_token_scores, sh, A, A, 0, 1001, A)
    expect(-1, ck.ck_token_scores, sh, A, A, 0, 1000, None)
    expect(-4, ck.ck_token_scores, sh, A, A + 4, 0, 1000, A)
    expect(-1, ck.ck_topk_select, 0, A, 1000, 0, 1000, 10, A, A)
    expect(-1, ck.ck_topk_select, 8, A, 1000, 0, 0, 10, A, A)
    expect(-1, ck.ck_topk_select, 8, A, 1000, 0, 1000, -1, A, A)
    expect(-1, ck.ck_topk_select, 8, A, 1000, 1, 1000, 10, A, A)        # range leaves the row
    expect(-1, ck.ck_topk_select, 8, A, 1000, 0, 1000, 10, A, None)
    expect(-1, ck.ck_recall_hits, 8, A, A, A, None, A)
    expect(-1, ck.ck_recall_hits, 70000, A, A, A, A, A)
    expect(-1, ck.ck_page_keys, sh, A, 0, 1000, 0, A)                   # page_size 0, stride 0
    expect(-1, ck.ck_page_keys, sh, A, 0, 1001, 16, A)
    expect(-1, ck.ck_expand_pages, 8, A, A, 0, 0, 1000, A, A)
    expect(-1, ck.ck_expand_pages, 8, A, None, 16, 0, 1000, A, A)

    # cluster cache
    two = ctypes.c_void_p * 2

    def cache_struct(cap=64, K0=A):
        return binding._CkClusterCache(two(K0, A), two(A, A), two(A, A), two(A, A), two(A, A),
                                       cap, 0)

    def cached(cache=None, B=16, parity=0, miss=A, nc=40, ws=A):
        ck.ck_cached_decode_step(sh, A, A, A, A, A, A, A, nc, B,
                                 cache_struct() if cache is None else cache, parity, A, A, A, A,
                                 miss, A, workspace=ws)

    expect(-1, cached, B=65)                                        # budget above the cache rows
    expect(-1, cached, parity=2)
    expect(-1, cached, miss=None)
    expect(-1, cached, nc=41)
    expect(-1, cached, cache=cache_struct(cap=0))
    expect(-1, cached, cache=cache_struct(K0=None))
    expect(-4, cached, cache=cache_struct(K0=A + 4))
    expect(-3, cached, ws=0)
    expect(-1, ck.ck_cache_reset, sh, cache_struct(cap=0))
    expect(-1, ck.ck_host_device_ptr, 0)


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        binding.load_library(build_if_missing=False)
