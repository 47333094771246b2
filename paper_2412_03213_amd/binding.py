"""ctypes binding of libclusterkv.so: argument marshalling only.

Functions carry the names of the C entry points (include/clusterkv.h) and take
torch tensors in the layouts documented there.  Work is enqueued on torch's
current stream; nothing here synchronises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

CK_BF16, CK_F32 = 0, 1
CK_SEL_WHOLE, CK_SEL_TRIM_LAST = 0, 1
CK_MAX_CLUSTERS = 2048
CK_METRIC_COSINE, CK_METRIC_L2, CK_METRIC_IP, CK_KM_UNTIL_CONVERGED = 0, 1, 2, 4
CK_WS_CLUSTER_KEYS, CK_WS_SPARSE_ATTN, CK_WS_OBJECTIVE = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libclusterkv.so")

EXPORTS = ("ck_version", "ck_strerror", "ck_last_error_detail", "ck_workspace_bytes",
           "ck_cluster_keys", "ck_cluster_keys_opt", "ck_kmeans_assign", "ck_kmeans_objective", "ck_build_metadata", "ck_kmeans_update",
           "ck_select_clusters", "ck_gather_indices", "ck_sparse_decode_attn", "ck_sparse_decode_attn_static", "ck_sparse_decode_attn_two_pass", "ck_decode_step",
           "ck_full_decode_attn", "ck_token_scores", "ck_topk_select", "ck_recall_hits",
           "ck_page_keys", "ck_expand_pages", "ck_host_device_ptr", "ck_cache_reset",
           "ck_cached_decode_step", "ck_probe_mfma_bf16")


class ClusterKVError(RuntimeError):
    def __init__(self, code: int, name: str, detail: str):
        super().__init__(f"{name} (code {code}): {detail}")
        self.code = code


class _CkShape(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("N_cap", ctypes.c_int64), ("C_cap", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


class _CkClusterCache(ctypes.Structure):
    _fields_ = [("K", ctypes.c_void_p * 2), ("V", ctypes.c_void_p * 2),
                ("clusters", ctypes.c_void_p * 2), ("starts", ctypes.c_void_p * 2),
                ("n_held", ctypes.c_void_p * 2), ("cap_tokens", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


@dataclass(frozen=True)
class Shape:
    S: int
    Hq: int
    Hkv: int
    N_cap: int
    C_cap: int
    d: int = 128
    dtype: int = CK_BF16

    def c(self) -> _CkShape:
        return _CkShape(self.S, self.Hq, self.Hkv, self.d, self.N_cap, self.C_cap, self.dtype)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == CK_BF16 else torch.float32


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load the in-tree library; build it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise RuntimeError(f"{LIB_PATH} is missing: run python -m paper_2412_03213_amd.build")
        from .build import build
        build(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    P, I32, I64, U32, SZ, F = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                               ctypes.c_size_t, ctypes.c_float)
    SH = ctypes.POINTER(_CkShape)
    lib.ck_version.restype = ctypes.c_int
    lib.ck_version.argtypes = []
    lib.ck_strerror.restype = ctypes.c_char_p
    lib.ck_strerror.argtypes = [ctypes.c_int]
    lib.ck_last_error_detail.restype = ctypes.c_char_p
    lib.ck_last_error_detail.argtypes = []
    lib.ck_workspace_bytes.restype = SZ
    lib.ck_workspace_bytes.argtypes = [SH, ctypes.c_int, I64, I32]
    lib.ck_cluster_keys.restype = ctypes.c_int
    lib.ck_cluster_keys.argtypes = [SH, P, I64, I64, I32, I32, I32, P, P, P, P, P, P, P, SZ, P]
    lib.ck_cluster_keys_opt.restype = ctypes.c_int
    lib.ck_cluster_keys_opt.argtypes = [SH, P, I64, I64, I32, I32, I32, U32, P, P, P, P, P, P, P,
                                        P, SZ, P]
    lib.ck_kmeans_assign.restype = ctypes.c_int
    lib.ck_kmeans_assign.argtypes = [SH, P, I64, I64, P, I32, I32, P, P, P]
    lib.ck_kmeans_objective.restype = ctypes.c_int
    lib.ck_kmeans_objective.argtypes = [SH, P, I64, I64, P, I32, I32, P, P, P, P, SZ, P]
    lib.ck_build_metadata.restype = ctypes.c_int
    lib.ck_build_metadata.argtypes = [SH, P, I64, I64, I32, I32, P, P, P, P, SZ, P]
    lib.ck_kmeans_update.restype = ctypes.c_int
    lib.ck_kmeans_update.argtypes = [SH, P, P, P, P, I32, I32, P, P, P, P]
    lib.ck_select_clusters.restype = ctypes.c_int
    lib.ck_select_clusters.argtypes = [SH, P, P, P, I32, I32, U32, P, P, P, P, P]
    lib.ck_gather_indices.restype = ctypes.c_int
    lib.ck_gather_indices.argtypes = [SH, P, P, P, P, I32, U32, P, I32, P, P]
    lib.ck_sparse_decode_attn.restype = ctypes.c_int
    lib.ck_sparse_decode_attn.argtypes = [SH, P, P, P, P, P, I32, I32, I64, I64, I64, F, P, P,
                                          SZ, P]
    lib.ck_sparse_decode_attn_two_pass.restype = ctypes.c_int
    lib.ck_sparse_decode_attn_two_pass.argtypes = lib.ck_sparse_decode_attn.argtypes
    lib.ck_sparse_decode_attn_static.restype = ctypes.c_int
    lib.ck_sparse_decode_attn_static.argtypes = [SH, P, P, P, P, P, I32, I32, I64, I64, I64, F, P, P]
    lib.ck_decode_step.restype = ctypes.c_int
    lib.ck_decode_step.argtypes = [SH, P, P, P, P, P, P, P, I32, I32, U32, I64, I64, I64, F,
                                   P, P, P, P, P, I32, P, P, P, SZ, P]
    lib.ck_full_decode_attn.restype = ctypes.c_int
    lib.ck_full_decode_attn.argtypes = [SH, P, P, P, I64, F, P, P, SZ, P]
    lib.ck_token_scores.restype = ctypes.c_int
    lib.ck_token_scores.argtypes = [SH, P, P, I64, I64, P, P]
    lib.ck_topk_select.restype = ctypes.c_int
    lib.ck_topk_select.argtypes = [I32, P, I64, I64, I32, I32, P, I32, P, P]
    lib.ck_recall_hits.restype = ctypes.c_int
    lib.ck_recall_hits.argtypes = [I32, P, P, I32, P, P, I32, P, P]
    lib.ck_page_keys.restype = ctypes.c_int
    lib.ck_page_keys.argtypes = [SH, P, I64, I64, I32, P, I64, P]
    lib.ck_expand_pages.restype = ctypes.c_int
    lib.ck_expand_pages.argtypes = [I32, P, P, I32, I32, I64, I64, P, I32, P, P]
    CC = ctypes.POINTER(_CkClusterCache)
    lib.ck_host_device_ptr.restype = ctypes.c_int
    lib.ck_host_device_ptr.argtypes = [P, ctypes.POINTER(ctypes.c_void_p)]
    lib.ck_cache_reset.restype = ctypes.c_int
    lib.ck_cache_reset.argtypes = [SH, CC, P]
    lib.ck_cached_decode_step.restype = ctypes.c_int
    lib.ck_cached_decode_step.argtypes = [SH, P, P, P, P, P, P, P, I32, I32, CC, I32, F, P, P, P,
                                          P, P, P, P, SZ, P]
    lib.ck_probe_mfma_bf16.restype = ctypes.c_int
    lib.ck_probe_mfma_bf16.argtypes = [I32, I32, P, P, P, ctypes.POINTER(ctypes.c_double), P]
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        lib = load_library()
        raise ClusterKVError(rc, lib.ck_strerror(rc).decode(),
                             lib.ck_last_error_detail().decode())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):          # raw address (used by the argument-validation tests)
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(t) -> int:
    if isinstance(t, torch.Tensor) and t.is_cuda:
        return torch.cuda.current_stream(t.device).cuda_stream
    return 0


def ck_version() -> int:
    return load_library().ck_version()


def ck_workspace_bytes(sh: Shape, which: int, n: int, c: int = 0) -> int:
    s = sh.c()
    return int(load_library().ck_workspace_bytes(ctypes.byref(s), which, n, c))


def _workspace(nbytes: int, like: torch.Tensor) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=like.device)


def ck_cluster_keys(sh: Shape, K, tok_begin, tok_count, c_begin, c_count, n_iter, init_idx,
                    centroids, labels, sizes, offsets, sorted_idx, workspace=None):
    lib = load_library()
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_CLUSTER_KEYS, tok_count, c_count), K)
    s = sh.c()
    _check(lib.ck_cluster_keys(ctypes.byref(s), _ptr(K), tok_begin, tok_count, c_begin, c_count,
                               n_iter, _ptr(init_idx), _ptr(centroids), _ptr(labels),
                               _ptr(sizes), _ptr(offsets), _ptr(sorted_idx), _ptr(workspace),
                               workspace.numel() if isinstance(workspace, torch.Tensor) else 0,
                               _stream(K)))
    return workspace


def ck_cluster_keys_opt(sh: Shape, K, tok_begin, tok_count, c_begin, c_count, max_iter, flags,
                        init_idx, centroids, labels, sizes, offsets, sorted_idx, iters_done=None,
                        workspace=None):
    lib = load_library()
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_CLUSTER_KEYS, tok_count, c_count), K)
    s = sh.c()
    _check(lib.ck_cluster_keys_opt(ctypes.byref(s), _ptr(K), tok_begin, tok_count, c_begin,
                                   c_count, max_iter, flags, _ptr(init_idx), _ptr(centroids),
                                   _ptr(labels), _ptr(sizes), _ptr(offsets), _ptr(sorted_idx),
                                   _ptr(iters_done), _ptr(workspace),
                                   workspace.numel() if isinstance(workspace, torch.Tensor)
                                   else 0, _stream(K)))
    return workspace


def ck_kmeans_assign(sh: Shape, K, tok_begin, tok_count, centroids_hat, c_begin, c_count, labels,
                     best_sim=None):
    lib = load_library()
    s = sh.c()
    _check(lib.ck_kmeans_assign(ctypes.byref(s), _ptr(K), tok_begin, tok_count,
                                _ptr(centroids_hat), c_begin, c_count, _ptr(labels),
                                _ptr(best_sim), _stream(K)))


def ck_kmeans_objective(sh: Shape, K, tok_begin, tok_count, centroids_hat, c_begin, c_count, labels,
                        J, D, workspace=None):
    """J, D: float64 [S, Hkv] outputs (norm-weighted and plain cosine objective)."""
    lib = load_library()
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_OBJECTIVE, tok_count), K)
    s = sh.c()
    _check(lib.ck_kmeans_objective(ctypes.byref(s), _ptr(K), tok_begin, tok_count,
                                   _ptr(centroids_hat), c_begin, c_count, _ptr(labels), _ptr(J),
                                   _ptr(D), _ptr(workspace),
                                   workspace.numel() if isinstance(workspace, torch.Tensor) else 0,
                                   _stream(K)))
    return workspace


def ck_build_metadata(sh: Shape, labels, tok_begin, tok_count, c_begin, c_count, sizes, offsets,
                      sorted_idx, workspace=None):
    lib = load_library()
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_CLUSTER_KEYS, tok_count, c_count),
                               labels)
    s = sh.c()
    _check(lib.ck_build_metadata(ctypes.byref(s), _ptr(labels), tok_begin, tok_count, c_begin,
                                 c_count, _ptr(sizes), _ptr(offsets), _ptr(sorted_idx),
                                 _ptr(workspace),
                                 workspace.numel() if isinstance(workspace, torch.Tensor) else 0,
                                 _stream(labels)))
    return workspace


def ck_kmeans_update(sh: Shape, K, sizes, offsets, sorted_idx, c_begin, c_count, centroids,
                     centroids_hat, centroids_f32=None):
    lib = load_library()
    s = sh.c()
    _check(lib.ck_kmeans_update(ctypes.byref(s), _ptr(K), _ptr(sizes), _ptr(offsets),
                                _ptr(sorted_idx), c_begin, c_count, _ptr(centroids),
                                _ptr(centroids_hat), _ptr(centroids_f32), _stream(K)))


def ck_select_clusters(sh: Shape, q, centroids, sizes, n_clusters, budget, flags, sel_clusters,
                       n_sel_clusters, n_sel_tokens, scores):
    lib = load_library()
    s = sh.c()
    _check(lib.ck_select_clusters(ctypes.byref(s), _ptr(q), _ptr(centroids), _ptr(sizes),
                                  n_clusters, budget, flags, _ptr(sel_clusters),
                                  _ptr(n_sel_clusters), _ptr(n_sel_tokens), _ptr(scores),
                                  _stream(q)))


def ck_gather_indices(sh: Shape, sel_clusters, n_sel_clusters, offsets, sorted_idx, budget, flags,
                      token_idx, n_tokens):
    lib = load_library()
    s = sh.c()
    stride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else budget
    _check(lib.ck_gather_indices(ctypes.byref(s), _ptr(sel_clusters), _ptr(n_sel_clusters),
                                 _ptr(offsets), _ptr(sorted_idx), budget, flags, _ptr(token_idx),
                                 stride, _ptr(n_tokens), _stream(sel_clusters)))


def ck_sparse_decode_attn(sh: Shape, q, K, V, token_idx, n_tokens, max_tokens, out, n_sink=0,
                          recent_begin=0, recent_end=0, softmax_scale=None, workspace=None,
                          two_pass=False):
    """two_pass=True calls ck_sparse_decode_attn_two_pass (merge by a second launch)."""
    lib = load_library()
    if softmax_scale is None:
        softmax_scale = sh.d ** -0.5
    n_recent = max(0, recent_end - recent_begin)
    if workspace is None:
        workspace = _workspace(
            ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, max_tokens + n_sink + n_recent), q)
    stride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else 0
    s = sh.c()
    fn = lib.ck_sparse_decode_attn_two_pass if two_pass else lib.ck_sparse_decode_attn
    _check(fn(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), _ptr(token_idx), _ptr(n_tokens), stride,
              max_tokens, n_sink, recent_begin, recent_end, softmax_scale, _ptr(out),
              _ptr(workspace), workspace.numel() if isinstance(workspace, torch.Tensor) else 0,
              _stream(q)))
    return workspace


def ck_sparse_decode_attn_static(sh: Shape, q, K, V, token_idx, n_tokens, max_tokens, out,
                                 n_sink=0, recent_begin=0, recent_end=0, softmax_scale=None):
    """ck_sparse_decode_attn on the library's built-in scratch buffer: no workspace."""
    lib = load_library()
    if softmax_scale is None:
        softmax_scale = sh.d ** -0.5
    stride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else 0
    s = sh.c()
    _check(lib.ck_sparse_decode_attn_static(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V),
                                            _ptr(token_idx), _ptr(n_tokens), stride, max_tokens,
                                            n_sink, recent_begin, recent_end, softmax_scale,
                                            _ptr(out), _stream(q)))


def ck_full_decode_attn(sh: Shape, q, K, V, n_ctx, out, softmax_scale=None, workspace=None):
    lib = load_library()
    if softmax_scale is None:
        softmax_scale = sh.d ** -0.5
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, n_ctx), q)
    s = sh.c()
    _check(lib.ck_full_decode_attn(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), n_ctx,
                                   softmax_scale, _ptr(out), _ptr(workspace),
                                   workspace.numel() if isinstance(workspace, torch.Tensor)
                                   else 0, _stream(q)))
    return workspace


def ck_token_scores(sh: Shape, q, K, tok_begin, tok_count, scores):
    lib = load_library()
    s = sh.c()
    _check(lib.ck_token_scores(ctypes.byref(s), _ptr(q), _ptr(K), tok_begin, tok_count,
                               _ptr(scores), _stream(q)))


def ck_topk_select(n_problems, scores, row_stride, begin, n, k, out_idx, n_out):
    lib = load_library()
    stride = out_idx.shape[-1] if isinstance(out_idx, torch.Tensor) else max(1, min(k, n))
    _check(lib.ck_topk_select(n_problems, _ptr(scores), row_stride, begin, n, k, _ptr(out_idx),
                              stride, _ptr(n_out), _stream(scores)))


def ck_recall_hits(n_problems, token_idx, n_tokens, ref_idx, n_ref, hits):
    lib = load_library()
    istride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else 1
    rstride = ref_idx.shape[-1] if isinstance(ref_idx, torch.Tensor) else 1
    _check(lib.ck_recall_hits(n_problems, _ptr(token_idx), _ptr(n_tokens), istride, _ptr(ref_idx),
                              _ptr(n_ref), rstride, _ptr(hits), _stream(token_idx)))


def ck_page_keys(sh: Shape, K, tok_begin, tok_count, page_size, page_keys):
    lib = load_library()
    stride = page_keys.shape[-2] if isinstance(page_keys, torch.Tensor) else 0
    s = sh.c()
    _check(lib.ck_page_keys(ctypes.byref(s), _ptr(K), tok_begin, tok_count, page_size,
                            _ptr(page_keys), stride, _stream(K)))


def ck_expand_pages(n_problems, page_idx, n_pages, page_size, tok_begin, tok_count, token_idx,
                    n_tokens):
    lib = load_library()
    pstride = page_idx.shape[-1] if isinstance(page_idx, torch.Tensor) else 1
    istride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else 1
    _check(lib.ck_expand_pages(n_problems, _ptr(page_idx), _ptr(n_pages), pstride, page_size,
                               tok_begin, tok_count, _ptr(token_idx), istride, _ptr(n_tokens),
                               _stream(page_idx)))


def ck_host_device_ptr(host) -> int:
    """Device-visible address of a pinned host tensor (or of a raw pinned address)."""
    lib = load_library()
    out = ctypes.c_void_p(0)
    addr = host if isinstance(host, int) else host.data_ptr()
    _check(lib.ck_host_device_ptr(addr, ctypes.byref(out)))
    return out.value


class ClusterCache:
    """Device buffers of the cluster-granularity cache (two generations) for one layer."""

    def __init__(self, sh: Shape, device, cap_tokens: int):
        self.sh, self.cap = sh, cap_tokens
        dt = sh.torch_dtype
        self.K = [torch.zeros(sh.S, sh.Hkv, cap_tokens, sh.d, dtype=dt, device=device)
                  for _ in range(2)]
        self.V = [torch.zeros(sh.S, sh.Hkv, cap_tokens, sh.d, dtype=dt, device=device)
                  for _ in range(2)]
        self.clusters = [torch.zeros(sh.S, sh.Hkv, sh.C_cap, dtype=torch.int32, device=device)
                         for _ in range(2)]
        self.starts = [torch.zeros(sh.S, sh.Hkv, sh.C_cap + 1, dtype=torch.int32, device=device)
                       for _ in range(2)]
        self.n_held = [torch.zeros(sh.S, sh.Hkv, dtype=torch.int32, device=device)
                       for _ in range(2)]
        self.miss_tokens = torch.zeros(sh.S, sh.Hkv, dtype=torch.int32, device=device)
        self.step = 0

    def c(self) -> _CkClusterCache:
        two = ctypes.c_void_p * 2
        return _CkClusterCache(two(*[_ptr(t) for t in self.K]), two(*[_ptr(t) for t in self.V]),
                               two(*[_ptr(t) for t in self.clusters]),
                               two(*[_ptr(t) for t in self.starts]),
                               two(*[_ptr(t) for t in self.n_held]), self.cap, 0)


def ck_cache_reset(sh: Shape, cache):
    lib = load_library()
    s = sh.c()
    c = cache.c() if isinstance(cache, ClusterCache) else cache
    _check(lib.ck_cache_reset(ctypes.byref(s), ctypes.byref(c) if c is not None else None,
                              _stream(cache.K[0]) if isinstance(cache, ClusterCache) else 0))
    if isinstance(cache, ClusterCache):
        cache.step = 0


def ck_cached_decode_step(sh: Shape, q, K_home, V_home, centroids, sizes, offsets, sorted_idx,
                          n_clusters, budget, cache, step_parity, scores, sel_clusters,
                          n_sel_clusters, n_sel_tokens, miss_tokens, out, softmax_scale=None,
                          workspace=None):
    """K_home / V_home: device tensors, or device-visible addresses (int) of pinned host
    memory as returned by ck_host_device_ptr."""
    lib = load_library()
    if softmax_scale is None:
        softmax_scale = sh.d ** -0.5
    if workspace is None:
        workspace = _workspace(ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, budget), q)
    s = sh.c()
    c = cache.c() if isinstance(cache, ClusterCache) else cache
    _check(lib.ck_cached_decode_step(ctypes.byref(s), _ptr(q), _ptr(K_home), _ptr(V_home),
                                     _ptr(centroids), _ptr(sizes), _ptr(offsets),
                                     _ptr(sorted_idx), n_clusters, budget,
                                     ctypes.byref(c) if c is not None else None, step_parity,
                                     softmax_scale, _ptr(scores), _ptr(sel_clusters),
                                     _ptr(n_sel_clusters), _ptr(n_sel_tokens), _ptr(miss_tokens),
                                     _ptr(out), _ptr(workspace),
                                     workspace.numel() if isinstance(workspace, torch.Tensor)
                                     else 0, _stream(q)))
    return workspace


def cached_decode_step(st, cache: ClusterCache, q, K_home, V_home):
    """One cached decode step on the clustered state `st`; alternates the generations."""
    ck_cached_decode_step(st.sh, q, K_home, V_home, st.centroids, st.sizes, st.offsets,
                          st.sorted_idx, st.n_clusters, st.budget, cache, cache.step & 1,
                          st.scores, st.sel_clusters, st.n_sel_clusters, st.n_sel_tokens,
                          cache.miss_tokens, st.out, workspace=st.attn_ws)
    cache.step += 1
    return st.out


def _probe_operands(t):
    if t is None:
        return None
    if t.numel() * t.element_size() < 16384:
        raise ValueError("probe operands need 16384 bytes")
    return _ptr(t)


def ck_probe_mfma_bf16(n_workgroups: int, iters: int, sink, operands=None, clocks=None) -> float:
    """Enqueue the MFMA probe; returns the flops of the launch.  operands: 16384 bytes
    on the device (per lane 8 A then 8 B fragments) or None for constants; clocks: two
    int64 on the device that receive shader cycles and 100 MHz ticks, or None."""
    lib = load_library()
    fl = ctypes.c_double(0.0)
    _check(lib.ck_probe_mfma_bf16(n_workgroups, iters,
                                  _probe_operands(operands),
                                  _ptr(clocks) if clocks is not None else None,
                                  _ptr(sink), ctypes.byref(fl), _stream(sink)))
    return fl.value


class ClusterState:
    """Device buffers of one layer's clustering result (centroid table + metadata)
    plus the per-step outputs of the decode calls, allocated once."""

    def __init__(self, sh: Shape, device, budget: int, idx_stride: int | None = None,
                 max_recent: int = 0, n_sink: int = 0):
        self.sh = sh
        S, H, N, C = sh.S, sh.Hkv, sh.N_cap, sh.C_cap
        i32 = dict(dtype=torch.int32, device=device)
        self.centroids = torch.zeros(S, H, C, sh.d, dtype=sh.torch_dtype, device=device)
        self.labels = torch.zeros(S, H, N, **i32)
        self.sizes = torch.zeros(S, H, C, **i32)
        self.offsets = torch.zeros(S, H, C + 1, **i32)
        self.sorted_idx = torch.zeros(S, H, N, **i32)
        self.n_clusters = 0
        self.budget = budget
        stride = idx_stride or ((budget + 3) // 4 * 4)
        self.sel_clusters = torch.zeros(S, H, C, **i32)
        self.n_sel_clusters = torch.zeros(S, H, **i32)
        self.n_sel_tokens = torch.zeros(S, H, **i32)
        self.scores = torch.zeros(S, H, C, dtype=torch.float32, device=device)
        self.token_idx = torch.zeros(S, H, stride, **i32)
        self.n_tokens = torch.zeros(S, H, **i32)
        self.out = torch.zeros(S, sh.Hq, sh.d, dtype=sh.torch_dtype, device=device)
        self.attn_ws = _workspace(
            ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, budget + n_sink + max_recent),
            self.centroids)
        self.cluster_ws = None

    def cluster(self, K, init_idx, tok_begin, tok_count, c_count, n_iter, flags=0,
                iters_done=None):
        need = ck_workspace_bytes(self.sh, CK_WS_CLUSTER_KEYS, tok_count, c_count)
        if self.cluster_ws is None or self.cluster_ws.numel() < need:
            self.cluster_ws = _workspace(need, K)
        ck_cluster_keys_opt(self.sh, K, tok_begin, tok_count, self.n_clusters, c_count, n_iter,
                            flags, init_idx, self.centroids, self.labels, self.sizes,
                            self.offsets, self.sorted_idx, iters_done, self.cluster_ws)
        self.n_clusters += c_count


def ck_decode_step(sh: Shape, q, K, V, centroids, sizes, offsets, sorted_idx, n_clusters, budget,
                   flags, scores, sel_clusters, n_sel_clusters, n_sel_tokens, token_idx, n_tokens,
                   out, n_sink=0, recent_begin=0, recent_end=0, softmax_scale=None,
                   workspace=None):
    lib = load_library()
    if softmax_scale is None:
        softmax_scale = sh.d ** -0.5
    n_recent = max(0, recent_end - recent_begin)
    if workspace is None:
        workspace = _workspace(
            ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, budget + n_sink + n_recent), q)
    stride = token_idx.shape[-1] if isinstance(token_idx, torch.Tensor) else budget
    s = sh.c()
    _check(lib.ck_decode_step(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), _ptr(centroids),
                              _ptr(sizes), _ptr(offsets), _ptr(sorted_idx), n_clusters, budget,
                              flags, n_sink, recent_begin, recent_end, softmax_scale,
                              _ptr(scores), _ptr(sel_clusters), _ptr(n_sel_clusters),
                              _ptr(n_sel_tokens), _ptr(token_idx), stride, _ptr(n_tokens),
                              _ptr(out), _ptr(workspace),
                              workspace.numel() if isinstance(workspace, torch.Tensor) else 0,
                              _stream(q)))
    return workspace


def decode_step(st: ClusterState, q, K, V, flags=CK_SEL_WHOLE, n_sink=0, recent_begin=0,
                recent_end=0, fused=True):
    """One decode step of the path on the current stream: the fused library call, or
    (fused=False) selection, index gather and sparse attention as three calls.
    Returns st.out."""
    sh = st.sh
    if fused:
        ck_decode_step(sh, q, K, V, st.centroids, st.sizes, st.offsets, st.sorted_idx,
                       st.n_clusters, st.budget, flags, st.scores, st.sel_clusters,
                       st.n_sel_clusters, st.n_sel_tokens, st.token_idx, st.n_tokens, st.out,
                       n_sink=n_sink, recent_begin=recent_begin, recent_end=recent_end,
                       workspace=st.attn_ws)
        return st.out
    ck_select_clusters(sh, q, st.centroids, st.sizes, st.n_clusters, st.budget, flags,
                       st.sel_clusters, st.n_sel_clusters, st.n_sel_tokens, st.scores)
    ck_gather_indices(sh, st.sel_clusters, st.n_sel_clusters, st.offsets, st.sorted_idx,
                      st.budget, flags, st.token_idx, st.n_tokens)
    ck_sparse_decode_attn(sh, q, K, V, st.token_idx, st.n_tokens, st.budget, st.out,
                          n_sink=n_sink, recent_begin=recent_begin, recent_end=recent_end,
                          workspace=st.attn_ws)
    return st.out
