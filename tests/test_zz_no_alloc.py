"""ck_sparse_decode_attn_static (the entry point for callers that cannot allocate)
against ck_sparse_decode_attn on the same inputs: two calls in a row on the shared
built-in scratch buffer, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2412_03213_amd as ck

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_pair(S, Hq, Hkv, N, n_max, seed, n_sink=0, recent=(0, 0)):
    g = torch.Generator(device=DEV).manual_seed(seed)
    sh = ck.Shape(S, Hq, Hkv, N, 8)
    K = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(torch.bfloat16)
    q = torch.randn(S, Hq, 128, generator=g, device=DEV).to(torch.bfloat16)
    stride = (n_max + 3) // 4 * 4
    lo, hi = n_sink, (recent[0] if recent[1] > recent[0] else N)
    idx = torch.stack([torch.randperm(hi - lo, generator=g, device=DEV)[:stride] + lo
                       for _ in range(S * Hkv)]).view(S, Hkv, stride).to(torch.int32)
    n_tok = torch.randint(1, n_max + 1, (S, Hkv), generator=g, device=DEV).to(torch.int32)
    n_tok[0, 0] = n_max
    want = torch.zeros(S, Hq, 128, dtype=torch.bfloat16, device=DEV)
    got = torch.full_like(want, float("nan"))
    ck.ck_sparse_decode_attn(sh, q, K, V, idx, n_tok, n_max, want, n_sink=n_sink,
                             recent_begin=recent[0], recent_end=recent[1])
    ck.ck_sparse_decode_attn_static(sh, q, K, V, idx, n_tok, n_max, got, n_sink=n_sink,
                                    recent_begin=recent[0], recent_end=recent[1])
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_attention_matches_workspace_attention():
    # same kernels, same launch shape, same order of additions: bit-equal
    want, got = run_pair(S=2, Hq=32, Hkv=8, N=8192, n_max=1024, seed=1)      # 16 splits per head-problem
    assert torch.isfinite(got.float()).all()
    assert torch.equal(want, got)
    # second call, smaller input: stale partials of the first call must not leak in
    want, got = run_pair(S=1, Hq=8, Hkv=2, N=2048, n_max=200, seed=2, n_sink=16,
                         recent=(2000, 2048))
    assert torch.isfinite(got.float()).all()
    assert torch.equal(want, got)


def test_static_scratch_rejects_oversized_shapes():
    sh = ck.Shape(512, 32, 8, 4096, 8)
    t = torch.zeros(1024, dtype=torch.int32, device=DEV)
    with pytest.raises(ck.ClusterKVError) as e:
        ck.ck_sparse_decode_attn_static(sh, t, t, t, t, t, 1024, t)
    assert e.value.code == -3
