"""The single-launch split merge (last workgroup of a head-problem merges the partials it
reads back with agent-scope loads) against the two-pass form (second kernel), which runs
the same merge arithmetic: outputs must be bit-identical, call after call, with inputs
that change between calls (a stale partial or ticket would show), in HIP-graph replays
and on both storage types."""
import numpy as np
import pytest
import torch

import paper_2412_03213_amd as ck
from ck_synth import Config, MixtureWorkload, sample_init_indices
from oracle import clusterkv_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def np64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def make(S, Hq, Hkv, N, n_max, seed, dtype=torch.bfloat16):
    g = torch.Generator(device=DEV).manual_seed(seed)
    K = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dtype)
    V = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(dtype)
    stride = (n_max + 3) // 4 * 4
    idx = torch.stack([torch.randperm(N, generator=g, device=DEV)[:stride]
                       for _ in range(S * Hkv)]).view(S, Hkv, stride).to(torch.int32)
    return g, K, V, idx


@pytest.mark.parametrize("S,Hq,Hkv,N,n_max,dtype", [
    (1, 32, 8, 8192, 1024, ck.CK_BF16),      # 16 splits per head-problem (the 32k layer's shape)
    (8, 32, 8, 4096, 2048, ck.CK_BF16),      # 8 splits, 64 head-problems
    (3, 16, 2, 4096, 700, ck.CK_BF16),       # G = 8, head-problem count not a multiple of 8
    (2, 4, 4, 2048, 500, ck.CK_F32),         # fp32 check mode, G = 1
])
def test_single_launch_merge_equals_two_pass(S, Hq, Hkv, N, n_max, dtype):
    tdt = torch.bfloat16 if dtype == ck.CK_BF16 else torch.float32
    g, K, V, idx = make(S, Hq, Hkv, N, n_max, seed=S * 1000 + n_max, dtype=tdt)
    sh = ck.Shape(S, Hq, Hkv, N, 8, dtype=dtype)
    ws = torch.empty(ck.ck_workspace_bytes(sh, 1, n_max), dtype=torch.uint8, device=DEV)
    ws.random_(0, 256)                                   # nothing in the workspace has to be zero
    ws2 = torch.empty_like(ws)
    a = torch.zeros(S, Hq, 128, dtype=tdt, device=DEV)
    b = torch.zeros_like(a)
    for it in range(40):
        q = torch.randn(S, Hq, 128, generator=g, device=DEV).to(tdt)
        n_tok = torch.randint(0, n_max + 1, (S, Hkv), generator=g, device=DEV).to(torch.int32)
        if it % 3 == 0:
            n_tok[0, 0] = n_max
        a.fill_(float("nan"))
        ck.ck_sparse_decode_attn(sh, q, K, V, idx, n_tok, n_max, a, workspace=ws)
        ck.ck_sparse_decode_attn(sh, q, K, V, idx, n_tok, n_max, b, workspace=ws2, two_pass=True)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16 if tdt == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if tdt == torch.bfloat16 else torch.int32)), it
    # and the two-pass form against the oracle on the last inputs
    for s, h in [(0, 0), (S - 1, Hkv - 1)]:
        G = Hq // Hkv
        n = int(n_tok[s, h])
        want = O.attention_over(np64(q[s, h * G:(h + 1) * G]), np64(K[s, h]), np64(V[s, h]),
                                idx[s, h, :n].cpu().numpy())
        got = np64(b[s, h * G:(h + 1) * G])
        tol = 2e-2 if dtype == ck.CK_BF16 else 1e-5
        assert np.abs(got - want).max() <= tol * max(np.abs(want).max(), 1e-30)


def test_decode_step_graph_replays_match_eager():
    """ck_decode_step captured in a HIP graph: the launch keeps its ticket epoch across
    replays, so the last workgroup must leave the tickets ready for the next replay.
    Five replays with new queries, eager work and synchronisations in between."""
    cfg = Config("graph", 1, 2, 4, 16, 128, 6000, 64, 48, 4, 1024, seed=77)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed).to(DEV)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    st.cluster(w.K, init, 0, cfg.N, cfg.C, cfg.n_iter)
    ref = ck.ClusterState(sh, DEV, budget=cfg.B)
    for name in ("centroids", "sizes", "offsets", "sorted_idx"):
        getattr(ref, name).copy_(getattr(st, name))
    ref.n_clusters = st.n_clusters
    q = w.query().clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ck.decode_step(st, q, w.K, w.V)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ck.decode_step(st, q, w.K, w.V)
    for r in range(5):
        q.copy_(w.query())
        graph.replay()
        torch.cuda.synchronize()
        ck.decode_step(ref, q, w.K, w.V)                 # eager, its own workspace
        torch.cuda.synchronize()
        assert torch.equal(st.n_tokens, ref.n_tokens)
        for s in range(cfg.S):
            for h in range(cfg.Hkv):
                n = int(ref.n_tokens[s, h])
                assert torch.equal(st.token_idx[s, h, :n], ref.token_idx[s, h, :n])
        assert torch.equal(st.out.view(torch.int16), ref.out.view(torch.int16)), r
