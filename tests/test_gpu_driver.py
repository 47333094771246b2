"""GPU test of the layer-stack driver: clustering on a side stream, attention sinks, the
unclustered recent window, periodic clustering of generated tokens and full-KV first
layers (paper Sections III-B, IV-B, V-A).  The asynchronous run must equal, bit for
bit, the same calls issued one after the other on one stream, and the oracle within the
attention tolerance."""
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


def rel_err(got, want):
    den = np.maximum(np.abs(want).max(axis=-1), 1e-30)
    return (np.abs(got - want).max(axis=-1) / den).max()


def test_layer_stack_matches_sequential_calls_and_oracle():
    L, S, Hkv, G, N0, steps, m, cp, C0, B, sink = 4, 1, 2, 2, 1040, 150, 64, 2, 16, 128, 16
    Hq = Hkv * G
    cfgs = [Config(f"l{l}", 1, S, Hkv, Hq, 128, N0, 24, C0, 10, B, 100 + l) for l in range(L)]
    ws = [MixtureWorkload(c, device=DEV, extra_tokens=steps) for c in cfgs]
    stack = ck.LayerStack(L, S, Hq, Hkv, N0, steps, C0, B, DEV, n_sink=sink, full_kv_layers=2,
                          m=m, c_plus=cp, n_iter=5)
    sh = stack.sh
    assert sh.N_cap == N0 + steps and sh.C_cap == C0 + cp * (steps // m)
    # reference: the same calls, all on the current stream
    ref = [None, None] + [ck.ClusterState(sh, DEV, B, max_recent=m, n_sink=sink) for _ in range(2)]
    ref_to = [sink] * L
    inits = [sample_init_indices(w.K, C0, 7, tok_begin=sink, tok_count=N0 - sink).to(DEV) for w in ws]
    for l in range(L):
        stack.cluster_prefill(l, ws[l].K, inits[l])      # all layers' clustering in flight at once
    for l in range(2, L):
        ref[l].cluster(ws[l].K, inits[l], sink, N0 - sink, C0, 5)
        ref_to[l] = N0
    full_ref = torch.zeros(S, Hq, 128, dtype=torch.bfloat16, device=DEV)
    events = 0
    for t in range(1, steps + 1):
        n_ctx = N0 + t
        for l in range(L):
            ws[l].append_token()
            q = ws[l].query()
            out = stack.decode(l, q, ws[l].K, ws[l].V, n_ctx).clone()
            if l < 2:
                ck.ck_full_decode_attn(sh, q, ws[l].K, ws[l].V, n_ctx, full_ref)
                want = full_ref
            else:
                want = ck.decode_step(ref[l], q, ws[l].K, ws[l].V, n_sink=sink,
                                      recent_begin=ref_to[l], recent_end=n_ctx)
            assert torch.equal(out, want), f"step {t} layer {l}"
            if l >= 2 and n_ctx - ref_to[l] >= m:
                init = sample_init_indices(ws[l].K, cp, 1000 + t, tok_begin=ref_to[l],
                                           tok_count=m).to(DEV)
                assert stack.cluster_generated(l, ws[l].K, n_ctx, init)
                ref[l].cluster(ws[l].K, init, ref_to[l], m, cp, 5)
                ref_to[l] += m
                events += 1
            elif l >= 2:
                assert not stack.cluster_generated(l, ws[l].K, n_ctx, None)
        if t in (1, 70, steps):
            # against the oracle: the recalled list the GPU used, sinks, recent window
            for l in (0, 3):
                q = ws[l].query()
                out = np64(stack.decode(l, q, ws[l].K, ws[l].V, n_ctx))
                for h in range(Hkv):
                    qg = np64(q[0, h * G:(h + 1) * G])
                    K, V = np64(ws[l].K[0, h]), np64(ws[l].V[0, h])
                    if l == 0:
                        want = O.full_attention(qg, K, V, n_ctx)
                    else:
                        st = stack.states[l]
                        idx = st.token_idx[0, h, :int(st.n_tokens[0, h])].cpu().numpy()
                        want = O.sparse_attention(qg, K, V, idx, sink, stack.clustered_to[l], n_ctx)
                        # the recalled list never contains sinks or unclustered tokens
                        assert idx.min() >= sink and idx.max() < stack.clustered_to[l]
                    assert rel_err(out[0, h * G:(h + 1) * G], want) <= 2e-2
    assert events == 2 * (steps // m)
    for l in range(2, L):
        assert stack.states[l].n_clusters == C0 + cp * (steps // m) == ref[l].n_clusters
        torch.cuda.synchronize()
        assert torch.equal(stack.states[l].sorted_idx, ref[l].sorted_idx)
        assert torch.equal(stack.states[l].centroids, ref[l].centroids)
