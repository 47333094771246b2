"""Decode with incremental clustering (Section III-B, decode stage): every m generated
tokens are clustered among themselves into C+ clusters appended to the table; the
newest tokens that no cluster covers yet are always attended.  Scaled-down version
of the incremental configuration, checked against the oracle at every step."""
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


@pytest.mark.parametrize("flags", [ck.CK_SEL_WHOLE, ck.CK_SEL_TRIM_LAST])
def test_incremental_decode_loop(flags):
    N0, C0, m, Cp, steps, B = 2048, 32, 64, 4, 200, 256
    cfg = Config("incr_small", 1, 2, 2, 8, 128, N0, 64, C0, 10, B, seed=11, decode_steps=steps,
                 m_incr=m, c_incr=Cp)
    w = MixtureWorkload(cfg, device=DEV, extra_tokens=steps)
    n_events = steps // m
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, N0 + steps, C0 + n_events * Cp)
    st = ck.ClusterState(sh, DEV, budget=B, max_recent=m)
    st.cluster(w.K, sample_init_indices(w.K, C0, cfg.seed, 0, N0).to(DEV), 0, N0, C0, cfg.n_iter)
    G = cfg.G
    near = checked = 0
    worst = 0.0
    for t in range(1, steps + 1):
        row = w.append_token()
        assert row == N0 + t - 1
        q = w.query()
        recent_begin = N0 + m * ((t - 1) // m)
        recent_end = N0 + t
        out = ck.decode_step(st, q, w.K, w.V, flags=flags, recent_begin=recent_begin,
                             recent_end=recent_end)
        if t % 7 == 0 or t % m in (0, 1):
            torch.cuda.synchronize()
            C = st.n_clusters
            for s in range(cfg.S):
                for h in range(cfg.Hkv):
                    keys, vals = np64(w.K[s, h]), np64(w.V[s, h])
                    mu = np64(st.centroids[s, h, :C])
                    sizes = st.sizes[s, h, :C].cpu().numpy()
                    offs = st.offsets[s, h, :C + 1].cpu().numpy()
                    sidx = st.sorted_idx[s, h].cpu().numpy()
                    assert offs[-1] == recent_begin           # every older token is clustered
                    qg = np64(q[s, h * G:(h + 1) * G])
                    r = O.decode_step(qg, keys, vals, mu, sizes, offs, sidx, B, flags,
                                      recent_begin=recent_begin, recent_end=recent_end)
                    n = int(st.n_tokens[s, h])
                    got_idx = st.token_idx[s, h, :n].cpu().numpy()
                    checked += 1
                    if O.selection_near_tie(r["scores"], r["order"], r["n_sel"]):
                        near += 1
                    else:
                        assert np.array_equal(got_idx, r["idx"]), (t, s, h)
                    want = O.sparse_attention(qg, keys, vals, got_idx, 0, recent_begin, recent_end)
                    got = np64(out[s, h * G:(h + 1) * G])
                    err = (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max()
                    worst = max(worst, err)
                    assert err <= 2e-2, (t, s, h, err)
        if t % m == 0:
            tb = N0 + t - m
            init = sample_init_indices(w.K, Cp, 1000 + t, tb, m)
            st.cluster(w.K, init.to(DEV), tb, m, Cp, cfg.n_iter)
    torch.cuda.synchronize()
    assert st.n_clusters == C0 + n_events * Cp
    # final table: exact metadata for the labels, appended clusters hold only their own slice
    for s in range(cfg.S):
        for h in range(cfg.Hkv):
            n_clustered = N0 + n_events * m
            lab = st.labels[s, h, :n_clustered].cpu().numpy()
            sz, of, si = O.build_metadata(lab, st.n_clusters)
            assert np.array_equal(st.sizes[s, h].cpu().numpy(), sz)
            assert np.array_equal(st.offsets[s, h].cpu().numpy(), of)
            assert np.array_equal(st.sorted_idx[s, h, :n_clustered].cpu().numpy(), si)
            for j in range(n_events):
                seg = lab[N0 + j * m:N0 + (j + 1) * m]
                assert seg.min() >= C0 + j * Cp and seg.max() < C0 + (j + 1) * Cp
            keys = np64(w.K[s, h, :n_clustered])
            mu_o, _ = O.update(keys, lab, np.zeros((st.n_clusters, 128)))
            got = np64(st.centroids[s, h])
            nz = sz > 0
            assert np.abs(got[nz] - mu_o[nz]).max() <= 2.0 ** -8 * np.abs(mu_o).max()
    print(f"incremental decode: {checked} head-problem steps checked, {near} selection near-ties, "
          f"worst attention rel err {worst:.2e}")
