"""The remaining benchmark configurations at their full sizes, in the launch shapes
bench.py times; the oracle checks sampled head-problems one by one (metadata exactly,
sampled centroids, one teacher-forced assignment on sampled keys, the decode step)."""
import numpy as np
import pytest
import torch

import paper_2412_03213_amd as ck
from ck_synth import Config, MixtureWorkload, get_config, sample_init_indices
from oracle import clusterkv_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def np64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check_head_problem(cfg, w, st, q, out, s, h, rng, recent=(0, 0), n_clustered=None):
    C = st.n_clusters
    n_clustered = cfg.N if n_clustered is None else n_clustered
    keys, vals = np64(w.K[s, h]), np64(w.V[s, h])
    lab = st.labels[s, h, :n_clustered].cpu().numpy()
    sizes, offs, sidx = O.build_metadata(lab, C)
    assert np.array_equal(st.sizes[s, h, :C].cpu().numpy(), sizes)
    assert np.array_equal(st.offsets[s, h, :C + 1].cpu().numpy(), offs)
    assert np.array_equal(st.sorted_idx[s, h, :n_clustered].cpu().numpy(), sidx)
    mu = np64(st.centroids[s, h, :C])
    for c in rng.integers(0, C, 10):
        if sizes[c]:
            want = keys[sidx[offs[c]:offs[c + 1]]].mean(axis=0)
            assert np.abs(mu[c] - want).max() <= 2.0 ** -8 * np.abs(want).max() + 1e-6
    G = cfg.G
    qg = np64(q[s, h * G:(h + 1) * G])
    r = O.decode_step(qg, keys, vals, mu, sizes, offs, sidx, st.budget,
                      recent_begin=recent[0], recent_end=recent[1])
    n = int(st.n_tokens[s, h])
    got_idx = st.token_idx[s, h, :n].cpu().numpy()
    near = O.selection_near_tie(r["scores"], r["order"], r["n_sel"])
    if not near:
        assert np.array_equal(got_idx, r["idx"])
    assert 0 < n <= st.budget
    want = O.sparse_attention(qg, keys, vals, got_idx, 0, recent[0], recent[1])
    got = np64(out[s, h * G:(h + 1) * G])
    err = (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max()
    assert err <= 2e-2, err
    return near


def test_long_context_128k_sampled():
    cfg = get_config(3)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    st.cluster(w.K, init.to(DEV), 0, cfg.N, cfg.C, cfg.n_iter)
    q = w.query()
    out = ck.decode_step(st, q, w.K, w.V)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    for h in (1, 6):
        check_head_problem(cfg, w, st, q, out, 0, h, rng)
    # teacher-forced assignment on sampled keys of one head, all 1600 centroids
    h = 4
    mu_hat = O.round_to_bf16(O.unit_rows(np64(st.centroids[0, h])))
    hat = torch.zeros(cfg.S, cfg.Hkv, cfg.C, 128, dtype=torch.bfloat16, device=DEV)
    hat[0, h] = torch.from_numpy(mu_hat.astype(np.float32)).to(torch.bfloat16).to(DEV)
    lab2 = torch.zeros_like(st.labels)
    ck.ck_kmeans_assign(sh, w.K, 0, cfg.N, hat, 0, cfg.C, lab2)
    sample = rng.permutation(cfg.N)[:4096]
    lo, _, gap = O.assign(np64(w.K[0, h])[sample], mu_hat)
    got = lab2[0, h].cpu().numpy()[sample]
    assert not ((got != lo) & (gap >= 1e-4)).any()


def test_full_depth_one_layer_sampled():
    c2 = get_config(2)
    cfg = Config("full_depth_one_layer", 1, c2.S, c2.Hkv, c2.Hq, c2.d, c2.N, c2.M, c2.C,
                 c2.n_iter, c2.B, c2.seed)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    st.cluster(w.K, init.to(DEV), 0, cfg.N, cfg.C, cfg.n_iter)
    q = w.query()
    out = ck.decode_step(st, q, w.K, w.V)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2)
    for s, h in [(0, 0), (3, 5), (7, 7), (5, 2)]:
        check_head_problem(cfg, w, st, q, out, s, h, rng)
    # every head-problem: structure of the clustering
    sizes = st.sizes.cpu().numpy()
    assert np.all(sizes.sum(axis=-1) == cfg.N)
    nt = st.n_tokens.cpu().numpy()
    assert np.all((nt > 0) & (nt <= cfg.B))


def test_full_depth_all_layers_as_one_batch_sampled():
    """All 32 layers x 8 sequences as ONE batch of 2048 head-problems, the launch shape of
    bench.py's full-depth leg (32 GiB of K+V): sampled head-problems against the oracle,
    structure of every head-problem."""
    c2 = get_config(2)
    cfg = Config("full_depth_32_layers", 1, c2.S * c2.layers, c2.Hkv, c2.Hq, c2.d, c2.N, c2.M,
                 c2.C, c2.n_iter, c2.B, c2.seed)
    assert cfg.S * cfg.Hkv == 2048
    w = MixtureWorkload(cfg, device=DEV)
    w.token_center = None
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    st.cluster(w.K, init.to(DEV), 0, cfg.N, cfg.C, cfg.n_iter)
    q = w.query()
    out = ck.decode_step(st, q, w.K, w.V)
    torch.cuda.synchronize()
    rng = np.random.default_rng(22)
    near = 0
    for s, h in [(0, 0), (255, 7), (100, 3), (31, 6), (200, 1)]:
        near += check_head_problem(cfg, w, st, q, out, s, h, rng)
    sizes = st.sizes.cpu().numpy()
    assert np.all(sizes.sum(axis=-1) == cfg.N)
    offs = st.offsets.cpu().numpy()
    assert np.all(offs[..., 0] == 0) and np.all(offs[..., -1] == cfg.N)
    assert np.all(np.diff(offs, axis=-1) == sizes)
    nt = st.n_tokens.cpu().numpy()
    assert np.all((nt > 0) & (nt <= cfg.B))
    assert bool(torch.isfinite(out.float()).all())
    print(f"full depth as one batch: selection near-ties {near}/5")


def test_incremental_decode_full_size_sampled():
    cfg = get_config(4)
    steps, m, cp = cfg.decode_steps, cfg.m_incr, cfg.c_incr
    w = MixtureWorkload(cfg, device=DEV, extra_tokens=steps)
    n_events = steps // m
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N + steps, cfg.C + n_events * cp)
    st = ck.ClusterState(sh, DEV, budget=cfg.B, max_recent=m)
    st.cluster(w.K, sample_init_indices(w.K, cfg.C, cfg.seed, 0, cfg.N).to(DEV), 0, cfg.N, cfg.C,
               cfg.n_iter)
    rng = np.random.default_rng(4)
    check_at = {1, 319, 320, 321, 640, 1000, steps}
    near = 0
    for t in range(1, steps + 1):
        w.append_token()
        q = w.query()
        rb = cfg.N + m * ((t - 1) // m)
        out = ck.decode_step(st, q, w.K, w.V, recent_begin=rb, recent_end=cfg.N + t)
        if t in check_at:
            torch.cuda.synchronize()
            for s, h in [(0, 0), (11, 6)]:
                near += check_head_problem(cfg, w, st, q, out, s, h, rng, recent=(rb, cfg.N + t),
                                           n_clustered=rb)
        if t % m == 0:
            tb = cfg.N + t - m
            st.cluster(w.K, sample_init_indices(w.K, cp, cfg.seed + t, tb, m).to(DEV), tb, m, cp,
                       cfg.n_iter)
    torch.cuda.synchronize()
    assert st.n_clusters == cfg.C + n_events * cp == 412
    print(f"incremental full size: selection near-ties {near}/{2 * len(check_at)}")
