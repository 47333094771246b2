"""Randomised sweep of the whole path on small shapes: random batch, head counts, GQA group,
context, cluster count, budget, sinks, recent window and budget mode.  Every case checks
the clustering invariants, fused == three-call decode (bit for bit) and the decode step
against the oracle on the GPU's own tables (index lists exact off near-ties, attention
within tolerance)."""
import os

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


N_SEEDS = int(os.environ.get("CK_SWEEP_SEEDS", "300"))    # more seeds for a longer soak


@pytest.mark.parametrize("seed", range(N_SEEDS))
def test_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    S = int(rng.integers(1, 3))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 4, 8]))
    N = int(rng.integers(40, 3000))
    n_sink = int(rng.choice([0, 0, 5, 16]))
    n_recent = int(rng.choice([0, 0, 7, 33]))
    if N - n_sink - n_recent < 2:                         # always something to cluster
        N = n_sink + n_recent + 2
    n_clu_tok = N - n_sink - n_recent
    C = int(rng.integers(1, min(n_clu_tok, 300) + 1))
    B = int(rng.integers(1, n_clu_tok + 50))
    mode = int(rng.choice([ck.CK_SEL_WHOLE, ck.CK_SEL_TRIM_LAST]))
    n_iter = int(rng.integers(1, 5))
    cfg = Config(f"r{seed}", 1, S, Hkv, Hkv * G, 128, N, max(2, C // 2), C, n_iter, B, seed)
    w = MixtureWorkload(cfg, device=DEV)
    sh = ck.Shape(S, Hkv * G, Hkv, N, C)
    st = ck.ClusterState(sh, DEV, budget=B, max_recent=n_recent, n_sink=n_sink)
    init = sample_init_indices(w.K, C, seed, n_sink, n_clu_tok)
    st.cluster(w.K, init.to(DEV), n_sink, n_clu_tok, C, n_iter)
    q = w.query()
    rb, re = N - n_recent, N
    out_f = ck.decode_step(st, q, w.K, w.V, flags=mode, n_sink=n_sink, recent_begin=rb,
                           recent_end=re, fused=True).clone()
    idx_f, n_f = st.token_idx.clone(), st.n_tokens.clone()
    out_3 = ck.decode_step(st, q, w.K, w.V, flags=mode, n_sink=n_sink, recent_begin=rb,
                           recent_end=re, fused=False).clone()
    torch.cuda.synchronize()
    assert torch.equal(out_f, out_3)
    assert torch.equal(n_f, st.n_tokens)
    for s in range(S):
        for h in range(Hkv):
            n = int(n_f[s, h])
            assert torch.equal(idx_f[s, h, :n], st.token_idx[s, h, :n])
            keys, vals = np64(w.K[s, h]), np64(w.V[s, h])
            lab = st.labels[s, h, n_sink:n_sink + n_clu_tok].cpu().numpy()
            sizes, offs, sidx = O.build_metadata(lab, C, tok_begin=n_sink)
            assert st.sizes[s, h].cpu().numpy().tolist() == sizes.tolist()
            assert st.offsets[s, h].cpu().numpy().tolist() == offs.tolist()
            assert st.sorted_idx[s, h, :n_clu_tok].cpu().numpy().tolist() == sidx.tolist()
            mu = np64(st.centroids[s, h])
            for c in range(C):
                if sizes[c]:
                    want = keys[n_sink:n_sink + n_clu_tok][lab == c].mean(axis=0)
                    assert np.allclose(mu[c], want, rtol=2 ** -7, atol=2e-3)
            qg = np64(q[s, h * G:(h + 1) * G])
            r = O.decode_step(qg, keys, vals, mu, sizes, offs, sidx, B, mode, n_sink, rb, re)
            got_idx = idx_f[s, h, :n].cpu().numpy()
            if not O.selection_near_tie(r["scores"], r["order"], r["n_sel"]):
                assert got_idx.tolist() == r["idx"].tolist()
            assert n <= B and (mode == ck.CK_SEL_WHOLE or n == min(B, n_clu_tok))
            want = O.sparse_attention(qg, keys, vals, got_idx, n_sink, rb, re)
            got = np64(out_f[s, h * G:(h + 1) * G])
            if len(got_idx) + n_sink + n_recent == 0:
                assert (got == 0).all()
            else:
                err = (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max()
                assert err <= 2e-2, err


N_MID = int(os.environ.get("CK_SWEEP_MID_SEEDS", "12"))


@pytest.mark.parametrize("seed", range(N_MID))
def test_random_midsize_assignment(seed):
    """Random mid-size clustering problems (thousands to tens of thousands of tokens, up to
    24 head-problems, up to 700 clusters, cosine or l2), one iteration from the given
    initial rows: a teacher-forced assignment in whatever kernel and launch shape the sizes
    select (table in LDS with one or several blocks per workgroup, or the table streamed in
    chunks).  Every key of two head-problems against the oracle, metadata exact."""
    rng = np.random.default_rng(7000 + seed)
    S = int(rng.integers(1, 4))
    Hkv = int(rng.integers(1, 9))
    N = int(rng.integers(3000, 60000))
    C = int(rng.integers(2, 700))
    l2 = bool(rng.integers(0, 2))
    cfg = Config(f"m{seed}", 1, S, Hkv, Hkv, 128, N, max(2, C // 2), C, 1, 64, 900 + seed)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, C, cfg.seed)
    sh = ck.Shape(S, Hkv, Hkv, N, C)
    st = ck.ClusterState(sh, DEV, budget=64)
    st.cluster(w.K, init.to(DEV), 0, N, C, 1, flags=ck.CK_METRIC_L2 if l2 else 0)
    torch.cuda.synchronize()
    for s, h in {(0, 0), (S - 1, Hkv - 1)}:
        keys = np64(w.K[s, h])
        rows = keys[init[s, h].numpy()]
        if l2:
            lo, gap = O.assign_metric(keys, O.round_to_bf16(rows), O.L2)
        else:
            lo, _, gap = O.assign(keys, O.round_to_bf16(O.unit_rows(rows)))
        got = st.labels[s, h].cpu().numpy()
        near = gap < 1e-4
        bad = (got != lo) & ~near
        assert not bad.any(), f"seed {seed} S={S} Hkv={Hkv} N={N} C={C} l2={l2}: {bad.sum()} mismatches"
        assert near.sum() < 0.02 * N
        sizes, offs, sidx = O.build_metadata(got, C)
        assert np.array_equal(st.sizes[s, h].cpu().numpy(), sizes)
        assert np.array_equal(st.offsets[s, h].cpu().numpy(), offs)
        assert np.array_equal(st.sorted_idx[s, h].cpu().numpy(), sidx)


@pytest.mark.parametrize("seed", range(N_MID))
def test_random_midsize_decode(seed):
    """Random mid-size decode steps (up to 96 head-problems, contexts of thousands to tens
    of thousands of tokens, up to 700 clusters, budgets up to 2048, both budget modes,
    sinks and a recent window): the one-launch step against the three calls bit for bit
    on every head-problem, and against the oracle on the GPU's own tables for three of
    them.  Covers the split counts, the one-wavefront selection and its fallback, and
    tables above 512 clusters (scores computed by a kernel of their own)."""
    rng = np.random.default_rng(9000 + seed)
    S = int(rng.integers(1, 13))
    Hkv = int(rng.integers(1, 9))
    G = int(rng.choice([1, 2, 4, 8]))
    N = int(rng.integers(2000, 40000))
    n_sink = int(rng.choice([0, 0, 16]))
    n_recent = int(rng.choice([0, 0, 40, 319]))
    n_clu_tok = N - n_sink - n_recent
    C = int(rng.integers(2, 700))
    B = int(rng.integers(16, 2049))
    mode = int(rng.choice([ck.CK_SEL_WHOLE, ck.CK_SEL_TRIM_LAST]))
    cfg = Config(f"d{seed}", 1, S, Hkv, Hkv * G, 128, N, max(2, C // 2), C, 2, B, 300 + seed)
    w = MixtureWorkload(cfg, device=DEV)
    sh = ck.Shape(S, Hkv * G, Hkv, N, C)
    st = ck.ClusterState(sh, DEV, budget=B, max_recent=n_recent, n_sink=n_sink)
    init = sample_init_indices(w.K, C, cfg.seed, n_sink, n_clu_tok)
    st.cluster(w.K, init.to(DEV), n_sink, n_clu_tok, C, 2)
    q = w.query()
    rb, re = N - n_recent, N
    out_f = ck.decode_step(st, q, w.K, w.V, flags=mode, n_sink=n_sink, recent_begin=rb,
                           recent_end=re, fused=True).clone()
    idx_f, n_f = st.token_idx.clone(), st.n_tokens.clone()
    out_3 = ck.decode_step(st, q, w.K, w.V, flags=mode, n_sink=n_sink, recent_begin=rb,
                           recent_end=re, fused=False).clone()
    torch.cuda.synchronize()
    what = f"seed {seed} S={S} Hkv={Hkv} G={G} N={N} C={C} B={B} mode={mode}"
    assert torch.equal(out_f, out_3), what
    assert torch.equal(n_f, st.n_tokens), what
    for s in range(S):
        for h in range(Hkv):
            n = int(n_f[s, h])
            assert torch.equal(idx_f[s, h, :n], st.token_idx[s, h, :n]), what
    if mode == ck.CK_SEL_WHOLE and n_sink == 0 and n_recent == 0:
        # the cached step (rows copied into a dense buffer first) gives the same bits; a
        # cold cache misses every recalled token, the same query again none
        cache = ck.ClusterCache(sh, DEV, cap_tokens=B)
        ck.ck_cache_reset(sh, cache)
        out_c = ck.cached_decode_step(st, cache, q, w.K, w.V).clone()
        miss1 = cache.miss_tokens.clone()
        out_c2 = ck.cached_decode_step(st, cache, q, w.K, w.V).clone()
        torch.cuda.synchronize()
        assert torch.equal(out_c, out_f) and torch.equal(out_c2, out_f), what
        assert torch.equal(miss1, n_f) and int(cache.miss_tokens.sum()) == 0, what
    picks = {(0, 0), (S - 1, Hkv - 1), (S // 2, Hkv // 2)}
    for s, h in picks:
        n = int(n_f[s, h])
        keys, vals = np64(w.K[s, h]), np64(w.V[s, h])
        lab = st.labels[s, h, n_sink:n_sink + n_clu_tok].cpu().numpy()
        sizes, offs, sidx = O.build_metadata(lab, C, tok_begin=n_sink)
        assert np.array_equal(st.sizes[s, h].cpu().numpy(), sizes), what
        assert np.array_equal(st.sorted_idx[s, h, :n_clu_tok].cpu().numpy(), sidx), what
        mu = np64(st.centroids[s, h])
        qg = np64(q[s, h * G:(h + 1) * G])
        r = O.decode_step(qg, keys, vals, mu, sizes, offs, sidx, B, mode, n_sink, rb, re)
        got_idx = idx_f[s, h, :n].cpu().numpy()
        if not O.selection_near_tie(r["scores"], r["order"], r["n_sel"]):
            assert np.array_equal(got_idx, r["idx"]), what
        assert n <= B and (mode == ck.CK_SEL_WHOLE or n == min(B, n_clu_tok)), what
        want = O.sparse_attention(qg, keys, vals, got_idx, n_sink, rb, re)
        got = np64(out_f[s, h * G:(h + 1) * G])
        if len(got_idx) + n_sink + n_recent == 0:           # nothing fits the budget: zeros
            assert (got == 0).all(), what
        else:
            err = (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max()
            assert err <= 2e-2, (what, err)
