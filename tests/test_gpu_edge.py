"""Edge cases of the GPU path: degenerate cluster counts, ragged tiles on both
assignment tile sizes, exact ties, zero keys, reproducibility, clamped inputs."""
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


def bf16_dev(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(DEV)


@pytest.mark.parametrize("N,C,Hkv", [(1000, 1, 1), (300, 300, 1), (70001, 64, 1), (1537, 33, 3),
                                     (2048, 2048, 1), (5000, 512, 1), (5000, 513, 1),
                                     (40000, 500, 2), (70, 5, 1)])
def test_cluster_keys_shapes(N, C, Hkv):
    """C = 1 (global mean), C = N (every token its own cluster), a token count that is
    not a multiple of either assignment tile (512 for large problems, 128 for small),
    the largest supported cluster count; the largest table the streaming assignment
    kernel keeps in LDS (512 rows), one row more (the chunk-streaming kernel), a ragged
    last tile at full LDS occupancy with several blocks per workgroup, and fewer tokens
    than one 64-key task."""
    cfg = Config("edge", 1, 1, Hkv, Hkv, 128, N, max(4, min(C, 64)), C, 3, 64, seed=N % 97)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, C, cfg.seed)
    sh = ck.Shape(1, Hkv, Hkv, N, C)
    st = ck.ClusterState(sh, DEV, budget=64)
    st.cluster(w.K, init.to(DEV), 0, N, C, cfg.n_iter)
    torch.cuda.synchronize()
    for h in range(Hkv):
        keys = np64(w.K[0, h])
        lab = st.labels[0, h].cpu().numpy()
        sizes, offs, sidx = O.build_metadata(lab, C)
        assert np.array_equal(st.sizes[0, h].cpu().numpy(), sizes)
        assert np.array_equal(st.offsets[0, h].cpu().numpy(), offs)
        assert np.array_equal(st.sorted_idx[0, h].cpu().numpy(), sidx)
        mu_o, _ = O.update(keys, lab, np.zeros((C, 128)))
        got = np64(st.centroids[0, h])
        nz = sizes > 0
        assert np.abs(got[nz] - mu_o[nz]).max() <= 2.0 ** -8 * np.abs(mu_o).max() + 1e-30
        if C == 1:
            assert np.all(lab == 0)
        if C == N:
            assert np.all(sizes == 1)                      # every token stays its own cluster
            assert np.array_equal(init[0, h].numpy()[lab], np.arange(N))
        # one more teacher-forced assignment from the final centroids, all keys checked
        mu_hat = O.round_to_bf16(O.unit_rows(got))
        hat = torch.zeros(1, Hkv, C, 128, dtype=torch.bfloat16, device=DEV)
        hat[0, h] = bf16_dev(mu_hat)
        lab2 = torch.zeros_like(st.labels)
        ck.ck_kmeans_assign(sh, w.K, 0, N, hat, 0, C, lab2)
        lo, _, gap = O.assign(keys, mu_hat)
        bad = (lab2[0, h].cpu().numpy() != lo) & (gap >= 1e-4)
        assert not bad.any()


@pytest.mark.parametrize("N", [600, 70000])
def test_assignment_exact_ties_and_zero_keys(N):
    """Duplicated centroids give bit-identical similarities: the lower id must win,
    wherever the two copies sit (same tile, other half of the tile, another tile).
    An all-zero key scores 0 against everything and gets label 0."""
    C = 200
    rng = np.random.default_rng(3)
    mu = rng.normal(size=(C, 128))
    mu_hat = O.round_to_bf16(O.unit_rows(mu))
    # (11, 34), (18, 65): same lane half, LATER tile, LOWER accumulator slot -- the copy in
    # the later tile carries the larger slot bits and must still lose; (7, 97): other half
    pairs = [(0, 1), (2, 6), (3, 35), (10, 150), (64, 199), (31, 32), (11, 34), (18, 65),
             (7, 97)]
    for a, b in pairs:
        mu_hat[b] = mu_hat[a]
    K = torch.randn(1, 1, N, 128, device=DEV).to(torch.bfloat16)
    K[0, 0, 5] = 0
    K[0, 0, N - 1] = 0
    # make sure many keys actually pick a duplicated centroid
    for j, (a, b) in enumerate(pairs):
        K[0, 0, 20 + j] = bf16_dev(3.0 * mu_hat[a])
    sh = ck.Shape(1, 1, 1, N, C)
    hat = bf16_dev(mu_hat)[None, None].contiguous()
    lab = torch.full((1, 1, N), -1, dtype=torch.int32, device=DEV)
    ck.ck_kmeans_assign(sh, K, 0, N, hat, 0, C, lab)
    got = lab[0, 0].cpu().numpy()
    lo, _, gap = O.assign(np64(K[0, 0]), mu_hat)
    dup_hi = {b for _, b in pairs}
    assert not (set(got.tolist()) & dup_hi)                 # the higher copy never wins
    assert got[5] == 0 and got[N - 1] == 0
    for j, (a, b) in enumerate(pairs):
        assert got[20 + j] == a
    # everything else as usual; exact ties (gap 0) are decided identically by both sides
    exact = (gap == 0.0)
    assert np.array_equal(got[exact], lo[exact])
    assert not ((got != lo) & (gap >= 1e-4)).any()


def test_clustering_is_bit_reproducible():
    cfg = Config("rep", 1, 2, 2, 2, 128, 5000, 40, 40, 5, 64, seed=5)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed).to(DEV)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    outs = []
    for _ in range(3):
        st = ck.ClusterState(sh, DEV, budget=64)
        st.cluster(w.K, init, 0, cfg.N, cfg.C, cfg.n_iter)
        torch.cuda.synchronize()
        outs.append(st)
    for st in outs[1:]:
        assert torch.equal(st.labels, outs[0].labels)
        assert torch.equal(st.sorted_idx, outs[0].sorted_idx)
        assert torch.equal(st.centroids.view(torch.int16), outs[0].centroids.view(torch.int16))


def test_attention_clamps_bad_counts_and_indices():
    """n_tokens above max_tokens is clamped; token ids outside [0, N_cap) are clamped to
    a valid row: the call must stay in bounds whatever the index buffer holds."""
    S, Hkv, Hq, N = 1, 2, 4, 300
    K = torch.randn(S, Hkv, N, 128, device=DEV).to(torch.bfloat16)
    V = torch.randn(S, Hkv, N, 128, device=DEV).to(torch.bfloat16)
    q = torch.randn(S, Hq, 128, device=DEV).to(torch.bfloat16)
    sh = ck.Shape(S, Hq, Hkv, N, 4)
    idx = torch.tensor([[[0, 7, -5, 10 ** 6] + [3] * 60, [1, 2, 3, 4] + [299] * 60]],
                       dtype=torch.int32, device=DEV)
    n_tok = torch.tensor([[4, 1000]], dtype=torch.int32, device=DEV)
    out = torch.zeros(S, Hq, 128, dtype=torch.bfloat16, device=DEV)
    ck.ck_sparse_decode_attn(sh, q, K, V, idx, n_tok, 64, out)
    torch.cuda.synchronize()
    want0 = O.attention_over(np64(q[0, 0:2]), np64(K[0, 0]), np64(V[0, 0]), [0, 7, 0, N - 1])
    want1 = O.attention_over(np64(q[0, 2:4]), np64(K[0, 1]), np64(V[0, 1]),
                             [1, 2, 3, 4] + [299] * 60)
    got = np64(out[0])
    for g, w in ((slice(0, 2), want0), (slice(2, 4), want1)):
        err = np.abs(got[g] - w).max() / np.abs(w).max()
        assert err <= 2e-2


@pytest.mark.parametrize("G,dtype", [(8, ck.CK_BF16), (8, ck.CK_F32), (1, ck.CK_F32)])
def test_fused_decode_other_group_sizes(G, dtype):
    Hkv, S, N, C, B = 2, 2, 2000, 60, 300
    Hq = Hkv * G
    tdt = torch.bfloat16 if dtype == ck.CK_BF16 else torch.float32
    rng = np.random.default_rng(G)
    g = torch.Generator(device=DEV).manual_seed(G)
    K = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn(S, Hkv, N, 128, generator=g, device=DEV).to(torch.bfloat16)
    q = torch.randn(S, Hq, 128, generator=g, device=DEV).to(torch.bfloat16)
    sh = ck.Shape(S, Hq, Hkv, N, C, dtype=dtype)
    st = ck.ClusterState(sh, DEV, budget=B, n_sink=8)
    tabs = {}
    for s in range(S):
        for h in range(Hkv):
            lab = rng.integers(0, C, N - 8)
            sizes, offs, sidx = O.build_metadata(lab, C, tok_begin=8)
            mu, _ = O.update(np64(K[s, h, 8:]), lab, np.zeros((C, 128)))
            mu = O.round_to_bf16(mu)
            st.centroids[s, h] = torch.from_numpy(mu.astype(np.float32)).to(tdt).to(DEV)
            st.sizes[s, h] = torch.from_numpy(sizes.astype(np.int32)).to(DEV)
            st.offsets[s, h] = torch.from_numpy(offs.astype(np.int32)).to(DEV)
            st.sorted_idx[s, h, :N - 8] = torch.from_numpy(sidx.astype(np.int32)).to(DEV)
            tabs[(s, h)] = (mu, sizes, offs, sidx)
    st.n_clusters = C
    out = ck.decode_step(st, q.to(tdt), K.to(tdt), V.to(tdt), n_sink=8)
    torch.cuda.synchronize()
    for (s, h), (mu, sizes, offs, sidx) in tabs.items():
        qg = np64(q[s, h * G:(h + 1) * G])
        r = O.decode_step(qg, np64(K[s, h]), np64(V[s, h]), mu, sizes, offs, sidx, B, n_sink=8)
        n = int(st.n_tokens[s, h])
        got_idx = st.token_idx[s, h, :n].cpu().numpy()
        if not O.selection_near_tie(r["scores"], r["order"], r["n_sel"]):
            assert np.array_equal(got_idx, r["idx"])
        want = O.sparse_attention(qg, np64(K[s, h]), np64(V[s, h]), got_idx, n_sink=8)
        got = np64(out[s, h * G:(h + 1) * G])
        tol = 2e-2 if dtype == ck.CK_BF16 else 1e-5
        assert (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max() <= tol


def test_mfma_probe_runs():
    sink = torch.zeros(4, device=DEV)
    flops = ck.ck_probe_mfma_bf16(64, 10, sink)
    torch.cuda.synchronize()
    assert flops == 64 * 4 * 16 * 10 * 32768
    assert float(sink.abs().sum()) == 0.0
