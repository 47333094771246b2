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


def bf16_dev(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(DEV)


def test_assignment_many_head_problems_all_keys_teacher_forced():
    """The launch shape of the full-depth and batch-16 configurations (64 head-problems,
    C = 400: the streaming kernel with the table in LDS, several 512-token blocks per
    workgroup): every key of three head-problems against the oracle's labels, given the
    oracle's own unit centroids of its second iteration."""
    c2 = get_config(2)
    cfg = Config("assign_64hp", 1, c2.S, c2.Hkv, c2.Hq, c2.d, c2.N, c2.M, c2.C, 2, c2.B, 202)
    assert cfg.S * cfg.Hkv == 64 and cfg.N == 32768 and cfg.C == 400
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    picks = [(0, 0), (4, 3), (7, 7)]
    hat = torch.zeros(cfg.S, cfg.Hkv, cfg.C, 128, dtype=torch.bfloat16, device=DEV)
    traces = {}
    for s, h in picks:
        _, _, _, tr = O.kmeans(np64(w.K[s, h]), init[s, h].numpy(), 2, "bf16")
        traces[s, h] = tr
        hat[s, h] = bf16_dev(tr.mu_hat[1])
    lab = torch.full((cfg.S, cfg.Hkv, cfg.N), -1, dtype=torch.int32, device=DEV)
    best = torch.zeros(cfg.S, cfg.Hkv, cfg.N, dtype=torch.float32, device=DEV)
    ck.ck_kmeans_assign(sh, w.K, 0, cfg.N, hat, 0, cfg.C, lab, best)
    torch.cuda.synchronize()
    flagged = 0
    for s, h in picks:
        tr = traces[s, h]
        got = lab[s, h].cpu().numpy()
        near = tr.gap[1] < 1e-4
        bad = (got != tr.labels[1]) & ~near
        assert not bad.any(), f"head-problem {(s, h)}: {bad.sum()} mismatches off near-ties"
        want_best = (np64(w.K[s, h]) * tr.mu_hat[1][tr.labels[1]]).sum(axis=1)
        assert np.allclose(best[s, h].cpu().numpy()[~near], want_best[~near], rtol=1e-5, atol=1e-5)
        flagged += int(near.sum())
    assert flagged < 0.01 * len(picks) * cfg.N              # the exact check is not vacuous
    print(f"assignment, 64 head-problems: near-tie keys {flagged}/{len(picks) * cfg.N}")
    # a head-problem whose table is all zero: every similarity ties at 0, lowest id wins
    assert int(lab[1, 1].max()) == 0 and int(lab[1, 1].min()) == 0


@pytest.mark.parametrize("C", [600, 1100])
def test_assignment_chunk_streaming_kernel_all_keys_teacher_forced(C):
    """Tables of more than 512 centroids take the kernel that streams the table through
    LDS in chunks: with 16 head-problems of 32768 tokens (more 1024-token tiles than
    compute units) C = 600 runs its four-wavefront form, C = 1100 the eight-wavefront one.
    Every key of two head-problems against the oracle, given unit centroids made from
    sampled key rows."""
    S, Hkv, N = 2, 8, 32768
    cfg = Config("assign_chunks", 1, S, Hkv, Hkv, 128, N, 1024, C, 1, 256, seed=400 + C)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, C, cfg.seed)
    sh = ck.Shape(S, Hkv, Hkv, N, C)
    picks = [(0, 1), (1, 6)]
    hat = torch.zeros(S, Hkv, C, 128, dtype=torch.bfloat16, device=DEV)
    tables = {}
    for s, h in picks:
        mu_hat = O.round_to_bf16(O.unit_rows(np64(w.K[s, h])[init[s, h].numpy()]))
        tables[s, h] = mu_hat
        hat[s, h] = bf16_dev(mu_hat)
    lab = torch.full((S, Hkv, N), -1, dtype=torch.int32, device=DEV)
    ck.ck_kmeans_assign(sh, w.K, 0, N, hat, 0, C, lab)
    torch.cuda.synchronize()
    flagged = 0
    for s, h in picks:
        lo, _, gap = O.assign(np64(w.K[s, h]), tables[s, h])
        near = gap < 1e-4
        bad = (lab[s, h].cpu().numpy() != lo) & ~near
        assert not bad.any(), f"C={C} head-problem {(s, h)}: {bad.sum()} mismatches off near-ties"
        flagged += int(near.sum())
    assert flagged < 0.01 * len(picks) * N
    print(f"assignment, C={C}, 16 head-problems: near-tie keys {flagged}/{len(picks) * N}")


@pytest.mark.parametrize("S,Hkv,C", [(1, 2, 200), (2, 8, 200), (1, 2, 600), (2, 8, 600)])
def test_l2_assignment_large_tiles_all_keys(S, Hkv, C):
    """The l2 metric (bias -|mu|^2/2 added in the assignment read-out) at 32768 tokens per
    head-problem: C = 200 takes the streaming kernel (table in LDS), C = 600 the
    chunk-streaming one, with 2 head-problems in its eight-wavefront form and with 16 in
    its four-wavefront form.  One iteration from the given initial rows is a teacher-forced
    assignment: the labels must be the oracle's nearest stored centroid off near-ties."""
    N = 32768
    cfg = Config("l2_big", 1, S, Hkv, Hkv, 128, N, 256, C, 1, 256, seed=31 + S)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, C, cfg.seed)
    sh = ck.Shape(S, Hkv, Hkv, N, C)
    st = ck.ClusterState(sh, DEV, budget=256)
    st.cluster(w.K, init.to(DEV), 0, N, C, 1, flags=ck.CK_METRIC_L2)
    torch.cuda.synchronize()
    flagged = 0
    for s, h in [(0, 0), (S - 1, Hkv - 1)]:
        keys = np64(w.K[s, h])
        table = O.round_to_bf16(keys[init[s, h].numpy()])
        lo, gap = O.assign_metric(keys, table, O.L2)
        got = st.labels[s, h].cpu().numpy()
        near = gap < 1e-4
        bad = (got != lo) & ~near
        assert not bad.any(), f"head-problem {(s, h)}: {bad.sum()} mismatches off near-ties"
        flagged += int(near.sum())
        sizes, offs, sidx = O.build_metadata(got, C)
        assert np.array_equal(st.sizes[s, h].cpu().numpy(), sizes)
        assert np.array_equal(st.sorted_idx[s, h].cpu().numpy(), sidx)
    assert flagged < 0.01 * 2 * N
    print(f"l2 assignment, {S * Hkv} head-problems: near-tie keys {flagged}/{2 * N}")


def test_llama_layer_every_iteration_teacher_forced_all_heads():
    """The 32k layer (the configuration the benchmark is quoted on), all 8 heads, all 10
    iterations: every assignment given the oracle's unit centroids of that iteration (all
    keys, labels exact off near-ties), every update given the oracle's labels (sizes exact,
    fp32 means within 1e-5 of the fp64 ones); then the free-running call against the
    oracle's own trajectory (label agreement and objective ratio, as for the small cases)."""
    cfg = get_config(1)
    w = MixtureWorkload(cfg, device=DEV)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    H, N, C = cfg.Hkv, cfg.N, cfg.C
    keys = [np64(w.K[0, h]) for h in range(H)]
    runs = [O.kmeans(keys[h], init[0, h].numpy(), cfg.n_iter, "bf16") for h in range(H)]
    flagged = 0
    for t in range(cfg.n_iter):
        hat = torch.stack([bf16_dev(runs[h][3].mu_hat[t]) for h in range(H)])[None].contiguous()
        lab = torch.full((1, H, N), -1, dtype=torch.int32, device=DEV)
        ck.ck_kmeans_assign(sh, w.K, 0, N, hat, 0, C, lab)
        lab_in = torch.stack([torch.from_numpy(runs[h][3].labels[t].astype(np.int32))
                              for h in range(H)])[None].contiguous().to(DEV)
        sizes_d = torch.zeros(1, H, C, dtype=torch.int32, device=DEV)
        offs_d = torch.zeros(1, H, C + 1, dtype=torch.int32, device=DEV)
        sidx_d = torch.zeros(1, H, N, dtype=torch.int32, device=DEV)
        ck.ck_build_metadata(sh, lab_in, 0, N, 0, C, sizes_d, offs_d, sidx_d)
        prev = [runs[h][3].mu[t - 1] if t else keys[h][init[0, h].numpy()] for h in range(H)]
        cent = torch.stack([bf16_dev(p) for p in prev])[None].contiguous()
        hat_out = torch.zeros_like(cent)
        f32 = torch.stack([torch.from_numpy(p.astype(np.float32)) for p in prev])[None] \
            .contiguous().to(DEV)
        ck.ck_kmeans_update(sh, w.K, sizes_d, offs_d, sidx_d, 0, C, cent, hat_out, f32)
        torch.cuda.synchronize()
        for h in range(H):
            tr = runs[h][3]
            got = lab[0, h].cpu().numpy()
            near = tr.gap[t] < 1e-4
            bad = (got != tr.labels[t]) & ~near
            assert not bad.any(), f"head {h} iteration {t}: {bad.sum()} label mismatches"
            flagged += int(near.sum())
            assert np.array_equal(sizes_d[0, h].cpu().numpy(), tr.sizes[t])
            want = tr.mu[t]
            assert np.abs(np64(f32[0, h]) - want).max() <= 1e-5 * np.abs(want).max()
            nz = tr.sizes[t] > 0
            assert np.abs(np64(cent[0, h])[nz] - want[nz]).max() <= 2.0 ** -8 * np.abs(want).max()
    total = cfg.n_iter * H * N
    assert flagged < 0.01 * total
    print(f"32k layer, teacher-forced: near-tie keys {flagged}/{total} = {flagged / total:.2e}")
    # free-running
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    st.cluster(w.K, init.to(DEV), 0, N, C, cfg.n_iter)
    torch.cuda.synchronize()
    for h in range(H):
        mu_o, lab_o, _, tr = runs[h]
        lab = st.labels[0, h].cpu().numpy()
        got = np64(st.centroids[0, h])
        agree = float((lab_o == lab).mean())
        J_gpu = O.weighted_objective(keys[h], O.unit_rows(got), lab)
        print(f"32k layer head {h}: free-running label agreement {agree:.4f}, "
              f"J gpu/oracle {J_gpu / tr.J[-1]:.6f}")
        assert agree > 0.9
        assert abs(J_gpu / tr.J[-1] - 1) < 2e-2
