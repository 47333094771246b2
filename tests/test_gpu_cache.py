"""GPU tests of the cluster-granularity cache (paper Sections IV-A, IV-D): the home copy
of K/V lives in pinned host memory and is read by the GPU itself; every step must
reproduce the output of the uncached decode step bit for bit, and the rows it reports
as loaded must be exactly those of the clusters the previous step did not hold (the
oracle's cache model applied to the GPU's own selections)."""
import numpy as np
import pytest
import torch

import paper_2412_03213_amd as ck
from ck_synth import Config, MixtureWorkload, sample_init_indices
from oracle import clusterkv_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def clustered(cfg, dtype=torch.bfloat16):
    w = MixtureWorkload(cfg, device=DEV)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, DEV, budget=cfg.B)
    init = sample_init_indices(w.K, cfg.C, cfg.seed).to(DEV)
    st.cluster(w.K, init, 0, cfg.N, cfg.C, 4)
    return w, sh, st


@pytest.mark.parametrize("home", ["pinned_host", "device"])
@pytest.mark.parametrize("S,Hkv,G,N,C,B", [(2, 2, 4, 3000, 40, 512), (1, 2, 1, 2048 + 37, 50, 300),
                                           (1, 1, 8, 700, 700, 64)])
def test_cached_steps_equal_uncached_and_count_misses(home, S, Hkv, G, N, C, B):
    cfg = Config("cache", 1, S, Hkv, Hkv * G, 128, N, 32, C, 10, B, 9)
    w, sh, st = clustered(cfg)
    HP = S * Hkv
    if home == "pinned_host":
        Kh = torch.empty(w.K.shape, dtype=w.K.dtype, pin_memory=True)
        Vh = torch.empty(w.V.shape, dtype=w.V.dtype, pin_memory=True)
        Kh.copy_(w.K)
        Vh.copy_(w.V)
        torch.cuda.synchronize()
        K_home, V_home = ck.ck_host_device_ptr(Kh), ck.ck_host_device_ptr(Vh)
    else:
        K_home, V_home = w.K, w.V
    cache = ck.ClusterCache(sh, DEV, cap_tokens=B + 5)
    ck.ck_cache_reset(sh, cache)
    ref = ck.ClusterState(sh, DEV, budget=B)            # same tables, uncached path
    for name in ("centroids", "sizes", "offsets", "sorted_idx"):
        getattr(ref, name).copy_(getattr(st, name))
    ref.n_clusters = st.n_clusters
    sizes = st.sizes.view(HP, -1).cpu().numpy()
    held = [[] for _ in range(HP)]
    total_hit = total = 0
    for step in range(8):
        q = w.query(sticky=0.7)
        out = ck.cached_decode_step(st, cache, q, K_home, V_home).clone()
        want = ck.decode_step(ref, q, w.K, w.V).clone()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"step {step}"
        n_sel = st.n_sel_clusters.view(HP).cpu().numpy()
        sel = st.sel_clusters.view(HP, -1).cpu().numpy()
        n_tok = st.n_sel_tokens.view(HP).cpu().numpy()
        miss = cache.miss_tokens.view(HP).cpu().numpy()
        for hp in range(HP):
            assert n_sel[hp] == int(ref.n_sel_clusters.view(HP)[hp])
            cur = sel[hp, :n_sel[hp]]
            hit_w, miss_w, held[hp] = O.cache_step(held[hp], cur, sizes[hp])
            assert miss[hp] == miss_w and n_tok[hp] == hit_w + miss_w
            if step == 0:
                assert miss[hp] == n_tok[hp]            # cold cache
            total_hit += hit_w
            total += hit_w + miss_w
            g = (cache.step - 1) & 1
            assert int(cache.n_held[g].view(HP)[hp]) == n_sel[hp]
            assert cache.clusters[g].view(HP, -1)[hp, :n_sel[hp]].cpu().tolist() == cur.tolist()
            # the cache rows are the recalled K rows in recalled order
            idx = ref.token_idx.view(HP, -1)[hp, :n_tok[hp]].long()
            s_, h_ = divmod(hp, Hkv)
            assert torch.equal(cache.K[g][s_, h_, :n_tok[hp]], w.K[s_, h_][idx])
            assert torch.equal(cache.V[g][s_, h_, :n_tok[hp]], w.V[s_, h_][idx])
    assert total > 0


def test_same_query_twice_is_all_hits_and_reset_empties():
    cfg = Config("cache2", 1, 1, 2, 8, 128, 4096, 64, 51, 10, 1024, 4)
    w, sh, st = clustered(cfg)
    cache = ck.ClusterCache(sh, DEV, cap_tokens=1024)
    ck.ck_cache_reset(sh, cache)
    q = w.query()
    ck.cached_decode_step(st, cache, q, w.K, w.V)
    first = cache.miss_tokens.clone()
    out1 = st.out.clone()
    ck.cached_decode_step(st, cache, q, w.K, w.V)
    torch.cuda.synchronize()
    assert int(cache.miss_tokens.sum()) == 0
    assert torch.equal(first, st.n_sel_tokens)
    assert torch.equal(out1, st.out)
    ck.ck_cache_reset(sh, cache)
    ck.cached_decode_step(st, cache, q, w.K, w.V)
    torch.cuda.synchronize()
    assert torch.equal(cache.miss_tokens, st.n_sel_tokens)


def test_host_pointer_of_unpinned_memory_is_an_error():
    t = torch.empty(1024, dtype=torch.uint8)            # pageable
    with pytest.raises(ck.ClusterKVError) as e:
        ck.ck_host_device_ptr(t)
    assert e.value.code == -5
    torch.zeros(4, device=DEV).sum().item()             # the runtime is still healthy
