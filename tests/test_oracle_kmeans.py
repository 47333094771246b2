"""Pins for the oracle's K-means (Section III-B): brute force against the
loop-only restatement, structural invariants, the objective that neither step
can increase, and special cases with a known answer."""
import numpy as np
import pytest
import torch

from oracle import clusterkv_oracle as O
from tests import loops


def mixture(rng, N, M, d, sigma=0.5):
    centers = rng.normal(size=(M, d))
    centers /= np.linalg.norm(centers, axis=1, keepdims=True)
    which = rng.integers(0, M, N)
    return 3.0 * centers[which] + sigma * rng.normal(size=(N, d)), centers, which


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e38 * 0 + 255.5]])
    x32 = x.astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(x32.astype(np.float64)), want)
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_to_bf16(1.00390625) == 1.0
    assert O.round_to_bf16(1.01171875) == 1.015625


@pytest.mark.parametrize("seed", range(5))
def test_kmeans_matches_loops(seed):
    rng = np.random.default_rng(seed)
    N, C, d = 48, 5, 8
    keys, _, _ = mixture(rng, N, 6, d)
    init = rng.permutation(N)[:C]
    mu, labels, sizes, tr = O.kmeans(keys, init, 4, storage="f64")
    lc, ll = loops.kmeans(keys.tolist(), init.tolist(), 4)
    assert ll == labels.tolist()
    assert np.allclose(lc, mu, rtol=1e-12, atol=1e-13)
    # a single step at a time as well
    la = loops.cosine_assign(keys.tolist(), tr.mu[0].tolist())
    assert la == O.assign(keys, O.unit_rows(tr.mu[0]))[0].tolist()


@pytest.mark.parametrize("storage", ["f64", "bf16"])
def test_kmeans_structure(storage):
    rng = np.random.default_rng(11)
    N, C, d = 600, 12, 32
    keys, _, _ = mixture(rng, N, 20, d)
    if storage == "bf16":
        keys = O.round_to_bf16(keys)
    init = rng.permutation(N)[:C]
    mu, labels, sizes, tr = O.kmeans(keys, init, 6, storage=storage)
    assert labels.shape == (N,) and labels.min() >= 0 and labels.max() < C
    assert sizes.sum() == N                                   # each token in exactly one cluster
    assert np.array_equal(sizes, np.bincount(labels, minlength=C))
    for c in range(C):                                        # centroid = mean of current members
        if sizes[c]:
            assert np.allclose(mu[c], keys[labels == c].mean(axis=0), rtol=1e-12, atol=1e-13)
    assert len(tr.labels) == 6 and np.array_equal(tr.labels[-1], labels)
    # the first assignment reads the normalised initial rows
    assert np.allclose(tr.mu_hat[0], O.storage_round(
        keys[init] / np.linalg.norm(keys[init], axis=1, keepdims=True), storage))


@pytest.mark.parametrize("seed", range(4))
def test_weighted_objective_never_increases(seed):
    """J = sum |k_i| (1 - cos(k_i, centroid)) cannot grow: the assignment picks
    the best centroid per key, and the direction of the member sum maximises
    sum <k_i, u> over unit u.  (Exact arithmetic; fp64 slack only.)"""
    rng = np.random.default_rng(20 + seed)
    N, C, d = 500, 10, 16
    keys, _, _ = mixture(rng, N, 25, d, sigma=1.0)
    init = rng.permutation(N)[:C]
    _, _, _, tr = O.kmeans(keys, init, 12, storage="f64")
    J = np.array(tr.J)
    assert np.all(np.diff(J) <= 1e-12 * J[0])
    assert J[-1] < J[0]
    # J agrees with its definition through the cosine
    knorm = np.linalg.norm(keys, axis=1)
    lab, mh = tr.labels[3], tr.mu_hat[3]
    cos = (keys * mh[lab]).sum(1) / knorm
    assert abs(tr.J[3] - (knorm * (1 - cos)).sum()) < 1e-9
    assert abs(tr.D[3] - (1 - cos).sum()) < 1e-9


def test_noise_free_mixture_is_recovered_in_one_iteration():
    rng = np.random.default_rng(31)
    M, d, N = 9, 16, 300
    keys, centers, which = mixture(rng, N, M, d, sigma=0.0)
    keys = keys * rng.uniform(0.5, 2.0, size=(N, 1))          # lengths must not matter
    init = np.array([np.nonzero(which == m)[0][0] for m in range(M)])
    mu, labels, sizes, tr = O.kmeans(keys, init, 3, storage="f64")
    assert np.array_equal(labels, which)
    for t in range(3):
        assert np.array_equal(tr.labels[t], which)            # fixed point from the start
    assert np.allclose(O.unit_rows(mu), centers, atol=1e-12)


def test_single_cluster_is_global_mean():
    rng = np.random.default_rng(32)
    keys = rng.normal(size=(77, 8))
    mu, labels, sizes, _ = O.kmeans(keys, [5], 2, storage="f64")
    assert np.all(labels == 0) and sizes.tolist() == [77]
    assert np.allclose(mu[0], keys.mean(axis=0))


def test_every_token_its_own_cluster():
    rng = np.random.default_rng(33)
    N = 40
    keys = rng.normal(size=(N, 8))
    init = rng.permutation(N)
    mu, labels, sizes, _ = O.kmeans(keys, init, 2, storage="f64")
    assert np.all(sizes == 1)
    assert np.array_equal(init[labels], np.arange(N))
    assert np.allclose(mu[labels], keys)


def test_empty_cluster_keeps_its_centroid():
    keys = np.array([[1.0, 0.0], [0.9, 0.1], [0.0, 1.0], [0.1, 0.9]])
    prev = np.array([[1.0, 0.0], [0.0, 1.0], [-1.0, -1.0]])
    labels, _, gap = O.assign(keys, O.unit_rows(prev))
    assert labels.tolist() == [0, 0, 1, 1]
    mu, sizes = O.update(keys, labels, prev)
    assert sizes.tolist() == [2, 2, 0]
    assert np.array_equal(mu[2], prev[2])
    assert np.allclose(mu[0], [0.95, 0.05]) and np.allclose(mu[1], [0.05, 0.95])


def test_assign_ties_and_gap():
    keys = np.array([[2.0, 0.0], [1.0, 1.0]])
    mu_hat = np.array([[1.0, 0.0], [1.0, 0.0], [0.0, 1.0]])
    labels, best, gap = O.assign(keys, mu_hat)
    assert labels.tolist() == [0, 0]                 # equal similarity -> lower id
    assert gap[0] == 0.0 and abs(gap[1]) < 1e-15
    # the gap is in cosine units: scaling a key leaves it unchanged
    l2, _, g2 = O.assign(keys * 7.0, np.array([[1.0, 0.0], [0.0, 1.0]]))
    l1, _, g1 = O.assign(keys, np.array([[1.0, 0.0], [0.0, 1.0]]))
    assert np.allclose(g1, g2) and l1.tolist() == l2.tolist()
    assert abs(g1[0] - 1.0) < 1e-15


def test_duplicate_initial_rows_rejected():
    keys = np.array([[1.0, 0.0], [1.0, 0.0], [0.0, 1.0]])
    with pytest.raises(ValueError):
        O.kmeans(keys, [0, 1], 1)


def test_synthetic_generator_feeds_oracle():
    """End-to-end on the tiny configuration's recipe (smaller N): the oracle runs
    on the shared generator's bf16 tensors and recovers mostly-pure clusters."""
    from ck_synth import Config, MixtureWorkload, sample_init_indices
    cfg = Config("t", 1, 1, 2, 2, 128, 512, 16, 16, 10, 128, seed=0)
    w = MixtureWorkload(cfg)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    keys = w.K[0, 1].float().numpy().astype(np.float64)
    assert np.array_equal(O.round_to_bf16(keys), keys)
    mu, labels, sizes, tr = O.kmeans(keys, init[0, 1].numpy(), cfg.n_iter, storage="bf16")
    tc = w.token_center[0, 1, :cfg.N].numpy()
    purity = sum(np.bincount(tc[labels == c]).max() for c in range(cfg.C) if sizes[c]) / cfg.N
    assert purity > 0.6
    assert tr.J[-1] < tr.J[0]
