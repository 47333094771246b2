"""Pins for the oracle's K-means variants: l2 / inner-product assignment (the
metrics compared in paper Section V-B) and the run-until-convergence loop of
Section III-B."""
import numpy as np
import pytest
from scipy.cluster.vq import kmeans2, vq

from oracle import clusterkv_oracle as O


def _mixture(rng, n, d, m, noise):
    centers = rng.standard_normal((m, d))
    centers /= np.linalg.norm(centers, axis=1, keepdims=True)
    which = rng.integers(0, m, size=n)
    return 3.0 * centers[which] + noise * rng.standard_normal((n, d)), which, centers


def test_l2_assignment_matches_library_vector_quantiser():
    rng = np.random.default_rng(1)
    keys = rng.standard_normal((700, 16))
    table = rng.standard_normal((23, 16))
    labels, gap = O.assign_metric(keys, table, O.L2)
    code, dist = vq(keys, table)
    assert labels.tolist() == code.tolist()
    # gap: half the difference of the two smallest squared distances over |k|
    d2 = ((keys[:, None, :] - table[None]) ** 2).sum(-1)
    d2.sort(axis=1)
    want = 0.5 * (d2[:, 1] - d2[:, 0]) / np.linalg.norm(keys, axis=1)
    assert np.allclose(gap, want, rtol=1e-12, atol=0)
    assert np.allclose(np.sqrt(d2[:, 0]), dist)


def test_l2_equals_biased_inner_product_form():
    """argmin |k-mu|^2 == argmax (<k,mu> - |mu|^2/2): the form a contraction kernel uses."""
    rng = np.random.default_rng(2)
    keys = rng.standard_normal((300, 8))
    table = rng.standard_normal((11, 8)) * 2.0
    labels, _ = O.assign_metric(keys, table, O.L2)
    v = keys @ table.T - 0.5 * (table * table).sum(axis=1)[None, :]
    assert labels.tolist() == np.argmax(v, axis=1).tolist()


def test_inner_product_assignment_loops_and_ties():
    rng = np.random.default_rng(3)
    keys = rng.integers(-2, 3, size=(40, 4)).astype(np.float64)
    table = rng.integers(-2, 3, size=(6, 4)).astype(np.float64)
    table[4] = table[1]                                    # an exact duplicate: lower id must win
    labels, _ = O.assign_metric(keys, table, O.INNER)
    for i in range(40):
        best, bj = None, -1
        for j in range(6):
            dot = sum(keys[i, c] * table[j, c] for c in range(4))
            if best is None or dot > best:
                best, bj = dot, j
        assert labels[i] == bj
    assert 4 not in labels.tolist()


def test_metrics_differ_only_by_centroid_length():
    """With unit-length centroids all three metrics pick the same centroid."""
    rng = np.random.default_rng(4)
    keys = rng.standard_normal((200, 8))
    table = O.unit_rows(rng.standard_normal((9, 8)))
    a, _ = O.assign_metric(keys, table, O.COSINE)
    b, _ = O.assign_metric(keys, table, O.INNER)
    c, _ = O.assign_metric(keys, table, O.L2)
    assert a.tolist() == b.tolist() == c.tolist()


def test_kmeans_run_cosine_fixed_count_equals_kmeans():
    rng = np.random.default_rng(5)
    keys, _, _ = _mixture(rng, 600, 16, 12, 0.5)
    keys = O.round_to_bf16(keys)
    init = rng.permutation(600)[:12]
    mu0, lab0, sz0, tr0 = O.kmeans(keys, init, 6)
    mu1, lab1, sz1, n_done, tr1 = O.kmeans_run(keys, init, 6)
    assert n_done == 6
    assert lab0.tolist() == lab1.tolist() and sz0.tolist() == sz1.tolist()
    assert np.array_equal(mu0, mu1)


@pytest.mark.parametrize("metric", [O.COSINE, O.L2, O.INNER])
def test_convergence_stop_is_a_fixed_point(metric):
    """Stopping at the first unchanged assignment gives the state that any larger
    fixed iteration count reaches, and the iteration count is the first repeat."""
    rng = np.random.default_rng(6)
    keys, _, _ = _mixture(rng, 500, 8, 6, 0.3)
    keys = O.round_to_f32(keys)
    init = rng.permutation(500)[:6]
    mu, lab, sz, n_done, tr = O.kmeans_run(keys, init, 50, "f32", metric, until_converged=True)
    assert 2 <= n_done < 50
    assert tr.labels[-1].tolist() == tr.labels[-2].tolist()
    for t in range(1, n_done - 1):
        assert tr.labels[t].tolist() != tr.labels[t - 1].tolist()
    mu2, lab2, sz2, n2, _ = O.kmeans_run(keys, init, n_done + 3, "f32", metric)
    assert n2 == n_done + 3
    assert lab2.tolist() == lab.tolist() and sz2.tolist() == sz.tolist()
    assert np.array_equal(mu2, mu)
    # every centroid is the mean of its members
    for c in range(6):
        if sz[c]:
            assert np.allclose(mu[c], keys[lab == c].mean(axis=0), rtol=1e-13, atol=1e-13)


def test_zero_noise_mixture_converges_at_second_assignment():
    rng = np.random.default_rng(7)
    keys, which, centers = _mixture(rng, 240, 8, 5, 0.0)
    keys = O.round_to_f32(keys)
    init = np.array([int(np.flatnonzero(which == c)[0]) for c in range(5)])
    for metric in (O.COSINE, O.L2, O.INNER):
        mu, lab, sz, n_done, _ = O.kmeans_run(keys, init, 20, "f32", metric, until_converged=True)
        assert n_done == 2
        assert lab.tolist() == which.tolist()


def test_l2_run_matches_library_lloyd_iterations():
    rng = np.random.default_rng(8)
    keys, _, _ = _mixture(rng, 400, 8, 5, 0.4)
    keys = O.round_to_f32(keys)
    init = rng.permutation(400)[:5]
    mu, lab, sz, n_done, tr = O.kmeans_run(keys, init, 7, "f32", O.L2)
    assert min(min(g) for g in tr.gap) > 1e-6              # no near-tie on this data
    cent, code = kmeans2(keys, keys[init].copy(), iter=7, minit="matrix")
    # library: labels from the table BEFORE its last update, centroids after it
    assert code.tolist() == lab.tolist()
    assert np.allclose(cent, mu, rtol=1e-6, atol=1e-6)


def test_l2_objective_never_increases():
    rng = np.random.default_rng(9)
    keys, _, _ = _mixture(rng, 800, 16, 20, 0.5)
    keys = O.round_to_f32(keys)
    init = rng.permutation(800)[:16]
    _, _, _, n_done, tr = O.kmeans_run(keys, init, 12, "f32", O.L2)
    prev = np.inf
    for t in range(n_done):
        # objective after the t-th update, with the labels it used (fp64 means)
        j = O.sum_squared_distance(keys, tr.mu[t], tr.labels[t])
        assert j <= prev * (1 + 1e-9)
        prev = j
