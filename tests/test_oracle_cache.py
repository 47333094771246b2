"""Pins for the oracle's cluster-granularity cache model (paper Section IV-D, R = 1)."""
import numpy as np

from oracle import clusterkv_oracle as O


def test_cache_closed_forms():
    sizes = np.array([3, 5, 0, 2, 7])
    assert O.cache_step([], [1, 3], sizes) == (0, 7, [1, 3])            # cold cache: all loaded
    assert O.cache_step([1, 3], [3, 1], sizes) == (7, 0, [3, 1])        # same set, other order
    assert O.cache_step([1, 3], [0, 4], sizes) == (0, 10, [0, 4])       # disjoint
    assert O.cache_step([1, 3], [4, 3, 2], sizes) == (2, 7, [4, 3, 2])  # empty cluster 2 costs nothing
    assert O.cache_step([0], [], sizes) == (0, 0, [])


def test_only_the_previous_step_is_kept():
    sizes = np.array([4, 4, 4])
    h1, m1, held = O.cache_step([], [0], sizes)
    h2, m2, held = O.cache_step(held, [1], sizes)
    h3, m3, held = O.cache_step(held, [0], sizes)      # cluster 0 was dropped at step 2
    assert (h1, m1, h2, m2, h3, m3) == (0, 4, 0, 4, 0, 4)
    assert O.cache_hit_rate([[0], [1], [0]], sizes) == 0.0
    assert O.cache_hit_rate([[0, 1], [1, 2], [2, 1]], sizes) == (0 + 4 + 8) / 24


def test_cluster_hits_equal_token_set_intersection():
    """Clusters partition the tokens, so hits counted per cluster equal the size of the
    intersection of consecutive recalled token lists (built by the index generation)."""
    rng = np.random.default_rng(2)
    n, C, B = 400, 20, 90
    labels = rng.integers(0, C, size=n)
    sizes, offsets, sorted_idx = O.build_metadata(labels, C)
    held, prev_tokens = [], set()
    for step in range(12):
        scores = rng.standard_normal(C)
        order, n_sel, n_tok = O.select_clusters(scores, sizes, B, O.WHOLE)
        tokens = set(O.gather_indices(order, n_sel, offsets, sorted_idx, B, O.WHOLE).tolist())
        hit, miss, held = O.cache_step(held, order[:n_sel], sizes)
        assert hit == len(tokens & prev_tokens)
        assert hit + miss == len(tokens) == n_tok
        prev_tokens = tokens
