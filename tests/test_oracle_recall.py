"""Pins for the oracle's evaluation helpers: exact top-B tokens, recall rate
(paper Section V-B) and the page-granular selector described in Section II-C."""
import numpy as np
import pytest

from oracle import clusterkv_oracle as O


def test_token_scores_is_sum_of_head_logits_loops():
    rng = np.random.default_rng(5)
    q = rng.standard_normal((3, 8))
    k = rng.standard_normal((17, 8))
    s = O.token_scores(q, k)
    for i in range(17):
        acc = 0.0
        for g in range(3):
            for c in range(8):
                acc += q[g, c] * k[i, c]
        assert abs(s[i] - acc) < 1e-12


def test_topk_hand_case_with_ties():
    # scores:      idx 0    1    2    3    4    5
    s = np.array([1.0, 5.0, 5.0, -2.0, 5.0, 0.5])
    # three equal maxima at 1, 2, 4: lower index first
    assert O.topk_indices(s, 1).tolist() == [1]
    assert O.topk_indices(s, 2).tolist() == [1, 2]
    assert O.topk_indices(s, 3).tolist() == [1, 2, 4]
    assert O.topk_indices(s, 4).tolist() == [0, 1, 2, 4]
    assert O.topk_indices(s, 0).tolist() == []
    assert O.topk_indices(s, 9).tolist() == [0, 1, 2, 3, 4, 5]


@pytest.mark.parametrize("n,k", [(1, 1), (64, 7), (1000, 256), (4097, 1024)])
def test_topk_matches_partition(n, k):
    """Distinct random scores: the set equals numpy's partition-based selection."""
    rng = np.random.default_rng(n + k)
    s = rng.permutation(n).astype(np.float64) * 0.37 - 11.0
    want = np.sort(np.argpartition(-s, k - 1)[:k])
    assert O.topk_indices(s, k).tolist() == want.tolist()


def test_topk_brute_force_small():
    rng = np.random.default_rng(0)
    for trial in range(50):
        n = int(rng.integers(1, 12))
        s = rng.integers(-3, 4, size=n).astype(np.float64)     # many ties
        k = int(rng.integers(0, n + 1))
        # selection by repeated removal of the best remaining (lowest index among equals)
        left = list(range(n))
        got = []
        for _ in range(k):
            b = left[0]
            for i in left:
                if s[i] > s[b]:
                    b = i
            got.append(b)
            left.remove(b)
        assert O.topk_indices(s, k).tolist() == sorted(got)


def test_recall_rate_closed_forms():
    assert O.recall_rate([1, 2, 3], [1, 2, 3]) == 1.0
    assert O.recall_rate([4, 5, 6], [1, 2, 3]) == 0.0
    assert O.recall_rate([1, 9, 3, 7], [1, 2, 3, 4]) == 0.5
    assert O.recall_rate([], [1, 2]) == 0.0
    assert O.recall_rate([3], []) == 1.0
    # duplicates in the selection count once
    assert O.recall_rate([1, 1, 1, 2], [1, 2, 3, 4]) == 0.5


def test_topk_near_tie_flag():
    s = np.array([3.0, 2.0, 2.0 - 1e-6, 0.0])
    assert O.topk_near_tie(s, 2)
    assert not O.topk_near_tie(s, 1)
    assert not O.topk_near_tie(s, 3)
    assert not O.topk_near_tie(s, 4)


def test_page_keys_hand_case():
    k = np.array([[1.0, -4.0], [0.5, -1.0], [-2.0, 3.0], [7.0, 2.0], [-1.0, -1.0]])
    rep = O.page_keys(k, 2)
    assert rep.tolist() == [[1.0, -1.0], [7.0, 3.0], [-1.0, -1.0]]     # last page is short
    rep = O.page_keys(k, 2, tok_begin=1, tok_count=3)
    assert rep.tolist() == [[0.5, 3.0], [7.0, 2.0]]


def test_page_score_bounds_every_member_for_nonnegative_queries():
    """For q >= 0 per channel, <q, per-channel max> >= <q, k> for every key of the page."""
    rng = np.random.default_rng(3)
    k = rng.standard_normal((160, 16))
    q = np.abs(rng.standard_normal((4, 16)))
    rep = O.page_keys(k, 16)
    ps = O.token_scores(q, rep)
    ts = O.token_scores(q, k)
    for p in range(10):
        assert ps[p] >= ts[p * 16:(p + 1) * 16].max() - 1e-12


def test_page_size_one_is_exact_topk():
    rng = np.random.default_rng(8)
    k = rng.standard_normal((300, 8))
    q = rng.standard_normal((2, 8))
    pages, toks = O.page_select(q, k, 1, 40)
    want = O.topk_indices(O.token_scores(q, k), 40)
    assert pages.tolist() == want.tolist() and toks.tolist() == want.tolist()
    assert O.recall_rate(toks, want) == 1.0


def test_expand_pages_and_budget():
    rng = np.random.default_rng(9)
    k = rng.standard_normal((100, 4))
    q = rng.standard_normal((1, 4))
    pages, toks = O.page_select(q, k, 16, 50)           # 3 pages
    assert len(pages) == 3
    assert toks.tolist() == O.expand_pages(pages, 16, 100).tolist()
    assert all(t // 16 in set(pages.tolist()) for t in toks)
    assert len(toks) <= 48
    # last (short) page: tokens stop at the context end
    assert O.expand_pages([6], 16, 100).tolist() == [96, 97, 98, 99]
    assert O.expand_pages([0, 2], 4, 100, tok_begin=10).tolist() == [10, 11, 12, 13, 18, 19, 20, 21]


def test_cluster_selection_with_one_token_per_cluster_has_recall_one():
    """C = N: cluster recall is the exact top-B (the goal stated in Section III-A)."""
    rng = np.random.default_rng(12)
    n, d, B = 96, 8, 20
    k = O.round_to_bf16(rng.standard_normal((n, d)))
    q = O.round_to_bf16(rng.standard_normal((2, d)))
    labels = np.arange(n)
    sizes, offsets, sorted_idx = O.build_metadata(labels, n)
    st = O.decode_step(q, k, k, k, sizes, offsets, sorted_idx, B)
    want = O.topk_indices(O.token_scores(q, k), B)
    assert O.recall_rate(st["idx"], want) == 1.0
