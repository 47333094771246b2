"""Pins for the oracle's metadata, selection, indexing and attention functions.

Sources of truth used here: the worked example the paper prints for Fig. 8
(tests/golden/fig8_indexing.txt), closed forms, library routines a special case
reduces to (torch SDPA in fp64, a plain top-k), invariants, and the loop-only
restatement in tests/loops.py on tiny inputs.
"""
import os

import numpy as np
import pytest
import torch

from oracle import clusterkv_oracle as O
from tests import loops

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig8_indexing.txt")


def read_golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":")
            out[k.strip()] = [int(x) for x in v.split()]
    return out


# ---------------------------------------------------------------- Fig. 8 example
def test_fig8_metadata_and_indexing():
    g = read_golden()
    labels = np.array(g["labels"])
    sizes, offsets, sorted_idx = O.build_metadata(labels, 3)
    # scores that realise the printed order "cluster 2, then 0, then 1"
    scores = np.zeros(3)
    for rank, c in enumerate(g["closest_order"]):
        scores[c] = 10.0 - rank
    B = g["budget"][0]
    for mode in (O.WHOLE, O.TRIM_LAST):
        order, n_sel, n_tok = O.select_clusters(scores, sizes, B, mode)
        assert order.tolist() == g["closest_order"]
        assert sizes[order].tolist() == g["reordered_sizes"]
        assert np.cumsum(sizes[order]).tolist() == g["reordered_prefix"]
        assert n_sel == g["n_selected_clusters"][0]
        sel = order[:n_sel]
        assert sizes[sel].tolist() == g["selected_sizes"]
        assert offsets[sel + 1].tolist() == g["selected_end_positions"]
        idx = O.gather_indices(order, n_sel, offsets, sorted_idx, B, mode)
        assert idx.tolist() == g["selected_tokens"]
        assert n_tok == len(idx)


def test_fig8_other_budgets():
    g = read_golden()
    labels = np.array(g["labels"])
    sizes, offsets, sorted_idx = O.build_metadata(labels, 3)
    assert sizes.tolist() == [1, 3, 2]
    assert offsets.tolist() == [0, 1, 4, 6]
    assert sorted_idx.tolist() == [1, 2, 3, 4, 0, 5]
    scores = np.array([2.0, 1.0, 3.0])
    # B=4: the third cluster (size 3) does not fit whole; the paper's rule trims it
    order, n_sel, n_tok = O.select_clusters(scores, sizes, 4, O.WHOLE)
    assert (n_sel, n_tok) == (2, 3)
    assert O.gather_indices(order, n_sel, offsets, sorted_idx, 4, O.WHOLE).tolist() == [0, 5, 1]
    order, n_sel, n_tok = O.select_clusters(scores, sizes, 4, O.TRIM_LAST)
    assert (n_sel, n_tok) == (3, 4)
    assert O.gather_indices(order, n_sel, offsets, sorted_idx, 4, O.TRIM_LAST).tolist() == [0, 5, 1, 4]
    for mode in (O.WHOLE, O.TRIM_LAST):
        order, n_sel, n_tok = O.select_clusters(scores, sizes, 6, mode)
        assert (n_sel, n_tok) == (3, 6)
        got = O.gather_indices(order, n_sel, offsets, sorted_idx, 6, mode).tolist()
        assert got == [0, 5, 1, 2, 3, 4]
    # B=1: best cluster (size 2) alone exceeds the budget
    order, n_sel, n_tok = O.select_clusters(scores, sizes, 1, O.WHOLE)
    assert (n_sel, n_tok) == (0, 0)
    order, n_sel, n_tok = O.select_clusters(scores, sizes, 1, O.TRIM_LAST)
    assert (n_sel, n_tok) == (1, 1)
    assert O.gather_indices(order, n_sel, offsets, sorted_idx, 1, O.TRIM_LAST).tolist() == [5]


# ---------------------------------------------------------------- metadata
@pytest.mark.parametrize("seed", range(4))
def test_metadata_invariants_and_loops(seed):
    rng = np.random.default_rng(seed)
    N, C = 200, 13
    labels = rng.integers(0, C, N)
    labels[labels == 5] = 6                       # an empty cluster
    sizes, offsets, sorted_idx = O.build_metadata(labels, C, tok_begin=16)
    assert sizes.sum() == N and sizes[5] == 0
    assert np.all(np.diff(offsets) == sizes) and offsets[0] == 0
    assert sorted(sorted_idx.tolist()) == list(range(16, 16 + N))
    for c in range(C):
        seg = sorted_idx[offsets[c]:offsets[c + 1]]
        assert np.all(labels[seg - 16] == c)
        assert np.all(np.diff(seg) > 0)
    ls, lo, lidx = loops.metadata(labels.tolist(), C)
    assert ls == sizes.tolist() and lo == offsets.tolist()
    assert [i + 16 for i in lidx] == sorted_idx.tolist()


# ---------------------------------------------------------------- scoring
def test_score_is_mean_member_logit():
    """With raw-mean centroids, q.mu_c equals the mean of q.k_i over the members
    (linearity), summed over the query heads of the group."""
    rng = np.random.default_rng(1)
    N, C, d, G = 300, 7, 16, 4
    keys = rng.normal(size=(N, d))
    labels = rng.integers(0, C, N)
    mu, sizes = O.update(keys, labels, np.zeros((C, d)))
    q = rng.normal(size=(G, d))
    s = O.score_clusters(q, mu)
    for c in range(C):
        member_logits = (keys[labels == c] @ q.T).sum(axis=1)
        assert abs(s[c] - member_logits.mean()) < 1e-12 * max(1.0, abs(s[c]))


# ---------------------------------------------------------------- selection
@pytest.mark.parametrize("seed", range(6))
def test_select_gather_invariants_and_loops(seed):
    rng = np.random.default_rng(100 + seed)
    N, C, d, G = 64, 8, 8, 2
    keys = rng.normal(size=(N, d))
    labels = rng.integers(0, C, N)
    if seed % 2:
        labels[labels == 3] = 2
    mu, sizes0 = O.update(keys, labels, rng.normal(size=(C, d)))
    sizes, offsets, sorted_idx = O.build_metadata(labels, C)
    assert np.array_equal(sizes, sizes0)
    q = rng.normal(size=(G, d))
    if seed == 5:
        mu[4] = mu[1]                              # exact score tie -> lower id first
    scores = O.score_clusters(q, mu)
    for B in (1, 5, 17, 40, 64, 100):
        for mode in (O.WHOLE, O.TRIM_LAST):
            order, n_sel, n_tok = O.select_clusters(scores, sizes, B, mode)
            idx = O.gather_indices(order, n_sel, offsets, sorted_idx, B, mode)
            # order: permutation, scores non-increasing, ties by id
            assert sorted(order.tolist()) == list(range(C))
            so = scores[order]
            assert np.all(np.diff(so) <= 0)
            for a, b in zip(order[:-1], order[1:]):
                if scores[a] == scores[b]:
                    assert a < b
            assert len(idx) == n_tok <= B
            assert len(set(idx.tolist())) == len(idx)
            if mode == O.WHOLE:
                want = set()
                for c in order[:n_sel]:
                    want |= set(np.nonzero(labels == c)[0].tolist())
                assert set(idx.tolist()) == want                 # whole clusters only
                if n_sel < C:
                    assert n_tok + sizes[order[n_sel]] > B       # the next one would not fit
            else:
                assert n_tok == min(B, N)
            ls, lorder, ln, lpicked = loops.select_and_gather(
                q.tolist(), mu.tolist(), sizes.tolist(), offsets.tolist(),
                sorted_idx.tolist(), B, trim=(mode == O.TRIM_LAST))
            assert np.allclose(ls, scores, rtol=1e-12, atol=1e-12)
            assert lorder == order.tolist()
            assert ln == n_sel and lpicked == idx.tolist()


def test_singleton_clusters_reduce_to_topk():
    """C = N with one token per cluster: cluster selection is the exact top-B of
    q.k_i, the goal stated in Section III-A."""
    rng = np.random.default_rng(7)
    N, d, B = 50, 8, 12
    keys = rng.normal(size=(N, d))
    labels = rng.permutation(N)                    # token i alone in cluster labels[i]
    mu, sizes = O.update(keys, labels, np.zeros((N, d)))
    sizes, offsets, sorted_idx = O.build_metadata(labels, N)
    q = rng.normal(size=(1, d))
    r = O.decode_step(q, keys, rng.normal(size=(N, d)), mu, sizes, offsets, sorted_idx, B)
    logits = torch.from_numpy(keys @ q[0])
    top = torch.topk(logits, B).indices.numpy()
    assert r["idx"].tolist() == top.tolist()


def test_selection_near_tie_flag():
    scores = np.array([5.0, 4.0, 4.0 + 1e-6, 1.0])
    order = np.argsort(-scores, kind="stable")
    assert O.selection_near_tie(scores, order, 2)        # pair (2,1) inside the prefix
    assert not O.selection_near_tie(scores, order, 1)    # only the pair (5, 4+1e-6) is looked at
    assert not O.selection_near_tie(scores, order, 0)
    assert not O.selection_near_tie(np.array([3.0, 2.0, 1.0]), np.array([0, 1, 2]), 3)


# ---------------------------------------------------------------- attention
@pytest.mark.parametrize("G", [1, 4])
def test_attention_matches_torch_sdpa(G):
    rng = np.random.default_rng(3)
    N, d = 97, 32
    K, V = rng.normal(size=(N, d)), rng.normal(size=(N, d))
    q = rng.normal(size=(G, d))
    ids = rng.permutation(N)[:40]
    got = O.attention_over(q, K, V, ids)
    tq = torch.from_numpy(q)[None, :, None, :]                      # [1, G, 1, d]
    tk = torch.from_numpy(K[ids])[None, None].expand(1, G, -1, -1)
    tv = torch.from_numpy(V[ids])[None, None].expand(1, G, -1, -1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    full = O.full_attention(q, K, V)
    tk = torch.from_numpy(K)[None, None].expand(1, G, -1, -1)
    tv = torch.from_numpy(V)[None, None].expand(1, G, -1, -1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    assert np.allclose(full, want, rtol=1e-12, atol=1e-13)


def test_attention_special_cases_and_loops():
    rng = np.random.default_rng(4)
    N, d, G = 30, 8, 2
    K, V = rng.normal(size=(N, d)), rng.normal(size=(N, d))
    q = rng.normal(size=(G, d))
    # one token -> its value
    assert np.allclose(O.attention_over(q, K, V, [11]), np.tile(V[11], (G, 1)))
    # identical keys -> plain mean of the values
    Ke = np.tile(K[0], (N, 1))
    ids = [3, 9, 20, 21]
    assert np.allclose(O.attention_over(q, Ke, V, ids), np.tile(V[ids].mean(0), (G, 1)))
    # order of the index list is irrelevant
    a = O.attention_over(q, K, V, [1, 5, 7, 2])
    b = O.attention_over(q, K, V, [7, 2, 1, 5])
    assert np.allclose(a, b, rtol=1e-13, atol=1e-14)
    # empty set -> zeros
    assert np.all(O.attention_over(q, K, V, []) == 0)
    # sinks and recent tokens join the recalled set
    got = O.sparse_attention(q, K, V, [10, 12], n_sink=2, recent_begin=27, recent_end=30)
    want = O.attention_over(q, K, V, [0, 1, 10, 12, 27, 28, 29])
    assert np.allclose(got, want)
    # loop-only restatement
    ids = [4, 8, 15, 16, 23]
    for g in range(G):
        want = loops.softmax_attention(q[g].tolist(), K.tolist(), V.tolist(), ids,
                                       1.0 / np.sqrt(d))
        assert np.allclose(O.attention_over(q, K, V, ids)[g], want, rtol=1e-12, atol=1e-13)


def test_budget_covering_everything_equals_full_attention():
    rng = np.random.default_rng(5)
    N, C, d, G = 120, 9, 16, 4
    keys, V = rng.normal(size=(N, d)), rng.normal(size=(N, d))
    init = rng.permutation(N)[:C]
    mu, labels, sizes, _ = O.kmeans(keys, init, 5, storage="f64")
    sizes, offsets, sorted_idx = O.build_metadata(labels, C)
    q = rng.normal(size=(G, d))
    for mode in (O.WHOLE, O.TRIM_LAST):
        r = O.decode_step(q, keys, V, mu, sizes, offsets, sorted_idx, N + 5, mode)
        assert sorted(r["idx"].tolist()) == list(range(N))
        assert np.allclose(r["out"], O.full_attention(q, keys, V), rtol=1e-12, atol=1e-13)
