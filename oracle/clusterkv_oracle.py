"""CPU oracle for the ClusterKV hot path -- TEST INFRASTRUCTURE, not product code.

A plain, slow, fp64 NumPy statement of what the path computes, written from the
paper: cosine K-means over the keys of one KV head (Section III-B), scoring of
the query against the cluster centroids and selection of clusters in score order
up to a token budget (Section III-C), generation of the selected token indices
from the clustering metadata (Section IV-C, Fig. 8) and softmax attention over
only the selected keys and values (Section II-B).  Only tests, the smoke check
and the benchmark's CPU-baseline leg may import it; it shares no code with the
GPU library and must never serve as a fallback for it.

Everything here works on ONE head-problem (one sequence, one KV head):
keys/values are [N, d] float64 arrays that hold exactly the values the GPU
stores (bf16 or fp32 bit patterns widened to fp64), queries are [G, d] for the
G query heads that share the KV head.

Readings taken where the paper is silent (each is listed in the design notes):
  * centroid = arithmetic mean of the raw (un-normalised) member keys; the
    assignment step compares keys with the unit-length copy of each centroid,
    rounded to the storage type of the centroid table;
  * an empty cluster keeps its previous centroid and stays in the table;
  * ties (equal similarity, equal score) go to the lower cluster id;
  * a fixed iteration count replaces the run-to-convergence loop by default;
    `kmeans_run` can also stop at the first assignment that changes no label;
  * cluster score = sum over the G query heads of <q_g, centroid>, no 1/sqrt(d);
  * budget: WHOLE keeps the longest prefix of the score order whose sizes sum to
    at most B; TRIM_LAST (the paper's rule) extends the prefix until the sum
    reaches B and cuts the last cluster, keeping its trailing entries.

Pin status: every function below is pinned by tests/test_oracle_*.py (worked
example of Fig. 8, closed forms, invariants, library cross-checks, loop-only
brute force).  The 10-iteration K-means trajectory as a whole has no printed
values to compare with: "parity unpinned" for `kmeans` and `kmeans_run` beyond
their per-step pins (the l2 variant is pinned as a whole against a library
Lloyd iteration on data without near-ties).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

WHOLE = 0
TRIM_LAST = 1


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_bf16(x):
    """Nearest bf16 value (8 significant bits, ties to even), returned as fp64.
    Assumes the bf16 normal range."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def round_to_f32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def storage_round(x, storage: str):
    if storage == "bf16":
        return round_to_bf16(x)
    if storage == "f32":
        return round_to_f32(x)
    if storage == "f64":
        return np.asarray(x, dtype=np.float64)
    raise ValueError(storage)


# --------------------------------------------------------------------------
# K-means (Section III-B)
# --------------------------------------------------------------------------
def unit_rows(mu):
    """mu_hat_c = mu_c / |mu_c| (zero rows stay zero)."""
    mu = np.asarray(mu, dtype=np.float64)
    n = np.sqrt((mu * mu).sum(axis=1, keepdims=True))
    out = np.zeros_like(mu)
    np.divide(mu, n, out=out, where=n > 0)
    return out


def assign(keys, mu_hat):
    """Assignment step: label_i = argmax_c <k_i, mu_hat_c> (the key's own length
    does not change the argmax of the cosine).  Returns (labels, best, gap) where
    gap is best minus runner-up similarity in cosine units (inf if C == 1)."""
    sim = keys @ mu_hat.T                                     # [N, C]
    labels = np.argmax(sim, axis=1)                           # first maximum wins
    best = sim[np.arange(len(keys)), labels]
    if sim.shape[1] > 1:
        part = np.partition(sim, -2, axis=1)
        second = part[:, -2]
        knorm = np.sqrt((keys * keys).sum(axis=1))
        gap = np.where(knorm > 0, (best - second) / np.where(knorm > 0, knorm, 1.0), 0.0)
    else:
        gap = np.full(len(keys), np.inf)
    return labels.astype(np.int64), best, gap


def update(keys, labels, mu_prev):
    """Update step: centroid = mean of the keys assigned to it; an empty cluster
    keeps mu_prev.  Returns (mu, sizes)."""
    C = mu_prev.shape[0]
    mu = np.array(mu_prev, dtype=np.float64, copy=True)
    sizes = np.zeros(C, dtype=np.int64)
    for c in range(C):
        members = keys[labels == c]
        sizes[c] = len(members)
        if len(members):
            mu[c] = members.sum(axis=0) / len(members)
    return mu, sizes


def weighted_objective(keys, mu_hat, labels):
    """J = sum_i |k_i| * (1 - cos(k_i, mu_hat_label_i)) = sum_i (|k_i| - <k_i, u_i>)
    for unit-length mu_hat; the quantity both K-means steps cannot increase."""
    knorm = np.sqrt((keys * keys).sum(axis=1))
    return float((knorm - (keys * mu_hat[labels]).sum(axis=1)).sum())


def cosine_objective(keys, mu_hat, labels):
    """Plain sum of the paper's distance D = 1 - cos(k_i, centroid)."""
    knorm = np.sqrt((keys * keys).sum(axis=1))
    dots = (keys * mu_hat[labels]).sum(axis=1)
    un = np.sqrt((mu_hat[labels] ** 2).sum(axis=1))
    den = knorm * un
    cos = np.divide(dots, den, out=np.zeros_like(dots), where=den > 0)
    return float((1.0 - cos).sum())


@dataclass
class KMeansTrace:
    """State of every iteration, so a GPU step can be checked with the oracle's
    own inputs to that step."""
    mu_hat: list = field(default_factory=list)    # table the t-th assignment read
    labels: list = field(default_factory=list)    # result of the t-th assignment
    gap: list = field(default_factory=list)       # near-tie measure per key
    mu: list = field(default_factory=list)        # fp64 centroids after the t-th update
    sizes: list = field(default_factory=list)
    J: list = field(default_factory=list)         # weighted objective after assignment t
    D: list = field(default_factory=list)         # cosine objective after assignment t


def kmeans(keys, init_idx, n_iter, storage="bf16"):
    """Cosine K-means of `keys` [N, d] with initial centroids keys[init_idx].
    Returns (mu, labels, sizes, trace): fp64 centroids after the last update,
    labels of the last assignment, cluster sizes, per-iteration trace."""
    init_idx = np.asarray(init_idx, dtype=np.int64)
    rows = keys[init_idx]
    if len({r.tobytes() for r in rows}) != len(rows):
        raise ValueError("initial centroids must be distinct key rows")
    mu = np.array(rows, dtype=np.float64, copy=True)
    sizes = np.zeros(len(init_idx), dtype=np.int64)
    labels = np.zeros(len(keys), dtype=np.int64)
    tr = KMeansTrace()
    for _ in range(n_iter):
        mu_hat = storage_round(unit_rows(mu), storage)
        labels, _, gap = assign(keys, mu_hat)
        tr.mu_hat.append(mu_hat)
        tr.labels.append(labels)
        tr.gap.append(gap)
        tr.J.append(weighted_objective(keys, mu_hat, labels))
        tr.D.append(cosine_objective(keys, mu_hat, labels))
        mu, sizes = update(keys, labels, mu)
        tr.mu.append(mu)
        tr.sizes.append(sizes)
    return mu, labels, sizes, tr


# --------------------------------------------------------------------------
# K-means variants: other distance metrics (the ablation of Section V-B) and
# the run-until-convergence loop of Section III-B
# --------------------------------------------------------------------------
COSINE = "cosine"
L2 = "l2"
INNER = "ip"


def assign_metric(keys, table, metric):
    """Assignment under one of the three metrics the paper compares.
      cosine: argmax_c <k, table_c>, table = unit-length centroids (as `assign`);
      ip:     argmax_c <k, table_c>, table = the centroids themselves;
      l2:     argmin_c |k - table_c|^2, table = the centroids themselves.
    Ties go to the lower id.  Returns (labels, gap): gap = distance between the
    best and the second-best candidate, expressed in units of <k, .>/|k| so that
    one tolerance serves all three (l2: half the difference of squared distances)."""
    keys = np.asarray(keys, dtype=np.float64)
    table = np.asarray(table, dtype=np.float64)
    if metric in (COSINE, INNER):
        labels, _, gap = assign(keys, table)
        return labels, gap
    if metric != L2:
        raise ValueError(metric)
    n, C = len(keys), len(table)
    labels = np.zeros(n, dtype=np.int64)
    gap = np.full(n, np.inf)
    for lo in range(0, n, 512):                               # key blocks only bound the memory
        blk = keys[lo:lo + 512]
        diff = blk[:, None, :] - table[None, :, :]
        d2 = (diff * diff).sum(axis=2)                        # [block, C]
        lab = np.argmin(d2, axis=1)                           # first minimum wins
        labels[lo:lo + 512] = lab
        if C > 1:
            part = np.partition(d2, 1, axis=1)
            knorm = np.sqrt((blk * blk).sum(axis=1))
            g = 0.5 * (part[:, 1] - part[:, 0])
            gap[lo:lo + 512] = np.where(knorm > 0, g / np.where(knorm > 0, knorm, 1.0), 0.0)
    return labels, gap


def metric_table(mu, metric, storage):
    """The centroid table an assignment under `metric` compares the keys with."""
    return storage_round(unit_rows(mu) if metric == COSINE else mu, storage)


def kmeans_run(keys, init_idx, max_iter, storage="bf16", metric=COSINE, until_converged=False):
    """K-means as in `kmeans`, under any of the three metrics, optionally stopping
    as soon as an assignment reproduces the labels of the previous one (Section
    III-B: the two steps alternate until the assignment no longer changes).  The
    confirming assignment counts as an iteration and is not followed by an update
    (it would recompute the same means).  Returns (mu, labels, sizes, n_done,
    trace); trace has the tables, labels, gaps and means of every iteration run."""
    keys = np.asarray(keys, dtype=np.float64)
    init_idx = np.asarray(init_idx, dtype=np.int64)
    rows = keys[init_idx]
    if len({r.tobytes() for r in rows}) != len(rows):
        raise ValueError("initial centroids must be distinct key rows")
    mu = np.array(rows, dtype=np.float64, copy=True)
    sizes = np.zeros(len(init_idx), dtype=np.int64)
    labels = None
    tr = KMeansTrace()
    n_done = 0
    for _ in range(max_iter):
        table = metric_table(mu, metric, storage)
        new_labels, gap = assign_metric(keys, table, metric)
        n_done += 1
        tr.mu_hat.append(table)
        tr.labels.append(new_labels)
        tr.gap.append(gap)
        if until_converged and labels is not None and np.array_equal(new_labels, labels):
            break
        labels = new_labels
        mu, sizes = update(keys, labels, mu)
        tr.mu.append(mu)
        tr.sizes.append(sizes)
    return mu, labels, sizes, n_done, tr


def sum_squared_distance(keys, mu, labels):
    """The textbook K-means objective (l2 metric)."""
    d = np.asarray(keys, dtype=np.float64) - np.asarray(mu, dtype=np.float64)[labels]
    return float((d * d).sum())


# --------------------------------------------------------------------------
# clustering metadata (Section IV-C, Fig. 8)
# --------------------------------------------------------------------------
def build_metadata(labels, C, tok_begin=0):
    """sizes[c], offsets (exclusive prefix sum of sizes, C+1 entries) and
    sorted_idx = token ids ordered by label, ascending token id inside a cluster.
    labels[i] belongs to token tok_begin + i."""
    labels = np.asarray(labels, dtype=np.int64)
    sizes = np.bincount(labels, minlength=C).astype(np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    sorted_idx = (np.argsort(labels, kind="stable") + tok_begin).astype(np.int64)
    return sizes, offsets, sorted_idx


# --------------------------------------------------------------------------
# selection (Section III-C) and indexing (Section IV-C)
# --------------------------------------------------------------------------
def score_clusters(q_group, mu):
    """s_c = sum_g <q_g, mu_c>; q_group [G, d], mu [C, d] (stored centroids)."""
    return (q_group @ mu.T).sum(axis=0)


def select_clusters(scores, sizes, budget, mode=WHOLE):
    """Clusters in descending score order (ties: lower id first) and how many of
    them are recalled.  Returns (order[C], n_sel_clusters, n_sel_tokens)."""
    scores = np.asarray(scores, dtype=np.float64)
    sizes = np.asarray(sizes, dtype=np.int64)
    C = len(scores)
    order = np.argsort(-scores, kind="stable")
    cum = np.cumsum(sizes[order])
    if mode == WHOLE:
        n_sel = int(np.searchsorted(cum, budget, side="right"))     # cum[j-1] <= B
        n_tok = int(cum[n_sel - 1]) if n_sel else 0
    elif mode == TRIM_LAST:
        j = int(np.searchsorted(cum, budget, side="left"))          # first cum >= B
        n_sel = min(j + 1, C)
        n_tok = int(min(cum[n_sel - 1], budget)) if n_sel else 0
    else:
        raise ValueError(mode)
    return order.astype(np.int64), n_sel, n_tok


def gather_indices(order, n_sel, offsets, sorted_idx, budget, mode=WHOLE):
    """I_T: the sorted_idx segments of the selected clusters, concatenated in
    selection order.  TRIM_LAST keeps the trailing entries of the last segment
    (the slice [end - kept, end) of Fig. 8's size / end-position gather)."""
    out = []
    total = 0
    for j in range(n_sel):
        c = int(order[j])
        beg, end = int(offsets[c]), int(offsets[c + 1])
        if mode == TRIM_LAST and total + (end - beg) > budget:
            beg = end - (budget - total)
        out.append(sorted_idx[beg:end])
        total += end - beg
    if not out:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate(out).astype(np.int64)


# --------------------------------------------------------------------------
# attention (Section II-A / II-B)
# --------------------------------------------------------------------------
def attention_over(q_group, K, V, token_ids, scale=None):
    """o_g = softmax(q_g K_T^T * scale) V_T over the rows `token_ids`; empty set
    gives zeros.  scale defaults to 1/sqrt(d)."""
    q_group = np.asarray(q_group, dtype=np.float64)
    d = q_group.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    token_ids = np.asarray(token_ids, dtype=np.int64)
    if token_ids.size == 0:
        return np.zeros((q_group.shape[0], V.shape[1]))
    Ks, Vs = K[token_ids], V[token_ids]
    logits = (q_group @ Ks.T) * scale                       # [G, n]
    logits = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(logits)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ Vs


def attended_set(token_idx, n_sink=0, recent_begin=0, recent_end=0):
    """T = [0, n_sink) + I_T + [recent_begin, recent_end): always-kept leading
    tokens, the recalled tokens, and the newest tokens no cluster covers yet."""
    parts = [np.arange(0, n_sink, dtype=np.int64),
             np.asarray(token_idx, dtype=np.int64),
             np.arange(recent_begin, max(recent_begin, recent_end), dtype=np.int64)]
    return np.concatenate(parts)


def sparse_attention(q_group, K, V, token_idx, n_sink=0, recent_begin=0, recent_end=0,
                     scale=None):
    return attention_over(q_group, K, V,
                          attended_set(token_idx, n_sink, recent_begin, recent_end), scale)


def full_attention(q_group, K, V, n_tokens=None, scale=None):
    n = len(K) if n_tokens is None else n_tokens
    return attention_over(q_group, K, V, np.arange(n), scale)


# --------------------------------------------------------------------------
# one decode step of the whole path for one head-problem
# --------------------------------------------------------------------------
def decode_step(q_group, K, V, mu_stored, sizes, offsets, sorted_idx, budget, mode=WHOLE,
                n_sink=0, recent_begin=0, recent_end=0):
    scores = score_clusters(q_group, mu_stored)
    order, n_sel, n_tok = select_clusters(scores, sizes, budget, mode)
    idx = gather_indices(order, n_sel, offsets, sorted_idx, budget, mode)
    out = sparse_attention(q_group, K, V, idx, n_sink, recent_begin, recent_end)
    return dict(scores=scores, order=order, n_sel=n_sel, n_tok=n_tok, idx=idx, out=out)


def selection_near_tie(scores, order, n_sel, tol=1e-4):
    """True when a pair of neighbours in the score order, at or before the
    boundary between the last recalled and the first rejected cluster, is closer
    than tol*(1+|s|): then a rounding difference may legitimately change the
    recalled list."""
    s = np.asarray(scores, dtype=np.float64)[order]
    hi = min(n_sel, len(s) - 1)
    for j in range(hi):
        if abs(s[j] - s[j + 1]) < tol * (1.0 + abs(s[j])):
            return True
    return False


# --------------------------------------------------------------------------
# evaluation of a selection: exact top-B tokens, recall rate, page selector
# (Section V-B "recall rate of important tokens"; Section II-C for the
# page-granular selector the recall curves are compared with)
# --------------------------------------------------------------------------
def token_scores(q_group, keys):
    """Importance of every token for one KV head: the attention logits of the G
    query heads of the group, summed (Section III-A states the goal as the
    tokens with the largest q.k; the group sum is the same reading as for the
    cluster scores)."""
    q = np.asarray(q_group, dtype=np.float64)
    return (np.asarray(keys, dtype=np.float64) @ q.T).sum(axis=1)


def topk_indices(scores, k):
    """Indices of the k largest scores (equal scores: the lower index is the
    larger), returned in ascending index order; all indices if k >= len."""
    s = np.asarray(scores, dtype=np.float64)
    k = max(0, min(int(k), len(s)))
    order = np.argsort(-s, kind="stable")[:k]
    return np.sort(order).astype(np.int64)


def topk_near_tie(scores, k, tol=1e-4):
    """True when the k-th and (k+1)-th largest scores are closer than
    tol*(1+|s|): the top-k set may then legitimately differ by rounding."""
    s = np.sort(np.asarray(scores, dtype=np.float64))[::-1]
    if k <= 0 or k >= len(s):
        return False
    return abs(s[k - 1] - s[k]) < tol * (1.0 + abs(s[k - 1]))


def recall_rate(selected, true_set):
    """|I_T intersect I_true| / |I_true| (Section V-B); 1.0 for an empty I_true."""
    t = np.unique(np.asarray(true_set, dtype=np.int64))
    if len(t) == 0:
        return 1.0
    sel = np.unique(np.asarray(selected, dtype=np.int64))
    return len(np.intersect1d(sel, t, assume_unique=True)) / len(t)


def page_keys(keys, page_size, tok_begin=0, tok_count=None):
    """Representative of every page of `page_size` consecutive tokens of
    [tok_begin, tok_begin + tok_count): the per-channel maximum of its keys, as
    Section II-C describes the page-granular selector.  The last page may be short."""
    k = np.asarray(keys, dtype=np.float64)
    n = (len(k) - tok_begin) if tok_count is None else tok_count
    n_pages = (n + page_size - 1) // page_size
    rep = np.empty((n_pages, k.shape[1]))
    for p in range(n_pages):
        lo = tok_begin + p * page_size
        rep[p] = k[lo:min(lo + page_size, tok_begin + n)].max(axis=0)
    return rep


def expand_pages(pages, page_size, n_tokens, tok_begin=0):
    """Token ids of the given pages (ascending page order, tokens ascending
    inside a page); the last page stops at tok_begin + n_tokens."""
    out = []
    for p in np.sort(np.asarray(pages, dtype=np.int64)):
        lo = tok_begin + p * page_size
        out.append(np.arange(lo, min(lo + page_size, tok_begin + n_tokens)))
    return np.concatenate(out).astype(np.int64) if out else np.zeros(0, dtype=np.int64)


def page_select(q_group, keys, page_size, budget, tok_begin=0, tok_count=None):
    """Page-granular selection: score every page by <sum_g q_g, representative>,
    keep the budget // page_size best pages, return (pages ascending, token ids)."""
    k = np.asarray(keys, dtype=np.float64)
    n = (len(k) - tok_begin) if tok_count is None else tok_count
    rep = page_keys(k, page_size, tok_begin, n)
    s = token_scores(q_group, rep)
    pages = topk_indices(s, budget // page_size)
    return pages, expand_pages(pages, page_size, n, tok_begin)


# --------------------------------------------------------------------------
# cluster-granularity cache of recalled K/V (Section IV-D), R = 1
# --------------------------------------------------------------------------
def cache_step(held_clusters, selected_clusters, sizes):
    """One decode step against a cache that holds the clusters recalled at the
    previous step: a selected cluster found there is a hit, every other one is
    loaded from the home copy.  Returns (hit_tokens, miss_tokens, new_held):
    token counts of both kinds and the cluster list the cache holds afterwards
    (exactly this step's selection, in its order)."""
    held = set(int(c) for c in held_clusters)
    hit = miss = 0
    for c in selected_clusters:
        if int(c) in held:
            hit += int(sizes[int(c)])
        else:
            miss += int(sizes[int(c)])
    return hit, miss, [int(c) for c in selected_clusters]


def cache_hit_rate(selections, sizes):
    """Token-weighted hit rate of a sequence of per-step selections (whole
    clusters), starting from an empty cache."""
    held, hit_t, all_t = [], 0, 0
    for sel in selections:
        h, m, held = cache_step(held, sel, sizes)
        hit_t += h
        all_t += h + m
    return hit_t / all_t if all_t else 0.0
