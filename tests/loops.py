"""Loop-only restatements of the path's definitions, used to pin the NumPy oracle.

Pure Python floats and lists, one scalar operation at a time, written from the
paper's definitions independently of oracle/ (no shared helpers, no NumPy
arithmetic).  Only usable on tiny inputs.
"""
import math


def dot(a, b):
    s = 0.0
    for x, y in zip(a, b):
        s += x * y
    return s


def cosine_assign(keys, cents):
    """label_i = index of the centroid with the largest cosine similarity
    (1 - D of Section III-B); first one on ties."""
    labels = []
    for k in keys:
        best, best_c = None, -1
        nk = math.sqrt(dot(k, k))
        for c, mu in enumerate(cents):
            nm = math.sqrt(dot(mu, mu))
            cos = dot(k, mu) / (nk * nm) if nk > 0 and nm > 0 else 0.0
            if best is None or cos > best:
                best, best_c = cos, c
        labels.append(best_c)
    return labels


def mean_update(keys, labels, cents):
    d = len(keys[0])
    out = []
    for c, old in enumerate(cents):
        acc = [0.0] * d
        n = 0
        for k, l in zip(keys, labels):
            if l == c:
                n += 1
                for j in range(d):
                    acc[j] += k[j]
        out.append([a / n for a in acc] if n else list(old))
    return out


def kmeans(keys, init_idx, n_iter):
    cents = [list(keys[i]) for i in init_idx]
    labels = None
    for _ in range(n_iter):
        labels = cosine_assign(keys, cents)
        cents = mean_update(keys, labels, cents)
    return cents, labels


def metadata(labels, C):
    sizes = [0] * C
    for l in labels:
        sizes[l] += 1
    offsets = [0]
    for c in range(C):
        offsets.append(offsets[-1] + sizes[c])
    sorted_idx = []
    for c in range(C):
        for i, l in enumerate(labels):
            if l == c:
                sorted_idx.append(i)
    return sizes, offsets, sorted_idx


def select_and_gather(q_group, cents, sizes, offsets, sorted_idx, budget, trim):
    C = len(cents)
    scores = []
    for mu in cents:
        s = 0.0
        for q in q_group:
            s += dot(q, mu)
        scores.append(s)
    remaining = list(range(C))
    order = []
    while remaining:                       # repeated selection of the maximum
        best = remaining[0]
        for c in remaining[1:]:
            if scores[c] > scores[best]:
                best = c
        order.append(best)
        remaining.remove(best)
    picked, total, n_sel = [], 0, 0
    for c in order:
        seg = sorted_idx[offsets[c]:offsets[c + 1]]
        if trim:
            if total >= budget:
                break
            room = budget - total
            if len(seg) > room:
                seg = seg[len(seg) - room:]
            picked.extend(seg)
            total += len(seg)
            n_sel += 1
        else:
            if total + len(seg) > budget:
                break
            picked.extend(seg)
            total += len(seg)
            n_sel += 1
    return scores, order, n_sel, picked


def softmax_attention(q, K, V, ids, scale):
    if not ids:
        return [0.0] * len(V[0])
    logits = [dot(q, K[i]) * scale for i in ids]
    m = max(logits)
    w = [math.exp(x - m) for x in logits]
    z = sum(w)
    out = [0.0] * len(V[0])
    for wi, i in zip(w, ids):
        for j in range(len(out)):
            out[j] += (wi / z) * V[i][j]
    return out
