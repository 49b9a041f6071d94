"""Link-prediction evaluation of the CPU oracle (TEST INFRASTRUCTURE ONLY): filtered ranks of
DistMult scores, MRR (Eq. 5) and Hits@k (Eq. 6) of the "Evaluation Metrics" section.

Plain NumPy in float64, one query at a time.  Nothing here is imported by the product package.

A *query* is (fixed entity, relation, true answer): for a test triple (h, r, t) the tail query
fixes h and asks for t, the head query fixes t and asks for h.  DistMult (Eq. 4) is symmetric in
its two entities, so both directions score a candidate e as  sum_k H[fixed][k] M[r][k] H[e][k].

Candidates are all entities except the true answer; the filtered setting also drops every
candidate whose triple is known to be true.  The rank of the true answer in the list sorted by
descending score is 1 + (candidates that score strictly higher); the paper does not say how equal
scores are ordered, so the number of candidates that score exactly the same is reported beside it
and the metrics place the true answer in the middle of its ties: rank = 1 + higher + equal / 2, the
mean position over all orders of the tied entries.
"""
from __future__ import annotations

import numpy as np


def queries_of(test_h, test_r, test_t):
    """Tail queries of all test triples, then head queries: (fixed, rel, true, side) with side 0 = the
    answer is the tail, 1 = the answer is the head."""
    h, r, t = (np.asarray(x, np.int64) for x in (test_h, test_r, test_t))
    n = len(h)
    return (np.concatenate([h, t]), np.concatenate([r, r]), np.concatenate([t, h]),
            np.concatenate([np.zeros(n, np.int64), np.ones(n, np.int64)]))


def known_answers(known_h, known_r, known_t):
    """Dictionaries (head, rel) -> set of tails and (tail, rel) -> set of heads of the known triples."""
    tails, heads = {}, {}
    for h, r, t in zip(np.asarray(known_h).tolist(), np.asarray(known_r).tolist(), np.asarray(known_t).tolist()):
        tails.setdefault((h, r), set()).add(t)
        heads.setdefault((t, r), set()).add(h)
    return tails, heads


def query_scores(H, M, fixed, rel):
    """Eq. 4 of one query against every entity, float64."""
    H = np.asarray(H, np.float64)
    return H @ (H[fixed] * np.asarray(M, np.float64)[rel])


def filtered_counts(H, M, test_h, test_r, test_t, known=None, tol=0.0):
    """For every query (tail queries first, then head queries): the number of remaining candidates that
    score higher than the true answer and the number that score the same.

    known: None (raw setting) or (known_h, known_r, known_t), the triples whose corruptions are dropped.
    tol > 0 returns instead the pair (lo, hi) that brackets any evaluation whose scores are within tol
    of the exact ones: lo = candidates above s_true + tol, hi = candidates at or above s_true - tol."""
    fixed, rel, true, side = queries_of(test_h, test_r, test_t)
    tails, heads = known_answers(*known) if known is not None else ({}, {})
    n_ent = np.asarray(H).shape[0]
    a = np.zeros(len(fixed), np.int64); b = np.zeros(len(fixed), np.int64)
    for q in range(len(fixed)):
        s = query_scores(H, M, fixed[q], rel[q])
        keep = np.ones(n_ent, bool)
        keep[true[q]] = False
        drop = (tails if side[q] == 0 else heads).get((int(fixed[q]), int(rel[q])), ())
        if drop:
            keep[np.fromiter(drop, np.int64)] = False
        st = s[true[q]]
        if tol > 0:
            a[q] = int(np.count_nonzero(keep & (s > st + tol)))
            b[q] = int(np.count_nonzero(keep & (s >= st - tol)))
        else:
            a[q] = int(np.count_nonzero(keep & (s > st)))
            b[q] = int(np.count_nonzero(keep & (s == st)))
    return a, b


def candidate_counts(H, M, fixed, rel, true, cand, tol=0.0):
    """The same two counts when every query brings its own candidate list cand[q] (the setting of the
    large citation graph: a fixed number of given negative targets per test edge).  An entry equal to the
    true answer is skipped."""
    H = np.asarray(H, np.float64); M = np.asarray(M, np.float64)
    cand = np.asarray(cand, np.int64)
    a = np.zeros(len(fixed), np.int64); b = np.zeros(len(fixed), np.int64)
    for q in range(len(fixed)):
        qv = H[fixed[q]] * M[rel[q]]
        st = float(H[true[q]] @ qv)
        c = cand[q][cand[q] != true[q]]
        s = H[c] @ qv
        if tol > 0:
            a[q] = int(np.count_nonzero(s > st + tol)); b[q] = int(np.count_nonzero(s >= st - tol))
        else:
            a[q] = int(np.count_nonzero(s > st)); b[q] = int(np.count_nonzero(s == st))
    return a, b


def ranks_of(higher, equal):
    return 1.0 + np.asarray(higher, np.float64) + 0.5 * np.asarray(equal, np.float64)


def metrics(higher, equal, ks=(1, 3, 10)):
    """MRR (Eq. 5) and Hits@k (Eq. 6) over all queries."""
    r = ranks_of(higher, equal)
    if len(r) == 0:
        return 0.0, [0.0 for _ in ks]
    return float(np.mean(1.0 / r)), [float(np.mean(r <= k)) for k in ks]
