"""Pins of the oracle's link-prediction evaluation ("Evaluation Metrics" section: filtered setting,
MRR Eq. 5, Hits@k Eq. 6) against the definition written out with sorted lists, a case worked by hand,
closed forms and a Monte-Carlo tie order."""
import itertools

import numpy as np
import pytest

from oracle import eval_oracle as ev


def random_model(seed, n=40, R=3, d=6):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(n, d)), rng.normal(size=(R, d))


def triples(seed, n, R, m):
    rng = np.random.default_rng(seed)
    return rng.integers(0, n, m), rng.integers(0, R, m), rng.integers(0, n, m)


def score(H, M, h, r, t):
    return sum(float(H[h][k]) * float(M[r][k]) * float(H[t][k]) for k in range(H.shape[1]))


def test_rank_is_the_position_in_the_sorted_list_of_unfiltered_corruptions():
    """The definition, literally: corrupt the tail (then the head) with every entity, drop corruptions
    that are known triples, sort positive + corruptions by descending score, read off the position."""
    n, R = 40, 3
    H, M = random_model(1, n, R)
    kh, kr, kt = triples(2, n, R, 300)
    th, tr, tt = triples(3, n, R, 25)
    known = set(zip(kh.tolist(), kr.tolist(), kt.tolist()))
    hi, eq = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt))
    assert not eq.any()                       # continuous random scores: no ties
    for i, (h, r, t) in enumerate(zip(th.tolist(), tr.tolist(), tt.tolist())):
        for side, q in ((0, i), (1, len(th) + i)):
            T = [((h, r, t), score(H, M, h, r, t))]
            for e in range(n):
                c = (h, r, e) if side == 0 else (e, r, t)
                if c == (h, r, t) or c in known:
                    continue
                T.append((c, score(H, M, *c)))
            T.sort(key=lambda x: -x[1])
            pos = [c for c, _ in T].index((h, r, t)) + 1
            assert pos == 1 + hi[q], (i, side)


def test_case_worked_by_hand():
    # one relation with m = 1, scalar embeddings 3, 1, 2, -1; test triple (0, r, 2)
    H = np.array([[3.0], [1.0], [2.0], [-1.0]]); M = np.array([[1.0]])
    th, tr, tt = np.array([0]), np.array([0]), np.array([2])
    # tail query: scores 3 * e = 9, 3, 6 (true), -3 -> entity 0 is above: rank 2
    # head query: scores e * 2 = 6 (true), 2, 4, -2 -> nothing above: rank 1
    hi, eq = ev.filtered_counts(H, M, th, tr, tt)
    assert hi.tolist() == [1, 0] and eq.tolist() == [0, 0]
    mrr, hits = ev.metrics(hi, eq, (1, 3))
    assert mrr == pytest.approx(0.75) and hits == [0.5, 1.0]
    # (0, r, 0) is a known triple: its corruption leaves the tail query's list
    hi, eq = ev.filtered_counts(H, M, th, tr, tt, (np.array([0]), np.array([0]), np.array([0])))
    assert hi.tolist() == [0, 0]
    assert ev.metrics(hi, eq, (1,)) == (1.0, [1.0])
    # a known triple with another relation or another head filters nothing
    hi, _ = ev.filtered_counts(np.hstack([H, H]), np.array([[1.0, 0.0], [0.0, 1.0]]), th, tr, tt,
                               (np.array([0, 1]), np.array([1, 0]), np.array([0, 0])))
    assert hi.tolist() == [1, 0]


def test_metrics_on_given_ranks():
    # ranks 1, 2, 4: MRR = (1 + 1/2 + 1/4) / 3, Hits@1 = 1/3, Hits@3 = 2/3, Hits@10 = 1
    mrr, hits = ev.metrics([0, 1, 3], [0, 0, 0], (1, 3, 10))
    assert mrr == pytest.approx(7.0 / 12.0)
    assert hits == pytest.approx([1 / 3, 2 / 3, 1.0])
    # ties: two entries tied with the truth -> positions 1, 2, 3 equally likely -> rank 2
    assert ev.ranks_of([0], [2]).tolist() == [2.0]


def test_filter_removes_exactly_the_known_entities_that_outscore():
    n, R = 60, 2
    H, M = random_model(5, n, R)
    kh, kr, kt = triples(6, n, R, 500)
    th, tr, tt = triples(7, n, R, 40)
    raw, _ = ev.filtered_counts(H, M, th, tr, tt)
    flt, _ = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt))
    assert (flt <= raw).all() and (flt < raw).any()
    for i in range(len(th)):
        h, r, t = int(th[i]), int(tr[i]), int(tt[i])
        outs = {int(e) for e in kt[(kh == h) & (kr == r)] if e != t and score(H, M, h, r, e) > score(H, M, h, r, t)}
        assert raw[i] - flt[i] == len(outs)
        outs = {int(e) for e in kh[(kt == t) & (kr == r)] if e != h and score(H, M, e, r, t) > score(H, M, h, r, t)}
        assert raw[len(th) + i] - flt[len(th) + i] == len(outs)


def test_a_model_that_knows_the_answers_scores_one():
    # orthonormal entity embeddings, test triples (i, 0, i): score(i, e) = [i == e]
    n = 12
    H = np.eye(n); M = np.ones((1, n))
    th = np.arange(n); tr = np.zeros(n, int)
    hi, eq = ev.filtered_counts(H, M, th, tr, th)
    assert not hi.any() and not eq.any()
    assert ev.metrics(hi, eq, (1,)) == (1.0, [1.0])
    # the sign of the relation flipped: the truth is the only negative score -> last of n
    hi, eq = ev.filtered_counts(H, -M, th, tr, th)
    assert (hi == n - 1).all() and not eq.any()
    mrr, hits = ev.metrics(hi, eq, (1, n - 1, n))
    assert mrr == pytest.approx(1.0 / n) and hits == [0.0, 0.0, 1.0]


def test_ties_take_the_mean_position_of_a_random_order():
    n = 9
    H = np.zeros((n, 4)); M = np.ones((2, 4))
    hi, eq = ev.filtered_counts(H, M, np.array([1]), np.array([0]), np.array([5]))
    assert hi.tolist() == [0, 0] and eq.tolist() == [n - 1, n - 1]
    r = ev.ranks_of(hi, eq)
    assert r.tolist() == [1 + (n - 1) / 2] * 2
    # every order of the tied list is equally likely: mean position of the truth over all rotations of a
    # shuffled list, by simulation
    rng = np.random.default_rng(0)
    pos = [int(np.nonzero(rng.permutation(n) == 0)[0][0]) + 1 for _ in range(20000)]
    assert abs(np.mean(pos) - r[0]) < 0.06
    # filtered ties leave the count
    hi, eq = ev.filtered_counts(H, M, np.array([1]), np.array([0]), np.array([5]),
                                (np.array([1, 1, 3]), np.array([0, 0, 0]), np.array([2, 3, 5])))
    assert eq.tolist() == [n - 3, n - 2]


def test_candidate_lists_and_the_tolerance_band():
    n, R = 50, 3
    H, M = random_model(9, n, R)
    th, tr, tt = triples(10, n, R, 30)
    fixed, rel, true, side = ev.queries_of(th, tr, tt)
    raw_hi, raw_eq = ev.filtered_counts(H, M, th, tr, tt)
    allc = np.tile(np.arange(n), (len(fixed), 1))
    c_hi, c_eq = ev.candidate_counts(H, M, fixed, rel, true, allc)
    np.testing.assert_array_equal(c_hi, raw_hi); np.testing.assert_array_equal(c_eq, raw_eq)
    # a shorter list: brute force
    rng = np.random.default_rng(11)
    cand = rng.integers(0, n, (len(fixed), 7))
    c_hi, _ = ev.candidate_counts(H, M, fixed, rel, true, cand)
    for q in range(len(fixed)):
        st = score(H, M, int(fixed[q]), int(rel[q]), int(true[q]))
        want = sum(1 for e in cand[q].tolist() if e != true[q] and score(H, M, int(fixed[q]), int(rel[q]), e) > st)
        assert c_hi[q] == want
    lo, hi = ev.filtered_counts(H, M, th, tr, tt, tol=1e-2)
    assert (lo <= raw_hi).all() and (raw_hi + raw_eq <= hi).all() and (lo < hi).any()
    lo0, hi0 = ev.filtered_counts(H, M, th, tr, tt, tol=1e-300)
    np.testing.assert_array_equal(lo0, raw_hi); np.testing.assert_array_equal(hi0, raw_hi)
