"""GPU parity of the link-prediction evaluation ("Evaluation Metrics" section: filtered ranks, MRR Eq. 5,
Hits@k Eq. 6) against the fp64 oracle.

Ranks are integers decided by comparing floating-point scores.  With small-integer embeddings every
score is exact in fp32 and fp64 alike, so the counts must agree bit for bit, ties included.  With
real-valued embeddings the fp32 scores differ from the fp64 ones in the last places: a candidate whose
score is that close to the answer's may fall on either side, so the counts are held to the bracket the
oracle computes with that margin, and must be equal wherever the bracket has closed."""
import sys

import numpy as np
import pytest

from oracle import eval_oracle as ev

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


def dev(x, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def integer_model(seed, n, R, d):
    rng = np.random.default_rng(seed)
    return rng.integers(-2, 3, (n, d)).astype(np.float32), rng.integers(-1, 2, (R, d)).astype(np.float32)


def real_model(seed, n, R, d):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(n, d)).astype(np.float32), rng.normal(size=(R, d)).astype(np.float32)


def triples(seed, n, R, m):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32))


def gpu_rank_all(kb, H, M, test, known, n, R):
    import torch
    filt = kb.EvalFilter(known[0], known[1], known[2], n, R) if known is not None else None
    hi, eq = kb.eval_rank_all(dev(H), dev(M), dev(test[0]), dev(test[1]), dev(test[2]), filt)
    torch.cuda.synchronize()
    return hi, eq


@pytest.mark.parametrize("n,R,d,n_test", [(777, 5, 100, 150), (300, 2, 256, 64), (130, 3, 4, 1)])
def test_the_two_kernels_give_a_pair_the_same_bits(kb, n, R, d, n_test):
    """The tile kernel's score of (query, answer) and the per-query kernel's are the same float, which is
    what makes subtracting the filtered entries exact; and all scores match the fp64 ones."""
    say("score bits", n, R, d, n_test)
    import torch
    H, M = real_model(1, n, R, d)
    th, tr, tt = triples(2, n, R, n_test)
    scores, ans = kb.eval_debug_scores(dev(H), dev(M), dev(th), dev(tr), dev(tt))
    torch.cuda.synchronize()
    fixed, rel, true, _ = ev.queries_of(th, tr, tt)
    picked = scores[torch.arange(2 * n_test, device="cuda"), dev(true)]
    assert torch.equal(picked.view(torch.int32), ans.view(torch.int32))
    want = np.stack([ev.query_scores(H, M, fixed[q], rel[q]) for q in range(2 * n_test)])
    assert np.abs(scores.cpu().numpy() - want).max() <= 1e-5 * np.abs(want).max()


@pytest.mark.parametrize("n,R,d,n_test,n_known", [(1000, 4, 32, 200, 6000), (129, 2, 8, 300, 900),
                                                   (5000, 30, 64, 40, 20000)])
def test_filtered_counts_exact_on_integer_embeddings(kb, n, R, d, n_test, n_known):
    say("integer", n, R, d, n_test, n_known)
    H, M = integer_model(3, n, R, d)
    th, tr, tt = triples(4, n, R, n_test)
    kh, kr, kt = triples(5, n, R, n_known)
    # the known set holds the test triples themselves, duplicates, and other answers of the same (h, r) / (r, t)
    kh = np.concatenate([kh, th, th, th[:50]]); kr = np.concatenate([kr, tr, tr, tr[:50]])
    kt = np.concatenate([kt, tt, tt, (tt[:50] + 1) % n]).astype(np.int32)
    hi, eq = gpu_rank_all(kb, H, M, (th, tr, tt), (kh, kr, kt), n, R)
    whi, weq = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt))
    assert weq.max() > 0                         # the case has ties
    np.testing.assert_array_equal(hi.cpu().numpy(), whi)
    np.testing.assert_array_equal(eq.cpu().numpy(), weq)
    raw_hi, raw_eq = gpu_rank_all(kb, H, M, (th, tr, tt), None, n, R)
    wr_hi, wr_eq = ev.filtered_counts(H, M, th, tr, tt)
    np.testing.assert_array_equal(raw_hi.cpu().numpy(), wr_hi)
    np.testing.assert_array_equal(raw_eq.cpu().numpy(), wr_eq)
    assert (whi < wr_hi).any()                   # and the filter matters
    # metrics: MRR and Hits@k in double
    import torch
    got = kb.eval_metrics(hi, eq, (1, 3, 10)).cpu().numpy()
    mrr, hits = ev.metrics(whi, weq, (1, 3, 10))
    np.testing.assert_allclose(got, [mrr] + hits, rtol=1e-12, atol=0)


def test_many_entity_tiles_per_block(kb):
    """Enough tiles that a block walks several entity tiles and keeps its counts across them."""
    say("several tiles per block")
    n, R, d, n_test = 300001, 3, 16, 130
    H, M = integer_model(7, n, R, d)
    th, tr, tt = triples(8, n, R, n_test)
    kh, kr, kt = triples(9, n, R, 50000)
    hi, eq = gpu_rank_all(kb, H, M, (th, tr, tt), (kh, kr, kt), n, R)
    whi, weq = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt))
    np.testing.assert_array_equal(hi.cpu().numpy(), whi)
    np.testing.assert_array_equal(eq.cpu().numpy(), weq)


@pytest.mark.parametrize("n,R,d,n_test", [(3000, 6, 128, 200), (1500, 3, 36, 77)])
def test_filtered_counts_on_real_embeddings(kb, n, R, d, n_test):
    say("real", n, R, d, n_test)
    H, M = real_model(11, n, R, d)
    th, tr, tt = triples(12, n, R, n_test)
    kh, kr, kt = triples(13, n, R, 30000)
    hi, eq = gpu_rank_all(kb, H, M, (th, tr, tt), (kh, kr, kt), n, R)
    hi, eq = hi.cpu().numpy(), eq.cpu().numpy()
    fixed, rel, true, _ = ev.queries_of(th, tr, tt)
    smax = max(np.abs(ev.query_scores(H, M, fixed[q], rel[q])).max() for q in range(0, 2 * n_test, 17))
    tol = 1e-6 * smax               # fp32 sums of d products against fp64: 2^-24 sqrt(d) of the terms' size, with margin
    lo, up = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt), tol=tol)
    assert (lo <= hi).all() and (hi + eq <= up).all()
    closed = lo == up
    assert closed.mean() > 0.95     # almost every bracket has closed: there the count is unique
    whi, weq = ev.filtered_counts(H, M, th, tr, tt, (kh, kr, kt))
    np.testing.assert_array_equal(hi[closed], whi[closed])
    assert not eq[closed].any()
    import torch
    got = kb.eval_metrics(dev(hi), dev(eq), (1, 10)).cpu().numpy()
    mrr, hits = ev.metrics(whi, weq, (1, 10))
    assert abs(got[0] - mrr) <= 1e-3 * mrr


@pytest.mark.parametrize("n_cand,d", [(1000, 128), (33, 128), (1, 128), (100, 8), (77, 48), (50, 200), (40, 400),
                                      (19, 1024)])
def test_candidate_lists(kb, n_cand, d):
    """The large citation graph's setting: every query ranks its answer against its own list.  The widths
    cover every lanes-per-row / pieces-per-lane form of the kernel."""
    say("candidates", n_cand, d)
    import torch
    n, R, nq = 4000, 1, 300
    rng = np.random.default_rng(21)
    fixed = rng.integers(0, n, nq).astype(np.int32); rel = np.zeros(nq, np.int32)
    answer = rng.integers(0, n, nq).astype(np.int32)
    cand = rng.integers(0, n, (nq, n_cand)).astype(np.int32)
    cand[::7, 0] = answer[::7]            # the answer inside its own list is skipped
    for make, exact in ((integer_model, True), (real_model, False)):
        H, M = make(22, n, R, d)
        hi, eq = kb.eval_rank_candidates(dev(H), dev(M), dev(fixed), dev(rel), dev(answer), dev(cand))
        torch.cuda.synchronize()
        hi, eq = hi.cpu().numpy(), eq.cpu().numpy()
        if exact:
            whi, weq = ev.candidate_counts(H, M, fixed, rel, answer, cand)
            np.testing.assert_array_equal(hi, whi); np.testing.assert_array_equal(eq, weq)
        else:
            tol = 1e-6 * 4.0 * d
            lo, up = ev.candidate_counts(H, M, fixed, rel, answer, cand, tol=tol)
            assert (lo <= hi).all() and (hi + eq <= up).all()
            whi, _ = ev.candidate_counts(H, M, fixed, rel, answer, cand)
            closed = lo == up
            np.testing.assert_array_equal(hi[closed], whi[closed])


def test_empty_inputs_and_errors(kb):
    say("edge cases")
    import torch
    H, M = integer_model(1, 50, 2, 8)
    e = torch.empty(0, dtype=torch.int32, device="cuda")
    hi, eq = kb.eval_rank_all(dev(H), dev(M), e, e, e)
    assert hi.numel() == 0
    out = kb.eval_metrics(hi, eq, (1,)).cpu().numpy()
    assert out.tolist() == [0.0, 0.0]
    # an empty filter is the raw setting
    th, tr, tt = triples(2, 50, 2, 20)
    f = kb.EvalFilter(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32), 50, 2)
    a = kb.eval_rank_all(dev(H), dev(M), dev(th), dev(tr), dev(tt), f)
    b = kb.eval_rank_all(dev(H), dev(M), dev(th), dev(tr), dev(tt), None)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    with pytest.raises(kb.KgeError):          # a filter built for other counts
        kb.eval_rank_all(dev(H), dev(M), dev(th), dev(tr), dev(tt), kb.EvalFilter(th, tr, tt, 51, 2))
    with pytest.raises(kb.KgeError):          # id out of range in the known triples
        kb.EvalFilter(np.array([50], np.int32), np.array([0], np.int32), np.array([0], np.int32), 50, 2)
    with pytest.raises(kb.KgeError):          # d not a multiple of 4
        kb.eval_rank_all(dev(H[:, :6].copy()), dev(M[:, :6].copy()), dev(th), dev(tr), dev(tt))
