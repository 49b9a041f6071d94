"""The entry point that allocates nothing, kge_eval_rank_all_static, against kge_eval_rank_all.

Both run the same kernels; the first keeps its scratch in a static device array inside the library
instead of a caller-provided workspace.  The outputs are integers (counts of entities scoring above /
exactly at the answer), so they must agree bit for bit - on two calls in a row, the second smaller
than the first (it must not see anything the first left in the shared array), and also against the
fp64 oracle where the embeddings are small integers (every score exact, ties included)."""
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


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def triples(seed, n, R, m):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32))


def both(kb, H, M, test, filt):
    """(higher, equal) of the workspace call and of the static-scratch call on the same inputs."""
    import torch
    th, tr, tt = (dev(x) for x in test)
    hi_w, eq_w = kb.eval_rank_all(H, M, th, tr, tt, filt)
    hi_s = torch.full((2 * len(test[0]),), -7, dtype=torch.int32, device="cuda")
    eq_s = torch.full_like(hi_s, -7)
    kb.eval_rank_all_static(H, M, th, tr, tt, hi_s, eq_s, filt)
    torch.cuda.synchronize()
    return hi_w.cpu().numpy(), eq_w.cpu().numpy(), hi_s.cpu().numpy(), eq_s.cpu().numpy()


def test_static_scratch_matches_workspace_call_twice_in_a_row(kb):
    n, R, d = 4099, 7, 72
    rng = np.random.default_rng(21)
    Hi = rng.integers(-2, 3, (n, d)).astype(np.float32)
    Mi = rng.integers(-1, 2, (R, d)).astype(np.float32)
    known = triples(22, n, R, 30000)
    big = triples(23, n, R, 700)          # 1400 queries: 11 query tiles, a ragged last one
    small = triples(24, n, R, 90)         # then 180 queries in the same array
    known = tuple(np.concatenate([k, b, s]) for k, b, s in zip(known, big, small))
    filt = kb.EvalFilter(known[0], known[1], known[2], n, R)
    H, M = dev(Hi), dev(Mi)
    for name, test in (("first call, 700 test triples", big), ("second call, 90 test triples", small)):
        say("static scratch:", name)
        hi_w, eq_w, hi_s, eq_s = both(kb, H, M, test, filt)
        np.testing.assert_array_equal(hi_s, hi_w)
        np.testing.assert_array_equal(eq_s, eq_w)
        whi, weq = ev.filtered_counts(Hi, Mi, test[0], test[1], test[2], known)
        assert weq.max() > 0
        np.testing.assert_array_equal(hi_s, whi)
        np.testing.assert_array_equal(eq_s, weq)
    # real-valued embeddings, raw setting (no filter), smaller again: still the workspace call's bits
    say("static scratch: third call, real embeddings, no filter")
    Hr = dev(rng.normal(size=(n, d)).astype(np.float32))
    Mr = dev(rng.normal(size=(R, d)).astype(np.float32))
    hi_w, eq_w, hi_s, eq_s = both(kb, Hr, Mr, triples(25, n, R, 33), None)
    np.testing.assert_array_equal(hi_s, hi_w)
    np.testing.assert_array_equal(eq_s, eq_w)


def test_static_scratch_refuses_what_does_not_fit(kb):
    """The size check is on the host: nothing is launched, the outputs stay as they were."""
    import torch
    n, R, d = 64, 2, 256
    H = torch.zeros((n, d), device="cuda"); M = torch.zeros((R, d), device="cuda")
    n_test = 40000                       # 80,000 queries x (1024 + 36) bytes > 32 MiB
    assert kb.eval_workspace_bytes(2 * n_test, d) > kb.EVAL_STATIC_BYTES
    t = torch.zeros(n_test, dtype=torch.int32, device="cuda")
    hi = torch.full((2 * n_test,), -7, dtype=torch.int32, device="cuda"); eq = torch.full_like(hi, -7)
    with pytest.raises(kb.KgeError) as e:
        kb.eval_rank_all_static(H, M, t, t, t, hi, eq)
    assert e.value.status == -2 and "static" in str(e.value)
    torch.cuda.synchronize()
    assert int(hi.min()) == -7 and int(eq.max()) == -7
    # an empty batch is fine and touches nothing
    kb.eval_rank_all_static(H, M, t[:0], t[:0], t[:0], hi[:0], eq[:0])
    torch.cuda.synchronize()
