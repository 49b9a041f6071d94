"""Pins of the oracle's counter-based negative sampler (Sec. 2.1, Sec. 3.3.1) and of the
DistMult score / cross-entropy loss (Eq. 4, Eq. 3)."""
import math
import os

import numpy as np
import pytest

from test_oracle_partition import tiny_graph


def test_philox_matches_an_independent_library_engine(orc, aten_philox):
    rng = np.random.default_rng(0)
    cases = [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (2**64 - 1, 2**64 - 1, 2**64 - 1)]
    for _ in range(200):
        cases.append(tuple(int(x) for x in rng.integers(0, 2**63, 3)))
    for seed, subseq, off in cases:
        ctr = [off & 0xFFFFFFFF, off >> 32, subseq & 0xFFFFFFFF, subseq >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        np.testing.assert_array_equal(orc.philox4x32_10(ctr, key), aten_philox(seed, subseq, off))


def test_philox_avalanche_and_bit_balance(orc):
    # A one-bit change of counter or key flips about half of the 128 output bits.
    rng = np.random.default_rng(1)
    flips = []
    for _ in range(300):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64).astype(np.uint32)
        base = orc.philox4x32_10(ctr, key)
        c2, k2 = ctr.copy(), key.copy()
        w = int(rng.integers(0, 6)); b = np.uint32(1 << int(rng.integers(0, 32)))
        if w < 4:
            c2[w] ^= b
        else:
            k2[w - 4] ^= b
        diff = base ^ orc.philox4x32_10(c2, k2)
        flips.append(sum(bin(int(x)).count("1") for x in diff))
    assert 58 < np.mean(flips) < 70


def test_negatives_stay_inside_the_partition_and_follow_the_draw(orc, aten_philox):
    head, rel, tail, n, R = tiny_graph(2, n=200, R=4, m=500)
    part = orc.build_partition(head, rel, tail, n, R, 4, 1, 2, 0)
    pos = np.arange(part["n_core"], dtype=np.int32)[::-1].copy()
    seed, step = 0x123456789ABCDEF, 7
    ne, ns = orc.sample_negatives(part, pos, 5, 1, seed, step)
    assert ne.shape == (len(pos), 5)
    cand = set(int(c) for c in part["cand"])
    core_ends = set(int(x) for x in part["core_h"]) | set(int(x) for x in part["core_t"])
    assert cand == core_ends                         # Sec. 3.3.1, domain 0: vertices of core edges
    assert set(int(x) for x in ne.ravel()) <= cand   # never outside the partition
    for p in (0, 3, len(pos) - 1):
        for k in range(5):
            x = aten_philox(seed, step, int(pos[p]) | (k << 32))
            assert ne[p, k] == part["cand"][(int(x[0]) * part["n_cand"]) >> 32]
            assert ns[p, k] == (1 if int(x[1]) >= 2**31 else 0)
    # tail-only mode never corrupts the head; same entity draw
    ne0, ns0 = orc.sample_negatives(part, pos, 5, 0, seed, step)
    assert (ns0 == 0).all()
    np.testing.assert_array_equal(ne0, ne)
    # a negative depends only on (core edge, slot, step, seed), not on its place in the batch
    ne_r, ns_r = orc.sample_negatives(part, pos[::-1].copy(), 5, 1, seed, step)
    np.testing.assert_array_equal(ne_r[::-1], ne)
    np.testing.assert_array_equal(ns_r[::-1], ns)
    ne_s, _ = orc.sample_negatives(part, pos, 5, 1, seed, step + 1)
    assert (ne_s != ne).mean() > 0.9


def test_negative_draws_are_uniform_and_the_coin_is_fair(orc):
    head, rel, tail, n, R = tiny_graph(3, n=64, R=2, m=400)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 1)
    n_cand = part["n_cand"]
    pos = np.arange(20000, dtype=np.int32)           # counter word only; indices need not exist
    ne, ns = orc.sample_negatives(part, pos, 50, 1, 99, 0)
    counts = np.bincount(ne.ravel(), minlength=part["n_vert"])[part["cand"]]
    T = ne.size
    chi2 = ((counts - T / n_cand) ** 2 / (T / n_cand)).sum()
    dof = n_cand - 1
    assert abs(chi2 - dof) < 6 * math.sqrt(2 * dof)
    assert abs(ns.mean() - 0.5) < 4 * 0.5 / math.sqrt(T)


def test_zero_embeddings_give_ln2_and_half_deltas(orc):
    head, rel, tail, n, R = tiny_graph(4)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    pos = np.arange(10, dtype=np.int32)
    ne, ns = orc.sample_negatives(part, pos, 3, 1, 1, 0)
    H = np.zeros((part["n_vert"], 4)); M = np.ones((R, 4))
    r = orc.distmult_score_loss(part, H, M, pos, ne, ns)
    assert (r["scores"] == 0).all()
    assert r["loss"] == pytest.approx(math.log(2.0), abs=1e-15)
    assert (r["dH"] == 0).all() and (r["dM"] == 0).all()


def test_scalar_case_by_hand(orc):
    # d = 1: one positive (h_s, m, h_t) = (2, .5, 3) -> g = 3; one tail-corrupted negative with
    # h_t' = -1 -> g' = -1.  L = [log(1+e^-3) + log(1+e^-1)] / 2.
    head = np.array([0], np.int32); rel = np.array([0], np.int32); tail = np.array([1], np.int32)
    part = orc.build_partition(np.array([0, 2], np.int32), np.array([0, 0], np.int32),
                               np.array([1, 0], np.int32), 3, 1, 1, 0, 2, 0)
    H = np.array([[2.0], [3.0], [-1.0]]); M = np.array([[0.5]])
    r = orc.distmult_score_loss(part, H, M, np.array([0], np.int32), np.array([[2]], np.int32),
                                np.array([[0]], np.uint8))
    np.testing.assert_allclose(r["scores"], [[3.0, -1.0]], rtol=1e-15)
    want = (math.log1p(math.exp(-3.0)) + math.log1p(math.exp(-1.0))) / 2
    assert r["loss"] == pytest.approx(want, rel=1e-14)
    sig = lambda x: 1 / (1 + math.exp(-x))
    dpos, dneg = (sig(3.0) - 1) / 2, sig(-1.0) / 2
    # dH_s = dpos*m*h_t + dneg*m*h_t',  dH_t = dpos*m*h_s,  dH_t' = dneg*m*h_s, dM = dpos*6 + dneg*(-2)
    np.testing.assert_allclose(r["dH"][:, 0], [dpos * 1.5 - dneg * 0.5, dpos * 1.0, dneg * 1.0], rtol=1e-13)
    np.testing.assert_allclose(r["dM"][0, 0], dpos * 6 - dneg * 2, rtol=1e-13)
    # head corruption: (s', r, t) with s' = vertex 2
    r2 = orc.distmult_score_loss(part, H, M, np.array([0], np.int32), np.array([[2]], np.int32),
                                 np.array([[1]], np.uint8))
    np.testing.assert_allclose(r2["scores"], [[3.0, -1.5]], rtol=1e-15)


def test_distmult_is_symmetric_and_matches_numpy(orc):
    head, rel, tail, n, R = tiny_graph(5, n=30, m=100)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(2)
    d = 5
    H = rng.normal(0, 1, (part["n_vert"], d)); M = rng.normal(0, 1, (R, d))
    pos = rng.permutation(part["n_core"])[:40].astype(np.int32)
    ne, ns = orc.sample_negatives(part, pos, 4, 1, 3, 0)
    r = orc.distmult_score_loss(part, H, M, pos, ne, ns)
    s = np.repeat(part["core_h"][pos][:, None], 5, 1); t = np.repeat(part["core_t"][pos][:, None], 5, 1)
    s[:, 1:] = np.where(ns == 1, ne, s[:, 1:]); t[:, 1:] = np.where(ns == 0, ne, t[:, 1:])
    rr = np.repeat(part["core_r"][pos][:, None], 5, 1)
    g = np.einsum("pkd,pkd,pkd->pk", H[s], M[rr], H[t])
    np.testing.assert_allclose(r["scores"], g, rtol=1e-12, atol=1e-13)
    g_sw = np.einsum("pkd,pkd,pkd->pk", H[t], M[rr], H[s])     # g(s,r,t) = g(t,r,s) for diagonal M_r
    np.testing.assert_allclose(r["scores"], g_sw, rtol=1e-12, atol=1e-13)
    y = np.zeros_like(g); y[:, 0] = 1
    p = 1 / (1 + np.exp(-g))
    want = -(y * np.log(p) + (1 - y) * np.log(1 - p)).mean()
    assert r["loss"] == pytest.approx(want, rel=1e-12)
