"""Pins of the oracle's dropout on layer inputs (large-graph training setting of Sec. 4: rate 0.2):
the mask against an independent Philox engine, the rate, independence across layers / steps /
columns, unbiasedness, and the backward pass against finite differences."""
import numpy as np
import pytest

from paper_2201_02791_amd import synth


def test_mask_follows_an_independent_philox_engine(orc, aten_philox):
    rng = np.random.default_rng(0)
    H = rng.normal(size=(9, 11))
    for p, seed, step, layer in [(0.2, 5, 0, 0), (0.5, 2**63 + 12345, 2**40 + 3, 1), (0.9, 77, 9, 3)]:
        out, mask = orc.dropout(H, p, seed, step, layer)
        thr = int(p * 2**32)
        for i in range(H.shape[0]):
            for k in range(H.shape[1]):
                x = aten_philox(seed ^ ((layer + 1) << 32), step, i | ((k // 4) << 32))[k % 4]
                keep = int(x) >= thr
                assert mask[i, k] == keep
                want = H[i, k] / (1.0 - p) if keep else 0.0
                assert out[i, k] == pytest.approx(want, rel=1e-15, abs=0)


def test_rate_zero_is_the_identity(orc):
    H = np.random.default_rng(1).normal(size=(17, 6))
    out, mask = orc.dropout(H, 0.0, 3, 4, 0)
    np.testing.assert_array_equal(out, H)
    assert mask.all()


@pytest.mark.parametrize("p", [0.2, 0.5])
def test_keep_rate_and_independence(orc, p):
    H = np.ones((4000, 64))
    _, m0 = orc.dropout(H, p, 11, 0, 0)
    n = m0.size
    sd = np.sqrt(p * (1 - p) / n)
    assert abs(m0.mean() - (1 - p)) < 5 * sd
    # every column and every row has the rate too (no column of the 4-word block is stuck)
    assert np.abs(m0.mean(0) - (1 - p)).max() < 5 * np.sqrt(p * (1 - p) / H.shape[0])
    # same arguments, same mask
    np.testing.assert_array_equal(orc.dropout(H, p, 11, 0, 0)[1], m0)
    # another layer, step or seed: a mask that agrees as often as two independent ones do
    agree = p * p + (1 - p) * (1 - p)
    for args in [(11, 0, 1), (11, 1, 0), (12, 0, 0), (11 + 2**32, 0, 0), (11, 2**32, 0)]:
        m1 = orc.dropout(H, p, *args)[1]
        assert abs((m1 == m0).mean() - agree) < 5 * np.sqrt(agree * (1 - agree) / n), args
    # neighbouring columns and rows are uncorrelated
    a = m0.astype(np.float64) - (1 - p)
    for sh, ax in [(1, 1), (2, 1), (3, 1), (4, 1), (1, 0)]:
        c = (a * np.roll(a, sh, axis=ax)).mean() / (p * (1 - p))
        assert abs(c) < 5 / np.sqrt(n), (sh, ax, c)


def test_unbiased_over_steps(orc):
    H = np.random.default_rng(2).normal(size=(50, 8))
    acc = np.zeros_like(H)
    T = 400
    for t in range(T):
        acc += orc.dropout(H, 0.2, 9, t, 0)[0]
    # variance of one draw of element x: x^2 p / (1 - p)
    sd = np.abs(H) * np.sqrt(0.2 / 0.8 / T)
    assert (np.abs(acc / T - H) < 5 * sd + 1e-12).all()


def test_backward_through_dropout_matches_finite_differences(orc):
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=60, n_triples=150, n_pos=4, d=6, n_bases=2)
    head, rel, tail = synth.make_triples(spec)
    part = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, 1, 0, 2, 0)
    params = synth.make_params(spec, part["n_vert"])
    # smooth activations so that finite differences are clean
    layers = [dict(V=np.asarray(params["V"][l], np.float64), a=np.asarray(params["a"][l], np.float64),
                   W0=np.asarray(params["W0"][l], np.float64), act=0) for l in range(2)]
    H0 = np.asarray(params["H0"], np.float64)
    rng = np.random.default_rng(3)
    Wt = rng.normal(size=(part["n_vert"], layers[-1]["W0"].shape[1]))
    drop = (0.3, 21, 5)

    def loss(H0_, layers_):
        Hs, _, _ = orc.rgcn_forward(part, layers_, H0_, drop=drop)
        return float((Hs[-1] * Wt).sum())

    Hs, pres, masks = orc.rgcn_forward(part, layers, H0, drop=drop)
    assert 0 < masks[0].mean() < 1 and 0 < masks[1].mean() < 1
    grads, dH0 = orc.rgcn_backward(part, layers, Hs, pres, Wt, True, drop=drop, masks=masks)
    # the network is multilinear in each parameter tensor without activations: central differences are exact
    eps = 1e-3
    for _ in range(12):
        i, k = int(rng.integers(0, H0.shape[0])), int(rng.integers(0, H0.shape[1]))
        Hp, Hm = H0.copy(), H0.copy(); Hp[i, k] += eps; Hm[i, k] -= eps
        fd = (loss(Hp, layers) - loss(Hm, layers)) / (2 * eps)
        assert dH0[i, k] == pytest.approx(fd, rel=1e-7, abs=1e-9)
        assert (dH0[i, k] == 0) or masks[0][i, k]
    for l in range(2):
        for name, g in (("V", "dV"), ("a", "da"), ("W0", "dW0")):
            for _ in range(4):
                idx = tuple(int(rng.integers(0, n)) for n in layers[l][name].shape)
                lp = [dict(x) for x in layers]; lm = [dict(x) for x in layers]
                lp[l][name] = layers[l][name].copy(); lp[l][name][idx] += eps
                lm[l][name] = layers[l][name].copy(); lm[l][name][idx] -= eps
                fd = (loss(H0, lp) - loss(H0, lm)) / (2 * eps)
                assert grads[l][g][idx] == pytest.approx(fd, rel=1e-7, abs=1e-9), (l, name, idx)
