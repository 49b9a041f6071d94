"""Central finite differences (fp64) pin every gradient the oracle's backward pass returns:
V, a, W_0 of both layers, the decoder diagonals M and the layer-1 input H0."""
import numpy as np
import pytest

from test_oracle_partition import tiny_graph
from test_oracle_rgcn import rand_layer


def setup_case(orc, acts, seed=0, P=1, pid=0):
    head, rel, tail, n, R = tiny_graph(40 + seed, n=24, R=2, m=70)
    part = orc.build_partition(head, rel, tail, n, R, P, pid, 2, 0)
    rng = np.random.default_rng(seed)
    d, B = 4, 3
    layers = [rand_layer(rng, 2 * R, B, d, d, a) for a in acts]
    H0 = rng.normal(0, 1, (part["n_vert"], d))
    M = rng.normal(0, 1, (R, d))
    pos = rng.permutation(part["n_core"])[:12].astype(np.int32)
    return part, layers, H0, M, pos


def loss_of(orc, part, layers, H0, M, pos):
    Hs, _ = orc.rgcn_forward(part, layers, H0)
    ne, ns = orc.sample_negatives(part, pos, 3, 1, 5, 0)
    return orc.distmult_score_loss(part, Hs[-1], M, pos, ne, ns)["loss"]


def fd(f, x, idx, eps=1e-6):
    old = x[idx]
    x[idx] = old + eps; lp = f()
    x[idx] = old - eps; lm = f()
    x[idx] = old
    return (lp - lm) / (2 * eps)


@pytest.mark.parametrize("acts,P,pid", [([0, 0], 1, 0), ([1, 0], 1, 0), ([1, 1], 1, 0), ([1, 0], 3, 1)])
def test_all_gradients_against_finite_differences(orc, acts, P, pid):
    part, layers, H0, M, pos = setup_case(orc, acts, seed=len(acts) + sum(acts), P=P, pid=pid)
    if part["n_core"] == 0:
        pytest.skip("empty partition")
    res = orc.train_step(part, layers, H0, M, pos, 3, 1, 5, 0)
    f = lambda: loss_of(orc, part, layers, H0, M, pos)
    assert res["loss"] == pytest.approx(f(), rel=1e-14)
    rng = np.random.default_rng(9)

    def check(arr, grad, name, n=12):
        flat_idx = rng.choice(arr.size, size=min(n, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            num = fd(f, arr, idx)
            assert grad[idx] == pytest.approx(num, rel=2e-5, abs=2e-9), (name, idx)

    for l, lay in enumerate(layers):
        check(lay["V"], res["grads"][l]["dV"], f"dV{l}")
        check(lay["a"], res["grads"][l]["da"], f"da{l}")
        check(lay["W0"], res["grads"][l]["dW0"], f"dW0{l}")
    check(M, res["dM"], "dM")
    check(H0, res["dH0"], "dH0", n=20)


def test_uniform_shift_of_one_row_matches_row_sum_of_dH(orc):
    # loss change under h_v += eps * 1 equals eps * sum_k dH0[v, k] to first order
    part, layers, H0, M, pos = setup_case(orc, [0, 0], seed=3)
    res = orc.train_step(part, layers, H0, M, pos, 3, 1, 5, 0)
    v = int(part["core_h"][pos[0]])
    eps = 1e-6
    Hp = H0.copy(); Hp[v] += eps
    Hm = H0.copy(); Hm[v] -= eps
    num = (loss_of(orc, part, layers, Hp, M, pos) - loss_of(orc, part, layers, Hm, M, pos)) / (2 * eps)
    assert res["dH0"][v].sum() == pytest.approx(num, rel=1e-5, abs=1e-10)
