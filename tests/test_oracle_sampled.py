"""The row-sampled / any-size checks used at full benchmark sizes, pinned here against the
whole-step C oracle on a small graph (which is itself pinned by brute force and finite differences)."""
import numpy as np
import pytest

from test_oracle_partition import tiny_graph
from test_oracle_rgcn import rand_layer


@pytest.fixture(scope="module")
def case(orc):
    from oracle import sampled
    head, rel, tail, n, R = tiny_graph(77, n=80, R=3, m=500)
    part = orc.build_partition(head, rel, tail, n, R, 2, 0, 2, 0)
    rng = np.random.default_rng(0)
    d, B = 8, 3
    layers = [rand_layer(rng, 2 * R, B, d, d, 1), rand_layer(rng, 2 * R, B, d, d, 0)]
    H0 = rng.normal(0, 1, (part["n_vert"], d)); M = rng.normal(0, 1, (R, d))
    pos = rng.permutation(part["n_core"])[:40].astype(np.int32)
    res = orc.train_step(part, layers, H0, M, pos, 3, 1, 5, 0)
    return sampled, part, layers, H0, res, sampled.EdgeView(part)


def test_sampled_rows_match_the_whole_step(case):
    sampled, part, layers, H0, res, ev = case
    rows = np.array([0, 3, 11, part["n_vert"] - 1])
    for l in (1, 0):
        lay, g = layers[l], res["grads"][l]
        Hin = res["Hs"][l]
        P = sampled.project_rows(Hin[rows], lay["V"])
        dP = sampled.transposed_rows(ev, rows, lay["a"], g["Gpre"])
        np.testing.assert_allclose(dP, g["dP"][rows], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(sampled.input_grad_rows(g["dP"][rows], g["Gpre"][rows], lay["V"], lay["W0"]),
                                   g["dH"][rows], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(sampled.self_weight_grad(Hin, g["Gpre"], chunk=16), g["dW0"], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(sampled.basis_weight_grad_column(Hin, g["dP"][:, 1, 2], chunk=16),
                                   g["dV"][1][:, 2], rtol=1e-11, atol=1e-13)
        Pfull = sampled.project_rows(Hin, lay["V"])
        da = sampled.coeff_grad_relations(ev, [0, 4], lambda ids: Pfull[ids], g["Gpre"], P.shape[1])
        for r, v in da.items():
            np.testing.assert_allclose(v, g["da"][r], rtol=1e-10, atol=1e-13)
        # pre-activations: exact ones, and ReLU outputs (equal wherever the gradient is non-zero)
        for pre in (res["pres"][l], res["Hs"][l + 1]):
            q = sampled.euler_quantity(pre, Hin, lay["W0"], g["Gpre"], chunk=16)
            assert q == pytest.approx(float(np.sum(lay["a"] * g["da"])), rel=1e-10)
            assert q == pytest.approx(float(np.sum(lay["V"] * g["dV"])), rel=1e-10)


def test_regrouped_helpers_match_the_whole_step(case, orc):
    """Run means, per-basis sums and the coefficient gradient from run means reproduce the C oracle."""
    sampled, part, layers, H0, res, ev = case
    lay, g = layers[0], res["grads"][0]
    S = part["n_seg"]
    runs = np.arange(S)
    Z = sampled.run_mean_rows(part, runs, H0)
    rows = np.arange(part["n_vert"])
    Y = sampled.basis_sum_rows(part, rows, lay["a"], lambda ids: Z[ids])
    pre = np.einsum("nbk,bkc->nc", Y, lay["V"]) + H0 @ lay["W0"]
    np.testing.assert_allclose(pre, res["pres"][0], rtol=1e-10, atol=1e-12)
    da = sampled.coeff_grad_relations_runs(part, [0, 1, 4], lambda ids: Z[ids], lay["V"], g["Gpre"])
    for r, v in da.items():
        np.testing.assert_allclose(v, g["da"][r], rtol=1e-9, atol=1e-12)


def test_relation_weight_helpers_match_the_whole_step(case, orc):
    sampled, part, layers, H0, res, ev = case
    lay, g = layers[0], res["grads"][0]
    S = part["n_seg"]; runs = np.arange(S)
    Z = sampled.run_mean_rows(part, runs, H0)
    U = sampled.relation_product_rows(part, runs, lambda ids: Z[ids], lay["a"], lay["V"])
    pre = H0 @ lay["W0"]
    np.add.at(pre, part["seg_dst"], U)
    np.testing.assert_allclose(pre, res["pres"][0], rtol=1e-10, atol=1e-12)
    # dP column and, through it, a column of dV
    col = sampled.transposed_column(ev, lay["a"], 1, g["Gpre"][:, 2])
    np.testing.assert_allclose(col, g["dP"][:, 1, 2], rtol=1e-11, atol=1e-13)
    # dz and the input gradient it gives: dH_j = sum_{e out of j} dz_run(e) / c + G_j W_0^T
    dZ = sampled.relation_product_t_rows(part, runs, g["Gpre"], lay["a"], lay["V"])
    lens = np.diff(part["seg_ptr"]); run_of_edge = np.repeat(runs, lens)
    dH = g["Gpre"] @ lay["W0"].T
    np.add.at(dH, part["col_src"], dZ[run_of_edge] / lens[run_of_edge][:, None])
    np.testing.assert_allclose(dH, g["dH"], rtol=1e-10, atol=1e-12)


def test_whole_size_reductions_match_the_whole_step(case):
    """The random projection of the basis gradients and the per-relation coefficient gradient from edges
    (the two checks that cover every vertex and edge at full size) against the C oracle's dV and da."""
    sampled, part, layers, H0, res, ev = case
    rng = np.random.default_rng(9)
    for l in (0, 1):
        lay, g = layers[l], res["grads"][l]
        Hin = res["Hs"][l]
        x, y = rng.normal(size=Hin.shape[1]), rng.normal(size=g["Gpre"].shape[1])
        want = np.einsum("k,bkc,c->b", x, g["dV"], y)
        np.testing.assert_allclose(sampled.basis_weight_grad_projection(ev, lay["a"], Hin, g["Gpre"], x, y), want,
                                   rtol=1e-10, atol=1e-13)
        # a coordinate pair picks out single elements: dV_b[k][c] for every b
        ek, ec = np.eye(Hin.shape[1])[3], np.eye(g["Gpre"].shape[1])[5]
        np.testing.assert_allclose(sampled.basis_weight_grad_projection(ev, lay["a"], Hin, g["Gpre"], ek, ec),
                                   g["dV"][:, 3, 5], rtol=1e-10, atol=1e-13)
        for r in (0, 2, 5):
            np.testing.assert_allclose(sampled.coeff_grad_relation_edges(ev, r, Hin, g["Gpre"], lay["V"], chunk=7),
                                       g["da"][r], rtol=1e-10, atol=1e-13)
