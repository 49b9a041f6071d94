"""Pins of the oracle's RGCN layer (Eq. 1, Eq. 2) and of the self-sufficiency of
expanded partitions (Sec. 3.2.2)."""
import numpy as np
import pytest

from test_oracle_partition import tiny_graph


def rand_layer(rng, R2, B, d_in, d_out, act):
    return dict(V=rng.normal(0, 0.3, (B, d_in, d_out)), a=rng.normal(0, 0.5, (R2, B)),
                W0=rng.normal(0, 0.3, (d_in, d_out)), act=act)


def brute_layer(head, rel, tail, vert_gid, R, dst_allowed, lay, H):
    """Eq. 1 edge by edge with W_r materialised from Eq. 2; c_{i,r} counted by dictionary.
    Works on global triples; only destinations in `dst_allowed` (local ids) receive messages."""
    lid = {int(g): k for k, g in enumerate(vert_gid)}
    W = np.einsum("rb,bio->rio", lay["a"], lay["V"])
    msgs = []
    for s, r, t in zip(head, rel, tail):
        s, r, t = int(s), int(r), int(t)
        if s in lid and t in lid:
            msgs.append((r, lid[t], lid[s]))
            msgs.append((r + R, lid[s], lid[t]))
    msgs = [m for m in msgs if m[1] in dst_allowed]
    c = {}
    for r, i, j in msgs:
        c[(r, i)] = c.get((r, i), 0) + 1
    pre = H @ lay["W0"]
    for r, i, j in msgs:
        pre[i] += (H[j] @ W[r]) / c[(r, i)]
    return pre, (np.maximum(pre, 0) if lay["act"] == 1 else pre)


@pytest.mark.parametrize("act", [0, 1])
def test_layer_equals_per_edge_brute_force(orc, act):
    head, rel, tail, n, R = tiny_graph(21, n=30, R=3, m=150)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(0)
    lay = rand_layer(rng, 2 * R, 3, 5, 7, act)
    H = rng.normal(0, 1, (part["n_vert"], 5))
    pre, out = orc.layer_forward(part, lay["V"], lay["a"], lay["W0"], act, H)
    bpre, bout = brute_layer(head, rel, tail, part["vert_gid"], R, set(range(part["n_vert"])), lay, H)
    np.testing.assert_allclose(pre, bpre, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out, bout, rtol=1e-12, atol=1e-12)


def test_one_basis_identity_is_the_neighbourhood_mean_hand_example(orc):
    # 3 vertices, triples (0,r0,2) and (1,r0,2).  With B = 1, a = 1, V_1 = I, W_0 = 0:
    #   vertex 2 receives the mean of h_0 and h_1 (relation r0);
    #   vertices 0 and 1 each receive h_2 over the inverse relation.
    head = np.array([0, 1], np.int32); rel = np.array([0, 0], np.int32); tail = np.array([2, 2], np.int32)
    part = orc.build_partition(head, rel, tail, 3, 1, 1, 0, 2, 0)
    H = np.array([[1.0, 2.0], [3.0, -4.0], [10.0, 20.0]])
    pre, out = orc.layer_forward(part, np.eye(2)[None], np.ones((2, 1)), np.zeros((2, 2)), 0, H)
    np.testing.assert_array_equal(out, np.array([[10.0, 20.0], [10.0, 20.0], [2.0, -1.0]]))
    # and with ReLU the negative entry is clipped
    _, out = orc.layer_forward(part, np.eye(2)[None], np.ones((2, 1)), np.zeros((2, 2)), 1, H)
    np.testing.assert_array_equal(out, np.array([[10.0, 20.0], [10.0, 20.0], [2.0, 0.0]]))
    # duplicate triple: c counts multiplicity, the mean is weighted
    head = np.array([0, 1, 1], np.int32); rel = np.zeros(3, np.int32); tail = np.array([2, 2, 2], np.int32)
    part = orc.build_partition(head, rel, tail, 3, 1, 1, 0, 2, 0)
    _, out = orc.layer_forward(part, np.eye(2)[None], np.ones((2, 1)), np.zeros((2, 2)), 0, H)
    np.testing.assert_allclose(out[2], (H[0] + 2 * H[1]) / 3, rtol=1e-15)


def test_one_basis_general_mean_per_relation(orc):
    # B = 1, a = 1: pre = (sum over relations of the per-relation neighbour mean) V_1 + H W_0.
    head, rel, tail, n, R = tiny_graph(4, n=25, R=2, m=90)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(1)
    N, d = part["n_vert"], 6
    H = rng.normal(0, 1, (N, d)); V = rng.normal(0, 1, (1, d, d)); W0 = rng.normal(0, 1, (d, d))
    pre, _ = orc.layer_forward(part, V, np.ones((2 * R, 1)), W0, 0, H)
    A = np.zeros((N, N))                     # dense normalised adjacency summed over relations
    sp = part["seg_ptr"]
    for s in range(part["n_seg"]):
        for e in range(sp[s], sp[s + 1]):
            A[part["seg_dst"][s], part["col_src"][e]] += 1.0 / (sp[s + 1] - sp[s])
    np.testing.assert_allclose(pre, A @ H @ V[0] + H @ W0, rtol=1e-11, atol=1e-12)


def test_zero_coefficients_leave_the_self_loop_gemm(orc):
    head, rel, tail, n, R = tiny_graph(6)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(2)
    lay = rand_layer(rng, 2 * R, 4, 8, 8, 1)
    H = rng.normal(0, 1, (part["n_vert"], 8))
    _, out = orc.layer_forward(part, lay["V"], np.zeros_like(lay["a"]), lay["W0"], 1, H)
    np.testing.assert_allclose(out, np.maximum(H @ lay["W0"], 0), rtol=1e-13, atol=1e-14)


def test_aggregate_is_linear_in_the_coefficients(orc):
    head, rel, tail, n, R = tiny_graph(7)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(3)
    lay = rand_layer(rng, 2 * R, 2, 4, 4, 0)
    H = rng.normal(0, 1, (part["n_vert"], 4))
    Z = np.zeros_like(lay["W0"])
    p1, _ = orc.layer_forward(part, lay["V"], lay["a"], Z, 0, H)
    p2, _ = orc.layer_forward(part, lay["V"], -2.5 * lay["a"], Z, 0, H)
    np.testing.assert_allclose(p2, -2.5 * p1, rtol=1e-12, atol=1e-13)


def test_vertex_relabelling_only_permutes_rows(orc):
    head, rel, tail, n, R = tiny_graph(8, n=20, m=100)
    # make sure every vertex occurs so local id == global id for P = 1
    head[:n] = np.arange(n)
    rng = np.random.default_rng(4)
    perm = rng.permutation(n).astype(np.int32)
    lay = rand_layer(rng, 2 * R, 2, 3, 3, 1)
    H = rng.normal(0, 1, (n, 3))
    p1 = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    p2 = orc.build_partition(perm[head], rel, perm[tail], n, R, 1, 0, 2, 0)
    H2 = np.empty_like(H); H2[perm] = H
    _, o1 = orc.layer_forward(p1, lay["V"], lay["a"], lay["W0"], 1, H)
    _, o2 = orc.layer_forward(p2, lay["V"], lay["a"], lay["W0"], 1, H2)
    np.testing.assert_allclose(o2[perm], o1, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("P,L", [(3, 2), (4, 1), (2, 3)])
def test_expanded_partition_is_self_sufficient(orc, P, L):
    """Sec. 3.2.2: after n-hop expansion an n-layer GNN gives, for every endpoint of a core
    edge, exactly the embedding it has on the whole graph."""
    head, rel, tail, n, R = tiny_graph(30 + P, n=60, R=3, m=140)
    rng = np.random.default_rng(5)
    d = 4
    layers = [rand_layer(rng, 2 * R, 2, d, d, 1 if l < L - 1 else 0) for l in range(L)]
    Hg = rng.normal(0, 1, (n, d))
    whole = orc.build_partition(head, rel, tail, n, R, 1, 0, L, 0)
    Hs_w, _ = orc.rgcn_forward(whole, layers, Hg[whole["vert_gid"]])
    gid_to_whole = {int(g): k for k, g in enumerate(whole["vert_gid"])}
    for pid in range(P):
        part = orc.build_partition(head, rel, tail, n, R, P, pid, L, 0)
        if part["n_core"] == 0:
            continue
        Hs_p, _ = orc.rgcn_forward(part, layers, Hg[part["vert_gid"]])
        for loc in part["cand"]:                    # neg_domain 0: cand = endpoints of core edges
            g = int(part["vert_gid"][loc])
            np.testing.assert_allclose(Hs_p[-1][loc], Hs_w[-1][gid_to_whole[g]], rtol=1e-12, atol=1e-13)
        # and the halo is not vacuous: some vertex outside S_0 differs or is absent
        assert part["n_vert"] >= part["n_cand"]


def test_layer_rows_matches_whole_layer(orc):
    head, rel, tail, n, R = tiny_graph(11, n=40, m=200)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(6)
    lay = rand_layer(rng, 2 * R, 3, 6, 6, 1)
    H = rng.normal(0, 1, (part["n_vert"], 6)).astype(np.float32)
    pre, out = orc.layer_forward(part, lay["V"], lay["a"], lay["W0"], 1, H)
    rows = np.array([0, 5, 17, part["n_vert"] - 1], np.int32)
    rpre, rout = orc.layer_rows(part, rows, lay["V"], lay["a"], lay["W0"], 1, H)
    np.testing.assert_allclose(rpre, pre[rows], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(rout, out[rows], rtol=1e-12, atol=1e-13)
