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


def test_bf16_message_storage_rounds_like_a_library_conversion(orc):
    """msg_bf16 rounds each projected message once to bfloat16 (nearest, ties to even).  With one
    basis, V = I, a = 1, W_0 = 0 and a single in-edge, the layer output IS the rounded message,
    which must equal PyTorch's float32 -> bfloat16 conversion, ties included."""
    import torch
    d = 256
    head = np.array([0], np.int32); rel = np.array([0], np.int32); tail = np.array([1], np.int32)
    part = orc.build_partition(head, rel, tail, 2, 1, 1, 0, 1, 0)
    rng = np.random.default_rng(0)
    h = (rng.standard_normal(d) * 10.0 ** rng.integers(-6, 6, d)).astype(np.float32)
    # exact ties: low 16 bits = 0x8000 with even and odd kept parts
    ties = np.array([0x3F808000, 0x3F818000, 0xBF808000, 0x40FF8000, 0x3F807FFF, 0x3F808001], np.uint32)
    h[:len(ties)] = ties.view(np.float32)
    H = np.zeros((2, d)); H[0] = h
    _, out = orc.layer_forward(part, np.eye(d)[None], np.ones((2, 1)), np.zeros((d, d)), 0, H, msg_bf16=True)
    want = torch.from_numpy(h).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(out[1], want)
    _, exact = orc.layer_forward(part, np.eye(d)[None], np.ones((2, 1)), np.zeros((d, d)), 0, H)
    np.testing.assert_array_equal(exact[1], h.astype(np.float64))


# ------------------------------------------------------------------ aggregate-first bf16 rounding (msg_bf16 = 2)
def _bf(x):
    import torch
    return torch.from_numpy(np.asarray(x, np.float64)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def _small_case(orc, seed, n=60, R=3, m=400, d_in=12, d_out=8, B=3):
    rng = np.random.default_rng(seed)
    head = rng.integers(0, n, m).astype(np.int32); rel = rng.integers(0, R, m).astype(np.int32)
    tail = rng.integers(0, n, m).astype(np.int32)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    V = rng.normal(0, 0.4, (B, d_in, d_out)); a = rng.normal(0, 1, (2 * R, B)); W0 = rng.normal(0, 0.4, (d_in, d_out))
    H = rng.normal(0, 1, (part["n_vert"], d_in)).astype(np.float32).astype(np.float64)
    return part, V, a, W0, H


def test_aggregate_first_bf16_mode_matches_a_numpy_emulation(orc):
    """Eq. 1-2 regrouped (run means z, per-basis sums y, one contraction with the stacked weights),
    every operand rounded with PyTorch's bfloat16 conversion, sums in float64."""
    part, V, a, W0, H = _small_case(orc, 4)
    S, N = part["n_seg"], part["n_vert"]
    lens = np.diff(part["seg_ptr"])
    run = np.repeat(np.arange(S), lens)
    Hq = _bf(H)
    Z = np.zeros((S, H.shape[1])); np.add.at(Z, run, Hq[part["col_src"]])
    Zq = _bf(Z / lens[:, None])
    Y = np.zeros((N, V.shape[0], H.shape[1]))
    np.add.at(Y, part["seg_dst"], a[part["seg_rel"]][:, :, None] * Zq[:, None, :])
    want = np.einsum("nbk,bkc->nc", _bf(Y), _bf(V)) + Hq @ _bf(W0)
    pre, out = orc.layer_forward(part, V, a, W0, 1, H, msg_bf16=2)
    np.testing.assert_allclose(pre, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_array_equal(out, np.maximum(pre, 0))
    exact, _ = orc.layer_forward(part, V, a, W0, 1, H)
    err = np.abs(pre - exact).max() / np.abs(exact).max()
    assert 0 < err < 2e-2                                       # rounded, and only by bf16 amounts
    rows = np.array([0, 7, N - 1], np.int32)
    rpre, rout = orc.layer_rows(part, rows, V, a, W0, 1, H.astype(np.float32), msg_bf16=2)
    np.testing.assert_allclose(rpre, pre[rows], rtol=1e-11, atol=1e-12)


def test_aggregate_first_bf16_mode_is_exact_on_bf16_representable_inputs(orc):
    """Small integers, power-of-two run lengths: no rounding point changes anything, so the regrouped
    evaluation must reproduce the exact layer (a regrouping mistake would not)."""
    n, R, d_in, d_out, B = 20, 2, 4, 4, 2
    rng = np.random.default_rng(1)
    # every (relation, destination) run gets 1, 2 or 4 edges
    head, rel, tail = [], [], []
    for t in range(n):
        for r in range(R):
            for j in rng.choice(n, size=int(rng.choice([1, 2, 4])), replace=False):
                head.append(j); rel.append(r); tail.append(t)
    head, rel, tail = (np.asarray(x, np.int32) for x in (head, rel, tail))
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 1, 0)
    lens = np.diff(part["seg_ptr"])
    fwd = part["seg_rel"] < R                       # inverse runs have arbitrary lengths: give them weight 0
    a = np.zeros((2 * R, B)); a[:R] = rng.integers(-2, 3, (R, B))
    assert set(lens[fwd]) <= {1, 2, 4}
    V = rng.integers(-2, 3, (B, d_in, d_out)).astype(np.float64)
    W0 = rng.integers(-2, 3, (d_in, d_out)).astype(np.float64)
    H = rng.integers(-4, 5, (part["n_vert"], d_in)).astype(np.float64)
    exact, _ = orc.layer_forward(part, V, a, W0, 0, H)
    got, _ = orc.layer_forward(part, V, a, W0, 0, H, msg_bf16=2)
    np.testing.assert_array_equal(got, exact)


def test_aggregate_first_bf16_backward(orc):
    """Mode 2 changes only da (through the rounded run means); every other gradient is the exact one."""
    part, V, a, W0, H = _small_case(orc, 9)
    pre, out = orc.layer_forward(part, V, a, W0, 1, H, msg_bf16=2)
    rng = np.random.default_rng(2)
    dH = rng.normal(0, 1, out.shape)
    g2 = orc.layer_backward(part, V, a, W0, 1, H, pre, dH, True, msg_bf16=2)
    g0 = orc.layer_backward(part, V, a, W0, 1, H, pre, dH, True, msg_bf16=0)
    for k in ("dV", "dW0", "dH", "dP", "Gpre"):
        np.testing.assert_array_equal(g2[k], g0[k])
    S = part["n_seg"]; lens = np.diff(part["seg_ptr"]); run = np.repeat(np.arange(S), lens)
    Z = np.zeros((S, H.shape[1])); np.add.at(Z, run, _bf(H)[part["col_src"]])
    Zq = _bf(Z / lens[:, None])
    G = g0["Gpre"][part["seg_dst"]]                                  # [S][d_out]
    per_run = np.einsum("sk,bkc,sc->sb", Zq, V, G)
    want = np.zeros_like(a); np.add.at(want, part["seg_rel"], per_run)
    np.testing.assert_allclose(g2["da"], want, rtol=1e-10, atol=1e-12)
    assert 0 < np.abs(g2["da"] - g0["da"]).max() / np.abs(g0["da"]).max() < 2e-2


# ------------------------------------------------------------------ relation-weight bf16 rounding (msg_bf16 = 3)
def test_relation_weight_bf16_mode_matches_a_numpy_emulation(orc):
    """Eq. 2 written out (W_r = sum_b a_rb V_b, rounded), run means z (rounded), one product z W_r per
    run (rounded when stored), summed per destination with the self-loop term."""
    part, V, a, W0, H = _small_case(orc, 14)
    S, N = part["n_seg"], part["n_vert"]
    lens = np.diff(part["seg_ptr"])
    run = np.repeat(np.arange(S), lens)
    Hq = _bf(H)
    Z = np.zeros((S, H.shape[1])); np.add.at(Z, run, Hq[part["col_src"]])
    Zq = _bf(Z / lens[:, None])
    Wr = _bf(np.einsum("rb,bkc->rkc", a, V))
    U = _bf(np.einsum("sk,skc->sc", Zq, Wr[part["seg_rel"]]))
    want = Hq @ _bf(W0)
    np.add.at(want, part["seg_dst"], U)
    pre, out = orc.layer_forward(part, V, a, W0, 1, H, msg_bf16=3)
    np.testing.assert_allclose(pre, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_array_equal(out, np.maximum(pre, 0))
    exact, _ = orc.layer_forward(part, V, a, W0, 1, H)
    assert 0 < np.abs(pre - exact).max() / np.abs(exact).max() < 2e-2
    rows = np.array([0, 7, N - 1], np.int32)
    rpre, _ = orc.layer_rows(part, rows, V, a, W0, 1, H.astype(np.float32), msg_bf16=3)
    np.testing.assert_allclose(rpre, pre[rows], rtol=1e-11, atol=1e-12)
    # backward: only da differs from the exact one, and it is the mode-2 value (same rounded run means)
    dH = np.random.default_rng(3).normal(0, 1, out.shape)
    g3 = orc.layer_backward(part, V, a, W0, 1, H, pre, dH, True, msg_bf16=3)
    g2 = orc.layer_backward(part, V, a, W0, 1, H, pre, dH, True, msg_bf16=2)
    for k in ("dV", "dW0", "dH", "dP", "Gpre", "da"):
        np.testing.assert_array_equal(g3[k], g2[k])


def test_relation_weight_bf16_mode_is_exact_on_bf16_representable_inputs(orc):
    n, R, d_in, d_out, B = 20, 2, 4, 4, 2
    rng = np.random.default_rng(1)
    head, rel, tail = [], [], []
    for t in range(n):
        for r in range(R):
            for j in rng.choice(n, size=int(rng.choice([1, 2, 4])), replace=False):
                head.append(j); rel.append(r); tail.append(t)
    head, rel, tail = (np.asarray(x, np.int32) for x in (head, rel, tail))
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 1, 0)
    a = np.zeros((2 * R, B)); a[:R] = rng.integers(-2, 3, (R, B))      # inverse runs (any length) get weight 0
    V = rng.integers(-2, 3, (B, d_in, d_out)).astype(np.float64)
    W0 = rng.integers(-2, 3, (d_in, d_out)).astype(np.float64)
    H = rng.integers(-4, 5, (part["n_vert"], d_in)).astype(np.float64)
    exact, _ = orc.layer_forward(part, V, a, W0, 0, H)
    got, _ = orc.layer_forward(part, V, a, W0, 0, H, msg_bf16=3)
    np.testing.assert_array_equal(got, exact)
