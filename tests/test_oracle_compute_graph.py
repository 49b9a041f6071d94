"""Pins of the oracle's per-batch computational sub-graph (Sec. 3.3, Algorithm 1 "getComputeGraph")
against set-based breadth-first search on the raw triples, sparse-matrix reachability, and the
property that defines it: rows outside the sub-graph cannot influence the batch's embeddings."""
import numpy as np
import pytest
import scipy.sparse as sp

from paper_2201_02791_amd import synth


def tiny(seed, n=60, R=3, m=150, P=1, pid=0):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32), n, R)


@pytest.mark.parametrize("seed,P,pid,L", [(1, 1, 0, 2), (2, 3, 1, 2), (3, 2, 0, 3), (4, 1, 0, 1)])
def test_matches_set_bfs_on_raw_triples(orc, seed, P, pid, L):
    head, rel, tail, n, R = tiny(seed)
    part = orc.build_partition(head, rel, tail, n, R, P, pid, L, 0)
    rng = np.random.default_rng(seed + 100)
    pos = rng.permutation(part["n_core"])[:5].astype(np.int32)
    neg = part["cand"][rng.integers(0, part["n_cand"], (len(pos), 2))].astype(np.int32)
    got = orc.compute_graph(part, pos, neg, L)

    gid = part["vert_gid"]
    batch = set(int(gid[v]) for v in orc.batch_vertices(part, pos, neg))
    # incoming message edges of the whole graph in global ids: s -> t and the inverse t -> s
    in_nbrs = {}
    for s, t in zip(head.tolist(), tail.tolist()):
        in_nbrs.setdefault(t, set()).add(s)
        in_nbrs.setdefault(s, set()).add(t)
    level = set(batch)
    want = [None] * L
    want[L - 1] = set(level)
    for l in range(L - 1, 0, -1):
        nxt = set(level)
        for v in level:
            nxt |= in_nbrs.get(v, set())
        level = nxt
        want[l - 1] = set(level)
    for l in range(L):
        got_set = set(int(gid[i]) for i in np.nonzero(got[l])[0])
        assert got_set == want[l], "layer %d" % l


def test_matches_sparse_reachability(orc):
    spec = synth.scaled(synth.WORKLOADS[2], n_entities=3000, n_triples=20000, n_pos=64)
    head, rel, tail = synth.make_triples(spec)
    part = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts, spec.part_id,
                               spec.n_hops, spec.neg_domain)
    pos = synth.make_batch(spec, part["n_core"])
    neg, _ = orc.sample_negatives(part, pos, 3, 1, 7, 0)
    got = orc.compute_graph(part, pos, neg, 2)
    N = part["n_vert"]
    dst = np.repeat(part["seg_dst"], np.diff(part["seg_ptr"]))
    A = sp.csr_matrix((np.ones(len(dst)), (dst, part["col_src"])), shape=(N, N))
    x1 = np.zeros(N); x1[orc.batch_vertices(part, pos, neg)] = 1
    x0 = ((A.T @ x1) > 0) | (x1 > 0)
    np.testing.assert_array_equal(got[1], x1.astype(np.uint8))
    np.testing.assert_array_equal(got[0], x0.astype(np.uint8))
    assert 0 < got[1].sum() < got[0].sum() < N


def test_rows_outside_the_subgraph_do_not_reach_the_batch(orc):
    """What the sub-graph is for: the batch rows of the last layer read layer-1 rows only on
    active[0] and input rows only on active[0] and its in-neighbours.  Changing every other input
    row leaves the batch embeddings bit-identical; changing an input row inside changes them."""
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=400, n_triples=900, n_pos=6)
    head, rel, tail = synth.make_triples(spec)
    part = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, 1, 0, 2, 0)
    params = synth.make_params(spec, part["n_vert"])
    layers = [dict(V=params["V"][l], a=params["a"][l], W0=params["W0"][l], act=spec.acts[l]) for l in range(2)]
    pos = synth.make_batch(spec, part["n_core"])
    neg, _ = orc.sample_negatives(part, pos, 1, 0, 3, 0)
    act = orc.compute_graph(part, pos, neg, 2)
    bv = orc.batch_vertices(part, pos, neg)
    N = part["n_vert"]
    # inputs that layer 1 reads for its active rows
    reads0 = act[0].copy()
    dst = np.repeat(part["seg_dst"], np.diff(part["seg_ptr"]))
    reads0[part["col_src"][act[0][dst] > 0]] = 1
    assert 0 < reads0.sum() < N
    H0 = np.asarray(params["H0"], np.float64)
    base = orc.rgcn_forward(part, layers, H0)[0][-1][bv]
    rng = np.random.default_rng(0)
    H1 = H0.copy()
    outside = np.nonzero(reads0 == 0)[0]
    H1[outside] = rng.normal(size=(len(outside), H0.shape[1]))
    np.testing.assert_array_equal(orc.rgcn_forward(part, layers, H1)[0][-1][bv], base)
    inside = np.nonzero(reads0)[0]
    for v in inside[:: max(1, len(inside) // 8)]:
        H2 = H0.copy(); H2[v] += 1.0
        assert np.abs(orc.rgcn_forward(part, layers, H2)[0][-1][bv] - base).max() > 0
