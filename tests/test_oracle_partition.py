"""Pins of the oracle's partitioning / Neighborhood Expansion / sorted edge runs
(Sec. 3.2.1, 3.2.2, Eq. 7) against set-based brute force and invariants."""
import numpy as np
import pytest


def tiny_graph(seed, n=40, R=3, m=120):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32), n, R)


def test_head_hash_values_worked_by_hand(orc):
    """part = ((head * 0x9E3779B1 mod 2^32) >> 8) mod P, worked out digit by digit:
      head 0: the product is 0                                           -> 0 for every P
      head 1: 0x9E3779B1 >> 8 = 0x9E3779; its last hex digits 0x79 = 0b0111_1001   -> mod 4 = 1, mod 8 = 1
      head 2: 2 * 0x9E3779B1 = 0x1_3C6EF362, low 32 bits 0x3C6EF362, >> 8 = 0x3C6EF3, 0xF3 = 0b1111_0011
                                                                         -> mod 4 = 3, mod 16 = 3
      head 3: 3 * 0x9E3779B1 = 0x1_DAA66D13, low 32 bits 0xDAA66D13, >> 8 = 0xDAA66D, 0x6D = 0b0110_1101
                                                                         -> mod 4 = 1, mod 8 = 5
              0xDAA66D = 14,329,453, digit sum 31                        -> mod 3 = 1
      head 1, P = 3: 0x9E3779 = 10,368,889, digit sum 52                 -> mod 3 = 1
    The multiplication wraps at 32 bits (head 2 and 3 overflow) and the low 8 bits are dropped."""
    for P in (1, 2, 3, 4, 7, 16):
        assert orc.part_of_head(0, P) == 0
    assert orc.part_of_head(1, 4) == 1 and orc.part_of_head(1, 8) == 1 and orc.part_of_head(1, 3) == 1
    assert orc.part_of_head(2, 4) == 3 and orc.part_of_head(2, 16) == 3
    assert orc.part_of_head(3, 4) == 1 and orc.part_of_head(3, 8) == 5 and orc.part_of_head(3, 3) == 1
    assert orc.part_of_head(1, 1 << 24) == 0x9E3779          # all 24 kept bits
    assert orc.part_of_head(2, 1 << 24) == 0x3C6EF3


def brute_partition(orc, head, rel, tail, n, R, P, pid, L, neg_domain):
    """Python sets and sorted tuples; the hash is the oracle's (pinned by hand-worked values above)."""
    M = len(head)
    core = [i for i in range(M) if orc.part_of_head(int(head[i]), P) == pid]
    S0 = set()
    for i in core:
        S0.add(int(head[i])); S0.add(int(tail[i]))
    medges = []                       # (rel, dst, src, id)
    for i in range(M):
        medges.append((int(rel[i]), int(tail[i]), int(head[i]), i))
    for i in range(M):
        medges.append((int(rel[i]) + R, int(head[i]), int(tail[i]), M + i))
    levels = [set(S0)]
    for _ in range(L):
        prev = levels[-1]
        nxt = set(prev)
        for (_, dst, src, _) in medges:
            if dst in prev:
                nxt.add(src)
        levels.append(nxt)
    verts = sorted(levels[-1])
    lid = {g: k for k, g in enumerate(verts)}
    dstset = levels[-2] if L >= 1 else set()
    kept = sorted((r, lid[dst], lid[src], eid) for (r, dst, src, eid) in medges if dst in dstset)
    seg_ptr, seg_rel, seg_dst = [], [], []
    for k, (r, dst, src, eid) in enumerate(kept):
        if k == 0 or (r, dst) != kept[k - 1][:2]:
            seg_ptr.append(k); seg_rel.append(r); seg_dst.append(dst)
    seg_ptr.append(len(kept))
    cand = [lid[g] for g in verts if (neg_domain == 1 or g in S0)]
    return dict(vert_gid=verts, core_eid=core, core_h=[lid[int(head[i])] for i in core],
                core_r=[int(rel[i]) for i in core], core_t=[lid[int(tail[i])] for i in core],
                seg_ptr=seg_ptr, seg_rel=seg_rel, seg_dst=seg_dst,
                col_src=[e[2] for e in kept], edge_id=[e[3] for e in kept], cand=cand)


@pytest.mark.parametrize("P,pid,L,dom", [(1, 0, 2, 0), (3, 1, 2, 0), (3, 0, 1, 1), (4, 2, 2, 1),
                                         (5, 4, 3, 0), (2, 0, 0, 0)])
def test_partition_matches_set_brute_force(orc, P, pid, L, dom):
    head, rel, tail, n, R = tiny_graph(10 + P + L)
    got = orc.build_partition(head, rel, tail, n, R, P, pid, L, dom)
    want = brute_partition(orc, head, rel, tail, n, R, P, pid, L, dom)
    for k, v in want.items():
        np.testing.assert_array_equal(got[k], np.asarray(v, dtype=got[k].dtype), err_msg=k)
    lens = np.diff(got["seg_ptr"])
    np.testing.assert_array_equal(got["inv_c"], (np.float32(1) / lens.astype(np.float32)))


def test_core_sets_are_a_disjoint_cover(orc):
    head, rel, tail, n, R = tiny_graph(3, n=60, m=300)
    P = 4
    seen = np.zeros(len(head), np.int32)
    for pid in range(P):
        part = orc.build_partition(head, rel, tail, n, R, P, pid, 2, 0)
        seen[part["core_eid"]] += 1
    assert (seen == 1).all()            # Sec. 3.2.1: disjoint edge sets covering the graph


def test_sorted_run_invariants(orc):
    head, rel, tail, n, R = tiny_graph(5, n=50, R=4, m=400)
    part = orc.build_partition(head, rel, tail, n, R, 2, 1, 2, 0)
    E, S = part["n_edge"], part["n_seg"]
    sp = part["seg_ptr"]
    assert sp[0] == 0 and sp[-1] == E and (np.diff(sp) > 0).all()
    key = part["seg_rel"].astype(np.int64) * part["n_vert"] + part["seg_dst"]
    assert (np.diff(key) > 0).all()                         # runs strictly ascending in (rel, dst)
    assert len(np.unique(part["edge_id"])) == E             # each message edge at most once
    for s in range(S):
        src = part["col_src"][sp[s]:sp[s + 1]]
        assert (np.diff(src) >= 0).all()
    # c_{i,r} recount by hashing (rel, dst) of every kept message edge
    M = len(head)
    lid = {int(g): k for k, g in enumerate(part["vert_gid"])}
    counts = {}
    for eid in part["edge_id"]:
        i = int(eid) % M
        if eid < M:
            k = (int(rel[i]), lid[int(tail[i])])
        else:
            k = (int(rel[i]) + R, lid[int(head[i])])
        counts[k] = counts.get(k, 0) + 1
    for s in range(S):
        c = counts[(int(part["seg_rel"][s]), int(part["seg_dst"][s]))]
        assert c == sp[s + 1] - sp[s]
        assert part["inv_c"][s] * np.float32(c) == pytest.approx(1.0, abs=1e-6)


def test_replication_factor_is_one_for_single_partition(orc):
    # Eq. 7 with p = 1 and no isolated vertex: RF = |V(E_1)| / |V| = 1.
    n = 30
    head = np.arange(n, dtype=np.int32)
    tail = ((np.arange(n) + 1) % n).astype(np.int32)
    rel = np.zeros(n, np.int32)
    part = orc.build_partition(head, rel, tail, n, 1, 1, 0, 2, 0)
    assert part["n_vert"] / n == 1.0
    assert part["n_edge"] == 2 * n and part["n_core"] == n


def test_replication_grows_towards_p_on_a_small_dense_graph(orc):
    # Table 2's qualitative behaviour: on a small dense KG the 2-hop expansion of each of
    # P partitions covers (almost) the whole graph, so RF approaches P.
    head, rel, tail, n, R = tiny_graph(9, n=80, R=3, m=1200)
    P = 4
    rf = sum(orc.build_partition(head, rel, tail, n, R, P, pid, 2, 0)["n_vert"] for pid in range(P)) / n
    assert 3.5 < rf <= 4.0


def test_zero_hops_and_empty_partition(orc):
    head, rel, tail, n, R = tiny_graph(1)
    part = orc.build_partition(head, rel, tail, n, R, 1, 0, 0, 0)
    assert part["n_edge"] == 0 and part["n_seg"] == 0 and part["n_vert"] > 0
    # a partition id nobody hashes to: everything empty
    head1 = np.array([0], np.int32); rel1 = np.array([0], np.int32); tail1 = np.array([1], np.int32)
    pid_used = orc.part_of_head(0, 7)
    other = (pid_used + 1) % 7
    part = orc.build_partition(head1, rel1, tail1, 2, 1, 7, other, 2, 0)
    assert part["n_vert"] == 0 and part["n_edge"] == 0 and part["n_core"] == 0 and part["n_cand"] == 0
