"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Integers bit-exact; fp32 embeddings/scores 1e-4, fp32 gradients 1e-3,
bf16-message runs 2e-2 (per-tensor relative error, max|x-y| / max|y|)."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import (SEED, STEP, align_mask_decisions, assert_partition_equal, assert_step_close, gpu_step,
                      layers_of, oracle_step, rel_err)

pytestmark = pytest.mark.gpu

TOL_VAL, TOL_GRAD, TOL_BF16 = 1e-4, 1e-3, 2e-2


def say(*a):
    print("[gpu-case]", *a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


def random_graph(seed, n, R, m):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32))


# ------------------------------------------------------------------ build_partition
@pytest.mark.parametrize("n,R,m,P,pid,L,dom", [
    (40, 3, 120, 1, 0, 2, 0), (40, 3, 120, 3, 1, 2, 0), (40, 3, 120, 3, 0, 1, 1), (500, 7, 4000, 4, 2, 2, 1),
    (500, 7, 4000, 5, 4, 3, 0), (40, 3, 120, 2, 0, 0, 0), (3000, 50, 70000, 2, 1, 2, 0),
    (70000, 3, 9000, 3, 0, 2, 0)])
def test_partition_bit_exact(kb, orc, n, R, m, P, pid, L, dom):
    say("partition", n, R, m, P, pid, L, dom)
    head, rel, tail = random_graph(n + m + P, n, R, m)
    gp = kb.build_partition(head, rel, tail, n, R, P, pid, L, dom)
    op = orc.build_partition(head, rel, tail, n, R, P, pid, L, dom)
    assert_partition_equal(gp, op)
    check_views(gp, op)
    # run-twice bit identity of the device build
    gp2 = kb.build_partition(head, rel, tail, n, R, P, pid, L, dom)
    for name in ("col_src", "edge_id", "seg_ptr", "dm_src", "sm_dst"):
        np.testing.assert_array_equal(gp.export(name), gp2.export(name))


def check_views(gp, op):
    """Destination-major / source-major views are stable re-orderings of the sorted edge list."""
    E, N = op["n_edge"], op["n_vert"]
    seg_of_edge = np.repeat(np.arange(op["n_seg"]), np.diff(op["seg_ptr"]))
    dst = op["seg_dst"][seg_of_edge]; rel = op["seg_rel"][seg_of_edge]; invc = op["inv_c"][seg_of_edge]
    src = op["col_src"]
    o = np.argsort(dst, kind="stable")
    np.testing.assert_array_equal(gp.export("dm_src"), src[o])
    np.testing.assert_array_equal(gp.export("dm_rel"), rel[o])
    np.testing.assert_array_equal(gp.export("dm_invc"), invc[o])
    np.testing.assert_array_equal(gp.export("dm_ptr"), np.searchsorted(dst[o], np.arange(N + 1)).astype(np.int32))
    o = np.argsort(src, kind="stable")
    np.testing.assert_array_equal(gp.export("sm_dst"), dst[o])
    np.testing.assert_array_equal(gp.export("sm_rel"), rel[o])
    np.testing.assert_array_equal(gp.export("sm_invc"), invc[o])
    np.testing.assert_array_equal(gp.export("sm_ptr"), np.searchsorted(src[o], np.arange(N + 1)).astype(np.int32))
    R2 = 2 * op["n_relations"]
    np.testing.assert_array_equal(gp.export("rel_ptr"),
                                  np.searchsorted(op["seg_rel"], np.arange(R2 + 1)).astype(np.int32))
    assert gp.max_in_degree == (np.bincount(dst, minlength=1).max() if E else 0)
    assert gp.max_out_degree == (np.bincount(src, minlength=1).max() if E else 0)


def test_partition_empty_and_errors(kb, orc):
    say("partition empty / errors")
    head = np.array([0], np.int32); rel = np.array([0], np.int32); tail = np.array([1], np.int32)
    other = (orc.part_of_head(0, 7) + 1) % 7
    gp = kb.build_partition(head, rel, tail, 2, 1, 7, other, 2, 0)
    assert gp.n_vert == 0 and gp.n_edge == 0 and gp.n_core == 0 and gp.n_cand == 0
    with pytest.raises(kb.KgeError) as e:
        kb.build_partition(np.array([5], np.int32), rel, tail, 2, 1, 1, 0, 2, 0)
    assert e.value.status == -4
    with pytest.raises(kb.KgeError) as e:
        kb.build_partition(head, rel, tail, 2, 1, 2, 2, 2, 0)
    assert e.value.status == -1


# ------------------------------------------------------------------ whole step, small shapes
SHAPES = [
    # name, n, R, m, d, B, n_pos, n_neg, mode, P, acts
    ("d32_B4", 300, 5, 2500, 32, 4, 200, 3, 1, 1, [1, 0]),
    ("d200_B10_ragged_lanes", 400, 6, 3000, 200, 10, 333, 5, 1, 1, [1, 0]),
    ("d128_B2", 500, 1, 4000, 128, 2, 257, 1, 0, 2, [1, 0]),
    ("d64_B3_odd_bases", 300, 4, 2000, 64, 3, 100, 2, 1, 3, [1, 1]),
    ("d8_B1", 100, 2, 700, 8, 1, 64, 4, 1, 1, [0, 0]),
    ("d256_B5", 200, 3, 1500, 256, 5, 90, 7, 1, 1, [1, 0]),
    ("d16_B20", 250, 9, 2200, 16, 20, 128, 2, 0, 2, [1, 0]),
    ("d96_B40_matrix_core_transpose", 300, 12, 2600, 96, 40, 150, 3, 1, 1, [1, 0]),
    ("d160_B70", 200, 5, 1500, 160, 70, 64, 2, 1, 2, [1, 1]),
    ("d32_B256_most_bases", 150, 4, 1200, 32, 256, 64, 2, 1, 1, [1, 0]),
]


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_step_small_shapes(kb, orc, shape):
    name, n, R, m, d, B, n_pos, n_neg, mode, P, acts = shape
    say("step", shape)
    spec = synth.scaled(synth.WORKLOADS[0], name=name, seed=17, n_entities=n, n_relations=R, n_triples=m,
                        d=d, n_bases=B, n_pos=n_pos, n_neg=n_neg, neg_mode=mode, n_parts=P, part_id=P - 1,
                        acts=acts, feature_std=0.5)
    head, rel, tail = random_graph(len(name) + n, n, R, m)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


def test_hub_vertex_and_isolated_rows(kb, orc):
    """A star: one vertex with in-degree far above 64 (several metadata batches per wavefront),
    many leaves with a single edge, a second relation, and duplicate triples."""
    say("hub")
    n, R = 700, 2
    leaves = np.arange(1, 601, dtype=np.int32)
    head = np.concatenate([leaves, leaves[:50], np.array([650, 651], np.int32)])
    tail = np.concatenate([np.zeros(600, np.int32), np.zeros(50, np.int32), np.array([651, 652], np.int32)])
    rel = np.concatenate([np.zeros(600, np.int32), np.ones(50, np.int32), np.array([0, 1], np.int32)])
    spec = synth.scaled(synth.WORKLOADS[0], name="hub", seed=5, n_entities=n, n_relations=R,
                        n_triples=len(head), d=64, n_bases=4, n_pos=300, n_neg=2, neg_mode=1)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert gp.max_in_degree >= 650
    assert_partition_equal(gp, op)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


@pytest.mark.parametrize("acts,n,m,d,B", [([0, 0], 600, 6000, 64, 8), ([1, 0], 6000, 90000, 64, 8),
                                          ([0, 0], 900, 9000, 96, 40), ([1, 0], 3000, 70000, 128, 64),
                                          ([1, 0], 2000, 30000, 224, 70)],
                         ids=["identity", "relu", "identity_B40_d96", "relu_B64_d128_hub_sources",
                              "relu_B70_d224_two_base_chunks"])
def test_bf16_messages_small(kb, orc, acts, n, m, d, B):
    """Messages stored as bf16 (fp32 accumulation): every output against the exact oracle at 2e-2.
    The ReLU mask of layer 1 is a decision taken from floating-point values; where a pre-activation
    lies inside the rounding band of its own sum the decision is the kernel's (align_mask_decisions
    asserts the band and that such elements are few), everything else is the oracle's arithmetic."""
    say("bf16 small", acts, n, m, d, B)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-small", seed=3, n_entities=n, n_relations=20,
                        n_triples=m, d=d, n_bases=B, n_pos=256, n_neg=4, n_parts=2, part_id=0, acts=acts)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    if B == 64:
        assert gp.max_out_degree >= 256, "this case is meant to have sources whose out-edges are cut into units"
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, acts, True, True)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_adopted)
    errs = assert_step_close(ts, res, TOL_BF16, TOL_BF16)
    say("bf16 errs vs the exact oracle", errs)


# ------------------------------------------------------------------ the scoring call alone, both forms
@pytest.mark.parametrize("indexed", [True, False], ids=["atomic_free", "atomics"])
@pytest.mark.parametrize("d,n_pos,n_neg,mode", [(4, 50, 3, 1), (72, 300, 5, 1), (200, 700, 9, 1), (256, 260, 64, 1),
                                                (260, 90, 2, 0), (512, 130, 7, 1), (32, 400, 0, 1), (64, 1, 1, 1)])
def test_scoring_call_alone(kb, orc, d, n_pos, n_neg, mode, indexed):
    """kge_distmult_score_loss on random embeddings against the oracle: scores, loss, dH, dM; widths that leave
    lanes idle, one and two 16-byte pieces per lane, negative counts that are not multiples of 4, no negatives,
    a single positive, and a hub entity that most triples name (a long occurrence list)."""
    import torch
    say("scoring alone", d, n_pos, n_neg, mode, "indexed" if indexed else "atomics")
    n, R, m = 900, 7, 6000
    head, rel, tail = random_graph(d + n_pos, n, R, m)
    head[: m // 3] = 5                                   # vertex 5 heads a third of the triples
    gp = kb.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    op = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    rng = np.random.default_rng(d)
    H = rng.normal(0, 0.5, (gp.n_vert, d)).astype(np.float32)
    M = rng.normal(0, 0.5, (R, d)).astype(np.float32)
    pos = rng.permutation(gp.n_core)[:n_pos].astype(np.int32)
    ne, ns = orc.sample_negatives(op, pos, n_neg, mode, SEED, STEP)
    want = orc.distmult_score_loss(op, H, M, pos, ne, ns)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    dH = torch.full((gp.n_vert, d), 7.0, device="cuda"); dM = torch.full((R, d), 7.0, device="cuda")
    scores = torch.empty((n_pos, 1 + n_neg), device="cuda"); loss = torch.full((1,), 7.0, device="cuda")
    idx = kb.ScoreIndex(gp, n_pos, n_neg, d) if indexed else None
    args = (gp, t(H), t(M), t(pos), t(ne.reshape(n_pos, -1)) if n_neg else None, t(ns.reshape(n_pos, -1)) if n_neg else None,
            n_neg, scores, loss, dH, dM)
    kb.distmult_score_loss(*args, index=idx)
    torch.cuda.synchronize()
    assert rel_err(scores.cpu().numpy(), want["scores"]) <= TOL_VAL
    assert abs(float(loss.cpu()[0]) - want["loss"]) <= TOL_VAL * want["loss"]
    assert rel_err(dH.cpu().numpy(), want["dH"]) <= TOL_GRAD
    assert rel_err(dM.cpu().numpy(), want["dM"]) <= TOL_GRAD
    untouched = np.abs(want["dH"]).max(axis=1) == 0
    assert untouched.any() or n_pos * (2 + n_neg) > 2000
    assert not dH.cpu().numpy()[untouched].any()
    assert gp.bad_ids() == 0
    if indexed:
        first = dH.clone()
        dH.fill_(3.0)
        kb.distmult_score_loss(*args, index=idx)
        torch.cuda.synchronize()
        assert torch.equal(first, dH), "the atomic-free form must repeat bit for bit"


@pytest.mark.parametrize("indexed", [False, True], ids=["atomic", "indexed"])
def test_ids_outside_the_partition_are_counted_and_never_addresses(kb, orc, indexed):
    """No id read from a device array becomes an address unchecked, in the sub-graph call or in either form of
    the scoring call: an entity or core-edge index outside the partition is skipped or replaced, and counted in
    the partition (the outputs of such a call are meaningless, but nothing is read or written out of bounds)."""
    import torch
    say("ids out of range", indexed)
    n, R, m, d, n_pos, n_neg = 300, 3, 2000, 32, 40, 4
    head, rel, tail = random_graph(5, n, R, m)
    gp = kb.build_partition(head, rel, tail, n, R, 1, 0, 2, 0)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    rng = np.random.default_rng(1)
    H = t(rng.normal(size=(gp.n_vert, d)).astype(np.float32)); M = t(rng.normal(size=(R, d)).astype(np.float32))
    pos = rng.permutation(gp.n_core)[:n_pos].astype(np.int32)
    ne = rng.integers(0, gp.n_vert, (n_pos, n_neg)).astype(np.int32); ns = np.zeros((n_pos, n_neg), np.uint8)
    good_pos, good_ne = pos.copy(), ne.copy()
    pos[3] = gp.n_core + 5; pos[7] = -1                 # two bad core-edge indices
    ne[0, 0] = gp.n_vert; ne[9, 2] = -4; ne[11, 3] = 2 ** 31 - 1      # three bad entities
    idx = kb.ScoreIndex(gp, n_pos, n_neg, d) if indexed else None
    dH = torch.empty((gp.n_vert, d), device="cuda"); dM = torch.empty((R, d), device="cuda")
    loss = torch.empty(1, device="cuda")
    assert gp.bad_ids() == 0
    kb.distmult_score_loss(gp, H, M, t(pos), t(ne), t(ns), n_neg, None, loss, dH, dM, index=idx)
    assert gp.bad_ids() == 5
    # the sub-graph call skips the same five and flags exactly what the good ids reach
    cg = kb.ComputeGraph(gp, 2)
    kb.compute_graph(gp, cg, t(pos), t(ne))
    assert gp.bad_ids() == 10
    got = cg.export()
    keep = np.ones(n_pos, bool); keep[[3, 7]] = False
    kb.compute_graph(gp, cg, t(good_pos[keep]), t(np.where(ne == good_ne, ne, good_ne[1, 1])))
    assert gp.bad_ids() == 10
    want = cg.export()
    np.testing.assert_array_equal(got[0], want[0])
    np.testing.assert_array_equal(got[1], want[1])
    if indexed:
        with pytest.raises(kb.KgeError):                 # a batch larger than the index was made for
            kb.distmult_score_loss(gp, H, M, t(np.zeros(n_pos + 1, np.int32)), None, None, 0, None, loss, dH, dM, index=idx)


def test_step_with_atomic_scoring(kb, orc):
    """The whole step with the scoring call's atomic form (no index)."""
    say("step, atomic scoring")
    spec = synth.scaled(synth.WORKLOADS[0], name="atomic", seed=17, n_entities=400, n_relations=6, n_triples=3000,
                        d=200, n_bases=10, n_pos=333, n_neg=5, neg_mode=1, feature_std=0.5)
    head, rel, tail = random_graph(3, 400, 6, 3000)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, score_index=False)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


def test_zero_negatives_and_empty_batch(kb, orc):
    say("n_neg = 0 / n_pos = 0")
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=200, n_triples=900, n_pos=50, n_neg=0)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)
    import torch
    ts.set_batch(np.zeros(0, np.int32), 3)
    ts.run(1, SEED, STEP)
    torch.cuda.synchronize()
    assert float(ts.loss.cpu()[0]) == 0.0
    assert float(ts.dH_out.abs().max().cpu()) == 0.0
    for g in ts.grads:
        assert float(g["dV"].abs().max().cpu()) == 0.0 and float(g["da"].abs().max().cpu()) == 0.0


def test_forward_is_bit_reproducible(kb):
    say("reproducibility")
    import torch
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=2000, n_triples=30000, d=64, n_bases=4)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    h1 = ts.H_out.clone(); ne1 = ts.neg_ent.clone(); sc1 = ts.scores.clone()
    ts.run(spec.neg_mode, SEED, STEP)
    torch.cuda.synchronize()
    assert torch.equal(h1, ts.H_out) and torch.equal(ne1, ts.neg_ent) and torch.equal(sc1, ts.scores)


def test_argument_errors(kb):
    say("argument errors")
    import torch
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=100, n_triples=500)
    head, rel, tail = synth.make_triples(spec)
    part = kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations)
    params = synth.make_params(spec, part.n_vert)
    dev = torch.device("cuda:0")
    t = lambda x: torch.from_numpy(x).to(dev)
    layers = [dict(V=t(params["V"][l]), a=t(params["a"][l]), W0=t(params["W0"][l]), act=1) for l in range(2)]
    need = kb.workspace_bytes(part, layers)
    H0 = t(params["H0"]); out = torch.empty_like(H0)
    small = torch.empty(max(need // 2, 256), dtype=torch.uint8, device=dev)
    with pytest.raises(kb.KgeError) as e:
        kb.rgcn_forward(part, layers, H0, small, out)
    assert e.value.status == -2
    bad = [dict(layers[0]), dict(layers[1])]
    bad[1]["V"] = torch.zeros((4, 16, 16), device=dev)       # d_in mismatch with layer 0's d_out
    with pytest.raises(kb.KgeError) as e:
        kb.workspace_bytes(part, bad)
    gone = [dict(layers[0], order=1), dict(layers[1], order=1)]      # the value of a removed evaluation order
    with pytest.raises(kb.KgeError, match="bad order"):
        kb.workspace_bytes(part, gone)
    odd = [dict(V=torch.zeros((2, 6, 6), device=dev), a=layers[0]["a"][:, :2].contiguous(),
                W0=torch.zeros((6, 6), device=dev), act=0)]
    with pytest.raises(kb.KgeError):
        kb.workspace_bytes(part, odd)                        # width not a multiple of 4


# ------------------------------------------------------------------ benchmark configurations
def test_config0_tiny_whole_step(kb, orc):
    spec = synth.WORKLOADS[0]
    say("config 0", spec.name)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert (gp.n_vert, gp.n_edge) == (1000, 10000)
    assert_partition_equal(gp, op)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


@pytest.fixture(scope="module")
def config1_oracle(orc):
    """configs[1] (the whole 14,541-entity graph as one partition, 30,000 positives x 10 negatives):
    the oracle's whole step, computed once for both evaluation orders."""
    spec = synth.WORKLOADS[1]
    head, rel, tail = synth.make_triples(spec)
    op = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts, spec.part_id,
                             spec.n_hops, spec.neg_domain)
    params = synth.make_params(spec, op["n_vert"])
    pos = synth.make_batch(spec, op["n_core"])
    say("config 1 oracle step")
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    return spec, (head, rel, tail), params, pos, op, res


@pytest.mark.parametrize("order", [0, 2], ids=["project_first", "relation_weights"])
def test_config1_mid_whole_graph_step(kb, orc, config1_oracle, order):
    spec, (head, rel, tail), params, pos, op, res = config1_oracle
    say("config 1", spec.name, "order", order)
    gp, ts, _, _ = gpu_step(spec, head, rel, tail, params=params, pos=pos, order=order)
    assert (gp.n_vert, gp.n_core) == (14541, 272115)       # one partition = the whole graph
    assert_partition_equal(gp, op)
    # 2.9 M pre-activations: one within fp32 rounding of zero may take the other side in the kernel's
    # fp32 sum; the ReLU decision is then taken in the kernel's precision
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, spec.acts, True, False)
    say("config 1 adopted ReLU decisions", n_adopted)
    assert n_adopted <= 8
    errs = assert_step_close(ts, res, TOL_VAL, TOL_GRAD)
    say("config 1 errs", errs)


def test_config2_mid_partition_whole_step(kb, orc):
    """Partition 0 of 8 of the 14,541-entity / 272,115-triple graph, d = 200, 10 bases, at its
    real shape (the expansion covers almost the whole graph); oracle runs the whole step."""
    spec = synth.WORKLOADS[2]
    say("config 2", spec.name)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    errs = assert_step_close(ts, res, TOL_VAL, TOL_GRAD)
    say("config 2 errs", errs)
