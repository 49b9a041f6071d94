"""GPU parity of the relation-weight order of Eq. 1-2, the library's product path (run means z,
W_r = sum_b a_rb V_b written out, one product z W_r per run), against the same oracle as the
project-first order: the orders are algebraically identical, so every output is held to the same
tolerances."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import (SEED, STEP, align_mask_decisions, assert_partition_equal, assert_step_close, gpu_step,
                      oracle_step, rel_err)

pytestmark = pytest.mark.gpu
TOL_VAL, TOL_GRAD = 1e-4, 1e-3
RELW = 2
ORDERS = [pytest.param(RELW, id="relation_weights")]


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


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


def test_runs_grouped_by_destination(kb, orc):
    say("dr view")
    head, rel, tail = random_graph(3, 500, 7, 6000)
    gp = kb.build_partition(head, rel, tail, 500, 7, 2, 1, 2, 0)
    op = orc.build_partition(head, rel, tail, 500, 7, 2, 1, 2, 0)
    S, N = op["n_seg"], op["n_vert"]
    order = np.lexsort((op["seg_rel"], op["seg_dst"]))            # by destination, then relation
    np.testing.assert_array_equal(gp.export("dr_seg"), order.astype(np.int32))
    np.testing.assert_array_equal(gp.export("dr_rel"), op["seg_rel"][order])
    want_ptr = np.searchsorted(op["seg_dst"][order], np.arange(N + 1)).astype(np.int32)
    np.testing.assert_array_equal(gp.export("dr_ptr"), want_ptr)
    assert gp.export("dr_ptr")[-1] == S
    # run id of every edge in source-major order (src, rel, dst, id)
    lens = np.diff(op["seg_ptr"])
    run_of_edge = np.repeat(np.arange(S), lens)
    dst_of_edge = op["seg_dst"][run_of_edge]; rel_of_edge = op["seg_rel"][run_of_edge]
    sm_order = np.lexsort((op["edge_id"], dst_of_edge, rel_of_edge, op["col_src"]))
    np.testing.assert_array_equal(gp.export("sm_seg"), run_of_edge[sm_order].astype(np.int32))


SHAPES = [
    # name, n, R, m, d, B, n_pos, n_neg, mode, P, acts
    ("d32_B4", 300, 5, 2500, 32, 4, 200, 3, 1, 1, [1, 0]),
    ("d200_B10_ragged_lanes", 400, 6, 3000, 200, 10, 333, 5, 1, 1, [1, 0]),
    ("d128_B2", 500, 1, 4000, 128, 2, 257, 1, 0, 2, [1, 0]),
    ("d64_B3_odd_bases", 300, 4, 2000, 64, 3, 100, 2, 1, 3, [1, 1]),
    ("d8_B1", 100, 2, 700, 8, 1, 64, 4, 1, 1, [0, 0]),
    ("d256_B5", 200, 3, 1500, 256, 5, 90, 7, 1, 1, [1, 0]),
    ("d16_B20", 250, 9, 2200, 16, 20, 128, 2, 0, 2, [1, 0]),
    ("d96_B40_matrix_core_sum", 300, 12, 2600, 96, 40, 150, 3, 1, 1, [1, 0]),
    ("d160_B70", 200, 5, 1500, 160, 70, 64, 2, 1, 2, [1, 1]),
    ("d32_B256_most_bases", 150, 4, 1200, 32, 256, 64, 2, 1, 1, [1, 0]),
    ("many_relations_few_runs", 400, 300, 3000, 32, 6, 100, 2, 1, 1, [1, 0]),
    ("one_relation_many_chunks", 9000, 1, 40000, 16, 2, 300, 1, 1, 1, [1, 0]),
]


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_step_relation_weights(kb, orc, shape, order):
    name, n, R, m, d, B, n_pos, n_neg, mode, P, acts = shape
    say("step, order", order, shape)
    spec = synth.scaled(synth.WORKLOADS[0], name=name, seed=17, n_entities=n, n_relations=R, n_triples=m,
                        d=d, n_bases=B, n_pos=n_pos, n_neg=n_neg, neg_mode=mode, n_parts=P, part_id=P - 1,
                        acts=acts, feature_std=0.5)
    head, rel, tail = random_graph(len(name) + n, n, R, m)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


def test_intermediate_run_means(kb, orc):
    """z (run means) of the LAST layer against their definition in fp64."""
    say("z")
    n, R, m, d, B = 600, 6, 7000, 64, 5
    spec = synth.scaled(synth.WORKLOADS[0], name="zy", seed=3, n_entities=n, n_relations=R, n_triples=m,
                        d=d, n_bases=B, n_pos=50, n_neg=1, feature_std=0.5)
    head, rel, tail = random_graph(77, n, R, m)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=RELW)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    H1 = res["Hs"][1]                       # input of the last layer
    lens = np.diff(op["seg_ptr"])
    run_of_edge = np.repeat(np.arange(op["n_seg"]), lens)
    Z = np.zeros((op["n_seg"], d))
    np.add.at(Z, run_of_edge, H1[op["col_src"]])
    Z /= lens[:, None]
    assert rel_err(ts.view(kb.WS_Z, 1).cpu().numpy(), Z) <= TOL_VAL


@pytest.mark.parametrize("order", ORDERS)
def test_hub_rows_relation_weights(kb, orc, order):
    """A run of 600 edges (split into units), a destination and a source with > 256 edges."""
    say("hub, order", order)
    n, R = 700, 2
    leaves = np.arange(1, 601, dtype=np.int32)
    head = np.concatenate([leaves, leaves[:50], np.array([650, 651], np.int32)])
    tail = np.concatenate([np.zeros(600, np.int32), np.zeros(50, np.int32), np.array([651, 652], np.int32)])
    rel = np.concatenate([np.zeros(600, np.int32), np.ones(50, np.int32), np.array([0, 1], np.int32)])
    spec = synth.scaled(synth.WORKLOADS[0], name="hub", seed=5, n_entities=n, n_relations=R,
                        n_triples=len(head), d=64, n_bases=4, n_pos=300, n_neg=2, neg_mode=1)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


@pytest.mark.parametrize("order", ORDERS)
def test_many_runs_per_destination(kb, orc, order):
    """One destination reached under 700 different relations: its list of runs is itself split."""
    say("heavy run list, order", order)
    n, R = 900, 700
    head = np.arange(1, 701, dtype=np.int32)
    tail = np.zeros(700, np.int32)
    rel = np.arange(700, dtype=np.int32)
    extra = random_graph(9, n, R, 1500)
    head = np.concatenate([head, extra[0]]); rel = np.concatenate([rel, extra[1]]); tail = np.concatenate([tail, extra[2]])
    spec = synth.scaled(synth.WORKLOADS[0], name="manyruns", seed=5, n_entities=n, n_relations=R,
                        n_triples=len(head), d=32, n_bases=3, n_pos=200, n_neg=1, neg_mode=1)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert np.diff(gp.export("dr_ptr")).max() >= 700
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD)


@pytest.mark.parametrize("order", ORDERS)
def test_relation_weights_with_compute_graph(kb, orc, order):
    say("sub-graph, order", order)
    n, R, m = 4000, 5, 14000
    spec = synth.scaled(synth.WORKLOADS[0], name="aggcone", seed=23, n_entities=n, n_relations=R, n_triples=m,
                        d=64, n_bases=4, n_pos=9, n_neg=2, neg_mode=1, feature_std=0.5)
    head, rel, tail = random_graph(31, n, R, m)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, cone=True, order=order)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    active, stats = ts.cg.export()
    np.testing.assert_array_equal(active, orc.compute_graph(op, pos, res["neg_ent"], 2))
    assert stats[1, 0] < stats[0, 0] < gp.n_vert
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD, batch_rows=orc.batch_vertices(op, pos, res["neg_ent"]))


TOL_BF16 = 2e-2


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("acts,n,m,d,B,cone", [([0, 0], 600, 6000, 64, 8, False), ([1, 0], 6000, 90000, 64, 8, False),
                                               ([0, 0], 900, 9000, 96, 40, False), ([1, 0], 5000, 60000, 128, 6, True),
                                               ([1, 0], 700, 7000, 40, 70, False)],
                         ids=["identity", "relu", "identity_B40_d96", "relu_subgraph", "relu_B70_d40_ragged_tiles"])
def test_bf16_relation_weights(kb, orc, acts, n, m, d, B, cone, order):
    """The bf16 pipeline of the relation-weight order (inputs, run means, W_r, the per-run products and W_0 are
    bf16 operands; sums fp32): every output against the exact oracle at 2e-2, ReLU decisions inside the
    rounding band taken as the kernel took them."""
    say("bf16, order", order, acts, n, m, d, B, cone)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-agg", seed=3, n_entities=n, n_relations=20,
                        n_triples=m, d=d, n_bases=B, n_pos=24 if cone else 256, n_neg=4, n_parts=2, part_id=0, acts=acts)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order, cone=cone)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    rows = orc.batch_vertices(op, pos, res["neg_ent"]) if cone else None
    active = orc.compute_graph(op, pos, res["neg_ent"], len(acts)) if cone else None
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, acts, True, True, rows=active)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_adopted)
    errs = assert_step_close(ts, res, TOL_BF16, TOL_BF16, batch_rows=rows)
    say("errs vs the exact oracle", errs)


@pytest.mark.parametrize("d_in,d", [(256, 128), (128, 256)], ids=["256_to_128", "128_to_256"])
def test_bf16_relation_weights_mixed_widths(kb, orc, d_in, d):
    """Layers whose input and output widths differ, at the widths the row-streaming kernels of the relation
    gradient and of the per-run products take (128 and 256): layer 1 is d_in -> d, layer 2 d -> d; relation chunks
    of every length (one run to several tiles).  Everything against the exact oracle at 2e-2."""
    say("bf16 relation order, widths", d_in, d)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-mixed", seed=9, n_entities=500, n_relations=12, n_triples=5000,
                        d=d, d_in=d_in, n_bases=8, n_pos=128, n_neg=4, n_parts=2, part_id=0, acts=[1, 0])
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=RELW)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, [1, 0], True, True)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_adopted)
    errs = assert_step_close(ts, res, TOL_BF16, TOL_BF16)
    say("errs vs the exact oracle", errs)


def test_bf16_ranges_ordered_by_destination_slab(kb, orc):
    """The transposed per-run products walk run ranges that are ordered by slab of the destination range and cut
    at slab borders; only a partition of more than 262,144 vertices gets more than one slab.  With the test hook a
    small graph gets eleven slabs and every relation is cut: the step must come out as without slabs (every run in
    exactly one range), to the bf16 tolerance against the exact oracle."""
    say("bf16 relation order with destination slabs")
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-slabs", seed=13, n_entities=2100, n_relations=3, n_triples=24000,
                        d=128, n_bases=4, n_pos=128, n_neg=4, n_parts=1, part_id=0, acts=[1, 0])
    head, rel, tail = synth.make_triples(spec)
    kb.set_rel_slab_for_tests(200, 40)
    try:
        gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=RELW)
    finally:
        kb.set_rel_slab_for_tests(0, 0)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, [1, 0], True, True)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_adopted)
    errs = assert_step_close(ts, res, TOL_BF16, TOL_BF16)
    say("errs vs the exact oracle", errs)


def test_bf16_run_means(kb, orc):
    """Run means z of the first layer (stored in bf16) against the exact means: each element within two
    bf16 roundings (of the input, of the mean) of mean|h| over its run, and 2e-2 as a tensor.  Runs of one edge
    keep no stored mean in this pipeline (the products read the source's row in place)."""
    say("bf16 z")
    import torch
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-z", seed=4, n_entities=800, n_relations=10, n_triples=9000,
                        d=64, n_bases=4, n_pos=64, n_neg=2, n_parts=1, part_id=0, acts=[1, 0])
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=RELW)
    op = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, 1, 0, 2, spec.neg_domain)
    H0 = np.asarray(params["H0"], np.float64)
    lens = np.diff(op["seg_ptr"]); run = np.repeat(np.arange(op["n_seg"]), lens)
    Z = np.zeros((op["n_seg"], spec.d)); np.add.at(Z, run, H0[op["col_src"]])
    Zabs = np.zeros_like(Z); np.add.at(Zabs, run, np.abs(H0[op["col_src"]]))
    Z /= lens[:, None]; Zabs /= lens[:, None]
    got = ts.view(kb.WS_Z, 0).to(torch.float64).cpu().numpy()
    multi = lens > 1
    assert multi.sum() > 100
    assert np.all(np.abs(got[multi] - Z[multi]) <= 2.0 * 2.0 ** -8 * Zabs[multi] + 1e-30)
    assert rel_err(got[multi], Z[multi]) <= TOL_BF16


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("d", [64, 72])
def test_bf16_many_small_relations(kb, orc, order, d):
    """800 relation ids over 5,000 runs: every row tile of the run list is a ragged handful of runs, a block's
    consecutive tiles belong to different relations (a new weight matrix per tile), and the per-relation
    contraction ranges of the outer products are one to a few runs long.  d = 64 takes the multi-tile form of
    the per-run products, d = 72 the one-tile form."""
    say("bf16, many small relations, order", order, d)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16-manyrel", seed=13, n_entities=1500, n_relations=400,
                        n_triples=4000, d=d, n_bases=4, n_pos=200, n_neg=3, n_parts=1, part_id=0, acts=[0, 0])
    head, rel, tail = random_graph(77, 1500, 400, 4000)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order)
    assert gp.n_seg > 4000 and len(np.unique(gp.export("seg_rel"))) > 700
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    errs = assert_step_close(ts, res, TOL_BF16, TOL_BF16)
    say("errs", errs)


@pytest.mark.parametrize("order", [pytest.param(0, id="project_first")] + ORDERS)
@pytest.mark.parametrize("dims,bf16", [((128, 32, 32), False), ((48, 96, 24), False), ((128, 32, 32), True),
                                       ((64, 128, 64), True), ((192, 64, 264), True), ((200, 40, 72), True), ((8, 248, 16), True),
                                       ((512, 256, 256), False), ((256, 256, 256), False), ((512, 320, 512), True),
                                       ((256, 256, 512), True)],
                         ids=["f32_128_32_32", "f32_48_96_24", "bf16_128_32_32", "bf16_64_128_64", "bf16_192_64_264_three_chunks_ragged_columns",
                              "bf16_200_40_72_ragged_tiles", "bf16_8_248_16_ragged_tiles",
                              "f32_512_256_256_widest", "f32_256_256_256_widest", "bf16_512_320_512_widest",
                              "bf16_256_256_512_widest"])
def test_feature_layer_with_different_widths(kb, orc, order, dims, bf16):
    """A feature-input layer whose width differs from the embedding width (the paper's large-graph
    setting: 128-d features, 32-d embeddings), and a widening layer, in every order."""
    say("d_in != d_out, order", order, dims, bf16)
    n, R, m, B = 700, 4, 6000, 3
    spec = synth.scaled(synth.WORKLOADS[4 if bf16 else 0], name="widths", seed=9, n_entities=n, n_relations=R,
                        n_triples=m, d=dims[2], n_bases=B, n_pos=150, n_neg=2, neg_mode=1, n_parts=1, part_id=0,
                        acts=[0, 0] if bf16 else [1, 0], feature_std=0.5)
    head, rel, tail = random_graph(41, n, R, m)
    too_wide = ("d_out <= 256" if order == 0 and max(dims[1:]) > 256 else
                "d_in <= 256" if order == RELW and not bf16 and max(dims[:2]) > 256 else None)
    if too_wide:
        # wider than the order's kernels take (see the header): a clean error before anything runs, not a fault
        part = kb.build_partition(head, rel, tail, n, R, 1, 0, 2, spec.neg_domain)
        with pytest.raises(kb.KgeError, match=too_wide):
            gpu_step(spec, head, rel, tail, params=dict(
                V=[np.zeros((B, dims[0], dims[1]), np.float32), np.zeros((B, dims[1], dims[2]), np.float32)],
                a=[np.zeros((2 * R, B), np.float32)] * 2,
                W0=[np.zeros((dims[0], dims[1]), np.float32), np.zeros((dims[1], dims[2]), np.float32)],
                M=np.zeros((R, dims[2]), np.float32), H0=np.zeros((part.n_vert, dims[0]), np.float32)), order=order)
        return
    rng = np.random.default_rng(5)
    g = lambda *shape: (rng.uniform(-1, 1, shape) * np.sqrt(6.0 / (shape[-2] + shape[-1]))).astype(np.float32)
    opart = orc.build_partition(head, rel, tail, n, R, 1, 0, 2, spec.neg_domain)
    params = dict(V=[g(B, dims[0], dims[1]), g(B, dims[1], dims[2])], a=[g(2 * R, B), g(2 * R, B)],
                  W0=[g(dims[0], dims[1]), g(dims[1], dims[2])],
                  M=(rng.standard_normal((R, dims[2])) * 0.1).astype(np.float32),
                  H0=(rng.standard_normal((opart["n_vert"], dims[0])) * 0.5).astype(np.float32))
    gp, ts, _, pos = gpu_step(spec, head, rel, tail, params=params, order=order)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    tol = (TOL_BF16, TOL_BF16) if bf16 else (TOL_VAL, TOL_GRAD)
    if not bf16:
        # a pre-activation within fp32 rounding of zero may take the other side in the kernel's fp32 sum
        # over up to 512 terms; the ReLU decision is then taken in the kernel's precision
        n_adopted, res = align_mask_decisions(orc, ts, op, res, params, spec.acts, True, False)
        say("adopted ReLU decisions", n_adopted)
        assert n_adopted <= 4
    assert_step_close(ts, res, *tol)
