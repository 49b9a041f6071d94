"""GPU parity of the per-batch computational sub-graph (Sec. 3.3, Algorithm 1 "getComputeGraph"):
the flags and counts are bit-exact against the oracle, and a step that propagates only the
sub-graph gives the batch embeddings, loss and gradients of the oracle's whole-partition step."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import (SEED, STEP, align_mask_decisions, assert_partition_equal, assert_step_close, gpu_step,
                      oracle_step)

pytestmark = pytest.mark.gpu
TOL_VAL, TOL_GRAD, TOL_BF16 = 1e-4, 1e-3, 2e-2


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


def check_flags(orc, ts, opart, pos, res, n_layers):
    want = orc.compute_graph(opart, pos, res["neg_ent"], n_layers)
    got, stats = ts.cg.export()
    np.testing.assert_array_equal(got, want)
    dst_of_edge = np.repeat(opart["seg_dst"], np.diff(opart["seg_ptr"]))
    for l in range(n_layers):
        assert stats[l, 0] == int(want[l].sum())
        assert stats[l, 1] == int(want[l][dst_of_edge].sum())
        assert stats[l, 2] == int(want[l][opart["seg_dst"]].sum())
        assert stats[l, 3] == int(want[l][opart["col_src"]].sum())
    # the rows of the first layer's input the batch reads: one hop beyond its active destinations
    flags, count = ts.cg.input_rows()
    want_in = orc.compute_graph(opart, pos, res["neg_ent"], n_layers + 1)[0]
    np.testing.assert_array_equal(flags, want_in)
    assert count == int(want_in.sum())
    return want, stats


CASES = [
    # name, n, R, m, d, B, n_pos, n_neg, mode, P, acts
    ("small_batch_d32_B4", 3000, 5, 12000, 32, 4, 8, 2, 1, 1, [1, 0]),
    ("d128_B2_parts", 5000, 1, 20000, 128, 2, 16, 1, 0, 2, [1, 0]),
    ("d200_B10_ragged", 1500, 6, 6000, 200, 10, 5, 3, 1, 1, [1, 1]),
    ("d96_B40_matrix_core_transpose", 1200, 12, 5000, 96, 40, 6, 2, 1, 1, [1, 0]),
    ("three_layers", 4000, 3, 9000, 16, 2, 3, 1, 1, 1, [1, 1, 0]),
    ("one_layer", 800, 3, 3000, 16, 2, 10, 1, 1, 1, [0]),
    ("full_batch_covers_everything", 300, 5, 2500, 32, 4, 200, 3, 1, 1, [1, 0]),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_cone_step_matches_whole_partition_oracle(kb, orc, case):
    name, n, R, m, d, B, n_pos, n_neg, mode, P, acts = case
    say("cone", case)
    spec = synth.scaled(synth.WORKLOADS[0], name=name, seed=23, n_entities=n, n_relations=R, n_triples=m,
                        d=d, n_bases=B, n_pos=n_pos, n_neg=n_neg, neg_mode=mode, n_parts=P, part_id=P - 1,
                        acts=acts, n_layers=len(acts), n_hops=len(acts), feature_std=0.5)
    rng = np.random.default_rng(len(name) + n)
    head = rng.integers(0, n, m).astype(np.int32); rel = rng.integers(0, R, m).astype(np.int32)
    tail = rng.integers(0, n, m).astype(np.int32)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, cone=True)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    assert_partition_equal(gp, op)
    want, stats = check_flags(orc, ts, op, pos, res, len(acts))
    if "covers" not in name and len(acts) > 1:
        assert 0 < stats[-1, 0] < stats[0, 0] <= gp.n_vert and stats[-1, 1] < gp.n_edge
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD, batch_rows=orc.batch_vertices(op, pos, res["neg_ent"]))


def test_cone_with_hub_rows(kb, orc):
    """A destination and a source with far more than 256 edges (split into units), inside and
    outside the batch's sub-graph."""
    say("cone hub")
    n, R = 1500, 2
    leaves = np.arange(1, 601, dtype=np.int32)
    leaves2 = np.arange(700, 1300, dtype=np.int32)
    # hub 0 collects 600 leaves; hub 650 collects another 600; a few chain edges
    head = np.concatenate([leaves, leaves2, np.array([0, 650, 1400], np.int32)])
    tail = np.concatenate([np.zeros(600, np.int32), np.full(600, 650, np.int32), np.array([1401, 1402, 1403], np.int32)])
    rel = np.concatenate([np.zeros(600, np.int32), np.ones(600, np.int32), np.array([0, 1, 0], np.int32)])
    spec = synth.scaled(synth.WORKLOADS[0], name="hub", seed=5, n_entities=n, n_relations=R,
                        n_triples=len(head), d=64, n_bases=4, n_pos=1, n_neg=0, neg_mode=1)
    for chosen in ([5], [1200], [1202], [3, 700, 1201]):      # batches that reach hub 0, hub 650, neither, both
        pos = np.asarray(chosen, np.int32)
        gp, ts, params, _ = gpu_step(spec, head, rel, tail, pos=pos, cone=True)
        op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
        check_flags(orc, ts, op, pos, res, 2)
        assert_step_close(ts, res, TOL_VAL, TOL_GRAD, batch_rows=orc.batch_vertices(op, pos, res["neg_ent"]))


@pytest.mark.parametrize("d,B", [(64, 8), (96, 40)], ids=["d64_B8", "d96_B40_matrix_core_transposed_sums"])
def test_cone_bf16_messages(kb, orc, d, B):
    say("cone bf16", d, B)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16cone", n_entities=5000, n_relations=20, n_triples=40000,
                        d=d, n_bases=B, n_pos=12, n_neg=4, n_parts=1, part_id=0, acts=[1, 0])
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, cone=True)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos)
    check_flags(orc, ts, op, pos, res, 2)
    active = orc.compute_graph(op, pos, res["neg_ent"], 2)
    n_adopted, res = align_mask_decisions(orc, ts, op, res, params, spec.acts, True, True, rows=active)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_adopted)
    assert_step_close(ts, res, TOL_BF16, TOL_BF16, batch_rows=orc.batch_vertices(op, pos, res["neg_ent"]))


def test_cone_empty_batch_and_errors(kb, orc):
    say("cone empty batch / wrong object")
    import torch
    spec = synth.scaled(synth.WORKLOADS[0], n_entities=200, n_triples=900, n_pos=20, n_neg=1)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, cone=True)
    ts.set_batch(np.zeros(0, np.int32), 2)
    ts.run(1, SEED, STEP)
    torch.cuda.synchronize()
    active, stats = ts.cg.export()
    assert not active.any() and not stats.any()
    assert float(ts.H_out.abs().max().cpu()) == 0.0 and float(ts.loss.cpu()[0]) == 0.0
    for g in ts.grads:
        assert float(g["dV"].abs().max().cpu()) == 0.0 and float(g["da"].abs().max().cpu()) == 0.0
    wrong = kb.ComputeGraph(gp, 3)           # layer count does not match the model
    with pytest.raises(kb.KgeError) as e:
        kb.rgcn_forward(gp, ts.layers, ts.H0, ts.workspace, ts.H_out, ts.msg_dtype, None, wrong)
    assert e.value.status == -1
    with pytest.raises(kb.KgeError):
        kb.ComputeGraph(gp, 0)
