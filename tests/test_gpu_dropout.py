"""GPU parity of dropout on the layer inputs (training setting of Sec. 4: rate 0.2 on the large
graphs): the keep decisions are bit-exact against the oracle's counter-based mask, and a whole step
with dropout matches the oracle in both evaluation orders, with and without the per-batch
sub-graph, in fp32 and with bf16 messages."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import (SEED, STEP, align_mask_decisions, assert_step_close, gpu_step, oracle_step, rel_err)

pytestmark = pytest.mark.gpu
TOL_VAL, TOL_GRAD, TOL_BF16 = 1e-4, 1e-3, 2e-2
PROJ, RELW = 0, 2
ORDERS = [pytest.param(PROJ, id="project_first"), pytest.param(RELW, id="relation_weights")]


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


def graph(seed, n, R, m):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, n, m).astype(np.int32), rng.integers(0, R, m).astype(np.int32),
            rng.integers(0, n, m).astype(np.int32))


def spec_of(name, n, R, m, d, B, n_pos, n_neg, acts, **kw):
    return synth.scaled(synth.WORKLOADS[0], name=name, seed=29, n_entities=n, n_relations=R, n_triples=m,
                        d=d, n_bases=B, n_pos=n_pos, n_neg=n_neg, neg_mode=1, n_parts=1, part_id=0,
                        acts=acts, n_layers=len(acts), n_hops=len(acts), feature_std=0.5, **kw)


@pytest.mark.parametrize("p", [0.2, 0.5, 0.9])
def test_keep_decisions_are_bit_exact(kb, orc, p):
    """The dropped copy of each layer's input has exactly the oracle's zero pattern (layer 1's input
    is an identity-activation output here, so it has no zeros of its own) and its kept values scaled."""
    say("mask", p)
    spec = spec_of("mask", 700, 4, 5000, 72, 3, 64, 2, [0, 0])
    head, rel, tail = graph(1, 700, 4, 5000)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, dropout=p)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos, dropout=p)
    pf = float(np.float32(p))
    for l in range(2):
        hd = ts.view(kb.WS_HD, l).cpu().numpy()
        m = res["masks"][l].astype(bool)
        assert abs(m.mean() - (1 - pf)) < 5 * np.sqrt(pf * (1 - pf) / m.size)
        np.testing.assert_array_equal(hd != 0, m & (res["Hs"][l] != 0))
        assert rel_err(hd, res["Hs"][l]) <= (1e-6 if l == 0 else TOL_VAL)
    # backward: the gradient with respect to H0 vanishes exactly where layer 0 dropped the element
    dh0 = ts.dH0.cpu().numpy()
    assert not dh0[~res["masks"][0].astype(bool)].any()


@pytest.mark.parametrize("cone", [False, True], ids=["whole_partition", "subgraph"])
@pytest.mark.parametrize("order", ORDERS)
def test_step_with_dropout(kb, orc, order, cone):
    say("step with dropout", order, cone)
    n, R, m = 2500, 6, 11000
    spec = spec_of("drop", n, R, m, 64, 5, 24 if cone else 300, 3, [1, 0])
    head, rel, tail = graph(7, n, R, m)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, cone=cone, order=order, dropout=0.2)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos, dropout=0.2)
    rows = orc.compute_graph(op, pos, res["neg_ent"], 2) if cone else None
    n_flip, res = align_mask_decisions(orc, ts, op, res, params, spec.acts, True, False, rows=rows)
    assert n_flip <= 8
    assert_step_close(ts, res, TOL_VAL, TOL_GRAD,
                      batch_rows=orc.batch_vertices(op, pos, res["neg_ent"]) if cone else None)


@pytest.mark.parametrize("order", ORDERS)
def test_step_with_dropout_bf16_messages(kb, orc, order):
    say("step with dropout, bf16", order)
    spec = synth.scaled(synth.WORKLOADS[4], name="bf16drop", n_entities=4000, n_relations=12, n_triples=30000,
                        d=64, n_bases=6, n_pos=200, n_neg=3, n_parts=1, part_id=0, acts=[1, 0])
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order, dropout=0.2)
    op, res = oracle_step(orc, spec, head, rel, tail, params, pos, dropout=0.2)
    # against the exact oracle; ReLU decisions inside the rounding band of their own sum (asserted, and few)
    # are taken as the kernel took them
    n_flip, res = align_mask_decisions(orc, ts, op, res, params, spec.acts, True, True)
    say("mask decisions inside the rounding band, taken as the kernel took them:", n_flip)
    assert_step_close(ts, res, TOL_BF16, TOL_BF16)


def test_masks_change_with_the_step_and_not_otherwise(kb):
    say("mask per step")
    import torch
    from paper_2201_02791_amd.step import TrainStep
    spec = spec_of("steps", 600, 3, 4000, 32, 2, 50, 1, [1, 0])
    head, rel, tail = graph(3, 600, 3, 4000)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=RELW, dropout=0.2)
    a = ts.view(kb.WS_HD, 0).clone()
    ts.run(spec.neg_mode, SEED, STEP); torch.cuda.synchronize()
    assert torch.equal(ts.view(kb.WS_HD, 0), a)
    ts.run(spec.neg_mode, SEED, STEP + 1); torch.cuda.synchronize()
    b = ts.view(kb.WS_HD, 0)
    same = ((a != 0) == (b != 0)).float().mean().item()
    assert abs(same - 0.68) < 0.02          # two independent masks of rate 0.2 agree on 0.2^2 + 0.8^2 of the elements


def test_rate_outside_the_unit_interval_is_refused(kb):
    say("bad rate")
    from paper_2201_02791_amd.step import TrainStep
    spec = spec_of("bad", 100, 2, 500, 16, 2, 10, 1, [1, 0])
    head, rel, tail = graph(4, 100, 2, 500)
    part = kb.build_partition(head, rel, tail, 100, 2, 1, 0, 2, 0)
    params = synth.make_params(spec, part.n_vert)
    for bad in (1.0, -0.1, float("nan")):
        with pytest.raises(kb.KgeError):
            TrainStep(part, params, spec.acts, kb.MSG_F32, dropout=bad)
