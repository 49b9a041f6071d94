"""GPU parity of the optimizer step (Algorithm 1, "optimizer.step()") against the oracle, and a short
training loop: forward, negatives, loss, backward, update - several times, against the same loop in
the oracle, with the loss going down."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import SEED, layers_of, rel_err

# the library takes float hyper-parameters: the oracle gets the same (float-rounded) values
LR, B1, B2, EPS = (float(np.float32(x)) for x in (0.01, 0.9, 0.999, 1e-8))

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


@pytest.mark.parametrize("kind", [0, 1], ids=["sgd", "adam"])
@pytest.mark.parametrize("n", [1, 255, 4096 + 3, 1 << 20])
def test_dense_step(kb, orc, kind, n):
    import torch
    say("dense optimizer step", kind, n)
    rng = np.random.default_rng(n + kind)
    p = rng.normal(0, 1, n).astype(np.float32); g = (rng.normal(0, 1, n) * 10.0 ** rng.integers(-4, 2, n)).astype(np.float32)
    m = rng.normal(0, 0.1, n).astype(np.float32); v = rng.uniform(0, 0.1, n).astype(np.float32)
    g[::7] = 0.0
    for t in (1, 9):
        dp, dg, dm, dv = (torch.from_numpy(x.copy()).cuda() for x in (p, g, m, v))
        kb.optimizer_step(kind, dp, dg, dm if kind else None, dv if kind else None, 0.01, 0.9, 0.999, 1e-8, t)
        torch.cuda.synchronize()
        op, om, ov = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
        orc.optimizer_step(kind, op, g, om, ov, LR, B1, B2, EPS, t)
        assert rel_err(dp.cpu().numpy(), op) <= 1e-6
        if kind:
            assert rel_err(dm.cpu().numpy(), om) <= 1e-6 and rel_err(dv.cpu().numpy(), ov) <= 1e-6


@pytest.mark.parametrize("use_mask", [True, False], ids=["mask", "nonzero_rows"])
def test_row_step(kb, orc, use_mask):
    import torch
    say("row optimizer step", use_mask)
    rng = np.random.default_rng(5)
    N, d = 1000, 72
    p = rng.normal(0, 1, (N, d)).astype(np.float32); g = rng.normal(0, 1, (N, d)).astype(np.float32)
    m = rng.normal(0, 0.1, (N, d)).astype(np.float32); v = rng.uniform(0, 0.1, (N, d)).astype(np.float32)
    touched = rng.random(N) < 0.3
    g[~touched] = 0.0
    g[np.nonzero(touched)[0][0], :-1] = 0.0          # a touched row with a single non-zero element
    mask = touched.astype(np.uint8)
    dp, dg, dm, dv = (torch.from_numpy(x.copy()).cuda() for x in (p, g, m, v))
    dmask = torch.from_numpy(mask).cuda() if use_mask else None
    kb.optimizer_step(1, dp, dg, dm, dv, 0.01, 0.9, 0.999, 1e-8, 3, rows=True, row_mask=dmask)
    torch.cuda.synchronize()
    op, om, ov = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    orc.optimizer_step(1, op, g, om, ov, LR, B1, B2, EPS, 3, row_mask=mask)
    assert rel_err(dp.cpu().numpy(), op) <= 1e-6 and rel_err(dm.cpu().numpy(), om) <= 1e-6
    assert rel_err(dv.cpu().numpy(), ov) <= 1e-6
    np.testing.assert_array_equal(dp.cpu().numpy()[~touched], p[~touched])       # untouched rows: bit-identical
    np.testing.assert_array_equal(dm.cpu().numpy()[~touched], m[~touched])


def test_training_loop_matches_the_oracle_and_the_loss_goes_down(kb, orc):
    """Algorithm 1 for one trainer: 5 mini-batch steps with Adam (lr 0.01) on a small graph."""
    import torch
    from paper_2201_02791_amd.step import TrainStep
    say("training loop")
    spec = synth.scaled(synth.WORKLOADS[0], name="loop", seed=11, n_entities=600, n_relations=6, n_triples=5000,
                        d=32, n_bases=3, n_pos=512, n_neg=2, neg_mode=1)
    head, rel, tail = synth.make_triples(spec)
    gp = kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, 1, 0, 2, spec.neg_domain)
    op = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, 1, 0, 2, spec.neg_domain)
    params = synth.make_params(spec, gp.n_vert)
    pos = synth.make_batch(spec, gp.n_core)
    ts = TrainStep(gp, params, spec.acts, kb.MSG_F32, cone=True, order=kb.ORDER_RELATION_WEIGHTS)
    ts.set_batch(pos, spec.n_neg)
    # the oracle's copy of every parameter and Adam state, float64
    P = dict(M=np.asarray(params["M"], np.float64), H0=np.asarray(params["H0"], np.float64))
    for l in range(2):
        for k in ("V", "a", "W0"):
            P["%s%d" % (k, l)] = np.asarray(params[k][l], np.float64).copy()
    st = {k: (np.zeros_like(x), np.zeros_like(x)) for k, x in P.items()}
    losses_g, losses_o = [], []
    for step in range(5):
        ts.run(spec.neg_mode, SEED, step)
        ts.optimizer_step(kb.OPT_ADAM, 0.01)
        torch.cuda.synchronize()
        losses_g.append(float(ts.loss.cpu()[0]))
        layers = [dict(V=P["V%d" % l], a=P["a%d" % l], W0=P["W0%d" % l], act=spec.acts[l]) for l in range(2)]
        res = orc.train_step(op, layers, P["H0"], P["M"], pos, spec.n_neg, spec.neg_mode, SEED, step)
        losses_o.append(res["loss"])
        grads = dict(M=res["dM"], H0=res["dH0"])
        for l in range(2):
            for k in ("V", "a", "W0"):
                grads["%s%d" % (k, l)] = res["grads"][l]["d" + k]
        for k in P:
            # the entity rows the step read: one hop beyond the first layer's active destinations
            mask = orc.compute_graph(op, pos, res["neg_ent"], 3)[0] if k == "H0" else None
            orc.optimizer_step(1, P[k], grads[k], st[k][0], st[k][1], LR, B1, B2, EPS, step + 1, row_mask=mask)
    say("losses gpu", losses_g, "oracle", losses_o)
    np.testing.assert_allclose(losses_g, losses_o, rtol=1e-4)
    # fresh negatives every step make single steps noisy; over the loop the loss must fall clearly
    assert losses_g[-1] < losses_g[0] - 0.02 and min(losses_g[1:]) < losses_g[0], "the loss must go down"
    c = lambda t: t.detach().cpu().numpy()
    assert rel_err(c(ts.M), P["M"]) <= 1e-3 and rel_err(c(ts.H0), P["H0"]) <= 1e-3
    for l in range(2):
        for k in ("V", "a", "W0"):
            assert rel_err(c(ts.layers[l][k]), P["%s%d" % (k, l)]) <= 1e-3, (k, l)
