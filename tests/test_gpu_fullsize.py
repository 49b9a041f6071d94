"""GPU parity at the benchmark's full sizes, in the launch configurations bench.py times.

The whole-step oracle is too slow there, so every kernel's output is checked against the EXACT (fp64)
oracle on samples it can compute one by one (rows, columns, runs, relations) or through reductions
that cost one pass over the edges at any size, all evaluated from the GPU's own stored layer inputs:

  build_partition   every array, bit-exact          sample_negatives   every draw, bit-exact
  sub-graph         flags and counts, bit-exact     distmult           all scores, loss, dH_out, dM
  forward           sampled rows of H_1, H_out (exact layer), of P or of the run means z / products u
  activation bwd    sampled rows of G (bit-exact)   input gradients    sampled rows of dH_1 (and dH0)
  transposed sums   sampled rows of dP, or of dz    dW0                whole, both layers
  dV  (both layers) sampled columns, and random projections x^T dV_b y of EVERY basis (every element of
                    every dV_b enters; one pass over the edges)
  da  (both layers) the two relations with the most edges and the rare ones, every basis, from edges;
                    the identity sum a*da = sum V*dV = sum <pre - h W0, G> as an extra

bf16-message workloads (configs[4]) are held to 2e-2 against the same exact oracle; fp32 ones to 1e-4
(values) and 1e-3 (gradients).
"""
import gc
import sys
import time

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import SEED, STEP, assert_partition_equal, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print("[gpu-case]", *a, file=sys.stderr, flush=True)


def pick_rows(rng, deg, edge_budget, n_max, allowed=None):
    """Random rows within an edge budget, plus one row that is cut into units (degree >= 256) and
    the heaviest row if they fit.  allowed: boolean mask of the rows that may be picked."""
    if allowed is not None:
        deg = np.where(allowed, deg, -1)
    order = rng.permutation(len(deg))
    order = order[deg[order] >= 0]
    rows, used = [], 0
    for v in order[:20000]:
        if deg[v] <= 200 and used + deg[v] <= 0.5 * edge_budget and len(rows) < n_max:
            rows.append(int(v)); used += int(deg[v])
    heavy = np.nonzero(deg >= 256)[0]
    if len(heavy):
        h = int(heavy[np.argmin(deg[heavy])])
        if deg[h] <= 0.25 * edge_budget:
            rows.append(h); used += int(deg[h])
        top = int(np.argmax(deg))
        if deg[top] <= 0.25 * edge_budget and top not in rows:
            rows.append(top)
    zero = np.nonzero(deg == 0)[0]
    if len(zero):
        rows.append(int(zero[0]))
    return np.array(sorted(set(rows)), np.int64)


class World:
    """Graph, GPU partition, oracle partition and edge view of one workload, built once per module and
    compared bit-exactly when built."""

    def __init__(self, kb, orc):
        self.kb, self.orc, self.cache = kb, orc, {}

    def get(self, cfg):
        if cfg in self.cache:
            return self.cache[cfg]
        from oracle import sampled
        kb, orc = self.kb, self.orc
        spec = synth.WORKLOADS[cfg]
        t0 = time.time()
        head, rel, tail = synth.make_triples(spec)
        gp = kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts, spec.part_id,
                                spec.n_hops, spec.neg_domain)
        say("config", cfg, "gpu partition N=%d E=%d S=%d (%.0f s)" % (gp.n_vert, gp.n_edge, gp.n_seg, time.time() - t0))
        op = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts, spec.part_id,
                                 spec.n_hops, spec.neg_domain)
        say("oracle partition done (%.0f s)" % (time.time() - t0))
        assert_partition_equal(gp, op)
        del head, rel, tail
        w = dict(gp=gp, op=op, ev=sampled.EdgeView(op), deg_in=np.diff(gp.export("dm_ptr")),
                 deg_out=np.diff(gp.export("sm_ptr")), params={})
        self.cache[cfg] = w
        return w


@pytest.fixture(scope="module")
def kb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2201_02791_amd import binding
    binding.load()
    return binding


@pytest.fixture(scope="module")
def world(kb, orc):
    return World(kb, orc)


def run_full_size(world, cfg, order="project", dropout=0.0, spec=None, da_layers=(0, 1)):
    """One step of workload `cfg` (or of `spec`, a variant on the same graph) on the GPU, every kernel's
    output against the exact oracle.  order "relation" runs on the batch's computational sub-graph (what
    bench.py times by default), "project" on the whole partition (the order the step is named in).
    da_layers: the layers whose coefficient gradient is recomputed from edges for the largest relations."""
    kb, orc = world.kb, world.orc
    relw = order == "relation"
    import torch
    from oracle import sampled
    from paper_2201_02791_amd.step import TrainStep
    spec = spec or synth.WORKLOADS[cfg]
    bf = spec.msg_dtype == "bf16"
    tol_v, tol_g = (2e-2, 2e-2) if bf else (1e-4, 1e-3)
    t0 = time.time()
    w = world.get(cfg)
    gp, op, ev, deg_in, deg_out = w["gp"], w["op"], w["ev"], w["deg_in"], w["deg_out"]
    N, d, B = gp.n_vert, spec.d, spec.n_bases
    d0 = spec.d_in or d
    if spec.name not in w["params"]:
        w["params"] = {spec.name: synth.make_params(spec, N)}
    params = w["params"][spec.name]
    pos = synth.make_batch(spec, gp.n_core)
    need_dH0 = not spec.fixed_features
    ts = TrainStep(gp, params, spec.acts, kb.MSG_BF16 if bf else kb.MSG_F32, need_dH0=need_dH0, cone=relw,
                   order=kb.ORDER_RELATION_WEIGHTS if relw else kb.ORDER_PROJECT_FIRST, dropout=dropout)
    ts.set_batch(pos, spec.n_neg)
    ne, ns = orc.sample_negatives(op, pos, spec.n_neg, spec.neg_mode, SEED, STEP)
    u_check = None
    run_len = np.diff(op["seg_ptr"])
    if relw:       # the per-run products of the last layer share their buffer with dz: look after forward only
        ts.set_dropout_state(SEED, STEP)
        ts.sample(spec.neg_mode, SEED, STEP); ts.compute_graph(); ts.forward()
        torch.cuda.synchronize()
        act_last = orc.compute_graph(op, pos, ne, 2)[1]
        okr = np.nonzero(act_last[op["seg_dst"]].astype(bool) & (run_len <= 2000))[0]
        uruns = np.random.default_rng(7).permutation(okr)[:120].astype(np.int64)
        tr = torch.from_numpy(uruns).to(ts.dev)
        u_check = (uruns, ts.view(kb.WS_U, 1)[:gp.n_seg * d].view(gp.n_seg, d)[tr].float().cpu().numpy(),
                   ts.view(kb.WS_Z, 1)[tr].float().cpu().numpy())
    ts.run(spec.neg_mode, SEED, STEP)
    torch.cuda.synchronize()
    say("gpu step done (%.0f s)" % (time.time() - t0))
    c = lambda t: t.detach().float().cpu().numpy()
    L = [dict(V=params["V"][l], a=params["a"][l], W0=params["W0"][l], act=spec.acts[l]) for l in range(2)]
    H0 = params["H0"]
    H1 = c(ts.view(kb.WS_H, 0)); Hout = c(ts.H_out)
    # what each layer read: its input, or with dropout the dropped copy - every element of it against the
    # oracle's mask (bit-exact zero pattern) and scaling, from the GPU's own layer outputs
    Hin0, Hin1, keep0, keep1, inv_keep = H0, H1, None, None, 1.0
    if dropout > 0:
        pf = float(np.float32(dropout))
        inv_keep = 1.0 / (1.0 - pf)
        Hin0, Hin1 = c(ts.view(kb.WS_HD, 0)), c(ts.view(kb.WS_HD, 1))
        for l, (src, got) in enumerate(((H0, Hin0), (H1, Hin1))):
            want, keep = orc.dropout(src, pf, SEED, STEP, l)
            np.testing.assert_array_equal(got != 0, (keep > 0) & (np.asarray(src) != 0))
            assert rel_err(got, want) <= 1e-6
            assert abs(keep.mean() - (1 - pf)) < 5 * np.sqrt(pf * (1 - pf) / keep.size)
            if l == 0:
                keep0 = keep
            else:
                keep1 = keep
            del want
        say("dropout masks checked (%.0f s)" % (time.time() - t0))
    rng = np.random.default_rng(123)
    errs = {}

    # ---- negatives and sub-graph: bit-exact
    np.testing.assert_array_equal(ts.neg_ent.cpu().numpy()[:, :spec.n_neg], ne)
    np.testing.assert_array_equal(ts.neg_side.cpu().numpy()[:, :spec.n_neg], ns)
    active = None
    if relw:
        active = orc.compute_graph(op, pos, ne, 2).astype(bool)
        got_active, stats = ts.cg.export()
        np.testing.assert_array_equal(got_active.astype(bool), active)
        for l in range(2):
            assert stats[l, 0] == int(active[l].sum()) and stats[l, 1] == int(deg_in[active[l]].sum())
        say("sub-graph (vertices, edges, runs) per layer:", stats.tolist())
        assert not Hout[~active[1]].any() and not H1[~active[0]].any()

    # ---- forward: sampled destination rows of both layers against the exact layer (the oracle projects
    # every neighbour on the spot: B d_in d_out multiply-adds per edge), and of the stored intermediates
    rows1 = pick_rows(rng, deg_in, 1.4e10 / (B * d0 * d), 300, None if active is None else active[0])
    rows2 = pick_rows(rng, deg_in, 1.4e10 / (B * d * d), 300, None if active is None else active[1])
    say("forward rows:", len(rows1), len(rows2), "edges:", int(deg_in[rows1].sum()), int(deg_in[rows2].sum()),
        "max deg:", int(deg_in[rows1].max()), int(deg_in[rows2].max()))
    _, want1 = orc.layer_rows(op, rows1, L[0]["V"], L[0]["a"], L[0]["W0"], L[0]["act"], Hin0)
    errs["H1 rows"] = (rel_err(H1[rows1], want1), tol_v)
    _, want2 = orc.layer_rows(op, rows2, L[1]["V"], L[1]["a"], L[1]["W0"], L[1]["act"], Hin1)
    errs["H_out rows"] = (rel_err(Hout[rows2], want2), tol_v)
    if relw:
        # run means of both layers on sampled runs into active destinations, from the GPU's own layer inputs.
        # The bf16 pipeline keeps no mean for a run of one edge (it reads the source's row of the layer input
        # in place, which is that mean): there, stored rows of z are sampled from longer runs only
        alias = bf
        for l, Hin in ((0, Hin0), (1, Hin1)):
            ok = active[l][op["seg_dst"]] & (run_len <= 2000) & ((run_len > 1) | (not alias))
            runs = rng.permutation(np.nonzero(ok)[0])[:400]
            runs = np.concatenate([runs, np.nonzero(ok & (run_len >= 256))[0][:2]]).astype(np.int64)
            zg = c(ts.view(kb.WS_Z, l)[torch.from_numpy(runs).to(ts.dev)])
            errs["z_%d runs" % (l + 1)] = (rel_err(zg, sampled.run_mean_rows(op, runs, Hin)), tol_v)
            gone = np.nonzero(~active[l][op["seg_dst"]] & ((run_len > 1) | (not alias)))[0][:50]   # outside: zero rows
            if len(gone):
                assert not c(ts.view(kb.WS_Z, l)[torch.from_numpy(gone).to(ts.dev)]).any()
        uruns, ug, zg_u = u_check
        if alias:       # single-edge runs: the operand is the source's row of the layer input
            one = run_len[uruns] == 1
            assert one.any() and not one.all()
            zg_u = zg_u.copy()
            zg_u[one] = Hin1[op["col_src"][op["seg_ptr"][uruns[one]]]]
        uw = sampled.relation_product_rows(op, uruns, lambda ids: zg_u, L[1]["a"], L[1]["V"])
        errs["u_2 runs"] = (rel_err(ug, uw), tol_v)
    else:
        trows = torch.from_numpy(rows1).to(ts.dev)
        P1 = c(ts.view(kb.WS_P, 0)[trows]).reshape(len(rows1), B, d)
        errs["P1 rows"] = (rel_err(P1, sampled.project_rows(Hin0[rows1], L[0]["V"])), tol_v)
        P2 = c(ts.view(kb.WS_P, 1)[trows]).reshape(len(rows1), B, d)
        errs["P2 rows"] = (rel_err(P2, sampled.project_rows(Hin1[rows1], L[1]["V"])), tol_v)
    say("forward checked (%.0f s)" % (time.time() - t0), errs)

    # ---- scoring: everything (fp32 in every workload)
    sl = orc.distmult_score_loss(op, Hout, params["M"], pos, ne, ns)
    errs["scores"] = (rel_err(c(ts.scores), sl["scores"]), 1e-4)
    errs["loss"] = (abs(float(ts.loss.cpu()[0]) - sl["loss"]) / sl["loss"], 1e-4)
    G2 = c(ts.dH_out)
    errs["dH_out"] = (rel_err(G2, sl["dH"]), 1e-3)
    errs["dM"] = (rel_err(c(ts.dM), sl["dM"]), 1e-3)
    del sl
    say("scoring checked (%.0f s)" % (time.time() - t0))

    # ---- backward
    srows = pick_rows(rng, deg_out, 40000, 60)
    tsrows = torch.from_numpy(srows).to(ts.dev)
    # layer 2 input gradient (dH_1) by definition from G2, and the activation backward
    dP2 = sampled.transposed_rows(ev, srows, L[1]["a"], G2)
    want = sampled.input_grad_rows(dP2, G2[srows], L[1]["V"], L[1]["W0"])
    if dropout > 0:        # chain rule through the dropped copy: the same mask and scale
        want = want * keep1[srows] * inv_keep
    dH1 = c(ts.view(kb.WS_DH, 1)[tsrows])
    errs["dH_1 rows"] = (rel_err(dH1, want), tol_g)
    G1 = c(ts.view(kb.WS_G, 0))
    np.testing.assert_array_equal(G1[srows], dH1 * (H1[srows] > 0))
    # layer 1 transposed sums from the GPU's own G1
    dP1w = sampled.transposed_rows(ev, srows, L[0]["a"], G1)
    if relw:
        # no dP in this order: the transposed per-run products dz of the last layer that produced an
        # input gradient are in the shared buffer
        lz, Gz = (0, G1) if need_dH0 else (1, G2)
        dz_w = d0 if lz == 0 else d
        zruns = np.random.default_rng(11).permutation(op["n_seg"])[:120].astype(np.int64)
        dzg = c(ts.view(kb.WS_U, lz)[:gp.n_seg * dz_w].view(gp.n_seg, dz_w)[torch.from_numpy(zruns).to(ts.dev)])
        errs["dz_%d runs" % (lz + 1)] = (rel_err(dzg, sampled.relation_product_t_rows(op, zruns, Gz, L[lz]["a"], L[lz]["V"])), tol_g)
        dP1 = dP1w
    else:
        X1 = ts.view(kb.WS_DP, 0)
        dP1 = c(X1[tsrows])[:, :B * d].reshape(len(srows), B, d)
        errs["dP_1 rows"] = (rel_err(dP1, dP1w), tol_g)
    if need_dH0:
        want = sampled.input_grad_rows(dP1, G1[srows], L[0]["V"], L[0]["W0"])
        if dropout > 0:
            want = want * keep0[srows] * inv_keep
        errs["dH0 rows"] = (rel_err(c(ts.dH0[tsrows]), want), tol_g)
    # self-loop weight gradients, whole
    errs["dW0_2"] = (rel_err(c(ts.grads[1]["dW0"]), sampled.self_weight_grad(Hin1, G2)), tol_g)
    errs["dW0_1"] = (rel_err(c(ts.grads[0]["dW0"]), sampled.self_weight_grad(Hin0, G1)), tol_g)
    say("rows and dW0 checked (%.0f s)" % (time.time() - t0))
    # basis gradients of both layers: two sampled columns each, and two random projections x^T dV_b y of
    # every basis - every element of every dV_b enters them, at the cost of one pass over the edges
    prng = np.random.default_rng(2024)
    for l, (Hin, G) in enumerate(((Hin0, G1), (Hin1, G2))):
        dV = c(ts.grads[l]["dV"]).astype(np.float64)
        di = dV.shape[1]
        for (b, col) in [(0, 0), (B - 1, d - 1)]:
            colv = sampled.transposed_column(ev, L[l]["a"], b, G[:, col])        # dP_l[:, b, col] by definition
            want = sampled.basis_weight_grad_column(Hin, colv)
            errs["dV_%d[%d][:,%d]" % (l + 1, b, col)] = (float(np.abs(dV[b][:, col] - want).max() / np.abs(dV[b]).max()), tol_g)
        for k in range(2):
            x, y = prng.standard_normal(di), prng.standard_normal(d)
            want = sampled.basis_weight_grad_projection(ev, L[l]["a"], Hin, G, x, y)
            got = np.einsum("k,bkc,c->b", x, dV, y)
            errs["dV_%d projection %d" % (l + 1, k)] = (rel_err(got, want), tol_g)
    say("dV checked (%.0f s)" % (time.time() - t0))
    # the identity sum a*da = sum V*dV = sum <pre - h W0, G> for both layers, as an extra
    for l, (pre, Hin, G) in enumerate([(H1, Hin0, G1), (Hout, Hin1, G2)]):
        q = sampled.euler_quantity(pre, Hin, L[l]["W0"], G)
        qa = float(np.sum(L[l]["a"].astype(np.float64) * c(ts.grads[l]["da"])))
        qv = float(np.sum(L[l]["V"].astype(np.float64) * c(ts.grads[l]["dV"])))
        scale = max(abs(q), 1e-30)
        errs["euler da layer %d" % (l + 1)] = (abs(qa - q) / scale, tol_g)
        errs["euler dV layer %d" % (l + 1)] = (abs(qv - q) / scale, tol_g)
    # coefficient gradients, every basis: the relations with the most edges (whose contraction ranges are
    # cut into chunks and accumulated atomically) straight from the edges, and rare ones
    cnt = np.bincount(ev.rel, minlength=2 * spec.n_relations)
    heads = np.argsort(cnt)[-2:]
    rare = np.nonzero((cnt > 0) & (cnt <= 3000))[0]
    rare = rare[np.argsort(cnt[rare])][-3:] if 2 * spec.n_relations > 8 else []
    for l, (Hin, G) in enumerate(((Hin0, G1), (Hin1, G2))):
        da = c(ts.grads[l]["da"])
        dmax = max(np.abs(da).max(), 1e-30)
        rels = list(rare) + (list(heads) if l in da_layers else [])
        for r in rels:
            v = sampled.coeff_grad_relation_edges(ev, int(r), Hin, G, L[l]["V"])
            errs["da_%d[rel %d, %d edges]" % (l + 1, r, cnt[r])] = (float(np.abs(da[r] - v).max() / max(np.abs(v).max(), 1e-3 * dmax)), tol_g)
    say("backward checked (%.0f s)" % (time.time() - t0))
    for k, v in errs.items():
        say("  %-34s %.3e (tol %.0e)" % (k, v[0], v[1]))
    bad = {k: v for k, v in errs.items() if not (v[0] <= v[1])}
    del ts
    gc.collect()
    torch.cuda.empty_cache()
    assert not bad, bad


def test_config3_full_size(world):
    """Partition 0 of 16 of the 2.9 M-vertex / 30 M-edge graph, d = 128, 2 bases, fp32; project-first order on
    the whole partition.  (Layer 1's coefficient gradient from all 59 M edges is recomputed in the next test.)"""
    run_full_size(world, 3, da_layers=(1,))


def test_config3_full_size_relation_weights_subgraph(world):
    """The launch configuration bench.py times by default: relation-weight order on the sub-graph."""
    run_full_size(world, 3, order="relation")


def test_config3_full_size_paper_setting(world):
    """The same graph with the hyper-parameters the paper trains its large graph with (Sec. 4): 128 fixed
    features -> 32-wide embeddings, 2 bases, dropout 0.2, 1 negative; bench.py --config 3 --paper-setting."""
    run_full_size(world, 3, order="relation", dropout=0.2, spec=synth.paper_large_setting())


def test_config4_full_size(world):
    """Partition 0 of 4 of the 1 M-entity / 20 M-triple / 1,000-relation graph, d = 256, 64 bases,
    bf16 messages; project-first order on the whole partition, against the exact oracle at 2e-2."""
    run_full_size(world, 4)


def test_config4_full_size_relation_weights_subgraph(world):
    """configs[4] as the bf16 relation-weight pipeline on the batch's computational sub-graph (bench.py's
    default), against the exact oracle at 2e-2."""
    run_full_size(world, 4, order="relation")


def test_config4_full_size_relation_weights_subgraph_dropout(world):
    """The benchmark's launch configuration with the large-graph setting's dropout of 0.2."""
    run_full_size(world, 4, order="relation", dropout=0.2)
