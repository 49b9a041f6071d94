"""Helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare."""
import numpy as np

from paper_2201_02791_amd import synth

SEED, STEP = 0x5EEDC0DE12345, 3


def rel_err(x, y):
    """Per-tensor relative error: max|x - y| / max|y| (y is the oracle)."""
    x = np.asarray(x, np.float64); y = np.asarray(y, np.float64)
    if y.size == 0:
        return 0.0
    scale = max(np.abs(y).max(), 1e-30)
    return float(np.abs(x - y).max() / scale)


def layers_of(params, acts):
    return [dict(V=params["V"][l], a=params["a"][l], W0=params["W0"][l], act=acts[l])
            for l in range(len(acts))]


def gpu_step(spec, head, rel, tail, params=None, pos=None, need_dH0=True, cone=False, order=0, dropout=0.0,
             score_index=True):
    """Build the partition and run one step on the GPU. Returns (part, step object, params, pos)."""
    from paper_2201_02791_amd import binding as kb
    from paper_2201_02791_amd.step import TrainStep
    import torch
    part = kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts,
                              spec.part_id, spec.n_hops, spec.neg_domain)
    if params is None:
        params = synth.make_params(spec, part.n_vert)
    if pos is None:
        pos = synth.make_batch(spec, part.n_core)
    msg = kb.MSG_BF16 if spec.msg_dtype == "bf16" else kb.MSG_F32
    ts = TrainStep(part, params, spec.acts, msg, need_dH0=need_dH0, cone=cone, order=order, dropout=dropout,
                   score_index=score_index)
    ts.set_batch(pos, spec.n_neg)
    ts.run(spec.neg_mode, SEED, STEP)
    torch.cuda.synchronize()
    return part, ts, params, pos


def oracle_step(orc, spec, head, rel, tail, params, pos, need_dH0=True, dropout=0.0):
    """The oracle's whole step in exact (double) arithmetic, whatever the workload's message type:
    bf16-message runs are compared with it under their wider tolerance."""
    part = orc.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts,
                               spec.part_id, spec.n_hops, spec.neg_domain)
    res = orc.train_step(part, layers_of(params, spec.acts), params["H0"], params["M"], pos,
                         spec.n_neg, spec.neg_mode, SEED, STEP, need_dH0,
                         dropout=float(np.float32(dropout)))      # the rate as the library's float field holds it
    return part, res


PART_ARRAYS = ["vert_gid", "core_eid", "core_h", "core_r", "core_t", "seg_ptr", "seg_rel", "seg_dst",
               "inv_c", "col_src", "edge_id", "cand"]


def assert_partition_equal(gpart, opart):
    for k in ("n_vert", "n_edge", "n_seg", "n_core", "n_cand"):
        assert getattr(gpart, k) == opart[k], k
    for name in PART_ARRAYS:
        got = gpart.export(name)
        want = opart[name]
        assert got.dtype == want.dtype, name
        if name == "inv_c":       # compared as bit patterns
            np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32), err_msg=name)
        else:
            np.testing.assert_array_equal(got, want, err_msg=name)


def elementwise_err(x, y):
    """max over elements of |x - y| / (|y| + rms(y)): a relative error per element with an absolute floor of
    the tensor's own rms, so that small entries count too (the per-tensor figure divides by max|y|)."""
    x = np.asarray(x, np.float64); y = np.asarray(y, np.float64)
    if y.size == 0:
        return 0.0
    rms = max(float(np.sqrt(np.mean(y * y))), 1e-30)
    return float((np.abs(x - y) / (np.abs(y) + rms)).max())


def assert_step_close(ts, res, tol_val, tol_grad, need_dH0=True, batch_rows=None):
    """Compare every output of a GPU step with the oracle's.  batch_rows: the step propagated only
    the batch's computational sub-graph, so H_out is compared on these rows and must be exactly
    zero on all others.  Beside the per-tensor relative errors (max|x - y| / max|y|), fp32 runs hold
    scores, the embedding gradient and the basis gradients element by element to 4x the tolerance
    relative to |y| + rms(y)."""
    c = lambda t: t.detach().cpu().numpy()
    errs = {}
    np.testing.assert_array_equal(c(ts.neg_ent)[:, :ts.n_neg], res["neg_ent"])
    np.testing.assert_array_equal(c(ts.neg_side)[:, :ts.n_neg], res["neg_side"])
    if batch_rows is None:
        errs["H_out"] = (rel_err(c(ts.H_out), res["Hs"][-1]), tol_val)
    else:
        rows = np.unique(batch_rows)
        h = c(ts.H_out)
        scale = max(np.abs(res["Hs"][-1]).max(), 1e-30)
        errs["H_out"] = (float(np.abs(h[rows] - res["Hs"][-1][rows]).max() / scale) if len(rows) else 0.0, tol_val)
        mask = np.ones(h.shape[0], bool); mask[rows] = False
        assert not h[mask].any(), "rows outside the batch must be zero"
    errs["scores"] = (rel_err(c(ts.scores), res["scores"]), tol_val)
    errs["loss"] = (abs(float(c(ts.loss)[0]) - res["loss"]) / abs(res["loss"]), tol_val)
    errs["dH_out"] = (rel_err(c(ts.dH_out), res["dH_out"]), tol_grad)
    errs["dM"] = (rel_err(c(ts.dM), res["dM"]), tol_grad)
    for l, g in enumerate(ts.grads):
        for k in ("dV", "da", "dW0"):
            errs["%s%d" % (k, l)] = (rel_err(c(g[k]), res["grads"][l][k]), tol_grad)
    if need_dH0:
        errs["dH0"] = (rel_err(c(ts.dH0), res["dH0"]), tol_grad)
    if tol_grad <= 1e-3:     # fp32 runs (a bf16 rounding of a large term is many times a small element)
        errs["scores (per element)"] = (elementwise_err(c(ts.scores), res["scores"]), 4 * tol_val)
        errs["dH_out (per element)"] = (elementwise_err(c(ts.dH_out), res["dH_out"]), 4 * tol_grad)
        for l, g in enumerate(ts.grads):
            errs["dV%d (per element)" % l] = (elementwise_err(c(g["dV"]), res["grads"][l]["dV"]), 4 * tol_grad)
    bad = {k: v for k, v in errs.items() if not (v[0] <= v[1])}
    assert not bad, "relative errors above tolerance: %s (all: %s)" % (bad, errs)
    return errs


# Unit roundoff of the arithmetic a pipeline sums in / stores messages in.
U_BF16, U_F32 = 2.0 ** -8, 2.0 ** -24


def mask_band(bf16):
    """Width of the band, relative to sum|terms| of a pre-activation, inside which its sign is not
    decided by the method but by rounding.  bf16 pipelines round at most four times on the way to a
    pre-activation (layer input, run mean or per-basis sum, weight, stored message or product), each by
    at most 2^-8 of the term: 4 * 2^-8.  fp32 pipelines only differ from the fp64 sums by summation
    order: an n-term fp32 sum is off by at most about sqrt(n) 2^-24 of sum|terms| in the random-walk
    model, n <= 4096 terms per element here: 64 * 2^-24."""
    return 4.0 * U_BF16 if bf16 else 64.0 * U_F32


def align_mask_decisions(orc, ts, opart, res, params, acts, need_dH0, bf16, rows=None, max_frac=None):
    """A ReLU mask is an integer decision taken from a floating-point value, and a pre-activation whose
    magnitude is below the rounding error of its own sum has no decided sign: the kernel's fp32 / bf16
    sums and the oracle's fp64 sums may put it on different sides of zero, and each such element moves
    the layer's gradients by a whole term.  The decision is then taken in the kernel's precision:

      * the oracle computes, from its own inputs, the bound  band * sum|terms|  for every pre-activation
        (the layer evaluated on absolute values of input and weights gives sum|terms| exactly);
      * every element where the kernel's mask differs from the oracle's must lie inside that bound
        (asserted - a sign difference anywhere else is an error), and they must be few (max_frac);
      * for those elements only, the oracle's backward pass is recomputed with the kernel's decision.

    Everything else - values, the other decisions, all arithmetic - stays the oracle's own.
    Returns (number of adopted decisions, res with updated gradients).
    rows: boolean [n_layers][N] of the rows that were propagated (None = all)."""
    from paper_2201_02791_amd import binding as kb
    band = mask_band(bf16)
    if max_frac is None:
        max_frac = 2e-2 if bf16 else 2e-5
    pres = [p.copy() for p in res["pres"]]
    n_flip = 0
    layers = layers_of(params, acts)
    for l, act in enumerate(acts):
        if act != 1:
            continue
        hg = ts.view(kb.WS_H, l).cpu().numpy()
        flip = (hg > 0) != (pres[l] > 0)
        if rows is not None:
            flip &= rows[l].astype(bool)[:, None]
        if not flip.any():
            continue
        lay = layers[l]
        abs_pre, _ = orc.layer_forward(opart, np.abs(lay["V"]), np.abs(lay["a"]), np.abs(lay["W0"]), 0,
                                       np.abs(res["Hs"][l]))
        worst = float((np.abs(pres[l][flip]) / abs_pre[flip]).max())
        assert worst <= band, "layer %d: a mask differs at |pre| = %.3g of sum|terms| (band %.3g)" % (l, worst, band)
        n_here = int(flip.sum())
        n_rows = hg.shape[0] if rows is None else int(rows[l].astype(bool).sum())
        assert n_here <= max(8, max_frac * n_rows * hg.shape[1]), \
            "layer %d: %d of %d mask decisions differ" % (l, n_here, n_rows * hg.shape[1])
        n_flip += n_here
        tiny = np.finfo(np.float64).tiny
        pres[l][flip] = np.where(hg[flip] > 0, tiny, -tiny)
    if n_flip == 0:
        return 0, res
    grads, dH0 = orc.rgcn_backward(opart, layers, res["Hs"], pres, res["dH_out"], need_dH0,
                                   res.get("drop"), res.get("masks"))
    out = dict(res); out["grads"] = grads; out["dH0"] = dH0
    return n_flip, out
