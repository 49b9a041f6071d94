#!/usr/bin/env python3
"""Benchmark: one training step (RGCN forward + in-partition negatives + DistMult/BCE +
RGCN backward) on one self-sufficient partition, on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]      (C = 4 by default; 3: the citation-shaped graph)

Prints ONE JSON line: whole-step throughput in message edges per second (inputs resident in
HBM), the roofline figures of the kernel that takes most of the step (HIP events recorded by
the library on the launch stream during the timed steps), and the CPU oracle timed on this
host as a baseline.  Data is synthetic and seeded (paper_2201_02791_amd/synth.py).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
# plain vector ALUs: 256 compute units x 4 SIMDs x 32 fp32 FMA lanes per clock x 2 flops x 2.4 GHz
PEAK_F32_VALU_TFLOPS = 256 * 4 * 32 * 2 * 2.4e9 / 1e12
# Adam's learning rate per workload.  The paper's 0.01 (Sec. 4) is kept where it trains; at configs[4]
# (64 bases, width 256: one Adam step of 0.01 on every a_rb and V_b moves each W_r entry by about four
# times its magnitude) it overshoots in three steps and then leaves every layer-1 ReLU dead, so that
# workload runs at 0.001, where the loss falls steadily.
DEFAULT_LR = {4: 1e-3}


def kernel_work(name, part, spec, dims, B, ep, n_pos, n_neg, cone=None, order="project", single_runs=0,
                n_input_rows=None, dropout=0.0):
    """Algorithmic work of ONE launch of a kernel: what the method itself must move or compute in this
    formulation, as the mean over the layers that launch it.  Returns a dict with "bytes" and / or "flops"
    (a contraction has both and the caller reports whichever ceiling takes longer at its peak), "unit"
    ("mfma" matrix cores, "alu" vector ALUs) for the flops, and "f32" when an fp32 contraction runs inside a
    bf16-message workload.  dims: [(d_in, d_out)] per layer; cone: None, or per layer the counts (active
    vertices, edges into them, runs into them, edges out of them) of the batch's computational sub-graph."""
    N, E, S = float(part.n_vert), float(part.n_edge), float(part.n_seg)
    R2 = 2.0 * part.n_relations
    L = len(dims)
    if name == "distmult":     # per scored group: h_s, h_t, M_r + one row per negative, read and accumulated
        d = dims[-1][1]
        return {"bytes": n_pos * (3.0 + n_neg) * d * 4.0 * 2.0 + n_pos * n_neg * 5.0}
    if name == "optimizer_rows":   # the entity table: a flag per vertex, 28 B per element of the rows the step reached
        nv0 = N if n_input_rows is None else float(n_input_rows)
        return {"bytes": N * 1.0 + nv0 * dims[0][0] * 28.0}
    Bg = 0 if order == "relation" else B      # relation-weight order: only the self-loop term W_0 goes through the dense GEMMs
    per_layer = []
    for l, (di, do) in enumerate(dims):
        nv, ne, ns = (N, E, S) if cone is None else (float(cone[l][0]), float(cone[l][1]), float(cone[l][2]))
        inactive = cone is not None
        w = None
        if name == "gather_fwd":   # per edge: P row + (src, rel, 1/c); per vertex: ptr (+ flag) + Self read + output write
            w = {"bytes": ne * (B * do * ep + 12.0) + N * ((5.0 if inactive else 4.0) + 4.0 * do) + nv * 4.0 * do + R2 * B * 4.0}
        elif name == "coeff_seg":  # per edge: P row + src; per run: ptr/dst/1/c + G row + B outputs
            w = {"bytes": ne * (B * do * ep + 4.0) + ns * (8.0 + 4.0 * do) + S * ((5.0 if inactive else 4.0) + 4.0 * B)}
        elif name == "gather_t":   # per edge: G row + (dst, rel, 1/c); per vertex: ptr + dP row write
            # the bf16 matrix-core form (>= 32 bases, width a multiple of 32) gathers the bf16 copy of G
            g_el = 2.0 if (ep == 2 and B >= 32 and do % 32 == 0) else 4.0
            w = {"bytes": ne * g_el * do + E * (13.0 if inactive else 12.0) + N * (4.0 + B * do * ep) + R2 * B * 4.0}
        elif name == "run_mean":   # per edge: source id + input row; per run: ptr/dst/1/c + z row written
            # single_runs: runs of one edge that the bf16 relation-weight pipeline neither reads nor writes
            # (their mean is the source's input row, read in place by the products), scaled to the sub-graph
            skip = single_runs * (ne / max(E, 1.0))
            w = {"bytes": (ne - skip) * (ep * di + 4.0) + S * 12.0 + (S - single_runs) * ep * di}
        elif name == "sum_runs":   # per run: u row + run id; per vertex: ptr + Self read + output write
            w = {"bytes": ns * (ep * do + 4.0) + N * (5.0 + 4.0 * do) + nv * 4.0 * do}
            if ep == 2 and l + 1 < len(spec.acts) and dropout == 0.0:   # it also writes the next layer's bf16 input
                w["bytes"] += N * 2.0 * do
        elif name == "sum_edges_out":  # per edge: dz row + (run id, 1/c); per vertex: ptr + Self read + output write
            if l == 0 and spec.fixed_features:
                continue               # no gradient with respect to fixed features
            eo = E if (cone is None or l == 0) else float(cone[l - 1][3])
            w = {"bytes": eo * (ep * di + 8.0) + N * (4.0 + 8.0 * di)}
        elif name in ("apply_rel", "apply_rel_t"):   # one (d_in x d_out) product per run: a row read and a row written
            if name == "apply_rel_t" and l == 0 and spec.fixed_features:
                continue
            w = {"flops": 2.0 * S * di * do, "bytes": S * (di + do) * ep + R2 * di * do * ep, "unit": "mfma"}
        elif name == "rel_outer":  # C_r = sum_runs z^T G: two rows read per run, C_r accumulated once
            w = {"flops": 2.0 * S * di * do, "bytes": S * (di + do) * ep + R2 * di * do * 4.0, "unit": "mfma"}
        elif name == "rel_weights":  # (2R x B) by (B x d_in d_out) on the vector ALUs; bf16: written in both orientations
            w = {"flops": 2.0 * R2 * B * di * do, "unit": "alu",
                 "bytes": B * di * do * 4.0 + R2 * di * do * (4.0 if ep == 4 else 2.0 * ep)}
        elif name == "basis_grad":   # the transposed product: C read once, dV written
            w = {"flops": 2.0 * R2 * B * di * do, "bytes": (R2 + B) * di * do * 4.0, "unit": "alu"}
        elif name == "coeff_contract":   # da_rb = <C_r, V_b>: C and V read once
            w = {"flops": 2.0 * R2 * di * do * B, "bytes": (R2 + B) * di * do * 4.0, "unit": "mfma", "f32": True}
        elif name == "project":    # H read, P and Self written
            w = {"flops": 2.0 * N * di * (Bg + 1) * do, "unit": "mfma",
                 "bytes": N * di * ep + N * Bg * do * ep + N * do * 4.0 + (Bg + 1) * di * do * ep}
        elif name == "weight_grad":  # H and [dP | G] read, the weight gradients accumulated
            w = {"flops": 2.0 * N * di * (Bg + 1) * do, "unit": "mfma",
                 "bytes": N * di * ep + N * (Bg + 1) * do * ep + (Bg + 1) * di * do * 4.0}
        elif name == "input_grad":   # [dP | G] read, dH written
            if l == 0 and spec.fixed_features:
                continue
            w = {"flops": 2.0 * N * di * (Bg + 1) * do, "unit": "mfma",
                 "bytes": N * (Bg + 1) * do * ep + N * di * 4.0 + (Bg + 1) * di * do * ep}
        elif name == "dropout":    # one fp32 matrix read and written; the mask is recomputed, never stored
            w = {"bytes": 8.0 * N * di}
            if not (l == 0 and spec.fixed_features):
                per_layer.append(w)    # and once more in backward, in place on the input gradient
        elif name == "act_bwd":
            if spec.acts[l] == 0:
                continue
            w = {"bytes": (12.0 + (2.0 if ep == 2 else 0.0)) * N * do}   # dH and H read, G written (bf16 messages: its bf16 copy too)
        elif name == "coeff_reduce":
            w = {"bytes": 4.0 * S * B}
        if w is not None:
            per_layer.append(w)
    if not per_layer:
        return {}
    out = dict(per_layer[0])
    for key in ("bytes", "flops"):
        if key in out:
            out[key] = sum(w[key] for w in per_layer) / len(per_layer)
    return out


def roof_of(work, avg_ms, ep):
    """Achieved rate of a kernel against the ceiling that binds: a contraction is charged to whichever of its
    two floors (flops at the matrix-core or vector-ALU peak, bytes at the HBM peak) takes longer."""
    t = avg_ms * 1e-3
    if not work or t <= 0:
        return None
    out = {}
    flop_peak = None
    if "flops" in work:
        if work.get("unit") == "alu":
            flop_peak, fb = PEAK_F32_VALU_TFLOPS, "alu"
        else:
            flop_peak, fb = (PEAK_F32_MFMA_TFLOPS if ep == 4 or work.get("f32") else PEAK_BF16_MFMA_TFLOPS), "mfma"
        out["frac_of_%s_peak" % fb] = work["flops"] / t / (flop_peak * 1e12)
    if "bytes" in work:
        out["frac_of_hbm_peak"] = work["bytes"] / t / (PEAK_HBM_GBS * 1e9)
    hbm_binds = "bytes" in work and ("flops" not in work or
                                     work["bytes"] / (PEAK_HBM_GBS * 1e9) >= work["flops"] / (flop_peak * 1e12))
    if hbm_binds:
        out.update(bound="hbm", achieved=work["bytes"] / t / 1e9, peak=PEAK_HBM_GBS, unit="GB/s")
    else:
        out.update(bound=fb, achieved=work["flops"] / t / 1e12, peak=flop_peak, unit="TFLOP/s")
    out["frac"] = out["achieved"] / out["peak"]
    return out


def measured_traffic(cfg_index, order, kernel, avg_ms):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this same benchmark (profiles/hbm_traffic.json), or None if there is no record for this workload and
    order - or if the record was taken when the kernel ran more than 15 % slower or faster than now (it
    then describes an older kernel and is not reported)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path)).get("configs[%d] %s" % (cfg_index, order), {}).get(kernel)
    if rec is None:
        return None
    was = rec.get("avg_ms")
    if was and abs(avg_ms - was) > 0.15 * was:
        return None
    return rec["bytes_per_launch"]


def cpu_baseline(spec, cfg_index):
    """The oracle as it stands, timed on this host (1 thread), on a bounded sample: the whole
    step on the same generator recipe, scaled down so that it takes roughly 10-30 s."""
    from paper_2201_02791_amd import synth
    from oracle import oracle as orc
    # oracle cost ~ 8 N B d^2 (projections, fwd+bwd, 2 layers) + 6 E B d  FMAs at roughly 5e9 FMA/s
    budget = 100e9
    per_vertex = 8.0 * spec.n_bases * spec.d * spec.d + 6.0 * 2.0 * (spec.n_triples / spec.n_entities) * spec.n_bases * spec.d
    n = int(min(spec.n_entities, max(200, budget / per_vertex)))
    scale = n / spec.n_entities
    m = max(400, int(spec.n_triples * scale))
    small = synth.scaled(spec, n_entities=n, n_triples=m, n_parts=1, part_id=0,
                         n_pos=max(16, int(spec.n_pos * scale)))
    head, rel, tail = synth.make_triples(small)
    part = orc.build_partition(head, rel, tail, small.n_entities, small.n_relations, 1, 0, small.n_hops,
                               small.neg_domain)
    params = synth.make_params(small, part["n_vert"])
    layers = [dict(V=params["V"][l], a=params["a"][l], W0=params["W0"][l], act=small.acts[l])
              for l in range(small.n_layers)]
    pos = synth.make_batch(small, part["n_core"])
    t0 = time.perf_counter()
    orc.train_step(part, layers, params["H0"], params["M"], pos, small.n_neg, small.neg_mode, 1, 0,
                   need_dH0=not small.fixed_features)
    dt = time.perf_counter() - t0
    return {"value": part["n_edge"] / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
            "host_cores": os.cpu_count(),
            "sample": "whole oracle step on the same recipe scaled to %d entities / %d triples "
                      "(%d message edges, d=%d, %d bases), %.1f s" % (n, m, part["n_edge"], small.d,
                                                                      small.n_bases, dt)}


def run_eval(args):
    """--eval: filtered link-prediction ranking ("Evaluation Metrics": MRR Eq. 5, Hits@k Eq. 6) instead of
    the training step.  all: every test triple's two queries against every entity of the workload's graph,
    known triples = the workload's training triples.  candidates: the large citation graph's setting, 1000
    given candidates per query.  Embeddings are random (no trained weights exist here): the arithmetic and
    the data movement are those of a trained model, the metric values are not."""
    import numpy as np
    import torch
    from paper_2201_02791_amd import binding as kb, synth
    kb.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    spec = synth.WORKLOADS[args.config]
    log = lambda *a: print("[bench]", *a, file=sys.stderr, flush=True)
    N, R, d = spec.n_entities, spec.n_relations, spec.d
    rng = np.random.default_rng(spec.seed + 77)
    n_test = args.eval_triples
    H = torch.from_numpy(rng.normal(0, 0.5, (N, d)).astype(np.float32)).cuda()
    M = torch.from_numpy(rng.normal(0, 1.0, (R, d)).astype(np.float32)).cuda()
    head, rel, tail = synth.make_triples(spec)
    pick = rng.permutation(len(head))[:n_test]       # test triples drawn like the graph's own
    th, tr, tt = (torch.from_numpy(np.ascontiguousarray(x[pick])).cuda() for x in (head, rel, tail))
    nq = 2 * n_test
    if args.eval == "all":
        t0 = time.time()
        filt = kb.EvalFilter(head, rel, tail, N, R)
        log("filter tables of %d known triples built in %.1f s (host sort, once per evaluation)" % (len(head), time.time() - t0))
        ws = torch.empty(kb.eval_workspace_bytes(nq, d), dtype=torch.uint8, device="cuda")
        step = lambda: kb.eval_rank_all(H, M, th, tr, tt, filt, ws)
        work_name, flops = "eval_count", 2.0 * nq * N * d
    else:
        n_cand = 1000
        fixed = torch.cat([th, tt]); rr = torch.cat([tr, tr]); ans = torch.cat([tt, th])
        cand = torch.from_numpy(rng.integers(0, N, (nq, n_cand)).astype(np.int32)).cuda()
        ws = torch.empty(kb.eval_workspace_bytes(nq, d), dtype=torch.uint8, device="cuda")
        step = lambda: kb.eval_rank_candidates(H, M, fixed, rr, ans, cand, ws)
        work_name, flops = "eval_cand", None
    del head, rel, tail
    for _ in range(args.warmup):
        hi, eq = step()
    torch.cuda.synchronize()
    kb.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        hi, eq = step()
        met = kb.eval_metrics(hi, eq, (1, 3, 10))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kb.profile_enable(False)
    prof = kb.profile_collect()
    for name, (tot, calls) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
        log("%-13s %9.3f ms/step  %4.1f launches" % (name, tot / args.steps, calls / args.steps))
    avg_ms = prof[work_name][0] / max(prof[work_name][1], 1)
    if flops is not None:        # dense contraction on the fp32 matrix cores
        roof = {"kernel": work_name, "bound": "mfma", "achieved": flops / (avg_ms * 1e-3) / 1e12,
                "peak": PEAK_F32_MFMA_TFLOPS, "unit": "TFLOP/s", "traffic": None, "avg_launch_ms": avg_ms}
    else:                        # gathers one entity row per (query, candidate)
        nbytes = nq * (1000 + 1) * (d * 4.0 + 4.0)
        roof = {"kernel": work_name, "bound": "hbm", "achieved": nbytes / (avg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "traffic": None, "avg_launch_ms": avg_ms}
    roof["frac"] = roof["achieved"] / roof["peak"]
    base = None
    if not args.no_cpu_baseline:
        from oracle import eval_oracle as evo
        Hc, Mc = H.cpu().numpy(), M.cpu().numpy()
        k = max(1, min(n_test, int(2e11 / (2.0 * N * d * 8))))      # about 10-30 s of fp64 matrix-vector products
        t0 = time.perf_counter()
        if args.eval == "all":
            evo.filtered_counts(Hc, Mc, th[:k].cpu().numpy(), tr[:k].cpu().numpy(), tt[:k].cpu().numpy())
        else:
            evo.candidate_counts(Hc, Mc, fixed[:2 * k].cpu().numpy(), rr[:2 * k].cpu().numpy(), ans[:2 * k].cpu().numpy(),
                                 cand[:2 * k].cpu().numpy())
        dtc = time.perf_counter() - t0
        base = {"value": 2 * k / dtc, "unit": "queries/s", "cores": 1, "kind": "oracle", "host_cores": os.cpu_count(),
                "sample": "%d of the %d queries (raw setting), %.1f s" % (2 * k, nq, dtc)}
    m = met.cpu().numpy()
    Hc = Mc = None
    del H, M, ws
    import gc
    gc.collect(); torch.cuda.empty_cache()
    return {"metric": "link-prediction ranking queries/s (filtered, DistMult) on 1 GPU", "value": nq / (dt / args.steps),
           "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "evaluation on configs[%d] %s" % (args.config, spec.name), "mode": args.eval,
                      "entities": N, "relations": R, "d": d, "test_triples": n_test, "queries": nq,
                      "known_triples": spec.n_triples if args.eval == "all" else 0,
                      "candidates_per_query": N - 1 if args.eval == "all" else 1000},
           "mrr_of_random_embeddings": float(m[0]), "hits_at_1_3_10": [float(x) for x in m[1:]],
           "roofline": roof, "cpu_baseline": base}


class Graphs:
    """Triples and partition of a workload, built once per process (several bench rows share a graph)."""

    def __init__(self, kb, synth, log):
        self.kb, self.synth, self.log, self.parts = kb, synth, log, {}

    def get(self, cfg):
        if cfg not in self.parts:
            spec = self.synth.WORKLOADS[cfg]
            t0 = time.time()
            head, rel, tail = self.synth.make_triples(spec)
            self.log("graph %s: %d entities, %d triples (%.1f s)" % (spec.name, spec.n_entities, len(head), time.time() - t0))
            t0 = time.time()
            part = self.kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts,
                                           spec.part_id, spec.n_hops, spec.neg_domain)
            self.log("partition %d/%d: N=%d E=%d S=%d core=%d cand=%d max_in=%d max_out=%d (%.1f s)" % (
                spec.part_id, spec.n_parts, part.n_vert, part.n_edge, part.n_seg, part.n_core, part.n_cand,
                part.max_in_degree, part.max_out_degree, time.time() - t0))
            self.parts[cfg] = part
        return self.parts[cfg]

    def drop(self, cfg):
        self.parts.pop(cfg, None)


ORDER_NAMES = {"project": "project-first", "relation": "relation-weight"}


def run_workload(graphs, cfg, order="relation", whole=False, dropout=0.0, steps=10, warmup=2, paper_setting=False,
                 optimizer=True, lr=None, calibrate=False):
    """Time `steps` training steps (Algorithm 1, one mini-batch each: negatives, sub-graph, forward, loss,
    backward, optimizer update) of one workload in one launch configuration.  Every step takes a fresh
    mini-batch, staged on the device before the timed region.  Returns the record of the run."""
    import gc
    import torch
    from paper_2201_02791_amd import binding as kb, synth
    from paper_2201_02791_amd.step import TrainStep
    log = graphs.log
    spec = synth.paper_large_setting() if paper_setting else synth.WORKLOADS[cfg]
    part = graphs.get(cfg)
    params = synth.make_params(spec, part.n_vert)
    msg = kb.MSG_BF16 if spec.msg_dtype == "bf16" else kb.MSG_F32
    lr = lr if lr is not None else DEFAULT_LR.get(cfg, 0.01)
    ts = TrainStep(part, params, spec.acts, msg, need_dH0=not spec.fixed_features, keep_scores=True,
                   cone=not whole,
                   order={"project": kb.ORDER_PROJECT_FIRST, "relation": kb.ORDER_RELATION_WEIGHTS}[order],
                   dropout=dropout)
    del params
    batches = [synth.make_batch(synth.scaled(spec, seed=spec.seed + 101 * i), part.n_core) for i in range(warmup + steps)]
    ts.set_batch(batches[0], spec.n_neg)
    staged = ts.stage_batches(batches)
    n_pos, n_neg = len(batches[0]), spec.n_neg
    log("%s, %s, %s: workspace %.2f GB" % (spec.name, ORDER_NAMES[order], "whole partition" if whole else "sub-graph",
                                           ts.ws_bytes / 1e9))
    if calibrate:     # known traffic: reads 1 GiB, writes 1 GiB
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def one_step(i):
        ts.use_batch(staged[i])
        ts.run(spec.neg_mode, 1234, i)
        if optimizer:
            ts.optimizer_step(kb.OPT_ADAM, lr)

    if optimizer:
        ts.init_optimizer(kb.OPT_ADAM)      # Adam moments allocated here, not inside a step
    losses = []
    for w in range(warmup):
        one_step(w)
        losses.append(float(ts.loss.cpu()[0]))
    torch.cuda.synchronize()
    kb.profile_enable(True)
    t0 = time.perf_counter()
    for k in range(steps):
        one_step(warmup + k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kb.profile_enable(False)
    prof = kb.profile_collect()
    losses.append(float(ts.loss.cpu()[0]))
    cone = n_input_rows = None
    if ts.cg is not None:
        cone = [tuple(int(x) for x in row) for row in ts.cg.export()[1]]
        n_input_rows = ts.cg.input_rows()[1]
        log("computational sub-graph (vertices, edges, runs, edges out) per layer, last step:", cone,
            "input rows read:", n_input_rows)

    ms_per_step = 1e3 * dt / steps
    E = part.n_edge
    single_runs = 0
    if order == "relation" and spec.msg_dtype == "bf16":
        single_runs = int((np.diff(part.export("seg_ptr")) == 1).sum())
    T = n_pos * (1 + n_neg)
    ep = 2 if spec.msg_dtype == "bf16" else 4
    dims = [(spec.d_in or spec.d, spec.d)] + [(spec.d, spec.d)] * (spec.n_layers - 1)
    kernels = {}
    if "distmult_gather" in prof:
        # the atomic-free scoring call is three steps (sort the batch's rows by entity, score, sum per entity):
        # its algorithmic bytes are those of the whole call, so the three are reported as one entry
        tot = sum(prof.pop(k)[0] for k in ("score_index", "distmult", "distmult_gather") if k in prof)
        prof["distmult"] = (tot, steps)
    if "project_self" in prof:
        # the projections of a bf16 layer with bases are two launches (the B basis products, then the self-loop
        # product): one entry, one launch pair per layer
        tot, calls = prof["project"]
        prof["project"] = (tot + prof.pop("project_self")[0], calls)
    for name, (tot_ms, calls) in prof.items():
        avg_ms = tot_ms / max(calls, 1)
        rec = {"ms_per_step": tot_ms / steps, "launches_per_step": calls / steps, "avg_ms": avg_ms}
        roof = roof_of(kernel_work(name, part, spec, dims, spec.n_bases, ep, n_pos, n_neg, cone, order, single_runs,
                                   n_input_rows, dropout), avg_ms, ep)
        if roof:
            rec.update(roof)
            if roof["frac"] > 1.0:
                # possible for a kernel whose rows repeat (hub vertices) and are served by the caches: it moves
                # fewer bytes than the algorithmic count
                rec["note"] = "above the HBM peak by algorithmic bytes: repeated rows are served by L2 / Infinity Cache"
        kernels[name] = rec
    rated = [k for k in kernels if "frac" in kernels[k]]
    dominant = max(rated, key=lambda k: kernels[k]["ms_per_step"]) if rated else None
    roof = None
    if dominant:
        kd = kernels[dominant]
        cfg_key = "%s%s" % (order, " whole" if whole else "")
        traffic = None if (paper_setting or dropout > 0) else measured_traffic(cfg, cfg_key, dominant, kd["avg_ms"])
        roof = {"kernel": dominant, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"], "traffic": traffic, "avg_launch_ms": kd["avg_ms"]}
        for key in ("frac_of_mfma_peak", "frac_of_hbm_peak", "frac_of_alu_peak"):
            if key in kd:
                roof[key] = kd[key]
    for name in sorted(kernels, key=lambda k: -kernels[k]["ms_per_step"]):
        kd = kernels[name]
        if "frac" in kd:
            log("%-14s %8.3f ms/step  %5.1f launches  %9.1f %s  (%.1f%% of the %s peak)" % (
                name, kd["ms_per_step"], kd["launches_per_step"], kd["achieved"], kd["unit"], 100 * kd["frac"], kd["bound"]))
        else:
            log("%-14s %8.3f ms/step  %5.1f launches" % (name, kd["ms_per_step"], kd["launches_per_step"]))
    out = {"metric": "train-step edges/s (RGCN fwd+bwd + DistMult) on 1 GPU",
           "value": E / (dt / steps), "unit": "edges/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16 messages, f32 accumulate" if ep == 2 else "f32",
           "data": "synthetic",
           "config": {"workload": "configs[%d] %s" % (cfg, spec.name), "n_vertices": part.n_vert,
                      "message_edges": E, "runs": part.n_seg, "d": spec.d, "d_in": spec.d_in or spec.d, "bases": spec.n_bases,
                      "relations_with_inverses": 2 * spec.n_relations, "layers": spec.n_layers,
                      "positives": n_pos, "negatives_per_positive": n_neg, "parallelism": "1 partition on 1 GPU",
                      "propagation": "whole partition" if cone is None else "batch computational sub-graph",
                      "batches": "a fresh mini-batch every step",
                      "optimizer": "adam, lr %g (inside the timed step)" % lr if optimizer else None,
                      "dropout": dropout, "order": ORDER_NAMES[order],
                      "subgraph_vertices_edgesin_runs_edgesout_per_layer": cone},
           "triples_per_s": T / (dt / steps), "loss": losses[-1], "loss_first_step": losses[0] if warmup else None,
           "roofline": roof, "kernels": kernels}
    del ts, staged
    gc.collect()
    torch.cuda.empty_cache()
    return out


def brief(rec):
    """A run's record with the ten longest kernels only: what the "also" list of the default run carries."""
    keep = ("avg_ms", "bound", "achieved", "unit", "frac", "frac_of_mfma_peak", "frac_of_hbm_peak")
    out = {"workload": rec["config"]["workload"], "order": rec["config"].get("order"),
           "propagation": rec["config"].get("propagation"), "dropout": rec["config"].get("dropout"),
           "optimizer": rec["config"].get("optimizer"), "steps": rec["steps"], "warmup": rec["warmup"],
           "ms_per_step": rec["ms_per_step"], "value": rec["value"], "unit": rec["unit"],
           "triples_per_s": rec.get("triples_per_s"), "loss": rec.get("loss"), "roofline": rec["roofline"]}
    if "kernels" in rec:
        top = sorted(rec["kernels"], key=lambda k: -rec["kernels"][k]["ms_per_step"])[:10]
        out["kernels"] = {k: {q: rec["kernels"][k][q] for q in keep if q in rec["kernels"][k]} for k in top}
    if rec["config"].get("mode"):
        out["mode"] = rec["config"]["mode"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4,
                    help="index into the workload list (0..4); default: the largest single-GPU workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--order", choices=["project", "relation"], default="relation",
                    help="order of Eq. 1-2: project-first (P = H V_b, then the neighbour sum; the order the step is "
                         "named in) or relation-weight (run means times W_r; the default, the library's product path, "
                         "same results)")
    ap.add_argument("--no-optimizer", action="store_true",
                    help="leave the optimizer step (Adam) out of the timed step")
    ap.add_argument("--lr", type=float, default=None, help="Adam's learning rate (default 0.01; 0.001 at configs[4])")
    ap.add_argument("--whole-partition", action="store_true",
                    help="propagate every vertex of the partition instead of the batch's computational sub-graph")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate on every layer's input (the paper's large-graph setting uses 0.2); "
                         "default 0: the benchmark's workload is quoted without it")
    ap.add_argument("--paper-setting", action="store_true",
                    help="with --config 3: the paper's large-graph hyper-parameters (128 features -> 32, 2 bases, "
                         "1 negative; add --dropout 0.2)")
    ap.add_argument("--eval", choices=["all", "candidates"], default=None,
                    help="time the link-prediction evaluation (filtered ranks, MRR, Hits@k) instead of the training step")
    ap.add_argument("--eval-triples", type=int, default=10000, help="test triples of --eval (two queries each)")
    ap.add_argument("--no-also", action="store_true",
                    help="default run only: skip the extra rows (configs[3], the named order, evaluation) that follow the headline")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one partition per GPU, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.eval:
        print(json.dumps(run_eval(args)))
        return

    import torch
    from paper_2201_02791_amd import binding as kb, synth
    kb.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    log = lambda *a: print("[bench]", *a, file=sys.stderr, flush=True)
    graphs = Graphs(kb, synth, log)
    assert not args.paper_setting or args.config == 3, "--paper-setting is the large citation graph's (config 3)"

    out = run_workload(graphs, args.config, args.order, args.whole_partition, args.dropout, args.steps, args.warmup,
                       args.paper_setting, not args.no_optimizer, args.lr, args.calibrate)
    # the default run (no workload flags) also carries, after the headline: the order the step is named in at
    # the same workload, configs[3] in both orders and with the paper's hyper-parameters, and the evaluation
    plain = (args.config == 4 and args.order == "relation" and not args.whole_partition and args.dropout == 0.0 and
             not args.no_optimizer and args.lr is None and not args.calibrate)
    if plain and not args.no_also:
        also = []
        t_also = time.time()
        log("--- also: configs[4] in the project-first order on the whole partition")
        also.append(brief(run_workload(graphs, 4, "project", True, 0.0, 2, 1)))
        ev = argparse.Namespace(config=4, eval="all", eval_triples=10000, steps=3, warmup=1, no_cpu_baseline=True)
        log("--- also: evaluation against all entities, configs[4]'s graph")
        also.append(brief(run_eval(ev)))
        graphs.drop(4)
        log("--- also: configs[3], relation-weight order on the sub-graph")
        also.append(brief(run_workload(graphs, 3, "relation", False, 0.0, 10, 2)))
        log("--- also: configs[3], project-first order on the whole partition")
        also.append(brief(run_workload(graphs, 3, "project", True, 0.0, 5, 1)))
        log("--- also: configs[3] with the paper's large-graph hyper-parameters (128 -> 32, 2 bases, dropout 0.2)")
        also.append(brief(run_workload(graphs, 3, "relation", False, 0.2, 10, 2, paper_setting=True)))
        ev = argparse.Namespace(config=3, eval="candidates", eval_triples=10000, steps=5, warmup=1, no_cpu_baseline=True)
        log("--- also: evaluation against 1000 candidates per query, configs[3]'s graph")
        also.append(brief(run_eval(ev)))
        graphs.drop(3)
        log("also-list took %.0f s" % (time.time() - t_also))
        out["also"] = also

    base = None
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        base = cpu_baseline(synth.paper_large_setting() if args.paper_setting else synth.WORKLOADS[args.config], args.config)
    out["cpu_baseline"] = base
    kernels = out.pop("kernels")
    out["kernels"] = kernels
    print(json.dumps(out))


if __name__ == "__main__":
    main()
