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


def kernel_work(name, part, spec, d, B, ep, n_pos, n_neg, cone=None, spec_order="project", single_runs=0):
    """Algorithmic bytes / flops of ONE launch of a kernel (what the method itself must move
    or compute in this formulation).  Returns (bound, work); the grouped contractions return
    ("mfma", flops, bytes) and the caller reports whichever ceiling binds.  cone: None, or the per-layer counts
    (active vertices, edges into them, runs into them) of the batch's computational sub-graph;
    the figure is then the mean over the layers' launches."""
    N, E, S = part.n_vert, part.n_edge, part.n_seg
    R2 = 2 * part.n_relations
    gemm_flops = 2.0 * N * d * (B + 1) * d
    if cone is not None and name in ("gather_fwd", "coeff_seg", "gather_t"):
        tot = 0.0
        for nv, ne, ns, _ in cone:
            if name == "gather_fwd":   # inactive rows: flag + ptr read, zero row written
                tot += ne * (B * d * ep + 12.0) + N * (5.0 + 4.0 * d) + nv * 4.0 * d + R2 * B * 4.0
            elif name == "coeff_seg":  # inactive runs: dst + flag read, B zeros written
                tot += ne * (B * d * ep + 4.0) + ns * (8.0 + 4.0 * d) + S * (5.0 + 4.0 * B)
            else:                      # every edge's metadata and flag, G rows of active destinations only
                tot += ne * 4.0 * d + E * 13.0 + N * (4.0 + B * d * ep) + R2 * B * 4.0
        return "hbm", tot / len(cone)
    if name == "gather_fwd":   # per edge: P row + (src, rel, 1/c); per vertex: ptr + Self read + output write
        return "hbm", E * (B * d * ep + 12.0) + N * (4.0 + 8.0 * d) + R2 * B * 4.0
    if name == "coeff_seg":    # per edge: P row + src; per run: ptr/dst/1/c + G row + B outputs
        return "hbm", E * (B * d * ep + 4.0) + S * (12.0 + 4.0 * d + 4.0 * B)
    if name == "gather_t":     # per edge: G row + (dst, rel, 1/c); per vertex: ptr + dP row write
        return "hbm", E * (4.0 * d + 12.0) + N * (4.0 + B * d * ep) + R2 * B * 4.0
    if name == "distmult":     # per scored group: h_s, h_t, M_r + one row per negative, read and atomically updated
        return "hbm", n_pos * (3.0 + n_neg) * d * 4.0 * 2.0 + n_pos * n_neg * 5.0
    ne_mean = E if cone is None else sum(c[1] for c in cone) / len(cone)
    ns_mean = S if cone is None else sum(c[2] for c in cone) / len(cone)
    nv_mean = N if cone is None else sum(c[0] for c in cone) / len(cone)
    if name == "run_mean":     # per edge: source id + input row; per run: ptr/dst/1/c + z row written
        # single_runs: runs of one edge that the bf16 relation-weight pipeline neither reads nor writes
        # (their mean is the source's input row, read in place by the products), scaled to the sub-graph
        skip = single_runs * (ne_mean / max(E, 1))
        return "hbm", (ne_mean - skip) * (ep * d + 4.0) + S * 12.0 + (S - single_runs) * ep * d
    if name == "aggregate":    # per run: z row + (run id, relation); per vertex: ptr + y row written
        return "hbm", ns_mean * (ep * d + 8.0) + N * 4.0 + nv_mean * B * d * ep + R2 * B * 4.0
    if name == "sum_runs":     # per run: u row + run id; per vertex: ptr + Self read + output write
        return "hbm", ns_mean * (ep * d + 4.0) + N * (5.0 + 4.0 * d) + nv_mean * 4.0 * d
    if name == "sum_edges_out":  # per edge: dz row + (run id, 1/c); per vertex: ptr + Self read + output write
        # rows outside the previous layer's active set are skipped (zero rows written); the first
        # layer's input gradient, when wanted, covers every vertex
        eo = E if cone is None else (sum(c[3] for c in cone[:-1]) + (0 if spec.fixed_features else E)) / max(
            len(cone) - (1 if spec.fixed_features else 0), 1)
        return "hbm", eo * (ep * d + 8.0) + N * (4.0 + 8.0 * d)
    if name in ("apply_rel", "apply_rel_t"):    # one (d x d) product per run: a row read and a row written per run
        return "mfma", 2.0 * S * d * d, S * 2.0 * d * ep + R2 * d * d * ep
    if name == "rel_weights" or name == "basis_grad":
        return "alu", 2.0 * R2 * B * d * d
    if name == "optimizer":    # dense tensors: p, g, m, v read, p, m, v written; small here, no figure given
        return "hbm", 0.0
    if name == "optimizer_rows":   # the entity table: gradient row read for every vertex, 28 B per touched element
        return "hbm", N * d * 4.0 + nv_mean * d * 24.0
    if name == "combine":
        return "mfma", gemm_flops
    if name == "rel_outer":    # C_r = sum_runs z^T G: 2 S d^2 flops; two rows read per run, C_r accumulated once
        return "mfma", 2.0 * S * d * d, S * 2.0 * d * ep + R2 * d * d * 4.0
    if name == "coeff_contract":
        return "mfma", 2.0 * R2 * d * d * B
    if spec_order == "relation":      # only the self-loop term W_0 goes through these
        gemm_flops = 2.0 * N * d * d
    if name == "project":
        return "mfma", gemm_flops
    if name == "weight_grad":
        return "mfma", gemm_flops
    if name == "input_grad":
        return "mfma", gemm_flops
    if name == "dropout":      # one fp32 matrix read and written; the mask is recomputed, never stored
        return "hbm", 8.0 * N * d
    if name == "act_bwd":
        return "hbm", 12.0 * N * d
    if name == "coeff_reduce":
        return "hbm", 4.0 * S * B
    return "hbm", 0.0


def measured_traffic(cfg_index, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this same benchmark (profiles/hbm_traffic.json), or None if not recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path)).get("configs[%d]" % cfg_index, {}).get(kernel)
    return None if rec is None else rec["bytes_per_launch"]


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
    out = {"metric": "link-prediction ranking queries/s (filtered, DistMult) on 1 GPU", "value": nq / (dt / args.steps),
           "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "evaluation on configs[%d] %s" % (args.config, spec.name), "mode": args.eval,
                      "entities": N, "relations": R, "d": d, "test_triples": n_test, "queries": nq,
                      "known_triples": spec.n_triples if args.eval == "all" else 0,
                      "candidates_per_query": N - 1 if args.eval == "all" else 1000},
           "mrr_of_random_embeddings": float(m[0]), "hits_at_1_3_10": [float(x) for x in m[1:]],
           "roofline": roof, "cpu_baseline": base}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4,
                    help="index into the workload list (0..4); default: the largest single-GPU workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--order", choices=["project", "aggregate", "relation"], default="relation",
                    help="order of Eq. 1-2: project-first (P = H V_b, then the neighbour sum), aggregate-first "
                         "(run means, per-basis sums, one contraction) or relation-weight (run means times W_r)")
    ap.add_argument("--no-optimizer", action="store_true",
                    help="leave the optimizer step (Adam, lr 0.01) out of the timed step")
    ap.add_argument("--whole-partition", action="store_true",
                    help="propagate every vertex of the partition instead of the batch's computational sub-graph")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate on every layer's input (the paper's large-graph setting uses 0.2); "
                         "default 0: the benchmark's workload is quoted without it")
    ap.add_argument("--eval", choices=["all", "candidates"], default=None,
                    help="time the link-prediction evaluation (filtered ranks, MRR, Hits@k) instead of the training step")
    ap.add_argument("--eval-triples", type=int, default=10000, help="test triples of --eval (two queries each)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one partition per GPU, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.eval:
        run_eval(args)
        return

    import torch
    from paper_2201_02791_amd import binding as kb, synth
    from paper_2201_02791_amd.step import TrainStep
    kb.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    spec = synth.WORKLOADS[args.config]
    log = lambda *a: print("[bench]", *a, file=sys.stderr, flush=True)

    t0 = time.time()
    head, rel, tail = synth.make_triples(spec)
    log("graph %s: %d entities, %d triples (%.1f s)" % (spec.name, spec.n_entities, len(head), time.time() - t0))
    t0 = time.time()
    part = kb.build_partition(head, rel, tail, spec.n_entities, spec.n_relations, spec.n_parts, spec.part_id,
                              spec.n_hops, spec.neg_domain)
    log("partition %d/%d: N=%d E=%d S=%d core=%d cand=%d max_in=%d max_out=%d (%.1f s)" % (
        spec.part_id, spec.n_parts, part.n_vert, part.n_edge, part.n_seg, part.n_core, part.n_cand,
        part.max_in_degree, part.max_out_degree, time.time() - t0))
    del head, rel, tail
    params = synth.make_params(spec, part.n_vert)
    pos = synth.make_batch(spec, part.n_core)
    msg = kb.MSG_BF16 if spec.msg_dtype == "bf16" else kb.MSG_F32
    ts = TrainStep(part, params, spec.acts, msg, need_dH0=not spec.fixed_features, keep_scores=True,
                   cone=not args.whole_partition,
                   order={"project": kb.ORDER_PROJECT_FIRST, "aggregate": kb.ORDER_AGGREGATE_FIRST,
                          "relation": kb.ORDER_RELATION_WEIGHTS}[args.order], dropout=args.dropout)
    ts.set_batch(pos, spec.n_neg)
    log("workspace %.2f GB" % (ts.ws_bytes / 1e9))

    if args.calibrate:     # known traffic: reads 1 GiB, writes 1 GiB
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    def one_step(i):          # Algorithm 1, one mini-batch: negatives, sub-graph, forward, loss, backward, update
        ts.run(spec.neg_mode, 1234, i)
        if not args.no_optimizer:
            ts.optimizer_step(kb.OPT_ADAM, 0.01)

    if not args.no_optimizer:
        ts.init_optimizer(kb.OPT_ADAM)      # Adam moments allocated here, not inside a step
    for w in range(args.warmup):
        one_step(w)
    torch.cuda.synchronize()
    kb.profile_enable(True)
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(args.warmup + k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kb.profile_enable(False)
    prof = kb.profile_collect()
    loss = float(ts.loss.cpu()[0])
    cone = None
    if ts.cg is not None:
        cone = [tuple(int(x) for x in row) for row in ts.cg.export()[1]]
        log("computational sub-graph (vertices, edges, runs) per layer:", cone)

    ms_per_step = 1e3 * dt / args.steps
    E = part.n_edge
    single_runs = 0
    if args.order == "relation" and spec.msg_dtype == "bf16":
        import numpy as np
        single_runs = int((np.diff(part.export("seg_ptr")) == 1).sum())
    n_pos, n_neg = len(pos), spec.n_neg
    T = n_pos * (1 + n_neg)
    ep = 2 if spec.msg_dtype == "bf16" else 4
    kernels = {}
    for name, (tot_ms, calls) in prof.items():
        kw = kernel_work(name, part, spec, spec.d, spec.n_bases, ep, n_pos, n_neg, cone, args.order, single_runs)
        bound, work = kw[0], kw[1]
        avg_ms = tot_ms / max(calls, 1)
        mfma_frac = None
        if len(kw) == 3:
            # a contraction with a byte figure: the roofline that binds is the one that takes longer at its peak
            # (flops / matrix-core peak against bytes / HBM peak), i.e. HBM below the ridge intensity
            peak_t = (PEAK_BF16_MFMA_TFLOPS if ep == 2 else PEAK_F32_MFMA_TFLOPS) * 1e12
            mfma_frac = kw[1] / (avg_ms * 1e-3) / peak_t
            if kw[2] / (PEAK_HBM_GBS * 1e9) > kw[1] / peak_t:
                bound, work = "hbm", kw[2]
        if bound == "hbm":
            ach, peak, unit = work / (avg_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        elif bound == "alu":
            ach, peak, unit = work / (avg_ms * 1e-3) / 1e12, PEAK_F32_MFMA_TFLOPS, "TFLOP/s"
        else:
            peak = PEAK_BF16_MFMA_TFLOPS if ep == 2 else PEAK_F32_MFMA_TFLOPS
            ach, unit = work / (avg_ms * 1e-3) / 1e12, "TFLOP/s"
        kernels[name] = {"ms_per_step": tot_ms / args.steps, "launches_per_step": calls / args.steps,
                         "avg_ms": avg_ms, "bound": bound, "achieved": ach, "peak": peak, "unit": unit,
                         "frac": ach / peak if peak else None}
        if mfma_frac is not None:
            kernels[name]["frac_of_mfma_peak"] = mfma_frac
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"]) if kernels else None
    roof = None
    if dominant:
        kd = kernels[dominant]
        traffic = measured_traffic(args.config, dominant)
        roof = {"kernel": dominant, "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"], "traffic": traffic, "avg_launch_ms": kd["avg_ms"]}
        if "frac_of_mfma_peak" in kd:
            roof["frac_of_mfma_peak"] = kd["frac_of_mfma_peak"]
        if traffic and kd["bound"] != "hbm":
            # a contraction under the matrix cores' ridge: its measured traffic at the HBM peak, for comparison
            roof["hbm_floor_ms"] = traffic / (PEAK_HBM_GBS * 1e9) * 1e3
            roof["frac_of_hbm_floor"] = roof["hbm_floor_ms"] / kd["avg_ms"]
    for name in sorted(kernels, key=lambda k: -kernels[k]["ms_per_step"]):
        kd = kernels[name]
        log("%-13s %8.3f ms/step  %5.1f launches  %9.1f %s  (%.1f%% of peak)" % (
            name, kd["ms_per_step"], kd["launches_per_step"], kd["achieved"], kd["unit"], 100 * kd["frac"]))

    base = None
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        base = cpu_baseline(spec, args.config)

    out = {"metric": "train-step edges/s (RGCN fwd+bwd + DistMult) on 1 GPU",
           "value": E / (dt / args.steps), "unit": "edges/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16 messages, f32 accumulate" if ep == 2 else "f32",
           "data": "synthetic",
           "config": {"workload": "configs[%d] %s" % (args.config, spec.name), "n_vertices": part.n_vert,
                      "message_edges": E, "runs": part.n_seg, "d": spec.d, "bases": spec.n_bases,
                      "relations_with_inverses": 2 * spec.n_relations, "layers": spec.n_layers,
                      "positives": n_pos, "negatives_per_positive": n_neg, "parallelism": "1 partition on 1 GPU",
                      "propagation": "whole partition" if cone is None else "batch computational sub-graph",
                      "optimizer": None if args.no_optimizer else "adam, lr 0.01 (inside the timed step)",
                      "dropout": args.dropout,
                      "order": {"project": "project-first", "aggregate": "aggregate-first", "relation": "relation-weight"}[args.order],
                      "subgraph_vertices_edgesin_runs_edgesout_per_layer": cone},
           "triples_per_s": T / (dt / args.steps), "loss": loss,
           "roofline": roof, "cpu_baseline": base, "kernels": kernels}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
