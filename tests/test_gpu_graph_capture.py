"""The calls of a step only launch kernels on the caller's stream (no allocation, no host
synchronisation, no memset nodes), so a step can be captured into a HIP graph and replayed.
Per-step scalars (sampler step, dropout step) are launch arguments: a replay repeats the
captured step number."""
import sys

import numpy as np
import pytest

from paper_2201_02791_amd import synth
from gpu_util import SEED, STEP, gpu_step, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print("[gpu-case]", *a, file=sys.stderr, flush=True)


@pytest.mark.parametrize("order,bf16,cone,d", [(0, False, False, 64), (2, False, True, 64), (2, True, True, 64),
                                               (0, True, False, 64), (2, True, True, 128), (0, True, False, 128)],
                         ids=["project_first_f32", "relation_weights_f32_subgraph", "relation_weights_bf16_subgraph",
                              "project_first_bf16", "relation_weights_bf16_subgraph_d128", "project_first_bf16_d128"])
def test_step_replays_from_a_hip_graph(order, bf16, cone, d):
    import torch
    say("graph capture, order", order, "bf16", bf16, "sub-graph", cone, "d", d)
    spec = synth.scaled(synth.WORKLOADS[4 if bf16 else 0], name="graph", seed=31, n_entities=3000, n_relations=12,
                        n_triples=20000, d=d, n_bases=4, n_pos=300, n_neg=4, neg_mode=1, n_parts=2, part_id=0,
                        acts=[1, 0], feature_std=0.5)
    head, rel, tail = synth.make_triples(spec)
    gp, ts, params, pos = gpu_step(spec, head, rel, tail, order=order, cone=cone)     # eager step
    torch.cuda.synchronize()
    names = ["H_out", "scores", "loss", "dH_out", "dM", "dH0", "neg_ent", "neg_side"]
    outs = {k: getattr(ts, k) for k in names}
    for l, g in enumerate(ts.grads):
        for k in ("dV", "da", "dW0"):
            outs["%s%d" % (k, l)] = g[k]
    eager = {k: v.clone() for k, v in outs.items()}

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ts.run(spec.neg_mode, SEED, STEP)
    for rep in range(3):
        for v in outs.values():          # the program's own eager work between replays: scribble over every output
            v.fill_(3)
        ts.workspace.fill_(0x5a)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            want, got = eager[k].cpu().numpy(), v.cpu().numpy()
            if k in ("neg_ent", "neg_side", "H_out", "scores"):      # integers; the forward pass is bit-reproducible
                np.testing.assert_array_equal(got, want, err_msg="%s, replay %d" % (k, rep))
            else:
                # sums accumulated with fp32 atomics differ in their last bits from run to run; in a bf16 pipeline
                # such a bit can move a rounding of the upstream gradient, one bf16 unit of one element
                tol = 1e-3 if bf16 else 1e-5
                assert rel_err(got.astype(np.float64), want.astype(np.float64)) <= tol, (k, rep)
