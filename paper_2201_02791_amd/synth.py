"""Seeded synthetic inputs: graphs, model parameters and edge mini-batches.

This module holds no arithmetic of the method itself (no message passing, no
scoring, no sampling of negatives).  It only draws random inputs with the
shapes and degree / relation statistics of the workloads the paper trains on
(Table 1: a 14,541-entity / 237-relation / 272,115-triple knowledge graph and
a 2.9 M-vertex / 30 M-edge single-relation citation graph with 128 features),
plus a tiny case and a larger many-relation stand-in.  The same arrays are
handed to the CPU oracle and to the GPU library.

Everything is NumPy ``default_rng(seed)``; integer outputs are int32, floating
point outputs are float32 (what the GPU path stores).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np


@dataclass
class WorkloadSpec:
    """Shape of one workload (one entry of the benchmark's config list)."""

    name: str
    seed: int
    n_entities: int
    n_relations: int          # R, before inverses are added
    n_triples: int
    head_dist: str            # "uniform" | "powerlaw"
    head_exponent: float      # tail exponent of the out-degree law (powerlaw only)
    head_cap: float           # weight cap (powerlaw only)
    tail_dist: str            # "uniform" | "powerlaw"
    tail_exponent: float
    tail_cap: float
    rel_zipf: float           # P(k) ~ (k+1)^-rel_zipf over R relations; 0 -> single relation
    n_parts: int
    part_id: int
    n_hops: int
    d: int
    n_bases: int
    n_layers: int
    msg_dtype: str            # "f32" | "bf16"
    feature_std: float        # std of the layer-1 input rows
    fixed_features: bool      # True: layer-1 input is a fixed feature matrix (no dH0)
    n_pos: int
    n_neg: int
    neg_mode: int             # 0 tail only, 1 head-or-tail with p = 0.5
    neg_domain: int = 0       # 0 endpoints of core edges, 1 all partition vertices
    acts: List[int] = field(default_factory=lambda: [1, 0])   # ReLU then identity
    d_in: Optional[int] = None   # width of the layer-1 input when it differs from d (fixed features)


def _w(name, seed, n, r, m, hd, he, hc, td, te, tc, rz, P, pid, d, B, dt, fstd, fixed,
       npos, nneg, mode):
    return WorkloadSpec(name=name, seed=seed, n_entities=n, n_relations=r, n_triples=m,
                        head_dist=hd, head_exponent=he, head_cap=hc,
                        tail_dist=td, tail_exponent=te, tail_cap=tc, rel_zipf=rz,
                        n_parts=P, part_id=pid, n_hops=2, d=d, n_bases=B, n_layers=2,
                        msg_dtype=dt, feature_std=fstd, fixed_features=fixed,
                        n_pos=npos, n_neg=nneg, neg_mode=mode)


#: The five benchmark workloads, index = config number.  (PAPER_LARGE below is a sixth, outside the list.)
WORKLOADS: List[WorkloadSpec] = [
    _w("tiny-kg", 0, 1_000, 10, 5_000, "uniform", 0, 0, "uniform", 0, 0, 1.1,
       1, 0, 32, 4, "f32", 0.1, False, 1_024, 1, 0),
    _w("mid-kg", 1, 14_541, 237, 272_115, "powerlaw", 2.1, 1e3, "uniform", 0, 0, 1.0,
       1, 0, 200, 10, "f32", 0.1, False, 30_000, 10, 1),
    _w("mid-kg-part0of8", 1, 14_541, 237, 272_115, "powerlaw", 2.1, 1e3, "uniform", 0, 0, 1.0,
       8, 0, 200, 10, "f32", 0.1, False, 8_192, 10, 1),
    _w("citation-part0of16", 2, 2_900_000, 1, 30_000_000, "powerlaw", 2.0, 1e4,
       "powerlaw", 2.0, 1e4, 0.0,
       16, 0, 128, 2, "f32", 1.0, True, 65_536, 1, 0),
    _w("big-kg-part0of4", 3, 1_000_000, 1_000, 20_000_000, "powerlaw", 2.1, 1e4,
       "uniform", 0, 0, 1.1,
       4, 0, 256, 64, "bf16", 0.1, False, 65_536, 64, 1),
]


def paper_large_setting() -> WorkloadSpec:
    """The citation-shaped workload with the hyper-parameters the paper trains its large graph with
    (Sec. 4): 128 fixed input features, 32-wide embeddings, 2 bases, 1 negative per positive; dropout 0.2
    is a run-time setting of the step.  Same graph, partition and batch as WORKLOADS[3]."""
    return scaled(WORKLOADS[3], name="citation-part0of16-paper-setting", d=32, d_in=128, n_bases=2, n_neg=1)


def scaled(spec: WorkloadSpec, **kw) -> WorkloadSpec:
    """Copy of ``spec`` with some fields replaced (reduced test variants)."""
    d = dict(spec.__dict__)
    d.update(kw)
    d["acts"] = list(d["acts"])
    return WorkloadSpec(**d)


def _powerlaw_weights(rng, n, exponent, cap):
    # w = min(u^(-1/(exponent-1)), cap), u ~ U(0,1]: degree tail ~ k^-exponent.
    u = 1.0 - rng.random(n)
    return np.minimum(u ** (-1.0 / (exponent - 1.0)), cap)


def _categorical(rng, weights, size):
    # `size` i.i.d. draws from Categorical(weights), as per-category counts (one multinomial
    # draw) expanded and shuffled: same distribution as drawing one by one, much faster.
    p = np.asarray(weights, np.float64)
    counts = rng.multinomial(size, p / p.sum())
    out = np.repeat(np.arange(len(p), dtype=np.int32), counts)
    rng.shuffle(out)
    return out


def make_triples(spec: WorkloadSpec):
    """(head, rel, tail) int32 arrays of the whole graph. Duplicates and
    head == tail triples are kept as drawn (the message graph is a multigraph)."""
    rng = np.random.default_rng(spec.seed)
    n, m = spec.n_entities, spec.n_triples
    if spec.head_dist == "uniform":
        head = rng.integers(0, n, size=m, dtype=np.int32)
    else:
        head = _categorical(rng, _powerlaw_weights(rng, n, spec.head_exponent, spec.head_cap), m)
    if spec.tail_dist == "uniform":
        tail = rng.integers(0, n, size=m, dtype=np.int32)
    else:
        tail = _categorical(rng, _powerlaw_weights(rng, n, spec.tail_exponent, spec.tail_cap), m)
    if spec.n_relations == 1 or spec.rel_zipf == 0.0:
        rel = np.zeros(m, dtype=np.int32)
    else:
        pk = (np.arange(spec.n_relations, dtype=np.float64) + 1.0) ** (-spec.rel_zipf)
        rel = _categorical(rng, pk, m)
    return head, rel, tail


def _glorot(rng, shape, fan_in, fan_out):
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=shape).astype(np.float32)


def make_params(spec: WorkloadSpec, n_vertices: int) -> Dict[str, object]:
    """Model parameters and the layer-1 input for a partition with
    ``n_vertices`` local vertices.

    Returns dict with ``H0`` [N,d], per-layer lists ``V`` [B,d,d], ``a`` [2R,B],
    ``W0`` [d,d], and ``M`` [R,d] (the decoder's diagonals), all float32; with ``spec.d_in`` set the
    layer-1 input and the first layer's V, W0 have that many rows."""
    rng = np.random.default_rng(spec.seed + 1_000_003)
    d, B, R2 = spec.d, spec.n_bases, 2 * spec.n_relations
    d0 = spec.d_in if spec.d_in else d
    out: Dict[str, object] = {"V": [], "a": [], "W0": []}
    for l in range(spec.n_layers):
        di = d0 if l == 0 else d
        out["V"].append(_glorot(rng, (B, di, d), di, d))
        out["a"].append(_glorot(rng, (R2, B), R2, B))
        out["W0"].append(_glorot(rng, (di, d), di, d))
    out["M"] = (rng.standard_normal((spec.n_relations, d)) * 0.1).astype(np.float32)
    # Row-chunked so the float64 temporaries of the big workloads stay small.
    H0 = np.empty((n_vertices, d0), dtype=np.float32)
    step = 1 << 18
    for s in range(0, n_vertices, step):
        e = min(n_vertices, s + step)
        H0[s:e] = rng.standard_normal((e - s, d0), dtype=np.float32) * np.float32(spec.feature_std)
    out["H0"] = H0
    return out


def make_batch(spec: WorkloadSpec, n_core: int, n_pos: Optional[int] = None) -> np.ndarray:
    """Indices (into the partition's core-edge list) of one edge mini-batch:
    the first ``n_pos`` entries of a seeded permutation of the core edges."""
    rng = np.random.default_rng(spec.seed + 2_000_003)
    n_pos = spec.n_pos if n_pos is None else n_pos
    n_pos = min(n_pos, n_core)
    if n_core <= (1 << 22):
        return rng.permutation(n_core)[:n_pos].astype(np.int32)
    # Large core sets: draw without replacement by rejection of duplicates.
    picked = np.unique(rng.integers(0, n_core, size=2 * n_pos))
    rng.shuffle(picked)
    return picked[:n_pos].astype(np.int32)
