"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``liborc.so`` built from ``kge_oracle.c`` (plain C, double precision,
single-threaded) and exposes its functions on NumPy arrays.  Nothing here is
imported by the product package; only tests, the smoke check and the
benchmark's cpu_baseline leg use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kge_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None


def build_lib(force: bool = False) -> str:
    """Compile the C oracle with gcc (no -march, so the library runs on any x86-64 host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-std=c99", "-fPIC", "-shared", "-fno-fast-math",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        build_lib()
        _lib = C.CDLL(_LIB)
        _lib.orc_build_partition.restype = C.c_void_p
        _lib.orc_part_of_head.restype = C.c_uint32
    return _lib


_I32, _F64, _F32, _U8, _I64 = C.c_int32, C.c_double, C.c_float, C.c_uint8, C.c_int64
_PART_ARRAYS = [("vert_gid", np.int32), ("core_eid", np.int32), ("core_h", np.int32),
                ("core_r", np.int32), ("core_t", np.int32), ("seg_ptr", np.int32),
                ("seg_rel", np.int32), ("seg_dst", np.int32), ("inv_c", np.float32),
                ("col_src", np.int32), ("edge_id", np.int32), ("cand", np.int32)]


def part_of_head(head: int, n_parts: int) -> int:
    return int(lib().orc_part_of_head(C.c_int32(head), C.c_int32(n_parts)))


def build_partition(head, rel, tail, n_entities, n_relations, n_parts=1, part_id=0, n_hops=2,
                    neg_domain=0) -> Dict[str, np.ndarray]:
    """Partition + expansion + sorted edge runs (Sec. 3.2).  Returns the arrays by name
    plus ``n_vert, n_edge, n_seg, n_core, n_cand`` and ``n_relations``."""
    L = lib()
    head = np.ascontiguousarray(head, np.int32)
    rel = np.ascontiguousarray(rel, np.int32)
    tail = np.ascontiguousarray(tail, np.int32)
    h = L.orc_build_partition(_p(head, _I32), _p(rel, _I32), _p(tail, _I32), C.c_int64(len(head)),
                              C.c_int32(n_entities), C.c_int32(n_relations), C.c_int32(n_parts),
                              C.c_int32(part_id), C.c_int32(n_hops), C.c_int32(neg_domain))
    h = C.c_void_p(h)
    sizes = np.zeros(5, np.int64)
    L.orc_partition_sizes(h, _p(sizes, _I64))
    n_vert, n_edge, n_seg, n_core, n_cand = (int(x) for x in sizes)
    lens = {"vert_gid": n_vert, "core_eid": n_core, "core_h": n_core, "core_r": n_core,
            "core_t": n_core, "seg_ptr": n_seg + 1, "seg_rel": n_seg, "seg_dst": n_seg,
            "inv_c": n_seg, "col_src": n_edge, "edge_id": n_edge, "cand": n_cand}
    out: Dict[str, object] = dict(n_vert=n_vert, n_edge=n_edge, n_seg=n_seg, n_core=n_core,
                                  n_cand=n_cand, n_relations=int(n_relations))
    for which, (name, dt) in enumerate(_PART_ARRAYS):
        arr = np.zeros(lens[name], dt)
        L.orc_partition_copy(h, C.c_int32(which), arr.ctypes.data_as(C.c_void_p))
        out[name] = arr
    L.orc_partition_free(h)
    return out


def _d(x):
    return np.ascontiguousarray(x, np.float64)


def layer_forward(part, V, a, W0, act, H):
    """One RGCN layer over the whole partition (Eq. 1-2). Returns (pre, H') in float64."""
    L = lib()
    V, a, W0, H = _d(V), _d(a), _d(W0), _d(H)
    B, d_in, d_out = V.shape
    N = part["n_vert"]
    assert H.shape == (N, d_in)
    P = np.empty((N, B, d_out))
    pre = np.empty((N, d_out))
    out = np.empty((N, d_out))
    L.orc_rgcn_layer_forward(C.c_int64(N), C.c_int64(part["n_seg"]), _p(part["seg_ptr"], _I32),
                             _p(part["seg_rel"], _I32), _p(part["seg_dst"], _I32),
                             _p(part["col_src"], _I32), C.c_int32(d_in), C.c_int32(d_out),
                             C.c_int32(B), _p(V, _F64), _p(a, _F64), _p(W0, _F64), C.c_int32(act),
                             _p(H, _F64), _p(P, _F64), _p(pre, _F64), _p(out, _F64))
    return pre, out


def dropout(H, p, seed, step, layer):
    """Inverted dropout on a layer's input with a counter-based mask.  Returns (dropped H, keep mask)."""
    H = _d(H)
    out = np.zeros_like(H); mask = np.zeros(H.shape, np.uint8)
    lib().orc_dropout(C.c_int64(H.shape[0]), C.c_int32(H.shape[1]), C.c_double(p), C.c_uint64(seed),
                      C.c_uint64(step), C.c_int32(layer), _p(H, _F64), _p(out, _F64), _p(mask, _U8))
    return out, mask


def rgcn_forward(part, layers: Sequence[dict], H0, drop=None):
    """All layers.  ``layers[l]`` has V [B,d,d], a [2R,B], W0 [d,d], act.  Returns the list of
    layer inputs/outputs ``Hs`` (len L+1, Hs[0] = H0) and pre-activations ``pres`` (len L).

    ``drop = (p, seed, step)`` applies :func:`dropout` to every layer's input; ``Hs[l]`` is then
    the input as the layer saw it (after dropout) for l < L, and the third result lists the keep
    masks."""
    Hs, pres, masks = [_d(H0)], [], []
    for l, lay in enumerate(layers):
        if drop is not None:
            Hs[-1], m = dropout(Hs[-1], drop[0], drop[1], drop[2], l)
            masks.append(m)
        pre, out = layer_forward(part, lay["V"], lay["a"], lay["W0"], lay["act"], Hs[-1])
        pres.append(pre)
        Hs.append(out)
    return (Hs, pres, masks) if drop is not None else (Hs, pres)


def layer_backward(part, V, a, W0, act, H, pre, dHout, need_dH=True):
    L = lib()
    V, a, W0, H, pre, dHout = _d(V), _d(a), _d(W0), _d(H), _d(pre), _d(dHout)
    B, d_in, d_out = V.shape
    N = part["n_vert"]
    P = np.empty((N, B, d_out)); dP = np.empty((N, B, d_out)); G = np.empty((N, d_out))
    dV = np.empty_like(V); da = np.empty_like(a); dW0 = np.empty_like(W0)
    dH = np.empty((N, d_in)) if need_dH else None
    L.orc_rgcn_layer_backward(C.c_int64(N), C.c_int64(part["n_seg"]), _p(part["seg_ptr"], _I32),
                              _p(part["seg_rel"], _I32), _p(part["seg_dst"], _I32),
                              _p(part["col_src"], _I32), C.c_int32(d_in), C.c_int32(d_out),
                              C.c_int32(B), C.c_int32(a.shape[0]), _p(V, _F64), _p(a, _F64),
                              _p(W0, _F64), C.c_int32(act), _p(H, _F64), _p(pre, _F64),
                              _p(dHout, _F64), _p(P, _F64), _p(dP, _F64), _p(G, _F64),
                              _p(dV, _F64), _p(da, _F64), _p(dW0, _F64),
                              _p(dH, _F64) if need_dH else None)
    return dict(dV=dV, da=da, dW0=dW0, dH=dH, dP=dP, Gpre=G)


def rgcn_backward(part, layers, Hs, pres, dH_out, need_dH0=True, drop=None, masks=None):
    """Reverse of :func:`rgcn_forward`. Returns per-layer grads (list) and dH0 (or None).  With
    dropout (``drop`` and the forward's ``masks``) the gradient handed to the layer below, and dH0,
    is the one with respect to the input before dropout."""
    grads: List[Optional[dict]] = [None] * len(layers)
    g = _d(dH_out)
    for l in range(len(layers) - 1, -1, -1):
        lay = layers[l]
        need = need_dH0 or l > 0
        r = layer_backward(part, lay["V"], lay["a"], lay["W0"], lay["act"], Hs[l], pres[l], g, need)
        grads[l] = r
        g = r["dH"]
        if drop is not None and g is not None:
            g = g * masks[l] / (1.0 - drop[0])
    return grads, g


def layer_rows(part, rows, V, a, W0, act, H_f32):
    """Layer output for the listed destination rows only, from the stored float32 input."""
    L = lib()
    rows = np.ascontiguousarray(rows, np.int32)
    V, a, W0 = _d(V), _d(a), _d(W0)
    B, d_in, d_out = V.shape
    H_f32 = np.ascontiguousarray(H_f32, np.float32)
    seg_dst = part["seg_dst"]
    order = np.argsort(seg_dst, kind="stable")
    sd = seg_dst[order]
    lo = np.searchsorted(sd, rows, side="left")
    hi = np.searchsorted(sd, rows, side="right")
    ptr = np.zeros(len(rows) + 1, np.int64)
    ptr[1:] = np.cumsum(hi - lo)
    segs = np.concatenate([order[l:h] for l, h in zip(lo, hi)] + [np.zeros(0, np.int64)]).astype(np.int64)
    pre = np.empty((len(rows), d_out)); out = np.empty((len(rows), d_out))
    L.orc_rgcn_layer_rows(C.c_int64(len(rows)), _p(rows, _I32), _p(ptr, _I64), _p(segs, _I64),
                          _p(part["seg_ptr"], _I32), _p(part["seg_rel"], _I32),
                          _p(part["col_src"], _I32), C.c_int32(d_in), C.c_int32(d_out), C.c_int32(B),
                          _p(V, _F64), _p(a, _F64), _p(W0, _F64), C.c_int32(act), _p(H_f32, _F32),
                          _p(pre, _F64), _p(out, _F64))
    return pre, out


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, np.uint32); k = np.ascontiguousarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def sample_negatives(part, pos_core_idx, n_neg, mode, seed, step):
    """In-partition negatives (Sec. 3.3.1). Returns (neg_ent [n_pos,n_neg] int32 local ids,
    neg_side uint8: 0 tail replaced, 1 head replaced)."""
    pos = np.ascontiguousarray(pos_core_idx, np.int32)
    ne = np.zeros((len(pos), n_neg), np.int32); ns = np.zeros((len(pos), n_neg), np.uint8)
    lib().orc_sample_negatives(_p(part["cand"], _I32), C.c_int64(part["n_cand"]), _p(pos, _I32),
                               C.c_int64(len(pos)), C.c_int32(n_neg), C.c_int32(mode),
                               C.c_uint64(seed), C.c_uint64(step), _p(ne, _I32), _p(ns, _U8))
    return ne, ns


def distmult_score_loss(part, H, M, pos_core_idx, neg_ent, neg_side):
    """Eq. 4 scores, Eq. 3 loss and their gradients.  Returns dict(scores, loss, dH, dM)."""
    H, M = _d(H), _d(M)
    N, d = H.shape
    pos = np.ascontiguousarray(pos_core_idx, np.int64)
    ph = np.ascontiguousarray(part["core_h"][pos]); pr = np.ascontiguousarray(part["core_r"][pos])
    pt = np.ascontiguousarray(part["core_t"][pos])
    neg_ent = np.ascontiguousarray(neg_ent, np.int32)
    n_neg = neg_ent.shape[1] if neg_ent.ndim == 2 else neg_ent.size // max(len(pos), 1)
    neg_ent = neg_ent.reshape(len(pos), n_neg)
    neg_side = np.ascontiguousarray(neg_side, np.uint8).reshape(len(pos), n_neg)
    scores = np.zeros((len(pos), 1 + n_neg)); loss = np.zeros(1)
    dH = np.zeros((N, d)); dM = np.zeros_like(M)
    lib().orc_distmult_score_loss(C.c_int64(N), C.c_int32(d), C.c_int32(M.shape[0]), _p(H, _F64),
                                  _p(M, _F64), C.c_int64(len(pos)), C.c_int32(n_neg), _p(ph, _I32),
                                  _p(pr, _I32), _p(pt, _I32), _p(neg_ent, _I32), _p(neg_side, _U8),
                                  _p(scores, _F64), _p(loss, _F64), _p(dH, _F64), _p(dM, _F64))
    return dict(scores=scores, loss=float(loss[0]), dH=dH, dM=dM)


def batch_vertices(part, pos_core_idx, neg_ent):
    """Local ids of every vertex a scored triple of the batch touches."""
    pos = np.ascontiguousarray(pos_core_idx, np.int64)
    return np.concatenate([part["core_h"][pos], part["core_t"][pos],
                           np.ascontiguousarray(neg_ent, np.int32).reshape(-1)]).astype(np.int32)


def compute_graph(part, pos_core_idx, neg_ent, n_layers):
    """Computational sub-graph of one edge batch (Sec. 3.3, Algorithm 1): uint8 [n_layers][N],
    row l = the vertices layer l+1 must produce an output for."""
    bv = np.ascontiguousarray(batch_vertices(part, pos_core_idx, neg_ent), np.int32)
    N = part["n_vert"]
    active = np.zeros((n_layers, N), np.uint8)
    lib().orc_compute_graph(C.c_int64(N), C.c_int64(part["n_seg"]), _p(part["seg_ptr"], _I32),
                            _p(part["seg_dst"], _I32), _p(part["col_src"], _I32), C.c_int64(len(bv)),
                            _p(bv, _I32), C.c_int32(n_layers), _p(active, _U8))
    return active


def optimizer_step(kind, p, g, m, v, lr=0.01, b1=0.9, b2=0.999, eps=1e-8, t=1, row_mask=None):
    """One optimizer step in place on float64 arrays (Algorithm 1, "optimizer.step()").  kind 0: plain
    gradient descent; 1: Adam.  row_mask (uint8 per row of a 2-D tensor): only those rows are touched."""
    assert p.dtype == np.float64 and p.flags.c_contiguous
    g = _d(g)
    if kind == 1:
        assert m.dtype == np.float64 and v.dtype == np.float64 and m.flags.c_contiguous and v.flags.c_contiguous
    if row_mask is None:
        n_rows, d, mk = 1, p.size, None
    else:
        n_rows, d = p.shape[0], p.size // max(p.shape[0], 1)
        mk = np.ascontiguousarray(row_mask, np.uint8)
    lib().orc_optimizer_step(C.c_int32(kind), _p(p, _F64), _p(g, _F64),
                             _p(m, _F64) if kind == 1 else None, _p(v, _F64) if kind == 1 else None,
                             C.c_int64(n_rows), C.c_int64(d), _p(mk, _U8) if mk is not None else None,
                             C.c_double(lr), C.c_double(b1), C.c_double(b2), C.c_double(eps), C.c_int64(t))


def train_step(part, layers, H0, M, pos_core_idx, n_neg, mode, seed, step, need_dH0=True, dropout=0.0):
    """One whole step: encoder forward, negatives, score + loss, encoder backward.  With
    ``dropout`` > 0 every layer's input is dropped with masks keyed by the step's (seed, step)."""
    drop = (float(dropout), seed, step) if dropout > 0 else None
    masks = None
    if drop is None:
        Hs, pres = rgcn_forward(part, layers, H0)
    else:
        Hs, pres, masks = rgcn_forward(part, layers, H0, drop)
    ne, ns = sample_negatives(part, pos_core_idx, n_neg, mode, seed, step)
    sl = distmult_score_loss(part, Hs[-1], M, pos_core_idx, ne, ns)
    grads, dH0 = rgcn_backward(part, layers, Hs, pres, sl["dH"], need_dH0, drop, masks)
    return dict(Hs=Hs, pres=pres, neg_ent=ne, neg_side=ns, scores=sl["scores"], loss=sl["loss"],
                dH_out=sl["dH"], dM=sl["dM"], grads=grads, dH0=dH0, masks=masks, drop=drop)
