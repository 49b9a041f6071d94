"""Thin ctypes binding of ``libkge_mi355.so``: argument marshalling only.

Function names mirror the C ABI (``include/kge_mi355.h``) without the ``kge_`` prefix.
PyTorch is used for device memory and streams; every step of the training path runs in
the library's HIP kernels.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkge_mi355.so")
_lib = None

EXPORTED = ["kge_build_partition", "kge_partition_info", "kge_partition_export",
            "kge_partition_destroy", "kge_workspace_bytes", "kge_workspace_slice", "kge_rgcn_forward",
            "kge_rgcn_backward", "kge_sample_negatives", "kge_distmult_score_loss",
            "kge_profile_enable", "kge_profile_collect", "kge_last_error", "kge_cgraph_create",
            "kge_cgraph_destroy", "kge_compute_graph", "kge_cgraph_export", "kge_optimizer_step",
            "kge_optimizer_step_rows", "kge_eval_filter_create", "kge_eval_filter_destroy",
            "kge_eval_workspace_bytes", "kge_eval_rank_all", "kge_eval_rank_candidates", "kge_eval_metrics",
            "kge_eval_debug_scores", "kge_eval_rank_all_static", "kge_cgraph_input_rows", "kge_score_index_create", "kge_score_index_destroy",
            "kge_partition_bad_ids", "kge_test_set_rel_slab"]

ACT_IDENTITY, ACT_RELU = 0, 1
ORDER_PROJECT_FIRST, ORDER_RELATION_WEIGHTS = 0, 2
OPT_SGD, OPT_ADAM = 0, 1
MSG_F32, MSG_BF16 = 0, 1
NEG_TAIL, NEG_HEAD_OR_TAIL = 0, 1
DOMAIN_CORE, DOMAIN_ALL = 0, 1
EVAL_STATIC_BYTES = 32 << 20      # KGE_EVAL_STATIC_BYTES

ARRAYS = {"vert_gid": (0, np.int32), "core_eid": (1, np.int32), "core_h": (2, np.int32),
          "core_r": (3, np.int32), "core_t": (4, np.int32), "seg_ptr": (5, np.int32),
          "seg_rel": (6, np.int32), "seg_dst": (7, np.int32), "inv_c": (8, np.float32),
          "col_src": (9, np.int32), "edge_id": (10, np.int32), "cand": (11, np.int32),
          "dm_ptr": (12, np.int32), "dm_src": (13, np.int32), "dm_rel": (14, np.int32),
          "dm_invc": (15, np.float32), "sm_ptr": (16, np.int32), "sm_dst": (17, np.int32),
          "sm_rel": (18, np.int32), "sm_invc": (19, np.float32), "rel_ptr": (20, np.int32),
          "dr_ptr": (21, np.int32), "dr_seg": (22, np.int32), "dr_rel": (23, np.int32),
          "sm_seg": (24, np.int32)}


class KgeError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("kge status %d: %s" % (status, msg))
        self.status = status


class _PartInfo(C.Structure):
    _fields_ = [("n_vert", C.c_int64), ("n_edge", C.c_int64), ("n_seg", C.c_int64),
                ("n_core", C.c_int64), ("n_cand", C.c_int64), ("n_triples", C.c_int64),
                ("n_entities", C.c_int32), ("n_relations", C.c_int32), ("n_parts", C.c_int32),
                ("part_id", C.c_int32), ("n_hops", C.c_int32), ("neg_domain", C.c_int32),
                ("max_in_degree", C.c_int32), ("max_out_degree", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("n_bases", C.c_int32), ("act", C.c_int32),
                ("order", C.c_int32), ("V", C.c_void_p), ("a", C.c_void_p), ("W0", C.c_void_p),
                ("dropout", C.c_float), ("drop_seed", C.c_uint64), ("drop_step", C.c_uint64)]


class _LayerGrad(C.Structure):
    _fields_ = [("dV", C.c_void_p), ("da", C.c_void_p), ("dW0", C.c_void_p)]


class _Opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("t", C.c_int64)]


class _ProfEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("total_ms", C.c_double), ("calls", C.c_int64)]


def load():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2201_02791_amd.build` "
                              "(there is no CPU fallback)" % LIB_PATH)
        # torch first: its bundled HIP runtime must be the one this process initialises; loading
        # the library before it brings in a second runtime that then finds no device
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        lib.kge_last_error.restype = C.c_char_p
        lib.kge_workspace_bytes.restype = C.c_size_t
        lib.kge_partition_destroy.restype = None
        lib.kge_cgraph_destroy.restype = None
        lib.kge_score_index_destroy.restype = None
        lib.kge_eval_filter_destroy.restype = None
        lib.kge_eval_workspace_bytes.restype = C.c_size_t
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise KgeError(rc, load().kge_last_error().decode())


def _ptr(t) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


class Partition:
    """Owner of a ``kge_partition*``."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)
        info = _PartInfo()
        _check(load().kge_partition_info(self._h, C.byref(info)))
        for name, _ in _PartInfo._fields_:
            setattr(self, name, int(getattr(info, name)))

    @property
    def handle(self):
        return self._h

    def export(self, name: str) -> np.ndarray:
        return partition_export(self, name)

    def bad_ids(self) -> int:
        """Ids outside the partition that the per-step kernels have met (and not used) so far; synchronises."""
        n = C.c_int64()
        _check(load().kge_partition_bad_ids(self._h, C.byref(n)))
        return int(n.value)

    def destroy(self):
        if self._h is not None and self._h.value:
            load().kge_partition_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def set_rel_slab_for_tests(vertices: int, min_runs: int = 0):
    """Test hook: slab size (destinations) and cutting threshold (runs) of the range order that partitions built
    afterwards give the transposed per-run products; (0, 0) restores the library's values."""
    load().kge_test_set_rel_slab(C.c_int32(vertices), C.c_int32(min_runs))


def build_partition(head, rel, tail, n_entities: int, n_relations: int, n_parts: int = 1,
                    part_id: int = 0, n_hops: int = 2, neg_domain: int = DOMAIN_CORE) -> Partition:
    head = np.ascontiguousarray(head, np.int32)
    rel = np.ascontiguousarray(rel, np.int32)
    tail = np.ascontiguousarray(tail, np.int32)
    assert len(head) == len(rel) == len(tail)
    out = C.c_void_p()
    _check(load().kge_build_partition(head.ctypes.data_as(C.c_void_p), rel.ctypes.data_as(C.c_void_p),
                                      tail.ctypes.data_as(C.c_void_p), C.c_int64(len(head)),
                                      C.c_int32(n_entities), C.c_int32(n_relations), C.c_int32(n_parts),
                                      C.c_int32(part_id), C.c_int32(n_hops), C.c_int32(neg_domain),
                                      C.byref(out)))
    return Partition(out.value)


def partition_info(part: Partition) -> dict:
    return {name: getattr(part, name) for name, _ in _PartInfo._fields_}


def partition_export(part: Partition, name: str) -> np.ndarray:
    which, dt = ARRAYS[name]
    n = {"vert_gid": part.n_vert, "core_eid": part.n_core, "core_h": part.n_core, "core_r": part.n_core,
         "core_t": part.n_core, "seg_ptr": part.n_seg + 1, "seg_rel": part.n_seg, "seg_dst": part.n_seg,
         "inv_c": part.n_seg, "col_src": part.n_edge, "edge_id": part.n_edge, "cand": part.n_cand,
         "dm_ptr": part.n_vert + 1, "dm_src": part.n_edge, "dm_rel": part.n_edge, "dm_invc": part.n_edge,
         "sm_ptr": part.n_vert + 1, "sm_dst": part.n_edge, "sm_rel": part.n_edge, "sm_invc": part.n_edge,
         "rel_ptr": 2 * part.n_relations + 1, "dr_ptr": part.n_vert + 1, "dr_seg": part.n_seg,
         "dr_rel": part.n_seg, "sm_seg": part.n_edge}[name]
    arr = np.empty(n, dt)
    _check(load().kge_partition_export(part.handle, C.c_int32(which), arr.ctypes.data_as(C.c_void_p),
                                       C.c_int64(arr.nbytes)))
    return arr


def partition_destroy(part: Partition):
    part.destroy()


def _layers(layers: Sequence[dict]):
    arr = (_Layer * len(layers))()
    for i, l in enumerate(layers):
        V, a, W0 = l["V"], l["a"], l["W0"]
        arr[i].n_bases, arr[i].d_in, arr[i].d_out = V.shape
        arr[i].act = int(l["act"])
        arr[i].order = int(l.get("order", ORDER_PROJECT_FIRST))
        arr[i].V, arr[i].a, arr[i].W0 = V.data_ptr(), a.data_ptr(), W0.data_ptr()
        arr[i].dropout = float(l.get("dropout", 0.0))
        arr[i].drop_seed, arr[i].drop_step = int(l.get("drop_seed", 0)), int(l.get("drop_step", 0))
    return arr


def workspace_bytes(part: Partition, layers: Sequence[dict], msg_dtype: int = MSG_F32) -> int:
    n = load().kge_workspace_bytes(part.handle, _layers(layers), C.c_int32(len(layers)), C.c_int32(msg_dtype))
    if n == 0:
        raise KgeError(-1, load().kge_last_error().decode())
    return int(n)


class ComputeGraph:
    """Owner of a ``kge_cgraph*``: the flags of one batch's computational sub-graph."""

    def __init__(self, part: Partition, n_layers: int):
        out = C.c_void_p()
        _check(load().kge_cgraph_create(part.handle, C.c_int32(n_layers), C.byref(out)))
        self._h = C.c_void_p(out.value)
        self.n_layers, self.n_vert = n_layers, part.n_vert

    @property
    def handle(self):
        return self._h

    def export(self):
        """(active uint8 [n_layers][N], counts int64 [n_layers][4] = vertices, edges in, runs, edges out)."""
        active = np.zeros((self.n_layers, self.n_vert), np.uint8)
        stats = np.zeros((self.n_layers, 4), np.int64)
        _check(load().kge_cgraph_export(self._h, active.ctypes.data_as(C.c_void_p),
                                        stats.ctypes.data_as(C.c_void_p)))
        return active, stats

    def input_rows_ptr(self) -> int:
        """Device address of the flags (uint8 [N]) of the first layer's input rows the batch reads."""
        ptr = C.c_void_p()
        _check(load().kge_cgraph_input_rows(self._h, C.byref(ptr), None, None))
        return ptr.value

    def input_rows(self):
        """(flags uint8 [N] on the host, their count): the first layer's input rows the batch reads."""
        flags = np.zeros(self.n_vert, np.uint8)
        count = C.c_int64()
        _check(load().kge_cgraph_input_rows(self._h, None, flags.ctypes.data_as(C.c_void_p), C.byref(count)))
        return flags, int(count.value)

    def destroy(self):
        if self._h is not None and self._h.value:
            load().kge_cgraph_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _cg(cg) -> C.c_void_p:
    return C.c_void_p(0) if cg is None else cg.handle


def compute_graph(part: Partition, cg: ComputeGraph, pos_core_idx, neg_ent=None, stream=None):
    n_neg_entries = 0 if neg_ent is None else neg_ent.numel()
    _check(load().kge_compute_graph(part.handle, cg.handle, _ptr(pos_core_idx), C.c_int64(pos_core_idx.numel()),
                                    _ptr(neg_ent if n_neg_entries else None), C.c_int64(n_neg_entries),
                                    _stream(stream)))


def rgcn_forward(part: Partition, layers: Sequence[dict], H0, workspace, H_out,
                 msg_dtype: int = MSG_F32, stream=None, cg: ComputeGraph = None):
    _check(load().kge_rgcn_forward(part.handle, _cg(cg), _layers(layers), C.c_int32(len(layers)), C.c_int32(msg_dtype),
                                   _ptr(H0), _ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                                   _ptr(H_out), _stream(stream)))


def rgcn_backward(part: Partition, layers: Sequence[dict], H0, workspace, dH_out, grads: Sequence[dict],
                  dH0=None, msg_dtype: int = MSG_F32, stream=None, cg: ComputeGraph = None):
    g = (_LayerGrad * len(layers))()
    for i, gr in enumerate(grads):
        g[i].dV, g[i].da, g[i].dW0 = gr["dV"].data_ptr(), gr["da"].data_ptr(), gr["dW0"].data_ptr()
    _check(load().kge_rgcn_backward(part.handle, _cg(cg), _layers(layers), C.c_int32(len(layers)), C.c_int32(msg_dtype),
                                    _ptr(H0), _ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                                    _ptr(dH_out), g, _ptr(dH0), _stream(stream)))


def sample_negatives(part: Partition, pos_core_idx, n_neg: int, mode: int, seed: int, step: int,
                     neg_ent, neg_side, stream=None):
    _check(load().kge_sample_negatives(part.handle, _ptr(pos_core_idx), C.c_int64(pos_core_idx.numel()),
                                       C.c_int32(n_neg), C.c_int32(mode), C.c_uint64(seed), C.c_uint64(step),
                                       _ptr(neg_ent), _ptr(neg_side), _stream(stream)))


class ScoreIndex:
    """Owner of a ``kge_score_index*``: scratch of the atomic-free scoring call for batches up to a given size."""

    def __init__(self, part: Partition, max_pos: int, max_neg: int, d: int):
        out = C.c_void_p()
        _check(load().kge_score_index_create(part.handle, C.c_int64(max_pos), C.c_int32(max_neg), C.c_int32(d),
                                             C.byref(out)))
        self._h = C.c_void_p(out.value)

    @property
    def handle(self):
        return self._h

    def destroy(self):
        if self._h is not None and self._h.value:
            load().kge_score_index_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def distmult_score_loss(part: Partition, H, M, pos_core_idx, neg_ent, neg_side, n_neg: int, scores, loss,
                        dH, dM, stream=None, index: "ScoreIndex" = None):
    _check(load().kge_distmult_score_loss(part.handle, index.handle if index is not None else C.c_void_p(0),
                                          _ptr(H), _ptr(M), C.c_int32(H.shape[1]),
                                          _ptr(pos_core_idx), C.c_int64(pos_core_idx.numel()),
                                          _ptr(neg_ent), _ptr(neg_side), C.c_int32(n_neg), _ptr(scores),
                                          _ptr(loss), _ptr(dH), _ptr(dM), _stream(stream)))


def profile_enable(on: bool):
    _check(load().kge_profile_enable(C.c_int32(1 if on else 0)))


def profile_collect() -> dict:
    """{kernel name: (total milliseconds, launches)} since profiling was enabled / last collected."""
    arr = (_ProfEntry * 64)()
    n = C.c_int32(0)
    _check(load().kge_profile_collect(arr, C.c_int32(64), C.byref(n)))
    return {arr[i].name.decode(): (float(arr[i].total_ms), int(arr[i].calls)) for i in range(n.value)}


WS_P, WS_H, WS_G, WS_DP, WS_DH, WS_Z, WS_U, WS_HD = 0, 1, 2, 3, 4, 5, 7, 8


def workspace_slice(part: Partition, layers: Sequence[dict], which: int, layer: int,
                    msg_dtype: int = MSG_F32):
    """(byte offset, byte size) of one intermediate inside the workspace."""
    off, nbytes = C.c_size_t(0), C.c_size_t(0)
    _check(load().kge_workspace_slice(part.handle, _layers(layers), C.c_int32(len(layers)), C.c_int32(msg_dtype),
                                      C.c_int32(which), C.c_int32(layer), C.byref(off), C.byref(nbytes)))
    return int(off.value), int(nbytes.value)


def optimizer_step(kind: int, param, grad, m=None, v=None, lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8, t=1,
                   rows: bool = False, row_mask=None, stream=None):
    """One optimizer step in place on device tensors.  rows=True: the row form on a 2-D tensor."""
    o = _Opt(kind, lr, beta1, beta2, eps, t)
    if rows:
        mask = C.c_void_p(row_mask) if isinstance(row_mask, int) else _ptr(row_mask)     # raw device address or tensor
        _check(load().kge_optimizer_step_rows(C.byref(o), _ptr(param), _ptr(grad), _ptr(m), _ptr(v),
                                              C.c_int64(param.shape[0]), C.c_int32(param.shape[1]),
                                              mask, _stream(stream)))
    else:
        _check(load().kge_optimizer_step(C.byref(o), _ptr(param), _ptr(grad), _ptr(m), _ptr(v),
                                         C.c_int64(param.numel()), _stream(stream)))


# ---- link-prediction evaluation (filtered ranks, MRR, Hits@k) ----------------------------------

class EvalFilter:
    """Owner of a ``kge_eval_filter*``: the known triples whose corruptions the filtered setting drops."""

    def __init__(self, head, rel, tail, n_entities: int, n_relations: int):
        head = np.ascontiguousarray(head, np.int32)
        rel = np.ascontiguousarray(rel, np.int32)
        tail = np.ascontiguousarray(tail, np.int32)
        assert len(head) == len(rel) == len(tail)
        out = C.c_void_p()
        _check(load().kge_eval_filter_create(head.ctypes.data_as(C.c_void_p), rel.ctypes.data_as(C.c_void_p),
                                             tail.ctypes.data_as(C.c_void_p), C.c_int64(len(head)),
                                             C.c_int32(n_entities), C.c_int32(n_relations), C.byref(out)))
        self._h = C.c_void_p(out.value)

    @property
    def handle(self):
        return self._h

    def destroy(self):
        if self._h is not None and self._h.value:
            load().kge_eval_filter_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def eval_workspace_bytes(n_queries: int, d: int) -> int:
    n = load().kge_eval_workspace_bytes(C.c_int64(n_queries), C.c_int32(d))
    if n == 0:
        raise KgeError(-1, load().kge_last_error().decode())
    return int(n)


def _eval_ws(n_queries, d, device, workspace):
    import torch
    need = eval_workspace_bytes(n_queries, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace


def eval_rank_all(H, M, test_h, test_r, test_t, filt: EvalFilter = None, workspace=None, stream=None):
    """(higher, equal) int32 [2 n_test] on the device: tail queries of all test triples, then head queries."""
    import torch
    n_test = test_h.numel()
    ws = _eval_ws(2 * n_test, H.shape[1], H.device, workspace)
    higher = torch.empty(2 * n_test, dtype=torch.int32, device=H.device)
    equal = torch.empty_like(higher)
    _check(load().kge_eval_rank_all(filt.handle if filt is not None else C.c_void_p(0), _ptr(H), C.c_int64(H.shape[0]),
                                    C.c_int32(H.shape[1]), _ptr(M), C.c_int32(M.shape[0]), _ptr(test_h), _ptr(test_r),
                                    _ptr(test_t), C.c_int64(n_test), _ptr(ws), C.c_size_t(ws.numel()), _ptr(higher),
                                    _ptr(equal), _stream(stream)))
    return higher, equal


def eval_rank_all_static(H, M, test_h, test_r, test_t, higher, equal, filt: EvalFilter = None, stream=None):
    """kge_eval_rank_all_static: the caller brings the outputs (int32 [2 n_test] each); nothing is allocated."""
    _check(load().kge_eval_rank_all_static(filt.handle if filt is not None else C.c_void_p(0), _ptr(H),
                                           C.c_int64(H.shape[0]), C.c_int32(H.shape[1]), _ptr(M), C.c_int32(M.shape[0]),
                                           _ptr(test_h), _ptr(test_r), _ptr(test_t), C.c_int64(test_h.numel()),
                                           _ptr(higher), _ptr(equal), _stream(stream)))


def eval_rank_candidates(H, M, fixed, rel, answer, cand, workspace=None, stream=None):
    """(higher, equal) int32 [n_queries] against each query's own candidate list cand [n_queries, n_cand]."""
    import torch
    nq = fixed.numel()
    ws = _eval_ws(nq, H.shape[1], H.device, workspace)
    higher = torch.empty(nq, dtype=torch.int32, device=H.device)
    equal = torch.empty_like(higher)
    _check(load().kge_eval_rank_candidates(_ptr(H), C.c_int64(H.shape[0]), C.c_int32(H.shape[1]), _ptr(M),
                                           C.c_int32(M.shape[0]), _ptr(fixed), _ptr(rel), _ptr(answer), C.c_int64(nq),
                                           _ptr(cand), C.c_int32(cand.shape[1] if cand.dim() == 2 else 0), _ptr(ws),
                                           C.c_size_t(ws.numel()), _ptr(higher), _ptr(equal), _stream(stream)))
    return higher, equal


def eval_metrics(higher, equal, ks=(1, 3, 10), stream=None):
    """Device tensor of doubles: MRR, then Hits@k for each k."""
    import torch
    out = torch.empty(1 + len(ks), dtype=torch.float64, device=higher.device)
    karr = (C.c_int32 * max(len(ks), 1))(*ks)
    _check(load().kge_eval_metrics(_ptr(higher), _ptr(equal), C.c_int64(higher.numel()), karr, C.c_int32(len(ks)),
                                   _ptr(out), _stream(stream)))
    return out


def eval_debug_scores(H, M, test_h, test_r, test_t, stream=None):
    """Test hook: (scores [2 n_test, n_entities] from the tile kernel, answer scores [2 n_test] from the
    per-query kernel)."""
    import torch
    n_test = test_h.numel()
    ws = _eval_ws(2 * n_test, H.shape[1], H.device, None)
    scores = torch.empty((2 * n_test, H.shape[0]), dtype=torch.float32, device=H.device)
    ans = torch.empty(2 * n_test, dtype=torch.float32, device=H.device)
    _check(load().kge_eval_debug_scores(_ptr(H), C.c_int64(H.shape[0]), C.c_int32(H.shape[1]), _ptr(M),
                                        C.c_int32(M.shape[0]), _ptr(test_h), _ptr(test_r), _ptr(test_t),
                                        C.c_int64(n_test), _ptr(ws), C.c_size_t(ws.numel()), _ptr(scores), _ptr(ans),
                                        _stream(stream)))
    return scores, ans
