"""One training step of Algorithm 1 on one partition: buffer ownership and call order.

Holds the torch tensors (device memory only) and issues the library calls in order on one
stream: negatives -> [computational sub-graph of the batch] -> encoder forward -> score/loss ->
encoder backward.  No arithmetic of the method happens in Python or torch.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from . import binding as kb


class TrainStep:
    def __init__(self, part: kb.Partition, params: Dict[str, object], acts: Sequence[int],
                 msg_dtype: int = kb.MSG_F32, need_dH0: bool = True, device: str = "cuda:0",
                 keep_scores: bool = True, cone: bool = False, order: int = kb.ORDER_PROJECT_FIRST,
                 dropout: float = 0.0, score_index: bool = True):
        import torch
        self.torch = torch
        self.part = part
        self.dev = torch.device(device)
        self.msg_dtype = msg_dtype
        t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)
        self.layers: List[dict] = []
        for V, a, W0, act in zip(params["V"], params["a"], params["W0"], acts):
            self.layers.append(dict(V=t(V), a=t(a), W0=t(W0), act=int(act), order=int(order),
                                    dropout=float(dropout), drop_seed=0, drop_step=0))
        self.M = t(params["M"])
        self.H0 = t(params["H0"])
        N = part.n_vert
        assert self.H0.shape[0] == N
        d_out = self.layers[-1]["V"].shape[2]
        self.H_out = torch.empty((N, d_out), dtype=torch.float32, device=self.dev)
        self.dH_out = torch.empty_like(self.H_out)
        self.dM = torch.empty_like(self.M)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self.grads = [dict(dV=torch.empty_like(l["V"]), da=torch.empty_like(l["a"]),
                           dW0=torch.empty_like(l["W0"])) for l in self.layers]
        self.dH0 = torch.empty_like(self.H0) if need_dH0 else None
        self.ws_bytes = kb.workspace_bytes(part, self.layers, msg_dtype)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.keep_scores = keep_scores
        # cone: propagate only the batch's computational sub-graph (Algorithm 1, getComputeGraph)
        self.cg = kb.ComputeGraph(part, len(self.layers)) if cone else None
        self.pos = None
        self.neg_ent = self.neg_side = self.scores = None
        self.n_neg = 0
        # score_index: the atomic-free form of the scoring call (its scratch is allocated with the batch)
        self.want_index = score_index
        self.index = None

    def set_batch(self, pos_core_idx: np.ndarray, n_neg: int):
        torch = self.torch
        self.pos = torch.from_numpy(np.ascontiguousarray(pos_core_idx, np.int32)).to(self.dev)
        n_pos = self.pos.numel()
        self.n_neg = int(n_neg)
        self.neg_ent = torch.empty((n_pos, max(n_neg, 1)), dtype=torch.int32, device=self.dev)
        self.neg_side = torch.empty((n_pos, max(n_neg, 1)), dtype=torch.uint8, device=self.dev)
        self.scores = (torch.empty((n_pos, 1 + n_neg), dtype=torch.float32, device=self.dev)
                       if self.keep_scores else None)
        self.index = (kb.ScoreIndex(self.part, max(n_pos, 1), self.n_neg, self.H_out.shape[1])
                      if self.want_index else None)

    def stage_batches(self, batches):
        """Copy several mini-batches (equal-length index arrays) to the device ahead of a loop; returns the
        tensor [n_batches, n_pos] whose rows `use_batch` takes."""
        torch = self.torch
        return torch.from_numpy(np.ascontiguousarray(np.stack(batches), np.int32)).to(self.dev)

    def use_batch(self, pos_dev):
        """Switch to another mini-batch of the size set_batch was given (a device tensor; nothing is allocated)."""
        assert pos_dev.numel() == self.pos.numel() and pos_dev.dtype == self.pos.dtype
        self.pos = pos_dev

    def view(self, which: int, layer: int):
        """Torch view [N, width] of one intermediate inside the workspace (see kge_workspace_slice)."""
        torch = self.torch
        off, nbytes = kb.workspace_slice(self.part, self.layers, which, layer, self.msg_dtype)
        raw = self.workspace[off:off + nbytes]
        bf = self.msg_dtype == kb.MSG_BF16 and which in (kb.WS_P, kb.WS_DP, kb.WS_Z, kb.WS_U)
        t = raw.view(torch.bfloat16 if bf else torch.float32)
        if which == kb.WS_U:          # flat: the caller reshapes to [S, d_out] (u) or [S, d_in] (dz)
            return t
        return t.view(self.part.n_seg if which == kb.WS_Z else self.part.n_vert, -1)

    # --- the four per-step calls, in Algorithm 1's order
    def compute_graph(self, stream=None):
        if self.cg is not None:
            kb.compute_graph(self.part, self.cg, self.pos, self.neg_ent if self.n_neg > 0 else None, stream)

    def forward(self, stream=None):
        kb.rgcn_forward(self.part, self.layers, self.H0, self.workspace, self.H_out, self.msg_dtype, stream,
                        self.cg)

    def sample(self, mode: int, seed: int, step: int, stream=None):
        kb.sample_negatives(self.part, self.pos, self.n_neg, mode, seed, step, self.neg_ent, self.neg_side, stream)

    def score_loss(self, stream=None):
        kb.distmult_score_loss(self.part, self.H_out, self.M, self.pos, self.neg_ent, self.neg_side,
                               self.n_neg, self.scores, self.loss, self.dH_out, self.dM, stream, self.index)

    def backward(self, stream=None):
        kb.rgcn_backward(self.part, self.layers, self.H0, self.workspace, self.dH_out, self.grads,
                         self.dH0, self.msg_dtype, stream, self.cg)

    def set_dropout_state(self, seed: int, step: int):
        """Seed and step of the dropout masks (Sec. 4 training setting); forward and backward of one
        step must see the same pair."""
        for lay in self.layers:
            lay["drop_seed"], lay["drop_step"] = int(seed), int(step)

    def run(self, mode: int, seed: int, step: int, stream=None):
        self.set_dropout_state(seed, step)
        self.sample(mode, seed, step, stream)
        self.compute_graph(stream)
        self.forward(stream)
        self.score_loss(stream)
        self.backward(stream)

    # --- Algorithm 1, "optimizer.step()": every parameter the step has a gradient for
    def optimizer_step(self, kind: int = kb.OPT_ADAM, lr: float = 0.01, beta1: float = 0.9, beta2: float = 0.999,
                       eps: float = 1e-8, stream=None):
        if not hasattr(self, "opt_t"):
            self.init_optimizer(kind)
        self.opt_t += 1
        # the entity table: only the rows the step read (flags of the sub-graph's input rows; without a
        # sub-graph the kernel skips rows whose gradient is all zero)
        mask = self.cg.input_rows_ptr() if self.cg is not None else None
        for name, p, g, rows in self._opt_pairs():
            m, v = self.opt_state.get(name, (None, None)) if kind == kb.OPT_ADAM else (None, None)
            kb.optimizer_step(kind, p, g, m, v, lr, beta1, beta2, eps, self.opt_t, rows=rows,
                              row_mask=mask if rows else None, stream=stream)

    def _opt_pairs(self):
        pairs = [("M", self.M, self.dM, False)]
        for l, (lay, g) in enumerate(zip(self.layers, self.grads)):
            pairs += [("V%d" % l, lay["V"], g["dV"], False), ("a%d" % l, lay["a"], g["da"], False),
                      ("W0%d" % l, lay["W0"], g["dW0"], False)]
        if self.dH0 is not None:
            pairs.append(("H0", self.H0, self.dH0, True))      # entity embeddings: only rows the step reached
        return pairs

    def init_optimizer(self, kind: int = kb.OPT_ADAM):
        """Allocate (zeroed) Adam moments for every parameter, so that no step allocates."""
        self.opt_t = 0
        self.opt_state = {}
        if kind == kb.OPT_ADAM:
            for name, p, _, _ in self._opt_pairs():
                self.opt_state[name] = (self.torch.zeros_like(p), self.torch.zeros_like(p))
