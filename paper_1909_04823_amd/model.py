"""One training step of LR / FM / W&D / DeepFM / DCN under DES on one MI355X, as a sequence of library calls.

Nothing is computed here: every tensor operation is a call into libdes (``des.py``); this module only
owns the device buffers and fixes the order of the calls --

    find -> partial_forward -> aggregate x3, fm_finalize                    (sparse operators, Sections 4.1-4.2, 5)
         -> dnn_partial_forward -> aggregate_bias_act -> dense layer -> head  (Section 4.3, tower, output unit)
         -> head backward -> tower backward -> dnn_backward -> backward_update -> dense_update

Model kinds follow the paper's table of shared components (Section 4): "lr" first order; "fm" first and
second order; "wd" first and high order; "deepfm" all three.  "dcn" (Section 4, the paragraph on DCN) puts a
cross network x_{l+1} = x_0 (x_l^T w_l) + b_l + x_l beside the tower, both on the pooled embeddings x_0; every
dot product over the d = F*D columns, the output unit's on the network's result included, is a DES
sub-operator (per-shard scalars, summed):

    pool -> [cross_partial -> aggregate -> cross_apply] x n -> cross_partial -> aggregate  (one logit term)

or, by default, all of them at once (cross_net_partial -> aggregate -> cross_net_forward): the layers only ever
add multiples of x_0 and biases, so the network needs one pass over x_0 for all its dot products.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import des

COMPONENTS = {"lr": ("lr",), "fm": ("lr", "fm"), "wd": ("lr", "dnn"), "deepfm": ("lr", "fm", "dnn"),
              "dcn": ("cross", "dnn")}


class Model:
    def __init__(self, table: des.Table, F: int, kind: str, tower: Optional[Dict[str, np.ndarray]], B_max: int,
                 opt_sparse: dict, opt_dense: dict, cross_fused: bool = True):
        """`table`: a des.Table whose state arrays fit `opt_sparse`; `tower`: initial dense parameters as numpy
        arrays -- W1[F*D,H1], b1[H1] (the layer under DES), W2[H1,H2], b2, ... Wn, bn (n >= 1 hidden layers),
        w_out[Hn], b0[1]; for "dcn" also cw1[d], cb1[d], ... (cross layers) and w_cross[d]; opt_*:
        des_optimizer_t fields."""
        self.t, self.F, self.D, self.K = table, int(F), table.dim, table.K
        self.parts = COMPONENTS[kind]
        self.opt_sparse, self.opt_dense = dict(opt_sparse), dict(opt_dense)
        self.step_no = 0
        self._aux = None
        dev = table.emb.device
        f = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
        z = lambda *shape: torch.zeros(shape, dtype=torch.float32, device=dev)
        B, D, K = int(B_max), self.D, self.K
        self.B_max = B
        self.P_lr, self.P_sum, self.P_sq = f(K, B), f(K, B, D), f(K, B)
        self.A_lr, self.A_sum, self.A_sq, self.fm2 = f(B), f(B, D), f(B), f(B)
        self.logit, self.p, self.g_logit, self.loss, self.db0 = f(B), f(B), f(B), f(1), f(1)
        self.n_uniq = torch.zeros(1, dtype=torch.int64, device=dev)
        self.rows = torch.empty(table.max_n, dtype=torch.int32, device=dev)
        self.dnn = "dnn" in self.parts
        H_max = 4
        self.grads = {}
        if self.dnn:
            self.params = {k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(dev) for k, v in tower.items()}
            if "cross" in self.parts:
                # the cross network's vectors side by side, U = [cw1 .. cwn, w_cross] and bias = [cb1 .. cbn]; the
                # per-parameter tensors are rows of these blocks, and so are their gradients
                n_cross = sum(1 for k in self.params if k.startswith("cw"))
                names = [f"cw{l + 1}" for l in range(n_cross)] + ["w_cross"]
                self.cU = torch.stack([self.params[k] for k in names]).contiguous()
                self.cB = torch.stack([self.params[f"cb{l + 1}"] for l in range(n_cross)]).contiguous() if n_cross else None
                self.dU = torch.empty_like(self.cU)
                self.dB = torch.empty_like(self.cB) if n_cross else None
                for i, k in enumerate(names):
                    self.params[k], self.grads[k] = self.cU[i], self.dU[i]
                for l in range(n_cross):
                    self.params[f"cb{l + 1}"], self.grads[f"cb{l + 1}"] = self.cB[l], self.dB[l]
            self.n_layers = sum(1 for k in self.params if k[0] == "W")
            self.H = [self.params[f"W{i + 1}"].shape[1] for i in range(self.n_layers)]       # widths H1..Hn
            H_max = max(self.H)
            self.pool, self.g_pool = f(B, F, D), f(B, F, D)
            # per layer i: partials Y (K shards for the first layer, one otherwise), activations a, their gradient da
            self.Yp = [f(K if i == 0 else 1, B, h) for i, h in enumerate(self.H)]
            self.a = [f(B, h) for h in self.H]
            self.da = [f(B, h) for h in self.H]
            ws_bytes = des.dnn_backward_bytes(B, F, D, self.H[0])
            for i in range(1, self.n_layers):
                ws_bytes = max(ws_bytes, des.dnn_backward_bytes(B, 1, self.H[i - 1], self.H[i]))
            self.dnn_ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            self.cross = "cross" in self.parts
            if self.cross:
                d = F * D
                self.n_cross = sum(1 for k in self.params if k.startswith("cw"))
                self.cross_fused = bool(cross_fused)
                self.cs = [f(B) for _ in range(self.n_cross + 1)]                       # aggregated scalars; last: logit term
                if self.cross_fused:
                    m = self.n_cross + 1
                    self.cP, self.ct, self.cgamma = f(K, B, m), f(B, m), f(B, m)
                    self.cross_ws = torch.empty(des.cross_net_bytes(B, d, self.n_cross), dtype=torch.uint8, device=dev)
                else:
                    self.xs = [self.pool] + [f(B, F, D) for _ in range(self.n_cross)]  # inputs of the cross layers, result
                    self.cP = f(K, B)
                    self.g_x = f(B, F, D)
                    self.cross_ws = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device=dev)
        else:
            self.cross = False
            self.params = {"b0": torch.from_numpy(np.ascontiguousarray(tower["b0"] if tower else np.zeros(1), dtype=np.float32)).to(dev)}
        for k, v in self.params.items():
            if k not in self.grads:
                self.grads[k] = torch.empty_like(v)
        self.s1 = {k: torch.zeros_like(v) for k, v in self.params.items()}
        self.s2 = {k: torch.zeros_like(v) for k, v in self.params.items()}
        self.ws = torch.empty(des.dense_workspace_bytes(H_max), dtype=torch.uint8, device=dev)

    # ------------------------------------------------------------------------------------------
    def forward(self, batch: des.Batch, rows: torch.Tensor, labels: torch.Tensor, backward_head: bool = True):
        """Forward pass and the output unit's gradients for `batch` (B <= B_max); returns views."""
        B, F, D = batch.B, self.F, self.D
        if B != self.B_max:
            raise ValueError("this driver keeps fixed-size buffers: batch.B must equal B_max")
        p = self.params
        fm = "fm" in self.parts
        self.t.partial_forward(batch, rows, self.P_lr, self.P_sum if fm else None, self.P_sq if fm else None,
                               self.pool if self.dnn else None)
        if fm:
            des.aggregate_forward(self.P_lr, self.P_sum, self.P_sq, self.A_lr, self.A_sum, self.A_sq, self.fm2)
        else:
            des.aggregate_forward(self.P_lr, None, None, self.A_lr)
        if self.dnn:
            x = self.pool                                   # [B, F, D]: the first layer is cut over the fields
            for i in range(self.n_layers):
                des.dnn_partial_forward(x, p[f"W{i + 1}"], self.K if i == 0 else 1, out=self.Yp[i])
                des.aggregate_bias_act(self.Yp[i], p[f"b{i + 1}"], True, self.a[i])
                x = self.a[i].view(B, 1, self.H[i])
        if self.cross and self.cross_fused:
            des.cross_net_partial(self.pool, self.cU, self.K, out=self.cP)
            des.aggregate_partials(self.cP.view(self.K, -1), self.ct.view(-1))
            des.cross_net_forward(self.ct, self.cU, self.cB, self.cgamma, self.cs[-1], self.cross_ws)
        elif self.cross:
            for l in range(self.n_cross):
                des.cross_partial(self.xs[l], p[f"cw{l + 1}"], self.K, out=self.cP)
                des.aggregate_partials(self.cP, self.cs[l])
                des.cross_apply(self.pool, self.xs[l], self.cs[l], p[f"cb{l + 1}"], out=self.xs[l + 1])
            des.cross_partial(self.xs[-1], p["w_cross"], self.K, out=self.cP)
            des.aggregate_partials(self.cP, self.cs[-1])
        des.head(labels, self.g_logit, self.ws,
                 A_lr=self.A_lr if "lr" in self.parts else (self.cs[-1] if self.cross else None),
                 fm2=self.fm2 if "fm" in self.parts else None,
                 a=self.a[-1] if self.dnn else None, w_out=p["w_out"] if self.dnn else None, b0=p["b0"],
                 logit=self.logit, p=self.p, loss=self.loss,
                 da=self.da[-1] if (self.dnn and backward_head) else None,
                 dw_out=self.grads["w_out"] if (self.dnn and backward_head) else None,
                 db0=self.grads["b0"])
        return self.loss

    def backward(self, batch: des.Batch, rows: torch.Tensor, dbg: Optional[dict] = None):
        """Tower backward, sparse backward + update, dense update.  Call after forward()."""
        self.backward_tower(batch)
        self.update(batch, rows, dbg)

    def backward_tower(self, batch: des.Batch):
        """Gradients of the dense parameters (self.grads) and of the pooled embeddings (self.g_pool)."""
        p, g = self.params, self.grads
        B = batch.B
        if self.dnn:
            for i in range(self.n_layers - 1, -1, -1):
                # da[i] becomes dZ[i] in place; then the layer's input gradient and weight gradient
                des.bias_act_backward(self.a[i], self.da[i], True, self.da[i], g[f"b{i + 1}"], self.ws)
                if i > 0:
                    des.dnn_backward(self.a[i - 1].view(B, 1, self.H[i - 1]), p[f"W{i + 1}"], self.da[i],
                                     self.da[i - 1].view(B, 1, self.H[i - 1]), g[f"W{i + 1}"], self.dnn_ws)
                else:
                    des.dnn_backward(self.pool, p["W1"], self.da[0], self.g_pool, g["W1"], self.dnn_ws)
        if self.cross and self.cross_fused:
            # added to what the tower left in g_pool
            des.cross_net_backward(self.pool, self.cU, self.cB, self.ct, self.cgamma, self.g_logit, self.g_pool, True,
                                   self.dU, self.dB, self.cross_ws)
        elif self.cross:
            # the cross network's result is a term of the logit; then layer by layer, every layer adding its share of
            # the gradient of x0 = pool to what the tower left in g_pool (the first layer's input gradient too)
            des.cross_partial_backward(self.xs[-1], p["w_cross"], self.g_logit, self.g_x, g["w_cross"], self.cross_ws)
            for l in range(self.n_cross - 1, -1, -1):
                des.cross_backward(self.pool, self.xs[l], p[f"cw{l + 1}"], self.cs[l], self.g_x,
                                   self.g_x if l > 0 else None, self.g_pool, True, g[f"cw{l + 1}"], g[f"cb{l + 1}"],
                                   self.cross_ws)

    def update(self, batch: des.Batch, rows: torch.Tensor, dbg: Optional[dict] = None):
        """Sparse backward with merge and row update, then the dense optimizer step."""
        g = self.grads
        self.step_no += 1
        sp = des.Optimizer(**dict(self.opt_sparse, step=self.step_no))
        gl = self.g_logit
        self.t.backward_update(batch, rows, sp,
                               g_lr=gl if "lr" in self.parts else None,
                               g_fm=gl if "fm" in self.parts else None,
                               A_sum=self.A_sum if "fm" in self.parts else None,
                               g_pool=self.g_pool if self.dnn else None,
                               dbg=dbg if dbg is not None else {"n_uniq": self.n_uniq})
        dn = des.Optimizer(**dict(self.opt_dense, step=self.step_no))
        for k in self.params:
            des.dense_update(self.params[k], g[k], dn, self.s1[k], self.s2[k])

    def train_step(self, batch: des.Batch, labels: torch.Tensor, insert: bool = True, overlap: bool = True):
        """find -> forward -> backward -> updates.  With `overlap` the row-sorting half of the sparse backward
        pass (des_backward_prepare, which needs only the rows) is issued on a second stream of default
        priority right after the lookup, so it runs beside the forward pass and the tower's matrix products."""
        rows = self.rows[:batch.nnz]
        self.t.find(batch.keys, des.MISS_INSERT if insert else des.MISS_ZERO, rows)
        if overlap:
            if self._aux is None:
                self._aux = torch.cuda.Stream()
                self._found, self._sorted = torch.cuda.Event(), torch.cuda.Event()
            main = torch.cuda.current_stream()
            self._found.record(main)
            self._aux.wait_event(self._found)
            with torch.cuda.stream(self._aux):
                self.t.backward_prepare(batch, rows)
                self._sorted.record(self._aux)
        self.forward(batch, rows, labels)
        self.backward_tower(batch)
        if overlap:
            torch.cuda.current_stream().wait_event(self._sorted)
        self.update(batch, rows)
        return self.loss


def auc(labels: np.ndarray, scores: np.ndarray) -> float:
    """Area under the ROC curve from host copies of labels and predictions (rank statistic with
    ties sharing their mean rank).  An evaluation metric for reports, not part of the training path."""
    labels = np.asarray(labels) > 0.5
    scores = np.asarray(scores, dtype=np.float64)
    order = np.argsort(scores, kind="stable")
    s = scores[order]
    ranks = np.empty(s.size, dtype=np.float64)
    i = 0
    bounds = np.flatnonzero(np.concatenate([[True], s[1:] != s[:-1], [True]]))
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        ranks[lo:hi] = 0.5 * (lo + hi - 1) + 1.0
    r = np.empty_like(ranks); r[order] = ranks
    n_pos, n_neg = int(labels.sum()), int((~labels).sum())
    if n_pos == 0 or n_neg == 0:
        return float("nan")
    return float((r[labels].sum() - n_pos * (n_pos + 1) / 2.0) / (n_pos * n_neg))
