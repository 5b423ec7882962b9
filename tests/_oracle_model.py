"""The CPU oracle's functions chained into one training step of LR / FM / W&D / DeepFM (test
infrastructure only).  Between stages every tensor is rounded to fp32 once, because that is the
precision in which the library's boundary hands tensors from one call to the next."""
from __future__ import annotations

import numpy as np

f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)

COMPONENTS = {"lr": ("lr",), "fm": ("lr", "fm"), "wd": ("lr", "dnn"), "deepfm": ("lr", "fm", "dnn"),
              "dcn": ("cross", "dnn")}


class OracleModel:
    def __init__(self, oracle, table, F, K, kind, tower, opt_sparse, opt_dense, policy=0):
        """`tower`: dict from synth.tower_init (copied); opt_*: dicts of optimizer fields."""
        self.o, self.t, self.F, self.K, self.policy = oracle, table, F, K, policy
        self.parts = COMPONENTS[kind]
        self.p = {k: v.copy() for k, v in tower.items()}
        self.s1 = {k: np.zeros_like(v) for k, v in tower.items()}
        self.s2 = {k: np.zeros_like(v) for k, v in tower.items()}
        self.opt_sparse, self.opt_dense = dict(opt_sparse), dict(opt_dense)
        self.step_no = 0

    def forward(self, batch, rows, labels):
        o, t, p, F, K = self.o, self.t, self.p, self.F, self.K
        B, D = batch.B, t.D
        c = {}
        P = t.partial_forward(B, F, batch.keys, batch.offsets, rows, K, self.policy, batch.vals, pool=False)
        c["A_lr"] = f32(o.aggregate(P["P_lr"])) if "lr" in self.parts else None
        c["A_sum"] = f32(o.aggregate(P["P_sum"]))
        c["fm2"] = f32(o.fm_finalize(o.aggregate(P["P_sum"]), o.aggregate(P["P_sq"]))) if "fm" in self.parts else None
        if "dnn" in self.parts:
            pool = t.partial_forward(B, F, batch.keys, batch.offsets, rows, 1, self.policy, batch.vals,
                                     lr=False, fm=False, pool=True)["P_pool"][0]
            c["pool"] = f32(pool)
            n_layers = sum(1 for k in p if k[0] == "W")
            x, c["a"] = c["pool"], []
            for i in range(n_layers):
                Y = o.aggregate(o.dnn_partial_forward(x, p[f"W{i + 1}"], K if i == 0 else 1))
                c["a"].append(f32(o.bias_act(Y, p[f"b{i + 1}"], True)))
                x = c["a"][i][:, None, :]
        if "cross" in self.parts:
            # cross network on x0 = pool; its result enters the logit through one more sharded dot product
            n_cross = sum(1 for k in p if k.startswith("cw"))
            c["xs"], c["cs"] = [c["pool"]], []
            for l in range(n_cross):
                s = f32(o.aggregate(o.cross_partial(c["xs"][l], p[f"cw{l + 1}"], K)))
                c["cs"].append(s)
                c["xs"].append(f32(o.cross_apply(c["pool"], c["xs"][l], s, p[f"cb{l + 1}"])))
            c["cs"].append(f32(o.aggregate(o.cross_partial(c["xs"][-1], p["w_cross"], K))))
            c["A_lr"] = c["cs"][-1]                      # an additive term of the logit, like the first-order sum
        c["head"] = o.head(labels, c["A_lr"], c["fm2"], c["a"][-1] if "dnn" in self.parts else None,
                           p["w_out"] if "dnn" in self.parts else None, float(p["b0"][0]))
        return c

    def loss(self, batch, rows, labels):
        return self.forward(batch, rows, labels)["head"]["loss"]

    def gradients(self, batch, rows, labels):
        """Forward cache plus dense gradients (float64) and the upstream gradients of the sparse path."""
        o, p = self.o, self.p
        c = self.forward(batch, rows, labels)
        h = c["head"]
        g = {"b0": np.array([h["db0"]])}
        c["g_logit"] = f32(h["g_logit"])
        c["g_pool"] = None
        if "dnn" in self.parts:
            g["w_out"] = h["dw_out"]
            da = f32(h["da"])
            for i in range(len(c["a"]) - 1, -1, -1):
                dZ, g[f"b{i + 1}"] = o.bias_act_backward(c["a"][i], da, True)
                x = c["a"][i - 1][:, None, :] if i > 0 else c["pool"]
                dx, g[f"W{i + 1}"] = o.dnn_backward(x, p[f"W{i + 1}"], f32(dZ))
                da = f32(dx[:, 0, :]) if i > 0 else None
                if i == 0:
                    c["g_pool"] = f32(dx)
        if "cross" in self.parts:
            n_cross = len(c["xs"]) - 1
            gx, g["w_cross"] = o.cross_partial_backward(c["xs"][-1], p["w_cross"], c["g_logit"])
            gx = f32(gx)
            g_pool = c["g_pool"]                          # fp32: what the tower's backward left
            for l in range(n_cross - 1, -1, -1):
                _, g_xl, g_x0, g[f"cw{l + 1}"], g[f"cb{l + 1}"] = o.cross_backward(c["pool"], c["xs"][l], p[f"cw{l + 1}"],
                                                                                 c["cs"][l], gx)
                share = g_x0 + (g_xl if l == 0 else 0.0)  # the first layer's input is x0 itself
                g_pool = f32(g_pool.astype(np.float64) + share)
                gx = f32(g_xl)
            c["g_pool"] = g_pool
        c["dense_grads"] = g
        return c

    def train_step(self, batch, labels, insert=True):
        o, t = self.o, self.t
        self.step_no += 1
        rows = t.find(batch.keys, insert_missing=insert)
        c = self.gradients(batch, rows, labels)
        gl = c["g_logit"]
        sp = o.Optimizer(**dict(self.opt_sparse, step=self.step_no))
        c["merge"] = t.backward_update(batch.B, self.F, batch.offsets, rows,
                                       gl if "lr" in self.parts else None,
                                       gl if "fm" in self.parts else None,
                                       c["A_sum"] if "fm" in self.parts else None,
                                       c["g_pool"], vals=batch.vals, optimizer=sp)
        dn = o.Optimizer(**dict(self.opt_dense, step=self.step_no))
        for k, grad in c["dense_grads"].items():
            o.dense_update(self.p[k], f32(grad), dn, self.s1[k], self.s2[k])
        c["rows"] = rows
        return c
