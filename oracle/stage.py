"""CPU oracle of one pipeline stage: forward / backward per micro-batch, gradient
accumulation over the M micro-batches of a mini-batch, one SGD update per mini-batch.

TEST INFRASTRUCTURE ONLY (see bapipe_oracle.c).  Follows the paper's stage semantics
(Sec. II-B, III-B-1): the forward and backward pass of a micro-batch use the same weights,
backward of a micro-batch needs the features its forward produced (kept here per in-flight
micro-batch, at most N-i+1 of them under 1F1B, Table I/II "Features memory"), and weights
change once, after the backward passes of the whole mini-batch.

storage="bf16" applies nearest-even bf16 rounding exactly where a tensor would be stored in
16 bits: each layer's output in forward (conv/linear/BN/add after bias and ReLU, average pool), each
input-gradient contribution in backward and their sum where a tensor feeds two layers, and
the working copy of conv/linear weight matrices.  Bias, gamma, beta, weight gradients,
BN statistics, softmax and loss are never rounded.  Inside an LSTM layer the input projection
of all steps and the pre-activation gradients are stored tensors too (rounded); the cell state
and the recurrent sums are not.  storage="exact" rounds nothing.
"""
import numpy as np

from stage_inputs import configs as C

from . import ops


class ScheduleError(Exception):
    pass


class OracleStage:
    def __init__(self, stage, params, storage=None, loss_scale=None, depth=None):
        self.stage = stage
        self.layers = stage["layers"]
        self.shapes = C.infer_shapes(stage)
        if storage is None:
            storage = "bf16" if stage["dtype"] == C.BF16 else "exact"
        assert storage in ("bf16", "exact")
        self.storage = storage
        self.q = ops.round_bf16 if storage == "bf16" else (lambda a: a)
        self.M = stage["n_micro"]
        i, N = stage["stage_index"], stage["n_stages"]
        mult = 2 if stage.get("schedule", C.SCHED_1F1B) == C.SCHED_1F1B_SO else 1
        self.depth = depth if depth is not None else min(self.M, mult * (N - i + 1))
        self.loss_scale = (1.0 / (stage["micro_batch"] * self.M)) if loss_scale is None else loss_scale
        self.w, self.b, self.dw, self.db = [], [], [], []
        for (w, b) in params:
            self.w.append(None if w is None else np.array(w, dtype=np.float64))
            self.b.append(None if b is None else np.array(b, dtype=np.float64))
            self.dw.append(None if w is None else np.zeros(w.shape))
            self.db.append(None if b is None else np.zeros(b.shape))
        self.stash = {}
        self.loss = {}
        self.trace = None          # set to {} to record, per (mb, layer), the masked output gradient and dx
        self.n_fwd = self.n_bwd = 0
        self.peak_in_flight = 0

    # ---- schedule bookkeeping -------------------------------------------------------
    def _claim(self, mb):
        if mb != self.n_fwd or mb >= self.M:
            raise ScheduleError("forward ids must be 0..M-1 ascending")
        if self.n_fwd - self.n_bwd >= self.depth:
            raise ScheduleError("stash depth exceeded")
        self.n_fwd += 1
        self.peak_in_flight = max(self.peak_in_flight, self.n_fwd - self.n_bwd)

    def _release(self, mb):
        if mb != self.n_bwd or mb >= self.n_fwd:
            raise ScheduleError("backward ids ascend and follow their forward")
        self.n_bwd += 1

    # ---- forward ------------------------------------------------------------------
    def forward(self, mb, x):
        self._claim(mb)
        q = self.q
        x = np.asarray(x, dtype=np.float64)
        outs, aux = [], []

        def src(t):
            return x if t < 0 else outs[t]

        for i, L in enumerate(self.layers):
            k = L["kind"]
            a = src(L["src0"])
            extra = None
            if k == C.CONV2D:
                y = ops.conv2d_fwd(a, q(self.w[i]), self.b[i], L["stride"], L["pad"])
                if L["fuse_relu"]:
                    y = ops.relu_fwd(y)
                y = q(y)
            elif k == C.RELU:
                y = ops.relu_fwd(a)
            elif k == C.MAXPOOL2D:
                y, extra = ops.maxpool_fwd(a, L["kh"], L["stride"], L["pad"])
            elif k == C.AVGPOOL2D:
                y = q(ops.avgpool_fwd(a, L["kh"]))
            elif k == C.BATCHNORM2D:
                y, mean, invstd = ops.bn_fwd(a, self.w[i], self.b[i], L["eps"])
                extra = (mean, invstd)
                if L["fuse_relu"]:
                    y = ops.relu_fwd(y)
                y = q(y)
            elif k == C.ADD:
                y = a + src(L["src1"])
                if L["fuse_relu"]:
                    y = ops.relu_fwd(y)
                y = q(y)
            elif k == C.FLATTEN:
                y = a.reshape(a.shape[0], -1, 1, 1)
            elif k == C.LINEAR:
                y = ops.linear_fwd(a.reshape(a.shape[0], -1), q(self.w[i]), self.b[i])
                if L["fuse_relu"]:
                    y = ops.relu_fwd(y)
                y = q(y).reshape(a.shape[0], -1, 1, 1)
            elif k == C.LSTM:
                y, extra = ops.lstm_fwd(a, q(self.w[i]), self.b[i], round16=self.storage == "bf16")
            elif k == C.SOFTMAX_XENT:
                y = ops.softmax_fwd(a.reshape(a.shape[0], -1)).reshape(a.shape)
            else:
                raise ValueError(k)
            outs.append(y)
            aux.append(extra)
        self.stash[mb] = (x, outs, aux)
        return outs[-1]

    # ---- backward -----------------------------------------------------------------
    def backward(self, mb, dy_or_labels):
        self._release(mb)
        q = self.q
        x, outs, aux = self.stash.pop(mb)
        need_in = bool(self.stage["need_input_grad"])
        G = {}

        def src(t):
            return x if t < 0 else outs[t]

        cur = [None]

        def give(t, c):
            if t < 0 and not need_in:
                return
            c = q(c)
            if self.trace is not None:
                self.trace[(mb, cur[0])]["dx"] = c
            G[t] = c if t not in G else q(G[t] + c)

        last = len(self.layers) - 1
        if self.layers[last]["kind"] != C.SOFTMAX_XENT:
            G[last] = np.asarray(dy_or_labels, dtype=np.float64)

        for i in range(last, -1, -1):
            L = self.layers[i]
            k = L["kind"]
            a = src(L["src0"])
            wants = L["src0"] >= 0 or need_in
            cur[0] = i
            if self.trace is not None:
                self.trace[(mb, i)] = {"x": a, "y": outs[i]}
            if k == C.SOFTMAX_XENT:
                z = a.reshape(a.shape[0], -1)
                loss, dz = ops.xent_bwd(z, dy_or_labels, self.loss_scale)
                self.loss[mb] = loss
                give(L["src0"], dz.reshape(a.shape))
                continue
            g = G.pop(i)
            if self.trace is not None:
                self.trace[(mb, i)]["gout"] = g      # total gradient of this layer's output, before its own gate
            if L["fuse_relu"] and k in (C.CONV2D, C.BATCHNORM2D, C.ADD, C.LINEAR):
                g = ops.relu_bwd(outs[i].reshape(g.shape), g)
            if self.trace is not None:
                self.trace[(mb, i)]["g"] = g
            if k == C.CONV2D:
                ops.conv2d_wgrad(a, g, self.dw[i], self.db[i], L["stride"], L["pad"])
                if wants:
                    give(L["src0"], ops.conv2d_dgrad(g, q(self.w[i]), a.shape, L["stride"], L["pad"]))
            elif k == C.RELU:
                give(L["src0"], ops.relu_bwd(outs[i], g))
            elif k == C.MAXPOOL2D:
                give(L["src0"], ops.maxpool_bwd(g, aux[i], a.shape, L["kh"], L["stride"], L["pad"]))
            elif k == C.AVGPOOL2D:
                give(L["src0"], ops.avgpool_bwd(g, a.shape, L["kh"]))
            elif k == C.BATCHNORM2D:
                mean, invstd = aux[i]
                dx = ops.bn_bwd(a, g, self.w[i], mean, invstd, self.dw[i], self.db[i])
                give(L["src0"], dx)
            elif k == C.ADD:
                give(L["src0"], g)
                give(L["src1"], g)
            elif k == C.FLATTEN:
                give(L["src0"], g.reshape(a.shape))
            elif k == C.LSTM:
                dx = ops.lstm_bwd(a, outs[i], q(self.w[i]), aux[i], g, self.dw[i], self.db[i], want_dx=wants,
                                  round16=self.storage == "bf16")
                if wants:
                    give(L["src0"], dx)
            elif k == C.LINEAR:
                a2 = a.reshape(a.shape[0], -1)
                g2 = g.reshape(g.shape[0], -1)
                ops.linear_wgrad(a2, g2, self.dw[i], self.db[i])
                if wants:
                    give(L["src0"], ops.linear_dgrad(g2, q(self.w[i])).reshape(a.shape))
            else:
                raise ValueError(k)
        return G.get(-1)

    # ---- update ---------------------------------------------------------------------
    def step(self, lr):
        if self.n_bwd != self.M:
            raise ScheduleError("step needs all M backward passes")
        for i in range(len(self.layers)):
            if self.w[i] is not None:
                ops.sgd_step(self.w[i], self.dw[i], lr)
                self.dw[i][...] = 0.0
            if self.b[i] is not None:
                ops.sgd_step(self.b[i], self.db[i], lr)
                self.db[i][...] = 0.0
        self.n_fwd = self.n_bwd = 0

    def pool_indices(self, mb, layer):
        return self.stash[mb][2][layer]


def one_f_one_b_order(M, depth):
    """[( 'F'|'B', mb )...]: depth warm-up forwards, then alternate B,F, then drain."""
    W = min(M, depth)
    order = [("F", m) for m in range(W)]
    for m in range(M - W):
        order += [("B", m), ("F", m + W)]
    order += [("B", m) for m in range(M - W, M)]
    return order
