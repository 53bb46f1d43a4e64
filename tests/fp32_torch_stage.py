"""A second, independent implementation of a bf16 stage for the CPU tests: PyTorch CPU ops in
float32 (library convolutions / matmuls with fp32 accumulation in the library's own blocked order)
with round-to-nearest-even bf16 rounding at the same points as the oracle's storage="bf16" mode -
layer outputs in forward, every input-gradient contribution and the sum at a fan-out in backward,
the working copy of the weight matrices.  It exists to answer one question on the CPU: how far apart
do two CORRECT implementations of the rounding-point contract end up, end to end, when they only
differ in the precision and order of their sums (fp32 here, fp64 in the oracle)?
Test infrastructure only; shares no code with the oracle or the HIP library."""
import numpy as np
import torch
import torch.nn.functional as F

from stage_inputs import configs as C


def _q(t):
    return t.to(torch.bfloat16).to(torch.float32)


class _RoundValue(torch.autograd.Function):
    """forward: round to bf16; backward: pass the gradient through unchanged"""
    @staticmethod
    def forward(ctx, t):
        return _q(t)

    @staticmethod
    def backward(ctx, g):
        return g


class _RoundGrad(torch.autograd.Function):
    """forward: identity; backward: round the gradient to bf16 (one stored gradient tensor)"""
    @staticmethod
    def forward(ctx, t):
        return t.view_as(t)

    @staticmethod
    def backward(ctx, g):
        return _q(g)


class Fp32TorchStage:
    """bug: None, or a deliberately planted mistake (to show that the acceptance test rejects it):
    "no_shortcut_grad" - the second input of every ADD receives no gradient;
    "gate_on_input"    - a fused ReLU's backward gates on the sign of the layer's INPUT sum's first
                         operand instead of the output (only for ADD layers)."""

    def __init__(self, stage, params, bug=None):
        self.stage, self.layers, self.bug = stage, stage["layers"], bug
        self.w = [None if w is None else torch.tensor(np.asarray(w, np.float32), requires_grad=True) for w, _ in params]
        self.b = [None if b is None else torch.tensor(np.asarray(b, np.float32), requires_grad=True) for _, b in params]
        self.scale = 1.0 / (stage["micro_batch"] * stage["n_micro"])
        self.loss = {}
        self._kept = {}

    def forward(self, mb, x):
        x = torch.tensor(np.asarray(x, np.float32), requires_grad=bool(self.stage["need_input_grad"]))
        outs = []

        def src(t):
            base = x if t < 0 else outs[t]
            return _RoundGrad.apply(base)             # this consumer's contribution is rounded on its own

        for i, L in enumerate(self.layers):
            k = L["kind"]
            a = src(L["src0"])
            relu = L["fuse_relu"]
            if k == C.CONV2D:
                y = F.conv2d(a, _RoundValue.apply(self.w[i]), self.b[i], stride=L["stride"], padding=L["pad"])
            elif k == C.RELU:
                y, relu = F.relu(a), 0
            elif k == C.MAXPOOL2D:
                y = F.max_pool2d(a, L["kh"], L["stride"], L["pad"])
            elif k == C.AVGPOOL2D:
                y = F.avg_pool2d(a, L["kh"])
            elif k == C.BATCHNORM2D:
                y = F.batch_norm(a, None, None, self.w[i], self.b[i], True, 0.0, L["eps"])
            elif k == C.ADD:
                b2 = src(L["src1"])
                if self.bug == "no_shortcut_grad":
                    b2 = b2.detach()
                y = a + b2
                if self.bug == "gate_on_input" and relu:
                    y, relu = torch.where(a > 0, y, torch.zeros_like(y)) * (y > 0), 0
            elif k == C.FLATTEN:
                y = a.reshape(a.shape[0], -1, 1, 1)
            elif k == C.LINEAR:
                y = F.linear(a.reshape(a.shape[0], -1), _RoundValue.apply(self.w[i]), self.b[i]).reshape(a.shape[0], -1, 1, 1)
            elif k == C.SOFTMAX_XENT:
                y = a                                  # logits; probabilities are taken below
            else:
                raise ValueError(k)
            if relu:
                y = F.relu(y)
            if k in (C.CONV2D, C.AVGPOOL2D, C.BATCHNORM2D, C.ADD, C.LINEAR):
                y = _RoundValue.apply(y)
            outs.append(_RoundGrad.apply(y))          # the sum of all consumers' contributions is rounded again
        self._kept[mb] = (x, outs)
        last = outs[-1]
        if self.layers[-1]["kind"] == C.SOFTMAX_XENT:
            return torch.softmax(last.reshape(last.shape[0], -1).detach().double(), 1).numpy().reshape(last.shape)
        return last.detach().double().numpy()

    def backward(self, mb, dy_or_labels):
        x, outs = self._kept.pop(mb)
        last = outs[-1]
        if self.layers[-1]["kind"] == C.SOFTMAX_XENT:
            z = last.reshape(last.shape[0], -1)
            loss = self.scale * F.cross_entropy(z, torch.tensor(np.asarray(dy_or_labels, np.int64)), reduction="sum")
            self.loss[mb] = float(loss)
            loss.backward()
        else:
            last.backward(torch.tensor(np.asarray(dy_or_labels, np.float32)))
        return None if x.grad is None else x.grad.double().numpy()

    def dw(self, i):
        return None if self.w[i] is None or self.w[i].grad is None else self.w[i].grad.double().numpy()

    def db(self, i):
        return None if self.b[i] is None or self.b[i].grad is None else self.b[i].grad.double().numpy()
