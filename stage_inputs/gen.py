"""Seeded synthetic tensors for the stage workloads (inputs only, no method arithmetic).

Every tensor is drawn from its own Philox counter stream keyed by (stage seed, stream id),
so any tensor can be regenerated alone.  Shapes follow the PyTorch conventions: activations
NCHW, conv weights OIHW, linear weights [out][in].  For bf16 stages the drawn fp32 values
are snapped to the nearest bf16-representable number so that the CPU oracle and the GPU
library start from identical values.
"""
import numpy as np

from . import configs as C

_S_INPUT, _S_GRAD, _S_LABEL, _S_PARAM = 1000, 2000, 3000, 10


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, int(stream)]))


def snap_bf16(a):
    """Nearest (ties to even) bf16-representable value of each finite fp32 element, as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _snap(stage, a):
    a = a.astype(np.float32)
    return snap_bf16(a) if stage["dtype"] == C.BF16 else a


def stage_input(stage, mb):
    shp = (stage["micro_batch"], stage["in_c"], stage["in_h"], stage["in_w"])
    return _snap(stage, _rng(stage["seed"], _S_INPUT + mb).standard_normal(shp, dtype=np.float32))


def output_shape(stage):
    return C.infer_shapes(stage)[-1]


def ends_in_loss(stage):
    return stage["layers"][-1]["kind"] == C.SOFTMAX_XENT


def upstream_grad(stage, mb):
    """N(0,1) gradient w.r.t. the stage output (NCHW) for micro-batch mb."""
    o = output_shape(stage)
    shp = (stage["micro_batch"],) + tuple(o)
    return _snap(stage, _rng(stage["seed"], _S_GRAD + mb).standard_normal(shp, dtype=np.float32))


def labels(stage, mb):
    classes = output_shape(stage)[0]
    return _rng(stage["seed"], _S_LABEL + mb).integers(0, classes, size=stage["micro_batch"],
                                                        dtype=np.int32)


def layer_params(stage, idx, perturb=False):
    """(w, b) fp32 master parameters of layer idx, or (None, None) if it has none.

    conv: Kaiming-normal std sqrt(2/fan_in), fan_in = cin*kh*kw ('kaiming' stages) ;
    linear: Xavier-uniform bound sqrt(6/(fan_in+fan_out)) ('xavier' stages) ;
    lstm: w [4*hidden][cin+hidden] and (perturbed) bias uniform in +-1/sqrt(hidden) ;
    batchnorm: w = gamma = 1, b = beta = 0 ; biases 0.
    perturb=True draws biases/beta ~ 0.1*N(0,1) and gamma ~ 1 + 0.1*N(0,1) instead, so that
    tests can see a dropped bias or scale term."""
    L = stage["layers"][idx]
    k = L["kind"]
    r = _rng(stage["seed"], _S_PARAM + 2 * idx)
    rb = _rng(stage["seed"], _S_PARAM + 2 * idx + 1)
    if k == C.CONV2D:
        shp = (L["cout"], L["cin"], L["kh"], L["kw"])
        fan_in = L["cin"] * L["kh"] * L["kw"]
        fan_out = L["cout"] * L["kh"] * L["kw"]
    elif k == C.LINEAR:
        shp = (L["cout"], L["cin"])
        fan_in, fan_out = L["cin"], L["cout"]
    elif k == C.LSTM:
        hd = L["cout"]
        bound = 1.0 / np.sqrt(hd)
        w = r.uniform(-bound, bound, size=(4 * hd, L["cin"] + hd)).astype(np.float32)
        b = np.zeros(4 * hd, np.float32)
        if perturb:
            b = rb.uniform(-bound, bound, size=4 * hd).astype(np.float32)
        return w, b
    elif k == C.BATCHNORM2D:
        g = np.ones(L["cout"], np.float32)
        b = np.zeros(L["cout"], np.float32)
        if perturb:
            g = (1.0 + 0.1 * r.standard_normal(L["cout"])).astype(np.float32)
            b = (0.1 * rb.standard_normal(L["cout"])).astype(np.float32)
        return g, b
    else:
        return None, None
    if stage["init"] == "xavier":
        bound = np.sqrt(6.0 / (fan_in + fan_out))
        w = r.uniform(-bound, bound, size=shp).astype(np.float32)
    else:
        w = (r.standard_normal(shp, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in)))
    b = None
    if L["has_bias"]:
        b = np.zeros(L["cout"], np.float32)
        if perturb:
            b = (0.1 * rb.standard_normal(L["cout"])).astype(np.float32)
    return w.astype(np.float32), b


def all_params(stage, perturb=False):
    return [layer_params(stage, i, perturb) for i in range(len(stage["layers"]))]


def default_loss_scale(stage):
    """1 / (micro_batch * M): the sum over micro-batches is the mini-batch mean."""
    return 1.0 / (stage["micro_batch"] * stage["n_micro"])
