"""Stage workloads: layer lists and shapes only (no arithmetic of the method).

A pipeline stage is a contiguous run of layers placed on one accelerator
(paper Sec. I / III-A); each workload below is one such stage together with its
position (i, N) in the pipeline, micro-batch size and micro-batch count M.
Both the CPU oracle and the HIP library consume these descriptions; neither
imports the other.

A layer is a dict with the integer fields of the C descriptor:
  kind, cin, cout, kh, kw, stride, pad, has_bias, fuse_relu, src0, src1, eps
`src0`/`src1` name the producing layer (index in the list), -1 = stage input.
"""

CONV2D, RELU, MAXPOOL2D, BATCHNORM2D, ADD, FLATTEN, LINEAR, SOFTMAX_XENT, AVGPOOL2D, LSTM = range(10)
KIND_NAMES = ["conv2d", "relu", "maxpool2d", "batchnorm2d", "add", "flatten",
              "linear", "softmax_xent", "avgpool2d", "lstm"]

FP32, BF16 = 0, 1
SCHED_1F1B, SCHED_1F1B_SO = 0, 1


def _layer(kind, cin=0, cout=0, k=0, stride=1, pad=0, has_bias=0, fuse_relu=0,
           src0=None, src1=-1, eps=0.0):
    return dict(kind=kind, cin=cin, cout=cout, kh=k, kw=k, stride=stride, pad=pad,
                has_bias=has_bias, fuse_relu=fuse_relu, src0=src0, src1=src1, eps=eps)


class _Builder:
    def __init__(self):
        self.layers = []

    def add(self, **kw):
        L = _layer(**kw)
        if L["src0"] is None:
            L["src0"] = len(self.layers) - 1
        self.layers.append(L)
        return len(self.layers) - 1

    def conv(self, cin, cout, k, stride=1, pad=None, bias=1, relu=0, src=None):
        return self.add(kind=CONV2D, cin=cin, cout=cout, k=k, stride=stride,
                        pad=(k // 2 if pad is None else pad), has_bias=bias,
                        fuse_relu=relu, src0=src)

    def pool(self, src=None, k=2, stride=2, pad=0):
        return self.add(kind=MAXPOOL2D, k=k, stride=stride, pad=pad, src0=src)

    def avgpool(self, k, src=None):
        """k x k mean, stride k, no padding (k = feature-map size: global average pool)."""
        return self.add(kind=AVGPOOL2D, k=k, stride=k, pad=0, src0=src)

    def relu(self, src=None):
        return self.add(kind=RELU, src0=src)

    def bn(self, c, relu=0, eps=1e-5, src=None):
        return self.add(kind=BATCHNORM2D, cin=c, cout=c, has_bias=1, fuse_relu=relu,
                        eps=eps, src0=src)

    def addl(self, a, b, relu=1):
        return self.add(kind=ADD, fuse_relu=relu, src0=a, src1=b)

    def flatten(self, src=None):
        return self.add(kind=FLATTEN, src0=src)

    def linear(self, cin, cout, relu=0, src=None):
        return self.add(kind=LINEAR, cin=cin, cout=cout, has_bias=1, fuse_relu=relu, src0=src)

    def lstm(self, cin, hidden, src=None):
        """LSTM over the H axis of a (cin, T, 1) tensor -> (hidden, T, 1); w [4*hidden][cin+hidden]."""
        return self.add(kind=LSTM, cin=cin, cout=hidden, has_bias=1, src0=src)

    def xent(self, src=None):
        return self.add(kind=SOFTMAX_XENT, src0=src)


def _stage(name, layers, dtype, in_chw, micro_batch, n_micro, stage_index, n_stages,
           need_input_grad, seed, init):
    return dict(name=name, layers=layers, dtype=dtype, in_c=in_chw[0], in_h=in_chw[1],
                in_w=in_chw[2], micro_batch=micro_batch, n_micro=n_micro,
                stage_index=stage_index, n_stages=n_stages, schedule=SCHED_1F1B,
                need_input_grad=need_input_grad, seed=seed, init=init)


BASE_SEED = 0x20121254


def tiny_stage(c=16, hw=32, micro_batch=4, n_micro=4, dtype=FP32, fused=True, cin=3):
    """conv3x3 cin->c +b+ReLU, conv3x3 c->c +b+ReLU, 2x2 maxpool (first stage of 2)."""
    b = _Builder()
    if fused:
        b.conv(cin, c, 3, relu=1, src=-1)
        b.conv(c, c, 3, relu=1)
    else:
        b.conv(cin, c, 3, relu=0, src=-1)
        b.relu()
        b.conv(c, c, 3, relu=0)
        b.relu()
    b.pool()
    return _stage("tiny", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 1, 2, 0,
                  BASE_SEED + 1, "kaiming")


def vgg16_stage1(c1=64, c2=128, hw=224, micro_batch=32, n_micro=8, dtype=BF16, cin=3):
    """conv1_1, conv1_2, pool, conv2_1, conv2_2, pool: stage 1 of a 4-way VGG-16 split."""
    b = _Builder()
    b.conv(cin, c1, 3, relu=1, src=-1)
    b.conv(c1, c1, 3, relu=1)
    b.pool()
    b.conv(c1, c2, 3, relu=1)
    b.conv(c2, c2, 3, relu=1)
    b.pool()
    return _stage("vgg16_stage1", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 1, 4, 0,
                  BASE_SEED + 2, "kaiming")


def vgg16_deep(cin=256, c=512, hw=28, micro_batch=64, n_micro=8, dtype=BF16):
    """conv4_1..4_3 at hw, pool, conv5_1..5_3 at hw/2, pool: stage 3 of 4."""
    b = _Builder()
    b.conv(cin, c, 3, relu=1, src=-1)
    b.conv(c, c, 3, relu=1)
    b.conv(c, c, 3, relu=1)
    b.pool()
    b.conv(c, c, 3, relu=1)
    b.conv(c, c, 3, relu=1)
    b.conv(c, c, 3, relu=1)
    b.pool()
    return _stage("vgg16_deep", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 3, 4, 1,
                  BASE_SEED + 3, "kaiming")


def vgg16_classifier(c=512, hw=7, hidden=4096, classes=1000, micro_batch=64, n_micro=16,
                     dtype=BF16):
    """flatten, FC+ReLU, FC+ReLU, FC, softmax cross-entropy: last stage of 4."""
    b = _Builder()
    b.flatten(src=-1)
    b.linear(c * hw * hw, hidden, relu=1)
    b.linear(hidden, hidden, relu=1)
    b.linear(hidden, classes, relu=0)
    b.xent()
    return _stage("vgg16_classifier", b.layers, dtype, (c, hw, hw), micro_batch, n_micro, 4, 4, 1,
                  BASE_SEED + 4, "xavier")


def _bottleneck(b, src, cin, mid, cout, stride, project):
    x = b.conv(cin, mid, 1, bias=0, src=src)
    x = b.bn(mid, relu=1)
    x = b.conv(mid, mid, 3, stride=stride, bias=0)
    x = b.bn(mid, relu=1)
    x = b.conv(mid, cout, 1, bias=0)
    main = b.bn(cout, relu=0)
    if project:
        s = b.conv(cin, cout, 1, stride=stride, bias=0, src=src)
        short = b.bn(cout, relu=0)
    else:
        short = src
    return b.addl(main, short, relu=1)


def resnet50_stage(cin=256, mid3=128, mid4=256, hw=56, n3=4, n4=6, micro_batch=32, n_micro=8,
                   dtype=BF16):
    """conv3_x (n3 bottlenecks) + conv4_x (n4 bottlenecks), stride 2 on the 3x3 of the
    first block of each group with a 1x1 stride-2 projection shortcut: stage 2 of 4."""
    b = _Builder()
    cur, c = -1, cin
    for i in range(n3):
        cur = _bottleneck(b, cur, c, mid3, 4 * mid3, 2 if i == 0 else 1, i == 0)
        c = 4 * mid3
    for i in range(n4):
        cur = _bottleneck(b, cur, c, mid4, 4 * mid4, 2 if i == 0 else 1, i == 0)
        c = 4 * mid4
    return _stage("resnet50_stage", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 2, 4, 1,
                  BASE_SEED + 5, "kaiming")


def vgg16_conv3(cin=128, c=256, hw=56, micro_batch=32, n_micro=8, dtype=BF16):
    """conv3_1..3_3 at hw, pool: the VGG-16 layers between stage 1 and the deep stage."""
    b = _Builder()
    b.conv(cin, c, 3, relu=1, src=-1)
    b.conv(c, c, 3, relu=1)
    b.conv(c, c, 3, relu=1)
    b.pool()
    return _stage("vgg16_conv3", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 2, 4, 1,
                  BASE_SEED + 6, "kaiming")


def resnet50_stem(c=64, hw=224, n2=3, micro_batch=32, n_micro=8, dtype=BF16, cin=3):
    """7x7 stride-2 conv, BN, ReLU, 3x3 stride-2 max-pool, conv2_x (n2 bottlenecks
    c -> c -> 4c, projection shortcut on the first): the head of ResNet-50."""
    b = _Builder()
    b.conv(cin, c, 7, stride=2, pad=3, bias=0, src=-1)
    b.bn(c, relu=1)
    cur = b.pool(k=3, stride=2, pad=1)
    ch = c
    for i in range(n2):
        cur = _bottleneck(b, cur, ch, c, 4 * c, 1, i == 0)
        ch = 4 * c
    return _stage("resnet50_stem", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 1, 4, 0,
                  BASE_SEED + 7, "kaiming")


def resnet50_tail(cin=1024, mid=512, hw=14, n5=3, classes=1000, micro_batch=32, n_micro=8,
                  dtype=BF16):
    """conv5_x (n5 bottlenecks, stride 2 in the first), global average pool, FC, softmax
    cross-entropy: the end of ResNet-50."""
    b = _Builder()
    cur, c = -1, cin
    for i in range(n5):
        cur = _bottleneck(b, cur, c, mid, 4 * mid, 2 if i == 0 else 1, i == 0)
        c = 4 * mid
    out_hw = (hw + 2 - 3) // 2 + 1
    b.avgpool(out_hw)
    b.flatten()
    b.linear(c, classes, relu=0)
    b.xent()
    return _stage("resnet50_tail", b.layers, dtype, (cin, hw, hw), micro_batch, n_micro, 4, 4, 1,
                  BASE_SEED + 8, "kaiming")


def gnmt_lstm_stage(hidden=1024, seq=50, n_layers=2, micro_batch=64, n_micro=8, dtype=BF16):
    """n_layers unidirectional LSTM layers of GNMT's width, each with the residual connection of
    the upper encoder / decoder layers (output = input + LSTM(input)): a middle stage of a
    4-way split of an 8-layer GNMT.  A sequence is a (hidden, seq, 1) tensor."""
    b = _Builder()
    cur = -1
    for _ in range(n_layers):
        y = b.lstm(hidden, hidden, src=cur)
        cur = b.addl(y, cur, relu=0)
    return _stage("gnmt_lstm_stage", b.layers, dtype, (hidden, seq, 1), micro_batch, n_micro, 2, 4, 1,
                  BASE_SEED + 11, "lstm")


def _concat(name, parts, micro_batch, n_micro, seed, init):
    """One stage holding the layers of consecutive stages (a whole network on one accelerator:
    what the per-layer profile is taken on before it is partitioned)."""
    layers = []
    for st in parts:
        base = len(layers)
        for L in st["layers"]:
            L = dict(L)
            L["src0"] = L["src0"] + base if L["src0"] >= 0 else base - 1
            if L["kind"] == ADD:
                L["src1"] = L["src1"] + base if L["src1"] >= 0 else base - 1
            layers.append(L)
    f = parts[0]
    return _stage(name, layers, f["dtype"], (f["in_c"], f["in_h"], f["in_w"]), micro_batch, n_micro,
                  1, 1, 0, seed, init)


def vgg16_full(micro_batch=32, n_micro=8, dtype=BF16, hw=224, width=64, hidden=4096, classes=1000):
    """All of VGG-16 (13 conv, 5 pool, 3 FC, loss) as one stage."""
    w = width
    parts = [vgg16_stage1(c1=w, c2=2 * w, hw=hw, micro_batch=micro_batch, dtype=dtype),
             vgg16_conv3(cin=2 * w, c=4 * w, hw=hw // 4, micro_batch=micro_batch, dtype=dtype),
             vgg16_deep(cin=4 * w, c=8 * w, hw=hw // 8, micro_batch=micro_batch, dtype=dtype),
             vgg16_classifier(c=8 * w, hw=hw // 32, hidden=hidden, classes=classes,
                              micro_batch=micro_batch, dtype=dtype)]
    return _concat("vgg16_full", parts, micro_batch, n_micro, BASE_SEED + 9, "kaiming")


def resnet50_full(micro_batch=32, n_micro=8, dtype=BF16, hw=224, width=64, classes=1000,
                  blocks=(3, 4, 6, 3)):
    """All of ResNet-50 (stem, conv2_x..conv5_x, average pool, FC, loss) as one stage."""
    w = width
    parts = [resnet50_stem(c=w, hw=hw, n2=blocks[0], micro_batch=micro_batch, dtype=dtype),
             resnet50_stage(cin=4 * w, mid3=2 * w, mid4=4 * w, hw=hw // 4, n3=blocks[1], n4=blocks[2],
                            micro_batch=micro_batch, dtype=dtype),
             resnet50_tail(cin=16 * w, mid=8 * w, hw=hw // 16, n5=blocks[3], classes=classes,
                           micro_batch=micro_batch, dtype=dtype)]
    return _concat("resnet50_full", parts, micro_batch, n_micro, BASE_SEED + 10, "kaiming")


FULL = {
    "tiny": tiny_stage,
    "vgg16_conv3": vgg16_conv3,
    "resnet50_stem": resnet50_stem,
    "resnet50_tail": resnet50_tail,
    "gnmt_lstm_stage": gnmt_lstm_stage,
    "vgg16_full": vgg16_full,
    "resnet50_full": resnet50_full,
    "vgg16_stage1": vgg16_stage1,
    "vgg16_deep": vgg16_deep,
    "vgg16_classifier": vgg16_classifier,
    "resnet50_stage": resnet50_stage,
}


def infer_shapes(stage):
    """Per-layer output shape (C, H, W) per sample; LINEAR/FLATTEN outputs are (F, 1, 1)."""
    shapes = []
    inp = (stage["in_c"], stage["in_h"], stage["in_w"])
    for idx, L in enumerate(stage["layers"]):
        s = inp if L["src0"] < 0 else shapes[L["src0"]]
        k = L["kind"]
        if k == CONV2D:
            assert s[0] == L["cin"], (idx, s, L)
            ho = (s[1] + 2 * L["pad"] - L["kh"]) // L["stride"] + 1
            wo = (s[2] + 2 * L["pad"] - L["kw"]) // L["stride"] + 1
            o = (L["cout"], ho, wo)
        elif k in (MAXPOOL2D, AVGPOOL2D):
            ho = (s[1] + 2 * L["pad"] - L["kh"]) // L["stride"] + 1
            wo = (s[2] + 2 * L["pad"] - L["kw"]) // L["stride"] + 1
            o = (s[0], ho, wo)
        elif k in (RELU, BATCHNORM2D, SOFTMAX_XENT):
            o = s
        elif k == ADD:
            s1 = inp if L["src1"] < 0 else shapes[L["src1"]]
            assert s == s1, (idx, s, s1)
            o = s
        elif k == FLATTEN:
            o = (s[0] * s[1] * s[2], 1, 1)
        elif k == LINEAR:
            assert s[0] * s[1] * s[2] == L["cin"], (idx, s, L)
            o = (L["cout"], 1, 1)
        elif k == LSTM:
            assert s[0] == L["cin"] and s[2] == 1, (idx, s, L)
            o = (L["cout"], s[1], 1)
        else:
            raise ValueError(k)
        shapes.append(o)
    return shapes


def conv_fc_macs_per_sample(stage):
    """Forward multiply-accumulates per sample over CONV2D, LINEAR and LSTM layers."""
    shapes = infer_shapes(stage)
    total = 0
    per_layer = []
    for L, o in zip(stage["layers"], shapes):
        m = 0
        if L["kind"] == CONV2D:
            m = o[0] * o[1] * o[2] * L["cin"] * L["kh"] * L["kw"]
        elif L["kind"] == LINEAR:
            m = L["cin"] * L["cout"]
        elif L["kind"] == LSTM:
            m = o[1] * 4 * L["cout"] * (L["cin"] + L["cout"])
        per_layer.append(m)
        total += m
    return total, per_layer


def flops_per_minibatch(stage):
    """2 FLOP per MAC for each of fwd, dgrad, wgrad over conv/FC layers; the dgrad of a
    layer fed by the stage input is not counted when the stage needs no input gradient."""
    total, per_layer = conv_fc_macs_per_sample(stage)
    fl = 0
    for L, m in zip(stage["layers"], per_layer):
        passes = 3
        if L["src0"] < 0 and not stage["need_input_grad"]:
            passes = 2
        fl += 2 * m * passes
    return fl * stage["micro_batch"] * stage["n_micro"]


def cut_crossings(stage):
    """For the cut after each layer l: (number of tensors, elements per sample) produced at or
    before l - the stage input included - and read by a layer after l.  A pipeline boundary
    placed at a cut has to send all of them; cuts crossed by one tensor are the ones a stage
    with a single input and a single output can be built for."""
    shapes = infer_shapes(stage)
    inp = (stage["in_c"], stage["in_h"], stage["in_w"])
    last_use = {}
    for i, L in enumerate(stage["layers"]):
        last_use[L["src0"]] = i
        if L["kind"] == ADD:
            last_use[L["src1"]] = i
    out = []
    for l in range(len(stage["layers"])):
        live = [t for t, u in last_use.items() if t <= l and u > l]
        elems = sum(int(inp[0] * inp[1] * inp[2]) if t < 0 else int(shapes[t][0] * shapes[t][1] * shapes[t][2])
                    for t in live)
        out.append((len(live), elems))
    return out
