"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on seeded workloads small enough for the oracle yet spanning several tiles with ragged tails."""
import math

import numpy as np
import pytest

from gpu_harness import GpuStage, compare_minibatch, stage_io
from oracle.stage import one_f_one_b_order
from paper_2012_12544_amd import binding as B
from stage_inputs import configs as C
from stage_inputs import gen

pytestmark = pytest.mark.gpu


def single(kind_builder, cin, hw, dtype, micro_batch=3, n_micro=2, need_input_grad=1, name="single"):
    b = C._Builder()
    kind_builder(b)
    return C._stage(name, b.layers, dtype, (cin, hw[0], hw[1]), micro_batch, n_micro, 1, 2,
                    need_input_grad, C.BASE_SEED + 77, "kaiming")


DT = [C.FP32, C.BF16]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("k,stride,cin,cout,hw,relu", [
    (3, 1, 3, 16, (9, 11), 1), (3, 1, 16, 24, (13, 10), 1), (3, 2, 8, 16, (15, 14), 0),
    (1, 1, 16, 40, (7, 9), 0), (1, 2, 24, 8, (9, 9), 1), (3, 1, 5, 7, (6, 5), 0),
])
def test_conv_layer(dtype, k, stride, cin, cout, hw, relu):
    st = single(lambda b: b.conv(cin, cout, k, stride=stride, relu=relu, src=-1), cin, hw, dtype)
    compare_minibatch(st, verbose="conv k%d s%d %d->%d" % (k, stride, cin, cout))


@pytest.mark.parametrize("k,stride,cin,cout,hw,mb", [
    (3, 1, 64, 64, (20, 23), 3),      # several pixel tiles, ragged last tile, K = 576
    (3, 1, 24, 136, (18, 18), 2),     # ragged K tile (216) and ragged channel tile (136 = 128 + 8)
    (3, 2, 32, 72, (21, 19), 3),      # stride-2 forward, strided dgrad
    (1, 1, 128, 256, (9, 7), 5),      # 1x1
    (1, 2, 72, 40, (15, 15), 2),      # 1x1 stride 2
    (3, 1, 8, 8, (5, 4), 1),          # smaller than one tile in every dimension
    (3, 1, 64, 64, (32, 48), 2),      # sides multiple of 16: halo-in-LDS kernel, 64-channel tile
    (3, 1, 128, 128, (16, 32), 3),    # halo kernel, two 64-channel input slices, 128-channel tile
    (3, 1, 128, 192, (32, 16), 1),    # halo kernel, 192 = 3 x 64 output channels
    (3, 1, 3, 64, (16, 32), 3),       # RGB input padded to 8 channels: first-layer kernel
    (3, 1, 3, 128, (32, 16), 2),      # ... two 64-channel output tiles
])
def test_conv_mfma_tiling(k, stride, cin, cout, hw, mb):
    st = single(lambda b: b.conv(cin, cout, k, stride=stride, relu=1, src=-1), cin, hw, C.BF16, micro_batch=mb)
    compare_minibatch(st, verbose="mfma conv k%d s%d %d->%d %s" % (k, stride, cin, cout, hw))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("layout", [B.NCHW, B.NHWC])
def test_relu_pool_layers_and_layouts(dtype, layout):
    def build(b):
        b.conv(8, 8, 3, relu=0, src=-1)
        b.relu()
        b.pool()
    st = single(build, 8, (10, 12), dtype)
    compare_minibatch(st, layout=layout, verbose="conv-relu-pool layout %d" % layout)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("c,hw,mb", [(16, (12, 10), 3), (6, (9, 7), 2), (64, (224, 224), 2), (512, (28, 28), 8)])
def test_pool_only_stage_indices_bit_exact(dtype, c, hw, mb):
    """Identical inputs on both sides: arg-max indices, outputs and routed gradients are exact."""
    st = single(lambda b: b.pool(src=-1), c, hw, dtype, micro_batch=mb, n_micro=1)
    xs, gs = stage_io(st)
    xs[0][:, :, 1, :] = xs[0][:, :, 0, :]                      # plant ties (vertical, horizontal, all four)
    xs[0][:, :, :, 3] = xs[0][:, :, :, 2]
    xs[0][0, 0, :4, :4] = 0.0
    from oracle.stage import OracleStage
    orc = OracleStage(st, gen.all_params(st))
    g = GpuStage(st, gen.all_params(st))
    y_ref, y = orc.forward(0, xs[0]), g.forward(0, xs[0])
    assert np.array_equal(orc.pool_indices(0, 0), g.pool_indices(0, 0))
    assert np.array_equal(y_ref, y)
    assert np.array_equal(orc.backward(0, gs[0]), g.backward(0, gs[0]))
    g.close()


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("k,stride,pad", [(3, 2, 1), (3, 2, 0), (3, 1, 1), (2, 1, 0), (2, 2, 1)])
@pytest.mark.parametrize("c,hw,mb", [(16, (12, 10), 3), (6, (9, 7), 2), (64, (112, 112), 2)])
def test_windowed_pool_only_stage_bit_exact(dtype, k, stride, pad, c, hw, mb):
    """Overlapping / padded windows (the ResNet stem's 3x3 stride-2 pool and relatives) on identical
    inputs: indices, outputs and the summed routed gradients agree exactly in fp32; in bf16 the sum
    of several routed gradients is rounded once on both sides."""
    if hw[0] > 100 and (k, stride, pad) != (3, 2, 1):
        pytest.skip("full stem shape only for the stem's own window")
    st = single(lambda b: b.pool(src=-1, k=k, stride=stride, pad=pad), c, hw, dtype, micro_batch=mb, n_micro=1)
    xs, gs = stage_io(st)
    xs[0][:, :, 1, :] = xs[0][:, :, 0, :]
    xs[0][:, :, :, 3] = xs[0][:, :, :, 2]
    xs[0][0, 0, :4, :4] = 0.0
    from oracle.stage import OracleStage
    orc = OracleStage(st, gen.all_params(st))
    g = GpuStage(st, gen.all_params(st))
    y_ref, y = orc.forward(0, xs[0]), g.forward(0, xs[0])
    assert np.array_equal(orc.pool_indices(0, 0), g.pool_indices(0, 0))
    assert np.array_equal(y_ref, y)
    dx_ref, dx = orc.backward(0, gs[0]), g.backward(0, gs[0])
    if dtype == C.FP32:
        assert np.allclose(dx_ref, dx, rtol=1e-6, atol=1e-6)       # up to four fp32 terms per input
    else:
        assert np.max(np.abs(dx_ref - dx)) <= 2.0 ** -7 * np.max(np.abs(dx_ref))   # one bf16 ulp of the largest
    assert np.array_equal(dx_ref == 0, dx == 0)
    g.close()


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("layout", [B.NCHW, B.NHWC])
def test_gated_windowed_pool_and_average_pool(dtype, layout):
    """ReLU-gated producers in front of both pools: the window maximum gates the max-pool gradient,
    the producer's own output gates the average pool's."""
    def build(b):
        x = b.conv(8, 16, 3, relu=1, src=-1)
        p = b.pool(k=3, stride=2, pad=1)
        c2 = b.conv(16, 16, 1, relu=1)
        b.avgpool(3)
    st = single(build, 8, (12, 12), dtype)
    compare_minibatch(st, layout=layout, verbose="conv-pool3x3-conv-avgpool layout %d" % layout)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("c,hw,k", [(16, (7, 7), 7), (6, (9, 6), 3), (2048, (7, 7), 7)])
def test_average_pool_only_stage(dtype, c, hw, k):
    st = single(lambda b: b.avgpool(k, src=-1), c, hw, dtype, micro_batch=4, n_micro=1)
    compare_minibatch(st, tol=1e-6 if dtype == C.FP32 else 2.0 ** -8, verbose="avgpool %s k%d" % (hw, k))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("hw,cout,mb", [((20, 18), 16, 2), ((64, 48), 64, 3)])
def test_stem_conv_7x7_stride_2(dtype, hw, cout, mb):
    st = single(lambda b: b.conv(3, cout, 7, stride=2, pad=3, bias=0, relu=0, src=-1), 3, hw, dtype, micro_batch=mb,
                need_input_grad=0)
    compare_minibatch(st, verbose="7x7 s2 conv %s" % (hw,))


@pytest.mark.parametrize("cin,hidden,T,mb,dtype", [
    (5, 7, 6, 3, C.FP32), (8, 8, 1, 2, C.FP32), (16, 24, 9, 4, C.FP32),
    (8, 16, 5, 3, C.BF16), (24, 40, 9, 4, C.BF16), (16, 16, 1, 5, C.BF16),
    (64, 64, 12, 70, C.BF16),                       # more sequences than one 64-row tile
])
@pytest.mark.parametrize("need_dx", [1, 0])
def test_lstm_layer(cin, hidden, T, mb, dtype, need_dx):
    st = single(lambda b: b.lstm(cin, hidden, src=-1), cin, (T, 1), dtype, micro_batch=mb, need_input_grad=need_dx)
    compare_minibatch(st, verbose="lstm %d->%d T=%d N=%d" % (cin, hidden, T, mb))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("layout", [B.NCHW, B.NHWC])
def test_lstm_stage_with_residual_connections(dtype, layout):
    st = C.gnmt_lstm_stage(hidden=16, seq=7, n_layers=2, micro_batch=3, n_micro=3, dtype=dtype)
    compare_minibatch(st, layout=layout, verbose="gnmt-like stage layout %d" % layout)


@pytest.mark.parametrize("dtype", DT)
def test_remaining_stages_small(dtype):
    """Shrunken copies of the VGG-16 conv3 block, the ResNet-50 head and the ResNet-50 end."""
    compare_minibatch(C.vgg16_conv3(cin=8, c=16, hw=16, micro_batch=2, n_micro=2, dtype=dtype), verbose="conv3 small")
    compare_minibatch(C.resnet50_stem(c=8, hw=32, n2=2, micro_batch=3, n_micro=2, dtype=dtype), verbose="stem small")
    compare_minibatch(C.resnet50_tail(cin=32, mid=8, hw=8, n5=2, classes=11, micro_batch=4, n_micro=2, dtype=dtype),
                      verbose="tail small")


def test_whole_networks_small_fp32():
    """Every layer of VGG-16 and of a one-block-per-group ResNet in one stage (what the per-layer
    profile is taken on), shrunken, fp32."""
    compare_minibatch(C.vgg16_full(micro_batch=2, n_micro=2, dtype=C.FP32, hw=32, width=4, hidden=24, classes=10),
                      verbose="vgg16 whole small")
    compare_minibatch(C.resnet50_full(micro_batch=4, n_micro=2, dtype=C.FP32, hw=64, width=4, classes=10,
                                      blocks=(1, 1, 1, 1)), verbose="resnet whole small")


@pytest.mark.parametrize("cin,cout,hw,mb", [(64, 64, (32, 16), 2), (64, 128, (16, 48), 2), (128, 64, (16, 16), 3)])
def test_conv_with_pool_in_its_epilogue(cin, cout, hw, mb):
    """16-aligned 3x3 conv (+ReLU) whose output only feeds a 2x2 max-pool: pooled values and arg-max
    indices come out of the conv kernel's epilogue and the conv output is never stored."""
    st = single(lambda b: (b.conv(cin, cout, 3, relu=1, src=-1), b.pool()), cin, hw, C.BF16, micro_batch=mb)
    compare_minibatch(st, verbose="conv+pool fused %d->%d %s" % (cin, cout, hw))


@pytest.mark.parametrize("dtype", DT)
def test_pool_odd_size_and_vector_tail(dtype):
    st = single(lambda b: (b.conv(6, 6, 1, relu=1, src=-1), b.pool()), 6, (9, 7), dtype)
    compare_minibatch(st, verbose="pool odd")


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("c,hw,mb", [(16, (6, 5), 5), (6, (7, 3), 5), (256, (4, 4), 5),
                                     # one-launch kernels (>= 128 channels, <= 2048 rows): one and two rows per
                                     # thread with a ragged tail, exactly at the row limit, just above it
                                     (128, (9, 7), 5), (136, (25, 11), 6), (256, (16, 16), 8), (128, (41, 10), 5),
                                     # above 2048 rows the producing conv hands over the statistics partials of its
                                     # pixel tiles (ragged last tile; more channels than one tile)
                                     (32, (40, 30), 2), (128, (33, 32), 8), (200, (29, 31), 3)])
def test_batchnorm_layer(dtype, c, hw, mb):
    # In bf16 a stored value one ulp apart on the two sides can flip a ReLU gate, and one flipped gate moves that
    # pixel's dx by more than the bound; with hundreds of thousands of gated elements that is no longer rare.
    # The large bf16 cases therefore compare dx at the pixels where both sides' gates agree in every channel
    # (the layers are 1x1, so other pixels' gates reach a pixel only through the per-channel sums) and bound
    # the share of disagreeing gates by 1e-3.
    big = dtype == C.BF16 and mb * hw[0] * hw[1] * c > 100000

    def build(b):
        b.conv(c, c, 1, bias=0, src=-1)
        b.bn(c, relu=1)
    st = single(build, c, hw, dtype, micro_batch=mb)
    compare_minibatch(st, verbose="bn c%d rows %d" % (c, mb * hw[0] * hw[1]), dx_where_output_gates_agree=big)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("c,c2,k,hw,mb", [(32, 24, 3, (40, 30), 2), (16, 136, 1, (25, 29), 3), (8, 8, 3, (6, 5), 2)])
def test_conv_bn_relu_conv_chain(dtype, c, c2, k, hw, mb):
    """A batch-norm between two convs: above 2048 rows (bf16) its forward statistics come out of the first conv's
    epilogue and the sums of its backward out of the second conv's input-gradient epilogue."""
    def build(b):
        b.conv(c, c, 1, bias=0, src=-1)
        b.bn(c, relu=1)
        b.conv(c, c2, k, bias=0)
    st = single(build, c, hw, dtype, micro_batch=mb)
    compare_minibatch(st, verbose="conv-bn-conv c%d rows %d" % (c, mb * hw[0] * hw[1]))


@pytest.mark.parametrize("dtype", DT)
def test_residual_block(dtype):
    st = C.resnet50_stage(cin=16, mid3=8, mid4=8, hw=8, n3=2, n4=1, micro_batch=3, n_micro=2, dtype=dtype)
    compare_minibatch(st, verbose="residual blocks")


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("layout", [B.NCHW, B.NHWC])
@pytest.mark.parametrize("hw,mb", [((6, 5), 3), ((30, 28), 3)])       # one-launch batch-norm; above its 2048 rows
def test_residual_unit_on_the_stage_input(dtype, layout, hw, mb):
    """conv 1x1 -> batch-norm -> (+ stage input) -> ReLU, then a second unit on that sum.  In bf16 the sum of each
    unit is stored by its batch-norm's normalisation pass, and the ADD's share of the gradient of the unit's input is
    added by the 1x1 conv's input-gradient epilogue instead of being copied first - for the first unit that input is
    the STAGE input, whose buffers (NHWC) are the caller's own."""
    def build(b):
        c1 = b.conv(16, 16, 1, bias=0, src=-1)
        n1 = b.bn(16)
        s1 = b.addl(n1, -1)
        b.conv(16, 16, 1, bias=0, src=s1)
        n2 = b.bn(16)
        b.addl(n2, s1)
    st = single(build, 16, hw, dtype, micro_batch=mb, n_micro=3, name="residual-on-input")
    compare_minibatch(st, layout=layout, verbose="residual units on the stage input, layout %d, rows %d" % (layout, mb * hw[0] * hw[1]))


@pytest.mark.parametrize("dtype", DT)
def test_classifier(dtype):
    st = C.vgg16_classifier(c=8, hw=3, hidden=40, classes=13, micro_batch=5, n_micro=3, dtype=dtype)
    for layout in (B.NCHW, B.NHWC):
        compare_minibatch(st, layout=layout, verbose="classifier layout %d" % layout)


def test_config1_tiny_fp32_full_size():
    compare_minibatch(C.tiny_stage(), perturb=False, verbose="cfg1 tiny")
    compare_minibatch(C.tiny_stage(), perturb=True, layout=B.NCHW, verbose="cfg1 tiny perturbed NCHW")


@pytest.mark.parametrize("name,stage", [
    ("vgg16_stage1", C.vgg16_stage1(c1=16, c2=24, hw=20, micro_batch=3, n_micro=5)),
    ("vgg16_deep", C.vgg16_deep(cin=16, c=24, hw=12, micro_batch=3, n_micro=3)),
    ("resnet50_stage", C.resnet50_stage(cin=16, mid3=8, mid4=16, hw=12, n3=2, n4=2, micro_batch=4, n_micro=4)),
])
def test_shrunken_workloads_bf16(name, stage):
    compare_minibatch(stage, verbose=name)


def test_profile_feeds_the_partition_explorer():
    """The per-layer profile measured on the device is what the host-side planner consumes."""
    st = C.vgg16_stage1(c1=16, c2=24, hw=20, micro_batch=3, n_micro=5)
    g = GpuStage(st, gen.all_params(st))
    prof = B.bapipe_profile_layers(g.h, 1, 2, len(st["layers"]))
    g.close()
    assert all(p["fwd_ms"] >= 0 and p["bwd_ms"] >= 0 for p in prof) and sum(p["fwd_ms"] + p["bwd_ms"] for p in prof) > 0
    f, b = [p["fwd_ms"] for p in prof], [p["bwd_ms"] for p in prof]
    sb, rep = B.bapipe_partition([f, f], [b, b], [p["out_feature_bytes"] for p in prof], [p["weight_bytes"] for p in prof],
                                 [p["stash_bytes"] for p in prof], n_micro=5, schedule=B.PLAN_1F1B_SO)
    assert sb[0] == 0 and sb[-1] == len(prof) and 0 < sb[1] < len(prof)
    total = sum(f) + sum(b)
    assert total / 2 * (1 - 1e-9) <= rep["bottleneck_ms"] <= total and math.isclose(rep["ideal_stage_ms"], total / 2, rel_tol=1e-9)


def test_profile_reports_layers_that_share_a_kernel_on_the_launching_layer():
    """Layers the stage runs as one kernel: the time is on the layer that launches it, the other reports 0 forward
    time - the max-pool behind a halo conv (bf16), the residual ADD behind a batch-norm."""
    st = C.vgg16_stage1(c1=64, c2=64, hw=32, micro_batch=2, n_micro=2)
    g = GpuStage(st, gen.all_params(st))
    prof = B.bapipe_profile_layers(g.h, 1, 2, len(st["layers"]))
    g.close()
    pools = [i for i, L in enumerate(st["layers"]) if L["kind"] == C.MAXPOOL2D]
    assert pools and all(prof[i]["fwd_ms"] == 0.0 and prof[i]["bwd_ms"] > 0.0 and prof[i - 1]["fwd_ms"] > 0.0 for i in pools)
    st = C.resnet50_stage(cin=16, mid3=8, mid4=8, hw=8, n3=2, n4=1, micro_batch=3, n_micro=2)
    g = GpuStage(st, gen.all_params(st))
    prof = B.bapipe_profile_layers(g.h, 1, 2, len(st["layers"]))
    g.close()
    adds = [i for i, L in enumerate(st["layers"]) if L["kind"] == C.ADD]
    assert adds and all(prof[i]["fwd_ms"] == 0.0 and prof[i - 1]["fwd_ms"] > 0.0 for i in adds)


@pytest.mark.parametrize("net", ["vgg16_full", "resnet50_full"])
def test_whole_network_profile_is_partitioned_into_four_stages(net):
    """The loop the profiler exists for (Sec. III-A / III-C): profile every layer of a whole network
    at its real layer shapes on the device, hand the profile to the partition explorer, and check the
    result against brute force over the measured numbers.  A cut inside a residual block is crossed
    by two tensors; it is priced at their total size, and with a finite link the explorer's own
    feature threshold a_th keeps boundaries out of the blocks."""
    from oracle import plan as P
    st = C.FULL[net](micro_batch=8, n_micro=4)
    g = GpuStage(st, gen.all_params(st))
    L = len(st["layers"])
    prof = B.bapipe_profile_layers(g.h, 1, 3, L)
    g.close()
    f, b = [p["fwd_ms"] for p in prof], [p["bwd_ms"] for p in prof]
    assert min(f) >= 0 and min(b) >= 0 and sum(f) > 0 and sum(b) > sum(f) * 0.5
    cross = C.cut_crossings(st)
    assert cross[-1] == (0, 0) and all(n >= 1 for n, _ in cross[:-1])
    if net == "vgg16_full":
        assert all(n == 1 for n, _ in cross[:-1])
    else:
        assert sum(1 for n, _ in cross[:-1] if n == 1) == 16 + 3 + 3       # after each block, stem layers, head
    esz = 2
    single = [e * esz * 8 for n, e in cross]
    assert all(prof[l]["out_feature_bytes"] == single[l] for l in range(L - 1) if cross[l][0] == 1 and
               st["layers"][l]["kind"] != C.SOFTMAX_XENT)
    out_bytes = [float(e * esz * 8) if n == 1 else 1e15 for n, e in cross]
    N = 4
    wb, sbts = [p["weight_bytes"] for p in prof], [p["stash_bytes"] for p in prof]
    total = sum(f) + sum(b)
    link = 1e15 / (total / N) / 10.0                  # a_th = T x link = 1e14: above every real tensor, below the penalty
    sb, rep = B.bapipe_partition([f] * N, [b] * N, out_bytes, wb, sbts, link_bytes_per_ms=link, n_micro=4,
                                 schedule=B.PLAN_1F1B_SNO)
    assert sb[0] == 0 and sb[-1] == L and all(sb[i] < sb[i + 1] for i in range(N))
    assert all(cross[sb[i] - 1][0] == 1 for i in range(1, N)), "a boundary fell inside a residual block"
    p = dict(fwd_ms=[f] * N, bwd_ms=[b] * N, out_bytes=out_bytes, weight_bytes=wb, stash_bytes=sbts,
             link_bytes_per_ms=link, n_micro=4, schedule=P.S_1F1B_SNO)
    legal = [l + 1 for l in range(L - 1) if cross[l][0] == 1]
    best = min(max(sum(f[lo:hi]) + sum(b[lo:hi]) for lo, hi in zip((0,) + c, c + (L,)))
               for c in __import__("itertools").combinations(legal, N - 1))
    assert math.isclose(rep["bottleneck_ms"], best, rel_tol=1e-9), (rep, best)
    assert math.isclose(rep["ideal_stage_ms"], total / N, rel_tol=1e-9)
    print("  %s: stages begin at %s, slowest %.3f ms vs ideal %.3f ms" % (net, sb, rep["bottleneck_ms"], total / N), flush=True)
    # every stage of the partition can be built and run as a stage of its own
    for i in range(N):
        sub = [dict(l) for l in st["layers"][sb[i]:sb[i + 1]]]
        for l in sub:
            l["src0"] = max(l["src0"] - sb[i], -1)
            if l["kind"] == C.ADD:
                l["src1"] = max(l["src1"] - sb[i], -1)
        shp = (st["in_c"], st["in_h"], st["in_w"]) if sb[i] == 0 else C.infer_shapes(st)[sb[i] - 1]
        part = C._stage("%s.part%d" % (net, i), sub, st["dtype"], shp, 8, 2, i + 1, N, 1 if i else 0, st["seed"], st["init"])
        gp = GpuStage(part, gen.all_params(part))
        per, depth = B.bapipe_stage_stash_bytes(gp.h)
        assert depth == min(2, N - i)
        gp.close()


def test_profile_sweep_over_micro_batch_sizes():
    st = C.vgg16_stage1(c1=16, c2=24, hw=20, micro_batch=4, n_micro=2)
    import torch
    alloc = B.TorchAllocator("cuda:0")
    opts = B.make_opts(st, io_layout=B.NHWC, stream=torch.cuda.current_stream().cuda_stream, allocator=alloc)
    sweep = B.bapipe_profile_sweep(st["layers"], [2, 4, 8], opts, warmup=1, iters=2)
    assert sorted(sweep) == [2, 4, 8]
    for mb, prof in sweep.items():
        assert len(prof) == len(st["layers"]) and all(p["fwd_ms"] >= 0 and p["bwd_ms"] >= 0 for p in prof)
    for i in range(len(st["layers"])):                      # sizes scale with the micro-batch, weights do not
        assert sweep[8][i]["out_feature_bytes"] == 4 * sweep[2][i]["out_feature_bytes"]
        assert sweep[8][i]["weight_bytes"] == sweep[2][i]["weight_bytes"]
    with pytest.raises(B.BapipeError) as e:
        B.bapipe_profile_sweep(st["layers"], [2, 0], opts)
    assert e.value.status == B.E_INVALID


def test_schedule_violations_and_stash_depth():
    st = C.vgg16_deep(cin=8, c=8, hw=4, micro_batch=2, n_micro=4)        # stage 3 of 4: depth 2
    g = GpuStage(st, gen.all_params(st))
    per, depth = B.bapipe_stage_stash_bytes(g.h)
    assert depth == 2 and per > 0
    xs, gs = stage_io(st)
    with pytest.raises(B.BapipeError) as e:
        g.backward(0, gs[0])
    assert e.value.status == B.E_ORDER
    with pytest.raises(B.BapipeError) as e:
        g.forward(1, xs[1])
    assert e.value.status == B.E_ORDER
    g.forward(0, xs[0])
    g.forward(1, xs[1])
    with pytest.raises(B.BapipeError) as e:
        g.forward(2, xs[2])                       # third in flight exceeds N-i+1 = 2
    assert e.value.status == B.E_ORDER
    with pytest.raises(B.BapipeError) as e:
        g.backward(1, gs[1])                      # FIFO
    assert e.value.status == B.E_ORDER
    with pytest.raises(B.BapipeError) as e:
        B.bapipe_stage_step(g.h, 0.1)
    assert e.value.status == B.E_ORDER
    g.backward(0, gs[0])
    g.forward(2, xs[2]); g.backward(1, gs[1]); g.forward(3, xs[3]); g.backward(2, gs[2]); g.backward(3, gs[3])
    B.bapipe_stage_step(g.h, 0.1)
    g.close()


def test_allocator_failure_is_reported_and_leaks_nothing():
    st = C.tiny_stage(c=4, hw=8, micro_batch=2, n_micro=2)
    for k in range(0, 6):
        alloc = B.TorchAllocator("cuda:0", fail_after=k)
        opts = B.make_opts(st, allocator=alloc)
        with pytest.raises(B.BapipeError) as e:
            B.bapipe_stage_create(st["layers"], 2, 2, opts)
        assert e.value.status == B.E_OOM
        assert not alloc.live


# ------------------------------------------------------------------------------ doubled warm-up (Table II, 1F1B-SO)
@pytest.mark.parametrize("name,stage,want", [
    # stage 3 of 4: 2(N-i+1) = 4 of 6 micro-batches in flight
    ("vgg16_deep", C.vgg16_deep(cin=16, c=24, hw=12, micro_batch=3, n_micro=6), 4),
    # stage 2 of 4: 2(N-i+1) = 6 exceeds M = 4, the ring holds the whole mini-batch
    ("resnet50_stage", C.resnet50_stage(cin=16, mid3=8, mid4=16, hw=12, n3=1, n4=1, micro_batch=4, n_micro=4), 4),
    # stage 1 of 2: 4 of 5
    ("tiny", C.tiny_stage(c=8, hw=12, micro_batch=2, n_micro=5), 4),
])
def test_1f1b_so_doubled_warm_up(name, stage, want):
    """1F1B-SO (Table II "Features memory" 2(N-i+1)a): the ring is twice as deep, the warm-up runs twice as
    many forwards before the first backward, results are those of the oracle under the same order, and one
    forward more than the depth is refused."""
    from gpu_harness import GpuStage
    so = dict(stage, schedule=C.SCHED_1F1B_SO)
    i, N, M = so["stage_index"], so["n_stages"], so["n_micro"]
    assert want == min(M, 2 * (N - i + 1))
    g = GpuStage(so, gen.all_params(so))
    per, depth = B.bapipe_stage_stash_bytes(g.h)
    assert depth == want
    plain = GpuStage(stage, gen.all_params(stage))
    assert B.bapipe_stage_stash_bytes(plain.h)[1] == min(M, N - i + 1)
    plain.close()
    xs, gs = stage_io(so)
    for m in range(depth):
        g.forward(m, xs[m])
    if depth < M:
        with pytest.raises(B.BapipeError) as e:
            g.forward(depth, xs[depth])
        assert e.value.status == B.E_ORDER
    g.close()
    order = one_f_one_b_order(M, want)
    assert [t for t, _ in order[:want]] == ["F"] * want            # doubled warm-up really is what runs
    compare_minibatch(so, order=order, verbose="1F1B-SO %s depth %d" % (name, want))


# ------------------------------------------------------------------------------ a stage that ends in FLATTEN
@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("layout", [B.NCHW, B.NHWC])
def test_stage_ending_in_flatten(dtype, layout):
    """A cut right after pool + flatten: the stage output (and the gradient coming back) is indexed
    c*H*W + h*W + w in either boundary layout, which is what the next stage's linear layer expects."""
    def build(b):
        b.conv(8, 16, 3, relu=1, src=-1)
        b.pool()
        b.flatten()
    st = single(build, 8, (6, 10), dtype, micro_batch=3)
    compare_minibatch(st, layout=layout, verbose="conv-pool-flatten layout %d" % layout)


def test_loss_of_the_previous_mini_batch_is_not_served_again():
    st = C.vgg16_classifier(c=8, hw=3, hidden=24, classes=7, micro_batch=4, n_micro=2)
    g = GpuStage(st, gen.all_params(st))
    xs, gs = stage_io(st)
    for m in range(2):
        g.forward(m, xs[m])
        g.backward(m, gs[m])
    assert B.bapipe_stage_get_loss(g.h, 1) > 0
    B.bapipe_stage_step(g.h, 0.1)
    assert B.bapipe_stage_get_loss(g.h, 1) > 0          # "the just finished mini-batch"
    g.forward(0, xs[0])
    for m in range(2):
        with pytest.raises(B.BapipeError) as e:
            B.bapipe_stage_get_loss(g.h, m)
        assert e.value.status == B.E_ORDER
    g.close()


# ------------------------------------------------------------------------------ run twice, compare bit for bit
@pytest.mark.parametrize("name,stage", [
    ("vgg16_stage1 64/128 channels", C.vgg16_stage1(c1=64, c2=128, hw=32, micro_batch=3, n_micro=3)),
    ("vgg16_deep 256 channels", C.vgg16_deep(cin=128, c=256, hw=12, micro_batch=5, n_micro=2)),
    ("resnet50_stage", C.resnet50_stage(cin=64, mid3=32, mid4=64, hw=24, n3=2, n4=2, micro_batch=4, n_micro=2)),
    ("classifier", C.vgg16_classifier(c=32, hw=3, hidden=136, classes=29, micro_batch=6, n_micro=3)),
    ("lstm", C.gnmt_lstm_stage(hidden=64, seq=9, n_layers=2, micro_batch=5, n_micro=2)),
    ("tiny fp32", C.tiny_stage()),
])
def test_same_mini_batch_twice_is_bit_identical(name, stage):
    """Every reduction runs in a fixed order (split partials added by a second kernel, no atomics), so two
    runs of the same mini-batch on fresh handles agree bit for bit; a race would show up here."""
    from gpu_harness import gpu_minibatch
    a, b = gpu_minibatch(stage), gpu_minibatch(stage)
    assert sorted(a) == sorted(b) and any(k.startswith("dw") for k in a)
    for k in a:
        assert np.array_equal(a[k], b[k]), (name, k)


# ------------------------------------------------------------------------------ overlap on further streams
OVERLAP_STAGES = [
    ("vgg16_stage1 64/128 channels", lambda: C.vgg16_stage1(c1=64, c2=128, hw=32, micro_batch=3, n_micro=6)),      # depth 4
    ("vgg16_deep 256 channels", lambda: C.vgg16_deep(cin=128, c=256, hw=12, micro_batch=5, n_micro=4)),            # depth 2
    ("resnet50_stage", lambda: C.resnet50_stage(cin=64, mid3=32, mid4=64, hw=24, n3=2, n4=2, micro_batch=4, n_micro=5)),  # depth 3
    ("classifier", lambda: C.vgg16_classifier(c=32, hw=3, hidden=136, classes=29, micro_batch=6, n_micro=3)),       # depth 1
    ("tiny fp32", lambda: C.tiny_stage()),
]


@pytest.mark.parametrize("name,make", OVERLAP_STAGES)
def test_further_streams_give_the_same_results_bit_for_bit(name, make):
    """A whole mini-batch enqueued at once with the backward passes and their weight-gradient kernels on streams of
    their own (passes overlap the forward passes of later micro-batches, ring slots are reused) against the same
    mini-batch on one stream; also each stream alone, and the static-workspace entry point."""
    from gpu_harness import gpu_minibatch
    ref = gpu_minibatch(make())
    for kw in (dict(backward_stream=True), dict(backward_stream=True, static=True), dict(backward_stream="no wgrad stream"),
               dict(wgrad_stream=True)):
        got = gpu_minibatch(make(), eager_sync=False, **kw)
        assert sorted(got) == sorted(ref)
        for k in ref:
            assert np.array_equal(got[k], ref[k]), (name, kw, k)


def test_further_streams_against_the_oracle_and_their_call_rules():
    st = C.resnet50_stage(cin=16, mid3=8, mid4=16, hw=12, n3=2, n4=2, micro_batch=4, n_micro=4)
    compare_minibatch(st, backward_stream=True, verbose="three streams, resnet blocks")
    compare_minibatch(C.vgg16_stage1(c1=16, c2=24, hw=20, micro_batch=3, n_micro=5), backward_stream=True, verbose="three streams, vgg stage 1")
    import torch
    g = GpuStage(st, gen.all_params(st))
    side, side2 = torch.cuda.Stream(device="cuda:0"), torch.cuda.Stream(device="cuda:0")
    xs, gs = stage_io(st)
    g.forward(0, xs[0])
    with pytest.raises(B.BapipeError) as e:                      # not in the middle of a mini-batch
        B.bapipe_stage_set_streams(g.h, side.cuda_stream, None)
    assert e.value.status == B.E_ORDER
    g.backward(0, gs[0])
    for m in range(1, 4):
        g.forward(m, xs[m])
        g.backward(m, gs[m])
    B.bapipe_stage_step(g.h, 0.1)
    with pytest.raises(B.BapipeError) as e:                      # the two streams must differ
        B.bapipe_stage_set_streams(g.h, side.cuda_stream, side.cuda_stream)
    assert e.value.status == B.E_INVALID
    B.bapipe_stage_set_streams(g.h, side.cuda_stream, side2.cuda_stream)    # between mini-batches: on, off, on again
    B.bapipe_stage_set_streams(g.h, None, None)
    B.bapipe_stage_set_streams(g.h, side.cuda_stream, None)
    g.close()


def test_measured_peaks_are_plausible_and_below_the_published_ones():
    """The probe behind bench.py's `measured_peaks` (register-resident MFMA loop, streaming copy): what it returns
    must lie under the published peaks of the part and well above what a broken probe (a loop the compiler removed,
    a copy that never ran) would give."""
    import ctypes as ct
    tf, gb = B.bapipe_measure_peaks()
    assert 800.0 < tf < 2500.0, tf          # bf16 dense MFMA: 2.5 PFLOP/s published
    assert 2000.0 < gb < 8000.0, gb         # HBM3E: 8 TB/s published (read + written bytes of a copy)
    tf2, gb2 = B.bapipe_measure_peaks()
    assert abs(tf2 - tf) < 0.1 * tf and abs(gb2 - gb) < 0.15 * gb
    one = ct.c_double(0)
    assert B.load().bapipe_measure_peaks(0, None, ct.byref(one)) == B.E_INVALID
    assert B.load().bapipe_measure_peaks(0, ct.byref(one), None) == B.E_INVALID
    # LDS read rates: 256 units x 128 bytes per clock x 2.4 GHz = 78.6 TB/s is what the instruction set documents
    # for a unit; the 64-bit transposing read moves half as much per instruction and cannot be faster than the
    # 128-bit read
    wide, tr = B.bapipe_measure_lds()
    assert 20.0 < tr <= 1.05 * wide < 200.0, (wide, tr)
    assert B.load().bapipe_measure_lds(0, None, ct.byref(one)) == B.E_INVALID
