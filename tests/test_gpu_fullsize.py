"""GPU parity at the full layer shapes of the bf16 workloads, in the launch configuration the
benchmark times (NHWC boundary, full micro-batch size): every kernel runs with the grid and
tiles of the real workload.  Only M, the number of micro-batches per mini-batch, is cut where it
changes no launch, so that the CPU oracle finishes within a minute or two per case.

Three kinds of check, all against the CPU oracle, none with an input or expected value from the GPU:

* end to end - the whole stage, every tensor.  The shallow stage (VGG-16 stage 1) is held to the 2e-2
  element-wise bound on everything, once at M = 2 and once in the benchmark's own configuration
  (M = 8, ring depth 4, slots reused).  Deeper stages cannot meet an element-wise bound end to end
  with ANY second implementation that sums in another order (a one-ulp difference in a stored
  activation flips ReLU gates / pool arg-max choices a few layers later and flips compound with
  depth; tests/test_flip_bound.py shows it on the CPU with an fp32 PyTorch implementation), so they
  are held to the rule of tests/flip_gate.py on every tensor - distance to the UN-ROUNDED oracle
  result at most 1.5 x the bf16 oracle's own distance to it - plus the element-wise bound wherever
  the depth allows it (forward outputs, the loss, and the classifier's gradients sample by sample).

* layer by layer, teacher-forced BY THE ORACLE - the oracle runs the whole stage once and, for
  every conv / linear / batch-norm / pool / ReLU / loss layer, its input x_l and its gated output
  gradient g_l are fed to a one-layer GPU stage of the same full shape: forward(x_l) is compared
  with the oracle's y_l, and backward(g_l) of a clone without the fused ReLU (the gate is
  already in g_l, so no decision is taken twice) with the oracle's dx_l, dw_l, db_l, all within
  2e-2 of max|ref|, pool indices bit-exact.

* slice by slice, teacher-forced the same way - runs of two to ten consecutive layers, so that the
  kernels that only exist where layers meet run at full shape under a gate: conv + ReLU + max-pool
  in one kernel, batch-norm statistics out of the producing conv's epilogue, batch-norm backward
  sums out of the consuming conv's input-gradient epilogue, the residual add and the gradient
  fan-out at a block input (whole bottleneck blocks).
"""
import time

import numpy as np
import pytest

import flip_gate
from gpu_harness import TOL, GpuStage, compare_minibatch, pool_index_gap, rel_err, stage_io
from oracle.stage import OracleStage, one_f_one_b_order
from paper_2012_12544_amd import binding as B
from stage_inputs import configs as C
from stage_inputs import gen

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------------------ end to end
@pytest.mark.timeout(1200)
def test_vgg16_stage1_end_to_end_benchmark_configuration():
    """Exactly what bench.py times: M = 8 micro-batches of 32, 1F1B with four in flight, every ring slot reused,
    backward passes on their own stream."""
    t0 = time.time()
    st = C.vgg16_stage1()
    assert st["n_micro"] == 8 and st["micro_batch"] == 32
    compare_minibatch(st, perturb=False, backward_stream=True, verbose="cfg2 vgg16_stage1 full shapes, M=8, depth 4, backward stream")
    print("  %.1f s" % (time.time() - t0), flush=True)


def _end_to_end_gated(stage, elementwise=("y", "loss"), rowwise_dx_outliers=None, with_exact=True):
    """Whole stage, M micro-batches in 1F1B order, every tensor under the rule of flip_gate; tensors whose name
    starts with one of `elementwise` also within the element-wise tolerance.  rowwise_dx_outliers = (k, bound):
    dx is held to the element-wise tolerance sample by sample, except for at most k samples per micro-batch
    (those in which a ReLU gate of a wide layer flipped), which stay within `bound`."""
    t0 = time.time()
    params = gen.all_params(stage)
    xs, gs = stage_io(stage)
    orc, gpu = OracleStage(stage, params), GpuStage(stage, params)
    # with_exact=False (the LSTM stage, whose oracle pass takes most of a minute): no un-rounded pass; the tensors named
    # in `elementwise` are held to the element-wise bound, the others to a plain L2 bound of five times it
    exact = OracleStage(stage, params, storage="exact") if with_exact else None
    tol = TOL[stage["dtype"]]
    pools = [i for i, L in enumerate(stage["layers"]) if L["kind"] == C.MAXPOOL2D]
    records, bad = [], []

    def judge(name, got, ref_b, ref_e):
        if ref_e is None:
            e = flip_gate.l2(got, ref_b)
            ok, rec = bool(np.all(np.isfinite(got))) and e <= 5 * tol, dict(name=name, e_impl=e, e_ref=0.0, e_pair=e, f_impl=0.0, f_ref=0.0)
        else:
            ok, rec = flip_gate.check(name, got, ref_b, ref_e, tol)
        rec["max_norm"] = rel_err(got, ref_b)
        records.append(rec)
        if not ok:
            bad.append(("flip_gate", rec))
        if name.startswith(tuple(elementwise)) and not rec["max_norm"] <= tol:
            bad.append(("element-wise", rec))

    for t, m in one_f_one_b_order(stage["n_micro"], orc.depth):
        if t == "F":
            y_b, y_e, y = orc.forward(m, xs[m]), (exact.forward(m, xs[m]) if exact else None), gpu.forward(m, xs[m])
            judge("y%d" % m, y, y_b, y_e)
            y_err = rel_err(y, y_b)
            for li in pools:
                ir, ig = orc.pool_indices(m, li), gpu.pool_indices(li, m)
                ie = exact.pool_indices(m, li) if exact else ir
                src = stage["layers"][li]["src0"]
                xin = orc.stash[m][0] if src < 0 else orc.stash[m][1][src]
                gap, frac, frac_ref = pool_index_gap(xin, ir, ig, stage["layers"][li]), float(np.mean(ir != ig)), float(np.mean(ir != ie))
                print("   pool layer %d mb %d: %.2e of windows differ (bf16 vs exact oracle: %.2e), worst gap %.2e of max" % (
                    li, m, frac, frac_ref, gap), flush=True)
                # the arg-max may differ only where the two candidates are as close as the tensors themselves are
                # (twice the error measured on this run's output), and not more often than rounding moves it
                assert gap <= max(2 * y_err, 2.0 ** -7), ("pool arg-max differs beyond a tie", li, m, gap, y_err)
                assert frac <= flip_gate.FACTOR * frac_ref + 1e-3, ("pool arg-max differs too often", li, m, frac, frac_ref)
        else:
            dx_b, dx_e, dx = orc.backward(m, gs[m]), (exact.backward(m, gs[m]) if exact else None), gpu.backward(m, gs[m])
            if dx_b is not None:
                judge("dx%d" % m, dx, dx_b, dx_e)
                if rowwise_dx_outliers:
                    k, bound = rowwise_dx_outliers
                    scale = np.max(np.abs(dx_b))
                    per_sample = np.max(np.abs(dx - dx_b).reshape(dx.shape[0], -1), axis=1) / scale
                    out = per_sample > tol
                    print("   dx%d: %d of %d samples beyond %.0e, worst %.2e" % (m, int(out.sum()), len(out), tol, per_sample.max()), flush=True)
                    if out.sum() > k or per_sample.max() > bound:
                        bad.append(("dx sample by sample", m, int(out.sum()), float(per_sample.max())))
            if gpu.is_loss:
                l_b, l = orc.loss[m], B.bapipe_stage_get_loss(gpu.h, m)
                assert abs(l - l_b) <= 1e-3 * abs(l_b), (l, l_b)
    for i, (w, b) in enumerate(params):
        if w is not None:
            dw, db = gpu.grads(i)
            judge("dw%d" % i, dw, orc.dw[i], exact.dw[i] if exact else None)
            if b is not None:
                judge("db%d" % i, db, orc.db[i], exact.db[i] if exact else None)
    gpu.close()
    for r in records:
        print("  " + flip_gate.fmt(r) + "  max-norm %.2e" % r["max_norm"], flush=True)
    print("  %s end to end: %d tensors, %.1f s" % (stage["name"], len(records), time.time() - t0), flush=True)
    assert not bad, bad


@pytest.mark.timeout(900)
def test_vgg16_deep_end_to_end_full_shapes():
    _end_to_end_gated(C.vgg16_deep(n_micro=1))


@pytest.mark.timeout(900)
def test_vgg16_deep_further_streams_same_bits_full_shapes():
    """Beside kernels of further streams the 14x14 layers take other pixel tiles than alone on the chip (a choice that
    only exists at full size): every output must still agree bit for bit with the one-stream run.  GPU only."""
    from gpu_harness import gpu_minibatch
    stage = C.vgg16_deep(n_micro=4)                 # depth 2: backward passes overlap later forward passes
    ref = gpu_minibatch(stage)
    got = gpu_minibatch(stage, eager_sync=False, backward_stream=True)
    assert sorted(got) == sorted(ref) and any(k.startswith("dw") for k in ref)
    for k in ref:
        assert np.array_equal(got[k], ref[k]), k


@pytest.mark.timeout(900)
def test_vgg16_classifier_end_to_end_full_shapes():
    # three layers deep: everything element-wise (weight and bias gradients included), the input gradient sample by
    # sample - one flipped ReLU gate among the 4096 units of a hidden layer moves that sample's dx by about
    # 1/sqrt(active units) = 2 % of the maximum, and 64 x 4096 x 2 gates leave a flip or two per micro-batch
    _end_to_end_gated(C.vgg16_classifier(n_micro=2), elementwise=("y", "loss", "dw", "db"), rowwise_dx_outliers=(3, 0.1))


@pytest.mark.timeout(900)
def test_resnet50_stage_end_to_end_full_shapes():
    _end_to_end_gated(C.resnet50_stage(n_micro=1), elementwise=("loss",))


# ------------------------------------------------------------------------------ layer by layer
def _one_layer_stage(stage, li, in_shape, fuse_relu, need_dx):
    L = dict(stage["layers"][li], src0=-1, src1=-1, fuse_relu=fuse_relu)
    return C._stage("%s.layer%d" % (stage["name"], li), [L], stage["dtype"], in_shape[1:], in_shape[0], 1, 1, 1,
                    1 if need_dx else 0, stage["seed"], stage["init"])


_TRACED = {}


def _oracle_pass(stage):
    """One traced oracle pass over micro-batch 0 of the whole stage, shared by the layer-by-layer and the slice
    tests of the same workload (only the latest workload is kept)."""
    key = (stage["name"], stage["micro_batch"])
    if key not in _TRACED:
        _TRACED.clear()
        t0 = time.time()
        params = gen.all_params(stage)
        xs, gs = stage_io(stage)
        orc = OracleStage(stage, params)
        orc.trace = {}
        orc.forward(0, xs[0])
        aux = orc.stash[0][2]
        dx_stage = orc.backward(0, gs[0])
        print("%s: oracle pass %.1f s" % (stage["name"], time.time() - t0), flush=True)
        _TRACED[key] = (params, gs, orc, aux, dx_stage)
    return _TRACED[key]


def _layerwise(stage, tag):
    t0 = time.time()
    tol = TOL[stage["dtype"]]
    params, gs, orc, aux, _ = _oracle_pass(stage)
    worst = {}
    tested = 0
    for li, L in enumerate(stage["layers"]):
        k = L["kind"]
        if k in (C.ADD, C.FLATTEN):
            continue                                    # two-input / aliasing layers: covered by the slice tests below
        tr = orc.trace[(0, li)]
        x = tr["x"]
        if x.ndim == 2:
            x = x.reshape(x.shape[0], -1, 1, 1)
        if k == C.LINEAR:
            x = x.reshape(x.shape[0], -1, 1, 1)
        x32 = x.astype(np.float32)
        need_dx = "dx" in tr
        p = [params[li]]
        # forward with the layer as configured
        st = _one_layer_stage(stage, li, x.shape, L["fuse_relu"], need_dx)
        g1 = GpuStage(st, p)
        y = g1.forward(0, x32)
        y_ref = tr["y"].reshape(y.shape)
        errs = {"y": rel_err(y, y_ref)}
        if k == C.MAXPOOL2D:
            assert np.array_equal(g1.pool_indices(0, 0), aux[li]), (tag, li, "pool indices")
        if k == C.SOFTMAX_XENT:
            dz = g1.backward(0, gs[0])
            errs["dx"] = rel_err(dz, tr["dx"].reshape(dz.shape))
            errs["loss"] = abs(B.bapipe_stage_get_loss(g1.h, 0) - orc.loss[0]) / abs(orc.loss[0])
            g1.close()
        else:
            g1.close()
            # backward on a clone without the fused ReLU, fed the oracle's already gated gradient
            st2 = _one_layer_stage(stage, li, x.shape, 0, need_dx)
            g2 = GpuStage(st2, p)
            g2.forward(0, x32)
            g = tr["g"].reshape(y.shape).astype(np.float32)
            dx = g2.backward(0, g)
            if need_dx:
                errs["dx"] = rel_err(dx, tr["dx"].reshape(dx.shape))
            if params[li][0] is not None:
                dw, db = g2.grads(0)
                errs["dw"] = rel_err(dw, orc.dw[li])
                if db is not None:
                    errs["db"] = rel_err(db, orc.db[li])
            g2.close()
        tested += 1
        for name, e in errs.items():
            worst[name] = max(worst.get(name, 0.0), e)
        bad = {n: e for n, e in errs.items() if not e <= tol}
        assert not bad, (tag, "layer %d (%s)" % (li, C.KIND_NAMES[k]), bad)
    print("%s: %d layers, worst errors %s, %.1f s" % (tag, tested, {n: "%.2e" % e for n, e in worst.items()},
                                                      time.time() - t0), flush=True)


@pytest.mark.timeout(900)
def test_vgg16_classifier_layerwise_full_shapes():
    _layerwise(C.vgg16_classifier(n_micro=1), "cfg4 layerwise")


# ------------------------------------------------------------------------------ slice by slice
def _slice_stage(stage, lo, hi, in_shape, need_dx, last_relu=None):
    """Layers lo..hi-1 of `stage` as a stage of their own, fed by the tensor that feeds layer lo."""
    t_in = stage["layers"][lo]["src0"]
    layers = []
    for i in range(lo, hi):
        L = dict(stage["layers"][i])
        for key in ("src0", "src1"):
            s0 = L[key]
            if key == "src1" and L["kind"] != C.ADD:
                continue
            if s0 == t_in:
                L[key] = -1
            else:
                assert lo <= s0 < hi, ("slice reads a tensor from outside", i, key, s0)
                L[key] = s0 - lo
        layers.append(L)
    for i, L in enumerate(stage["layers"]):                  # the slice's input must have no reader outside the slice
        if not lo <= i < hi:
            assert L["src0"] != t_in and not (L["kind"] == C.ADD and L["src1"] == t_in), (i, t_in)
    if last_relu is not None:
        layers[-1]["fuse_relu"] = last_relu
    return C._stage("%s[%d:%d]" % (stage["name"], lo, hi), layers, stage["dtype"], in_shape[1:], in_shape[0], 1, 1, 1,
                    1 if need_dx else 0, stage["seed"], stage["init"])


def _slices(stage, ranges, tag):
    """Teacher-forced runs of consecutive layers: input, gated output gradient and every expected value from
    one oracle pass over the whole stage.  Forward output and pool indices as for single layers; the gradients
    (input, weights, bias), which the slice's inner ReLU gates shape, in L2 (half the tolerance) with at most 1e-3
    of their elements (one element of a small tensor) beyond the element-wise bound."""
    t0 = time.time()
    tol = TOL[stage["dtype"]]
    params, gs, orc, aux, dx_stage = _oracle_pass(stage)
    for lo, hi in ranges:
        first, last = stage["layers"][lo], stage["layers"][hi - 1]
        x = orc.trace[(0, lo)]["x"]
        t_in = first["src0"]
        need_dx = t_in >= 0 or bool(stage["need_input_grad"])
        dx_ref = (orc.trace[(0, t_in)]["gout"] if t_in >= 0 else dx_stage) if need_dx else None
        p = params[lo:hi]
        g1 = GpuStage(_slice_stage(stage, lo, hi, x.shape, need_dx), p)
        y = g1.forward(0, x.astype(np.float32))
        y_ref = orc.trace[(0, hi - 1)]["y"].reshape(y.shape)
        errs = {"y": rel_err(y, y_ref)}
        for i in range(lo, hi):
            if stage["layers"][i]["kind"] == C.MAXPOOL2D:
                ig = g1.pool_indices(i - lo, 0)
                if not np.array_equal(ig, aux[i]):
                    # the pool's input comes out of this slice's own conv: candidates must be a rounding apart at most
                    src = stage["layers"][i]["src0"]
                    gap = pool_index_gap(orc.trace[(0, src)]["y"], aux[i], ig, stage["layers"][i])
                    assert gap <= 2.0 ** -7 and np.mean(ig != aux[i]) <= 1e-3, (tag, i, gap, float(np.mean(ig != aux[i])))
        g1.close()
        # backward on a clone whose last layer has no fused ReLU, fed the oracle's gated gradient
        g2 = GpuStage(_slice_stage(stage, lo, hi, x.shape, need_dx, last_relu=0), p)
        g2.forward(0, x.astype(np.float32))
        g = orc.trace[(0, hi - 1)]["g"].reshape(y.shape).astype(np.float32)
        dx = g2.backward(0, g)
        back = {}
        if need_dx:
            back["dx"] = (dx, dx_ref.reshape(dx.shape))
        for i in range(lo, hi):
            if params[i][0] is not None:
                dw, db = g2.grads(i - lo)
                back["dw%d" % i] = (dw, orc.dw[i])
                if db is not None:
                    back["db%d" % i] = (db, orc.db[i])
        g2.close()
        # gradients inside a slice pass the slice's own ReLU gates (and batch-norm scales by 1/std, which singles out
        # channels of small variance): L2 within half the tolerance, at most 1e-3 of the elements beyond the
        # element-wise bound (an element behind a flipped gate can be off by its whole value, so no cap on those)
        off, worst = {}, {}
        for name, (got, ref) in back.items():
            errs[name + "_l2"] = 2 * flip_gate.l2(got, ref)
            worst[name] = rel_err(got, ref)
            off[name] = flip_gate.off_fraction(got, ref, tol)
        print("%s layers %d..%d: %s, beyond tol %s, worst element %s" % (
            tag, lo, hi - 1, {n: "%.2e" % e for n, e in errs.items()}, {n: "%.1e" % e for n, e in off.items() if e > 0},
            {n: "%.1e" % e for n, e in worst.items() if e > tol}), flush=True)
        bad = {n: e for n, e in errs.items() if not e <= tol}
        bad.update({n + "_off": e for n, e in off.items() if e * back[n][1].size > max(1.0, 1e-3 * back[n][1].size)})
        assert not bad, (tag, (lo, hi), bad)
    print("%s: %d slices, %.1f s" % (tag, len(ranges), time.time() - t0), flush=True)


def _blocks(stage):
    """[lo, hi) of every residual block: it ends with an ADD and starts after the previous one."""
    out, lo = [], 0
    for i, L in enumerate(stage["layers"]):
        if L["kind"] == C.ADD:
            out.append((lo, i + 1))
            lo = i + 1
    return out


def _conv_pool_pairs(stage):
    return [(i, i + 2) for i, L in enumerate(stage["layers"][:-1])
            if L["kind"] == C.CONV2D and stage["layers"][i + 1]["kind"] == C.MAXPOOL2D and stage["layers"][i + 1]["src0"] == i]


@pytest.mark.timeout(900)
def test_vgg16_stage1_layers_and_conv_pool_slices_full_shapes():
    st = C.vgg16_stage1(n_micro=1)
    _layerwise(st, "cfg2 layerwise")
    assert _conv_pool_pairs(st) == [(1, 3), (4, 6)]
    _slices(st, _conv_pool_pairs(st) + [(3, 6)], "cfg2 slices")


@pytest.mark.timeout(900)
def test_vgg16_deep_layers_and_conv_pool_slices_full_shapes():
    st = C.vgg16_deep(n_micro=1)
    _layerwise(st, "cfg3 layerwise")
    _slices(st, _conv_pool_pairs(st), "cfg3 slices")


@pytest.mark.timeout(900)
def test_resnet50_stage_layers_and_bottleneck_blocks_full_shapes():
    st = C.resnet50_stage(n_micro=1)
    _layerwise(st, "cfg5 layerwise")
    blocks = _blocks(st)
    assert len(blocks) == 10
    _slices(st, blocks, "cfg5 blocks")


# ------------------------------------------------------------------------------ the remaining stages
@pytest.mark.timeout(900)
def test_vgg16_conv3_full_shapes():
    _end_to_end_gated(C.vgg16_conv3(n_micro=1))
    _layerwise(C.vgg16_conv3(n_micro=1), "vgg16 conv3 layerwise")


@pytest.mark.timeout(900)
def test_resnet50_stem_full_shapes():
    _end_to_end_gated(C.resnet50_stem(n_micro=1), elementwise=("loss",))
    _layerwise(C.resnet50_stem(n_micro=1), "resnet50 stem layerwise")


@pytest.mark.timeout(900)
def test_resnet50_tail_full_shapes():
    _end_to_end_gated(C.resnet50_tail(n_micro=1), elementwise=("loss",))
    _layerwise(C.resnet50_tail(n_micro=1), "resnet50 tail layerwise")


@pytest.mark.timeout(900)
def test_gnmt_lstm_stage_full_shapes():
    _end_to_end_gated(C.gnmt_lstm_stage(n_micro=1), with_exact=False)
    _layerwise(C.gnmt_lstm_stage(n_micro=1), "gnmt lstm layerwise")
