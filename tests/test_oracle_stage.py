"""Pins for the oracle's stage runner: whole-stage finite differences on shrunken copies of
the five workloads, micro-batch gradient accumulation == full-batch gradient, 1F1B order
independence, the stash-depth closed form of the paper's Tables I/II, and the update rule."""
import numpy as np
import pytest

from oracle.stage import OracleStage, ScheduleError, one_f_one_b_order
from stage_inputs import configs as C
from stage_inputs import gen

RNG = np.random.default_rng(777)


def small_stages():
    return {
        "tiny": C.tiny_stage(c=4, hw=8, micro_batch=2, n_micro=2),
        "tiny_unfused": C.tiny_stage(c=4, hw=8, micro_batch=2, n_micro=2, fused=False),
        "vgg16_stage1": C.vgg16_stage1(c1=4, c2=6, hw=8, micro_batch=2, n_micro=2),
        "vgg16_deep": C.vgg16_deep(cin=4, c=6, hw=8, micro_batch=2, n_micro=2),
        "vgg16_classifier": C.vgg16_classifier(c=4, hw=3, hidden=10, classes=7, micro_batch=3, n_micro=2),
        "resnet50_stage": C.resnet50_stage(cin=8, mid3=4, mid4=6, hw=8, n3=2, n4=2, micro_batch=3, n_micro=2),
        "vgg16_conv3": C.vgg16_conv3(cin=4, c=6, hw=8, micro_batch=2, n_micro=2),
        "resnet50_stem": C.resnet50_stem(c=4, hw=16, n2=2, micro_batch=3, n_micro=2),
        "resnet50_tail": C.resnet50_tail(cin=8, mid=4, hw=4, n5=2, classes=5, micro_batch=3, n_micro=2),
        "gnmt_lstm_stage": C.gnmt_lstm_stage(hidden=5, seq=6, n_layers=2, micro_batch=3, n_micro=2),
    }


def run_minibatch(orc, stage, order=None, xs=None, gs=None):
    M = stage["n_micro"]
    xs = xs or [gen.stage_input(stage, m) for m in range(M)]
    if gs is None:
        gs = [gen.labels(stage, m) if gen.ends_in_loss(stage) else gen.upstream_grad(stage, m)
              for m in range(M)]
    ys, dxs = {}, {}
    order = order or [(t, m) for m in range(M) for t in ("F", "B")]
    for t, m in order:
        if t == "F":
            ys[m] = orc.forward(m, xs[m])
        else:
            dxs[m] = orc.backward(m, gs[m])
    return ys, dxs


def scalar_objective(stage, params, xs, gs):
    """sum_m <stage(x_m), g_m> for regression stages, sum_m loss_m for the classifier."""
    orc = OracleStage(stage, params, storage="exact", depth=stage["n_micro"])
    tot = 0.0
    for m in range(stage["n_micro"]):
        y = orc.forward(m, xs[m])
        if gen.ends_in_loss(stage):
            orc.backward(m, gs[m])
            tot += orc.loss[m]
        else:
            tot += float(np.sum(y * gs[m]))
            orc.n_bwd += 1
    return tot


@pytest.mark.parametrize("name", list(small_stages()))
def test_whole_stage_finite_differences(name):
    stage = dict(small_stages()[name])
    stage["need_input_grad"] = 1
    stage["dtype"] = C.FP32
    params = [(None if w is None else w.astype(np.float64), None if b is None else b.astype(np.float64))
              for (w, b) in gen.all_params(stage, perturb=True)]
    M = stage["n_micro"]
    xs = [gen.stage_input(stage, m).astype(np.float64) for m in range(M)]
    gs = [gen.labels(stage, m) if gen.ends_in_loss(stage) else gen.upstream_grad(stage, m).astype(np.float64)
          for m in range(M)]
    orc = OracleStage(stage, params, storage="exact")
    _, dxs = run_minibatch(orc, stage, xs=xs, gs=gs)
    h = 1e-6
    checked = 0
    # weights / biases
    for li, (w, b) in enumerate(params):
        for arr, grad in ((w, orc.dw[li]), (b, orc.db[li])):
            if arr is None:
                continue
            for _ in range(2):
                ix = tuple(int(RNG.integers(0, s)) for s in arr.shape)
                old = arr[ix]
                arr[ix] = old + h
                fp = scalar_objective(stage, params, xs, gs)
                arr[ix] = old - h
                fm = scalar_objective(stage, params, xs, gs)
                arr[ix] = old
                num = (fp - fm) / (2 * h)
                assert abs(num - grad[ix]) <= 2e-5 * max(1.0, abs(num)), (name, li, ix, num, grad[ix])
                checked += 1
    # stage input
    for m in range(M):
        for _ in range(3):
            ix = tuple(int(RNG.integers(0, s)) for s in xs[m].shape)
            old = xs[m][ix]
            xs[m][ix] = old + h
            fp = scalar_objective(stage, params, xs, gs)
            xs[m][ix] = old - h
            fm = scalar_objective(stage, params, xs, gs)
            xs[m][ix] = old
            num = (fp - fm) / (2 * h)
            assert abs(num - dxs[m][ix]) <= 2e-5 * max(1.0, abs(num)), (name, m, ix, num, dxs[m][ix])
            checked += 1
    assert checked >= 8


@pytest.mark.parametrize("name", ["tiny", "vgg16_stage1", "vgg16_deep", "vgg16_classifier"])
def test_microbatch_accumulation_equals_full_batch(name):
    stage = dict(small_stages()[name])
    stage["dtype"] = C.FP32
    params = gen.all_params(stage, perturb=True)
    M, b = stage["n_micro"], stage["micro_batch"]
    xs = [gen.stage_input(stage, m) for m in range(M)]
    loss = gen.ends_in_loss(stage)
    gs = [gen.labels(stage, m) if loss else gen.upstream_grad(stage, m) for m in range(M)]
    orc = OracleStage(stage, params, storage="exact")
    run_minibatch(orc, stage, xs=xs, gs=gs)
    big = dict(stage, micro_batch=M * b, n_micro=1)
    orc1 = OracleStage(big, params, storage="exact", loss_scale=orc.loss_scale)
    orc1.forward(0, np.concatenate(xs))
    orc1.backward(0, np.concatenate(gs))
    for li in range(len(stage["layers"])):
        if orc.dw[li] is not None:
            np.testing.assert_allclose(orc.dw[li], orc1.dw[li], rtol=1e-11, atol=1e-12)
        if orc.db[li] is not None:
            np.testing.assert_allclose(orc.db[li], orc1.db[li], rtol=1e-11, atol=1e-12)
    if loss:
        assert abs(sum(orc.loss.values()) - orc1.loss[0]) < 1e-12


@pytest.mark.parametrize("name", ["vgg16_deep", "resnet50_stage"])
@pytest.mark.parametrize("storage", ["exact", "bf16"])
def test_1f1b_order_gives_the_same_results(name, storage):
    stage = dict(small_stages()[name], n_micro=5)
    params = gen.all_params(stage, perturb=True)
    a = OracleStage(stage, params, storage=storage)
    ya, da = run_minibatch(a, stage)
    b = OracleStage(stage, params, storage=storage)
    order = one_f_one_b_order(stage["n_micro"], b.depth)
    yb, dbb = run_minibatch(b, stage, order=order)
    assert b.peak_in_flight == b.depth
    for m in range(stage["n_micro"]):
        assert np.array_equal(ya[m], yb[m]) and np.array_equal(da[m], dbb[m])
    for li in range(len(stage["layers"])):
        if a.dw[li] is not None:
            assert np.array_equal(a.dw[li], b.dw[li])


@pytest.mark.parametrize("M,i,N,so", [(8, 1, 4, 0), (8, 3, 4, 0), (8, 4, 4, 0), (2, 1, 4, 0), (8, 2, 4, 1),
                                      (8, 1, 4, 1), (1, 1, 1, 0)])
def test_stash_depth_closed_form(M, i, N, so):
    """Features memory (N-i+1)*a for 1F1B and 2(N-i+1)*a with doubled warm-up (Tables I/II)."""
    stage = dict(small_stages()["tiny"], n_micro=M, stage_index=i, n_stages=N,
                 schedule=C.SCHED_1F1B_SO if so else C.SCHED_1F1B)
    orc = OracleStage(stage, gen.all_params(stage))
    want = min(M, (2 if so else 1) * (N - i + 1))
    assert orc.depth == want
    order = one_f_one_b_order(M, orc.depth)
    assert [m for t, m in order if t == "B"] == list(range(M))        # FIFO backward
    assert sum(1 for t, _ in order if t == "F") == M
    run_minibatch(orc, stage, order=order)
    assert orc.peak_in_flight == want


def test_schedule_violations_raise():
    stage = small_stages()["tiny"]
    orc = OracleStage(stage, gen.all_params(stage), depth=1)
    x, g = gen.stage_input(stage, 0), gen.upstream_grad(stage, 0)
    with pytest.raises(ScheduleError):
        orc.backward(0, g)
    with pytest.raises(ScheduleError):
        orc.forward(1, x)
    orc.forward(0, x)
    with pytest.raises(ScheduleError):
        orc.forward(1, x)                      # depth 1 exceeded
    with pytest.raises(ScheduleError):
        orc.step(0.1)
    orc.backward(0, g)
    orc.forward(1, x)
    orc.backward(1, g)
    orc.step(0.1)


def test_step_is_plain_sgd_and_clears_gradients():
    stage = small_stages()["vgg16_classifier"]
    params = gen.all_params(stage, perturb=True)
    orc = OracleStage(stage, params, storage="exact")
    run_minibatch(orc, stage)
    w0 = [None if w is None else w.copy() for w in orc.w]
    g0 = [None if g is None else g.copy() for g in orc.dw]
    orc.step(0.5)
    for li in range(len(stage["layers"])):
        if w0[li] is not None:
            np.testing.assert_allclose(orc.w[li], w0[li] - 0.5 * g0[li], rtol=0, atol=1e-15)
            assert not orc.dw[li].any()
    assert orc.n_fwd == 0 and orc.n_bwd == 0


def test_bf16_storage_outputs_are_representable_and_close_to_exact():
    from oracle import ops
    for name, tol in (("resnet50_stage", None), ("vgg16_deep", 0.05)):
        stage = small_stages()[name]
        params = gen.all_params(stage, perturb=True)
        a = OracleStage(stage, params, storage="bf16")
        b = OracleStage(stage, params, storage="exact")
        ya, da = run_minibatch(a, stage)
        yb, db_ = run_minibatch(b, stage)
        for m in ya:
            assert np.array_equal(ops.round_bf16(ya[m]), ya[m])
            assert np.array_equal(ops.round_bf16(da[m]), da[m])
            if tol:       # (the tiny BN stage flips ReLU masks under rounding; no closeness claim)
                assert np.max(np.abs(ya[m] - yb[m])) <= tol * np.max(np.abs(yb[m]))
                assert np.max(np.abs(da[m] - db_[m])) <= 5 * tol * np.max(np.abs(db_[m]))   # pool argmax flips


def test_workload_shapes_and_flop_table():
    """MAC counts per sample fixed by the layer shapes of the workloads; the whole networks add up
    to the well-known 15.47 GMAC (VGG-16) and 4.09 GMAC (ResNet-50, stride on the 3x3)."""
    want = {"tiny": 2.80e6, "vgg16_stage1": 4.711e9, "vgg16_deep": 6.011e9,
            "vgg16_classifier": 123.6e6, "resnet50_stage": 2.492e9, "vgg16_conv3": 4.624e9,
            "resnet50_stem": 785.9e6, "resnet50_tail": 811.3e6, "vgg16_full": 15.47e9,
            "resnet50_full": 4.089e9, "gnmt_lstm_stage": 2 * 50 * 4 * 1024 * 2048}
    for name, f in C.FULL.items():
        st = f()
        macs, _ = C.conv_fc_macs_per_sample(st)
        assert abs(macs - want[name]) / want[name] < 2e-3, (name, macs)
    assert abs(C.flops_per_minibatch(C.vgg16_stage1()) - 7.19e12) / 7.19e12 < 2e-3
    assert abs(C.flops_per_minibatch(C.vgg16_deep()) - 18.47e12) / 18.47e12 < 2e-3
    st5 = C.resnet50_stage()
    assert C.infer_shapes(st5)[-1] == (1024, 14, 14)
    assert sum(1 for L in st5["layers"] if L["kind"] == C.BATCHNORM2D) == 32
    v, r = C.vgg16_full(), C.resnet50_full()
    assert sum(1 for L in v["layers"] if L["kind"] == C.CONV2D) == 13
    assert sum(1 for L in v["layers"] if L["kind"] == C.LINEAR) == 3
    assert C.infer_shapes(v)[-1] == (1000, 1, 1) and C.infer_shapes(r)[-1] == (1000, 1, 1)
    assert sum(1 for L in r["layers"] if L["kind"] == C.CONV2D) == 53       # 1 + 3*16 + 4 projections
    assert sum(1 for L in r["layers"] if L["kind"] == C.BATCHNORM2D) == 53
    assert C.infer_shapes(C.resnet50_stem())[-1] == (256, 56, 56)
    assert C.infer_shapes(C.resnet50_tail())[-3] == (2048, 1, 1)


def test_input_generators_are_deterministic_and_bf16_representable():
    st = C.vgg16_deep(cin=8, c=8, hw=4, micro_batch=2)
    a, b = gen.stage_input(st, 3), gen.stage_input(st, 3)
    assert np.array_equal(a, b) and not np.array_equal(a, gen.stage_input(st, 4))
    assert np.array_equal(gen.snap_bf16(a), a)
    w, bias = gen.layer_params(st, 0)
    assert abs(w.std() - np.sqrt(2 / (8 * 9))) < 0.02 and not bias.any()
    cls = C.vgg16_classifier(c=8, hw=2, hidden=16, classes=5, micro_batch=4)
    w, _ = gen.layer_params(cls, 1)
    assert np.abs(w).max() <= np.sqrt(6 / (32 + 16))
    lab = gen.labels(cls, 0)
    assert lab.dtype == np.int32 and lab.min() >= 0 and lab.max() < 5
