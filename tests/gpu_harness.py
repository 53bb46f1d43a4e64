"""Shared helpers of the GPU parity tests: run a workload through the C ABI (via the ctypes
binding) and through the CPU oracle on the same seeded inputs, and compare tensor by tensor.
Only marshalling happens here (dtype / layout conversion of inputs and outputs)."""
import ctypes as ct

import numpy as np
import torch

from oracle.stage import OracleStage, one_f_one_b_order
from paper_2012_12544_amd import binding as B
from stage_inputs import configs as C
from stage_inputs import gen

DEV = "cuda:0"
TOL = {C.FP32: 1e-4, C.BF16: 2e-2}     # max|gpu-ref| / max|ref|, per tensor


def tdtype(stage):
    return torch.bfloat16 if stage["dtype"] == C.BF16 else torch.float32


def to_dev(stage, a_nchw, layout):
    """numpy NCHW float32 -> device tensor of the stage's storage type in the io layout."""
    t = torch.from_numpy(np.ascontiguousarray(a_nchw)).to(DEV)
    if layout == B.NHWC and t.dim() == 4:
        t = t.permute(0, 2, 3, 1)
    return t.contiguous().to(tdtype(stage))


def from_dev(t, shape_nchw, layout):
    """device tensor in io layout -> numpy float64 NCHW."""
    t = t.to(torch.float32)
    if layout == B.NHWC and len(shape_nchw) == 4:
        n, c, h, w = shape_nchw
        t = t.reshape(n, h, w, c).permute(0, 3, 1, 2)
    return t.contiguous().cpu().numpy().astype(np.float64).reshape(shape_nchw)


def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.all(np.isfinite(got)):
        return float("inf")
    d = np.max(np.abs(got - ref)) if ref.size else 0.0
    m = np.max(np.abs(ref)) if ref.size else 0.0
    return d / m if m > 0 else d


class GpuStage:
    def __init__(self, stage, params, layout=B.NHWC, loss_scale=0.0, use_torch_alloc=True, stream=None,
                 backward_stream=False, wgrad_stream=False):
        self.stage = stage
        self.layout = layout
        self.alloc = B.TorchAllocator(DEV) if use_torch_alloc else None
        self.stream = stream if stream is not None else torch.cuda.Stream(device=DEV)
        self.opts = B.make_opts(stage, io_layout=layout, stream=self.stream.cuda_stream,
                                allocator=self.alloc, loss_scale=loss_scale)
        self.h = B.bapipe_stage_create(stage["layers"], stage["micro_batch"], stage["n_micro"], self.opts)
        self.shapes = C.infer_shapes(stage)
        self.params = params
        for i, (w, b) in enumerate(params):
            if w is not None:
                B.bapipe_stage_set_params(self.h, i, w, b)
        self.keep = []
        self.is_loss = gen.ends_in_loss(stage)
        self.bstream = self.wstream = None
        if backward_stream:       # backward passes, and their weight-gradient kernels, on streams of their own
            self.bstream = torch.cuda.Stream(device=DEV)
            self.wstream = torch.cuda.Stream(device=DEV) if backward_stream != "no wgrad stream" else None
            B.bapipe_stage_set_streams(self.h, self.bstream.cuda_stream, None if self.wstream is None else self.wstream.cuda_stream)
        elif wgrad_stream:
            self.wstream = torch.cuda.Stream(device=DEV)
            B.bapipe_stage_set_streams(self.h, None, self.wstream.cuda_stream)

    def close(self):
        if self.h is not None:
            B.bapipe_stage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def out_shape(self):
        return (self.stage["micro_batch"],) + tuple(self.shapes[-1])

    def in_shape(self):
        s = self.stage
        return (s["micro_batch"], s["in_c"], s["in_h"], s["in_w"])

    def forward(self, mb, x_nchw):
        x = to_dev(self.stage, x_nchw, self.layout)
        n = int(np.prod(self.out_shape()))
        y = torch.empty(n, dtype=torch.float32 if self.is_loss else tdtype(self.stage), device=DEV)
        torch.cuda.synchronize()
        B.bapipe_stage_forward(self.h, mb, x.data_ptr(), y.data_ptr())
        torch.cuda.synchronize()
        return from_dev(y, self.out_shape(), self.layout)

    def backward(self, mb, dy_or_labels, want_dx=True, static=False):
        if self.is_loss:
            g = torch.from_numpy(np.ascontiguousarray(dy_or_labels, np.int32)).to(DEV)
        else:
            g = to_dev(self.stage, dy_or_labels, self.layout)
        dx = None
        if self.stage["need_input_grad"] and want_dx:
            dx = torch.empty(int(np.prod(self.in_shape())), dtype=tdtype(self.stage), device=DEV)
        torch.cuda.synchronize()
        entry = B.bapipe_stage_backward_static if static else B.bapipe_stage_backward
        entry(self.h, mb, g.data_ptr(), None if dx is None else dx.data_ptr())
        torch.cuda.synchronize()
        return None if dx is None else from_dev(dx, self.in_shape(), self.layout)

    def grads(self, i):
        w, b = self.params[i]
        return B.bapipe_stage_get_grads(self.h, i, None if w is None else w.shape, None if b is None else b.shape)

    def get_params(self, i):
        w, b = self.params[i]
        return B.bapipe_stage_get_params(self.h, i, None if w is None else w.shape, None if b is None else b.shape)

    def pool_indices(self, layer, mb):
        shp = (self.stage["micro_batch"],) + tuple(self.shapes[layer])
        return B.bapipe_stage_get_pool_indices(self.h, layer, mb, shp)


def stage_io(stage):
    M = stage["n_micro"]
    xs = [gen.stage_input(stage, m) for m in range(M)]
    if gen.ends_in_loss(stage):
        gs = [gen.labels(stage, m) for m in range(M)]
    else:
        gs = [gen.upstream_grad(stage, m) for m in range(M)]
    return xs, gs


def gpu_minibatch(stage, static=False, layout=B.NHWC, backward_stream=False, eager_sync=True, wgrad_stream=False):
    """One mini-batch in 1F1B order on the GPU alone: every output the library hands back (y and dx
    per micro-batch, losses, all weight gradients), by name.  eager_sync=False enqueues the whole
    mini-batch without waiting in between (inputs uploaded beforehand), so that passes really overlap
    when there is a backward stream."""
    params = gen.all_params(stage, perturb=True)
    xs, gs = stage_io(stage)
    g = GpuStage(stage, params, layout=layout, backward_stream=backward_stream, wgrad_stream=wgrad_stream)
    if not eager_sync:
        return _minibatch_enqueued_at_once(stage, g, params, xs, gs, static)
    _, depth = B.bapipe_stage_stash_bytes(g.h)
    out = {}
    for t, m in one_f_one_b_order(stage["n_micro"], depth):
        if t == "F":
            out["y%d" % m] = g.forward(m, xs[m])
        else:
            dx = g.backward(m, gs[m], static=static)
            if dx is not None:
                out["dx%d" % m] = dx
            if g.is_loss:
                out["loss%d" % m] = np.float64(B.bapipe_stage_get_loss(g.h, m))
    for i, (w, b) in enumerate(params):
        if w is not None:
            dw, db = g.grads(i)
            out["dw%d" % i] = dw
            if db is not None:
                out["db%d" % i] = db
    g.close()
    return out


def _minibatch_enqueued_at_once(stage, g, params, xs, gs, static):
    M = stage["n_micro"]
    _, depth = B.bapipe_stage_stash_bytes(g.h)
    dxs = [to_dev(stage, x, g.layout) for x in xs]
    if g.is_loss:
        dgs = [torch.from_numpy(np.ascontiguousarray(v, np.int32)).to(DEV) for v in gs]
    else:
        dgs = [to_dev(stage, v, g.layout) for v in gs]
    n_out = int(np.prod(g.out_shape()))
    ys = [torch.empty(n_out, dtype=torch.float32 if g.is_loss else tdtype(stage), device=DEV) for _ in range(M)]
    need_dx = bool(stage["need_input_grad"])
    dxo = [torch.empty(int(np.prod(g.in_shape())), dtype=tdtype(stage), device=DEV) if need_dx else None for _ in range(M)]
    torch.cuda.synchronize()
    entry = B.bapipe_stage_backward_static if static else B.bapipe_stage_backward
    for t, m in one_f_one_b_order(M, depth):
        if t == "F":
            B.bapipe_stage_forward(g.h, m, dxs[m].data_ptr(), ys[m].data_ptr())
        else:
            entry(g.h, m, dgs[m].data_ptr(), dxo[m].data_ptr() if need_dx else None)
    torch.cuda.synchronize()
    out = {}
    for m in range(M):
        out["y%d" % m] = from_dev(ys[m], g.out_shape(), g.layout)
        if need_dx:
            out["dx%d" % m] = from_dev(dxo[m], g.in_shape(), g.layout)
        if g.is_loss:
            out["loss%d" % m] = np.float64(B.bapipe_stage_get_loss(g.h, m))
    for i, (w, b) in enumerate(params):
        if w is not None:
            dw, db = g.grads(i)
            out["dw%d" % i] = dw
            if db is not None:
                out["db%d" % i] = db
    g.close()
    return out


def pool_index_gap(layer_in, idx_ref, idx_gpu, L):
    """Largest gap, over the windows whose arg-max differs, between the oracle's values at its own
    and at the GPU's arg-max position, relative to max|layer_in| (0 when the indices agree)."""
    bad = np.argwhere(idx_ref != idx_gpu)
    kw, st, pad = L["kw"], L["stride"], L["pad"]
    worst = 0.0
    for n, c, p, q in bad:
        a, b = int(idx_ref[n, c, p, q]), int(idx_gpu[n, c, p, q])
        va = layer_in[n, c, p * st + a // kw - pad, q * st + a % kw - pad]
        vb = layer_in[n, c, p * st + b // kw - pad, q * st + b % kw - pad]
        worst = max(worst, abs(va - vb))
    return worst / max(float(np.max(np.abs(layer_in))), 1e-30)


def compare_minibatch(stage, layout=B.NHWC, perturb=True, order=None, lr=0.05, check_pool=True,
                      tol=None, verbose=None, dx_where_output_gates_agree=False, backward_stream=False):
    """Full parity of one mini-batch: y, dx per micro-batch, pool indices, loss, every weight
    gradient after M micro-batches and the updated weights after step.  Returns the worst
    relative errors by tensor name.
    dx_where_output_gates_agree: for stages of 1x1 layers ending in a fused ReLU (a pixel's input
    gradient depends on that pixel's gates only): dx is compared at the pixels where the two sides'
    output gates (y > 0) agree in every channel, and the share of disagreeing gates is bounded."""
    tol = TOL[stage["dtype"]] if tol is None else tol
    params = gen.all_params(stage, perturb=perturb)
    xs, gs = stage_io(stage)
    orc = OracleStage(stage, params)
    gpu = GpuStage(stage, params, layout=layout, backward_stream=backward_stream)
    M = stage["n_micro"]
    order = order or one_f_one_b_order(M, orc.depth)
    per, depth = B.bapipe_stage_stash_bytes(gpu.h)
    assert depth == orc.depth
    errs = {}
    bf16 = stage["dtype"] == C.BF16
    pools = [i for i, L in enumerate(stage["layers"]) if L["kind"] == C.MAXPOOL2D]
    exact_pool = True
    gate_ok = {}
    for t, m in order:
        if t == "F":
            y_ref = orc.forward(m, xs[m])
            y = gpu.forward(m, xs[m])
            errs["y%d" % m] = rel_err(y, y_ref)
            if dx_where_output_gates_agree:
                flipped = (y > 0) != (y_ref > 0)
                assert np.mean(flipped) <= 1e-3, ("ReLU gates differ too often", m, float(np.mean(flipped)))
                gate_ok[m] = ~np.any(flipped, axis=1)                # [n, h, w]
            if check_pool:
                for li in pools:
                    ir, ig = orc.pool_indices(m, li), gpu.pool_indices(li, m)
                    assert ig.max() < stage["layers"][li]["kh"] * stage["layers"][li]["kw"]
                    if not np.array_equal(ir, ig):
                        exact_pool = False
                        src = stage["layers"][li]["src0"]
                        xin = orc.stash[m][0] if src < 0 else orc.stash[m][1][src]
                        # End to end the pool inputs of the two sides are only equal up to the error the tensors
                        # themselves show, so the arg-max is unique only up to that: where the indices differ the
                        # oracle's two candidates must be no further apart than twice the error measured on this
                        # micro-batch's output (at least one bf16 rounding step of the largest value), and such
                        # windows must be rare.  (With identical inputs the indices are bit-exact: see the pool-only
                        # stages in test_gpu_stage.py.)
                        gap, frac = pool_index_gap(xin, ir, ig, stage["layers"][li]), float(np.mean(ir != ig))
                        if verbose:
                            print("   pool layer %d mb %d: %.2e of windows differ, worst gap %.2e of max" % (li, m, frac, gap), flush=True)
                        bound = max(2 * errs["y%d" % m], 2.0 ** -7) if bf16 else 1e-6
                        assert gap <= bound, ("pool arg-max differs beyond a tie", li, m, gap, bound)
                        assert frac <= (1e-3 if bf16 else 1e-5), frac
        else:
            dx_ref = orc.backward(m, gs[m])
            dx = gpu.backward(m, gs[m])
            if dx_ref is not None and dx_where_output_gates_agree:
                assert dx.shape[2:] == gate_ok[m].shape[1:]
                keep = np.broadcast_to(gate_ok[m][:, None], dx.shape)
                errs["dx%d" % m] = float(np.max(np.abs(dx - dx_ref)[keep]) / np.max(np.abs(dx_ref)))
                if verbose:
                    print("   mb %d: dx compared at %.4f of the pixels" % (m, float(np.mean(gate_ok[m]))), flush=True)
            elif dx_ref is not None:
                errs["dx%d" % m] = rel_err(dx, dx_ref)
            if gpu.is_loss:
                l_ref, l = orc.loss[m], B.bapipe_stage_get_loss(gpu.h, m)
                errs["loss%d" % m] = abs(l - l_ref) / max(abs(l_ref), 1e-30)
    for i, (w, b) in enumerate(params):
        if w is None:
            continue
        dw, db = gpu.grads(i)
        errs["dw%d" % i] = rel_err(dw, orc.dw[i])
        if b is not None:
            errs["db%d" % i] = rel_err(db, orc.db[i])
    orc.step(lr)
    B.bapipe_stage_step(gpu.h, lr)
    for i, (w, b) in enumerate(params):
        if w is None:
            continue
        w2, b2 = gpu.get_params(i)
        errs["w%d" % i] = rel_err(w2, orc.w[i])
        if b is not None:
            errs["b%d" % i] = rel_err(b2, orc.b[i])
        dw, db = gpu.grads(i)
        assert not dw.any(), "step must clear the accumulators"
    gpu.close()
    worst = max(errs.values())
    if verbose:
        print(verbose, "worst rel err %.3e" % worst, "exact pool idx" if exact_pool else "pool idx tie-level diffs",
              {k: "%.2e" % v for k, v in sorted(errs.items(), key=lambda kv: -kv[1])[:4]}, flush=True)
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, (stage["name"], bad)
    return errs
