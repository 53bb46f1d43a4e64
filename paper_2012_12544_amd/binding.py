"""ctypes binding of libbapipe_stage.so (include/bapipe_stage.h): argument marshalling only.

Every arithmetic step runs in the library's HIP kernels; PyTorch supplies device memory
(tensors whose data_ptr() is handed over) and the HIP stream.  Loading fails loudly if the
library has not been built (`python -m paper_2012_12544_amd.build`); there is no fallback.
"""
import ctypes as ct
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbapipe_stage.so")

OK, E_INVALID, E_SHAPE, E_ORDER, E_OOM, E_DEVICE, E_UNSUPPORTED = range(7)
STATUS_NAMES = ["OK", "E_INVALID", "E_SHAPE", "E_ORDER", "E_OOM", "E_DEVICE", "E_UNSUPPORTED"]
FP32, BF16 = 0, 1
NCHW, NHWC = 0, 1
SCHED_1F1B, SCHED_1F1B_SO = 0, 1
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "bapipe_stage_create", "bapipe_stage_forward", "bapipe_stage_backward", "bapipe_stage_backward_static",
    "bapipe_stage_set_streams",
    "bapipe_stage_step",
    "bapipe_profile_layers", "bapipe_profile_sweep", "bapipe_stage_set_params", "bapipe_stage_get_params",
    "bapipe_stage_get_grads", "bapipe_stage_get_pool_indices", "bapipe_stage_get_loss",
    "bapipe_stage_stash_bytes", "bapipe_last_error", "bapipe_stage_destroy",
    "bapipe_stage_kernel_timing", "bapipe_stage_kernel_timing_read", "bapipe_measure_peaks", "bapipe_measure_lds",
    "bapipe_schedule_cost", "bapipe_schedule_choose", "bapipe_partition",
]
PLAN_1F1B_AS, PLAN_FBP_AS, PLAN_1F1B_SNO, PLAN_1F1B_SO = range(4)
KC_CONV_GATHER_MFMA, KC_CONV_WGRAD_MFMA, KC_CONV_DIRECT, KC_POOL, KC_BATCHNORM, KC_ELEMENTWISE = range(6)


class LayerDesc(ct.Structure):
    _fields_ = [("kind", ct.c_int32), ("cin", ct.c_int32), ("cout", ct.c_int32), ("kh", ct.c_int32),
                ("kw", ct.c_int32), ("stride", ct.c_int32), ("pad", ct.c_int32),
                ("has_bias", ct.c_int32), ("fuse_relu", ct.c_int32), ("src0", ct.c_int32),
                ("src1", ct.c_int32), ("eps", ct.c_float)]


ALLOC_FN = ct.CFUNCTYPE(ct.c_void_p, ct.c_size_t, ct.c_void_p)
FREE_FN = ct.CFUNCTYPE(None, ct.c_void_p, ct.c_void_p)


class Allocator(ct.Structure):
    _fields_ = [("alloc", ALLOC_FN), ("free", FREE_FN), ("ctx", ct.c_void_p)]


class StageOpts(ct.Structure):
    _fields_ = [("dtype", ct.c_int32), ("in_c", ct.c_int32), ("in_h", ct.c_int32), ("in_w", ct.c_int32),
                ("io_layout", ct.c_int32), ("stage_index", ct.c_int32), ("n_stages", ct.c_int32),
                ("schedule", ct.c_int32), ("need_input_grad", ct.c_int32), ("loss_scale", ct.c_float),
                ("hip_stream", ct.c_void_p), ("mem", Allocator)]


class LayerProfile(ct.Structure):
    _fields_ = [("fwd_ms", ct.c_double), ("bwd_ms", ct.c_double), ("weight_bytes", ct.c_uint64),
                ("out_feature_bytes", ct.c_uint64), ("stash_bytes", ct.c_uint64)]


class BapipeError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 7 else status, message))
        self.status = status


_lib = None


def load():
    """Load the built library; raise if it is missing (no CPU or eager fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libbapipe_stage.so is not built: run `python -m paper_2012_12544_amd.build` "
                           "(hipcc, gfx950); the library has no fallback path")
    lib = ct.CDLL(LIB_PATH)
    vp, i32 = ct.c_void_p, ct.c_int
    lib.bapipe_stage_create.argtypes = [ct.POINTER(LayerDesc), i32, i32, i32, ct.POINTER(StageOpts), ct.POINTER(vp)]
    lib.bapipe_stage_forward.argtypes = [vp, i32, vp, vp]
    lib.bapipe_stage_backward.argtypes = [vp, i32, vp, vp]
    lib.bapipe_stage_backward_static.argtypes = [vp, i32, vp, vp]
    lib.bapipe_stage_set_streams.argtypes = [vp, vp, vp]
    lib.bapipe_stage_step.argtypes = [vp, ct.c_float]
    lib.bapipe_profile_layers.argtypes = [vp, i32, i32, ct.POINTER(LayerProfile), i32, ct.POINTER(i32)]
    fp = ct.POINTER(ct.c_float)
    lib.bapipe_stage_set_params.argtypes = [vp, i32, fp, fp]
    lib.bapipe_stage_get_params.argtypes = [vp, i32, fp, fp]
    lib.bapipe_stage_get_grads.argtypes = [vp, i32, fp, fp]
    lib.bapipe_stage_get_pool_indices.argtypes = [vp, i32, i32, ct.POINTER(ct.c_uint8)]
    lib.bapipe_stage_get_loss.argtypes = [vp, i32, fp]
    lib.bapipe_stage_stash_bytes.argtypes = [vp, ct.POINTER(ct.c_uint64), ct.POINTER(i32)]
    lib.bapipe_stage_kernel_timing.argtypes = [vp, i32]
    lib.bapipe_stage_kernel_timing_read.argtypes = [vp, ct.POINTER(ct.c_double), ct.POINTER(ct.c_uint64),
                                                    ct.POINTER(ct.c_double), ct.POINTER(ct.c_double)]
    lib.bapipe_measure_peaks.argtypes = [vp, ct.POINTER(ct.c_double), ct.POINTER(ct.c_double)]
    lib.bapipe_measure_lds.argtypes = [vp, ct.POINTER(ct.c_double), ct.POINTER(ct.c_double)]
    lib.bapipe_last_error.argtypes = [vp]
    lib.bapipe_last_error.restype = ct.c_char_p
    lib.bapipe_stage_destroy.argtypes = [vp]
    lib.bapipe_stage_destroy.restype = None
    for name in EXPORTS:
        if name not in ("bapipe_last_error", "bapipe_stage_destroy"):
            getattr(lib, name).restype = ct.c_int
    _lib = lib
    return lib


def _check(status, handle=None):
    if status != OK:
        raise BapipeError(status, (load().bapipe_last_error(handle) or b"").decode())


class TorchAllocator:
    """Backs the library's device allocations with torch tensors (PyTorch caching allocator)."""

    def __init__(self, device="cuda:0", fail_after=None):
        import torch
        self._torch = torch
        self.device = device
        self.live = {}
        self.fail_after = fail_after      # test hook: the n-th allocation returns NULL
        self.count = 0
        self._a = ALLOC_FN(self._alloc)
        self._f = FREE_FN(self._free)

    def _alloc(self, nbytes, ctx):
        self.count += 1
        if self.fail_after is not None and self.count > self.fail_after:
            return None
        try:
            t = self._torch.empty(int(nbytes) + 256, dtype=self._torch.uint8, device=self.device)
        except Exception:                       # out of memory -> NULL, reported as E_OOM
            return None
        p = (t.data_ptr() + 255) // 256 * 256
        self.live[p] = t
        return p

    def _free(self, ptr, ctx):
        self.live.pop(ptr, None)

    def struct(self):
        return Allocator(self._a, self._f, None)


def make_layer_array(layers):
    arr = (LayerDesc * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = LayerDesc(L["kind"], L["cin"], L["cout"], L["kh"], L["kw"], L["stride"], L["pad"],
                           L["has_bias"], L["fuse_relu"], L["src0"], L["src1"], L["eps"])
    return arr


def bapipe_stage_create(layers, micro_batch, n_micro, opts):
    """layers: list of dicts with the LayerDesc fields; opts: StageOpts.  Returns the handle."""
    lib = load()
    arr = make_layer_array(layers)
    h = ct.c_void_p()
    st = lib.bapipe_stage_create(arr, len(layers), micro_batch, n_micro, ct.byref(opts), ct.byref(h))
    _check(st, None)
    return h


def bapipe_stage_forward(h, mb_id, x_ptr, y_ptr):
    _check(load().bapipe_stage_forward(h, mb_id, x_ptr, y_ptr), h)


def bapipe_stage_backward(h, mb_id, dy_or_labels_ptr, dx_ptr):
    _check(load().bapipe_stage_backward(h, mb_id, dy_or_labels_ptr, dx_ptr), h)


def bapipe_stage_backward_static(h, mb_id, dy_or_labels_ptr, dx_ptr):
    _check(load().bapipe_stage_backward_static(h, mb_id, dy_or_labels_ptr, dx_ptr), h)


def bapipe_stage_set_streams(h, backward_stream, wgrad_stream):
    _check(load().bapipe_stage_set_streams(h, backward_stream, wgrad_stream), h)


def bapipe_stage_step(h, lr):
    _check(load().bapipe_stage_step(h, lr), h)


def bapipe_profile_layers(h, warmup, iters, n_layers):
    out = (LayerProfile * n_layers)()
    n = ct.c_int(0)
    _check(load().bapipe_profile_layers(h, warmup, iters, out, n_layers, ct.byref(n)), h)
    return [dict(fwd_ms=out[i].fwd_ms, bwd_ms=out[i].bwd_ms, weight_bytes=out[i].weight_bytes,
                 out_feature_bytes=out[i].out_feature_bytes, stash_bytes=out[i].stash_bytes)
            for i in range(n.value)]


def bapipe_profile_sweep(layers, micro_batches, opts, warmup=1, iters=3):
    """Per-layer profile at each micro-batch size: {size: [record per layer]}."""
    descs = make_layer_array(layers)
    sizes = (ct.c_int * len(micro_batches))(*[int(m) for m in micro_batches])
    out = (LayerProfile * (len(layers) * len(micro_batches)))()
    _check(load().bapipe_profile_sweep(descs, len(layers), sizes, len(micro_batches), ct.byref(opts), warmup, iters, out))
    n = len(layers)
    return {int(m): [dict(fwd_ms=out[k * n + i].fwd_ms, bwd_ms=out[k * n + i].bwd_ms, weight_bytes=out[k * n + i].weight_bytes,
                          out_feature_bytes=out[k * n + i].out_feature_bytes, stash_bytes=out[k * n + i].stash_bytes)
                     for i in range(n)] for k, m in enumerate(micro_batches)}


def _fptr(a):
    return None if a is None else a.ctypes.data_as(ct.POINTER(ct.c_float))


def bapipe_stage_set_params(h, layer, w, b):
    w = None if w is None else np.ascontiguousarray(w, np.float32)
    b = None if b is None else np.ascontiguousarray(b, np.float32)
    _check(load().bapipe_stage_set_params(h, layer, _fptr(w), _fptr(b)), h)


def bapipe_stage_get_params(h, layer, w_shape, b_shape):
    w = None if w_shape is None else np.empty(w_shape, np.float32)
    b = None if b_shape is None else np.empty(b_shape, np.float32)
    _check(load().bapipe_stage_get_params(h, layer, _fptr(w), _fptr(b)), h)
    return w, b


def bapipe_stage_get_grads(h, layer, w_shape, b_shape):
    w = None if w_shape is None else np.empty(w_shape, np.float32)
    b = None if b_shape is None else np.empty(b_shape, np.float32)
    _check(load().bapipe_stage_get_grads(h, layer, _fptr(w), _fptr(b)), h)
    return w, b


def bapipe_stage_get_pool_indices(h, layer, mb_id, shape):
    idx = np.empty(shape, np.uint8)
    _check(load().bapipe_stage_get_pool_indices(h, layer, mb_id, idx.ctypes.data_as(ct.POINTER(ct.c_uint8))), h)
    return idx


def bapipe_stage_get_loss(h, mb_id):
    v = ct.c_float(0)
    _check(load().bapipe_stage_get_loss(h, mb_id, ct.byref(v)), h)
    return v.value


def bapipe_stage_stash_bytes(h):
    per = ct.c_uint64(0)
    depth = ct.c_int(0)
    _check(load().bapipe_stage_stash_bytes(h, ct.byref(per), ct.byref(depth)), h)
    return per.value, depth.value


def bapipe_stage_kernel_timing(h, kernel_class):
    _check(load().bapipe_stage_kernel_timing(h, kernel_class), h)


def bapipe_stage_kernel_timing_read(h):
    ms, n, fl, by = ct.c_double(0), ct.c_uint64(0), ct.c_double(0), ct.c_double(0)
    _check(load().bapipe_stage_kernel_timing_read(h, ct.byref(ms), ct.byref(n), ct.byref(fl), ct.byref(by)), h)
    return dict(total_ms=ms.value, launches=n.value, flop=fl.value, bytes=by.value)


def bapipe_measure_peaks(stream=0):
    """(bf16 MFMA TFLOP/s of a register-resident loop, GB/s of a streaming copy) on the current device."""
    tf, gb = ct.c_double(0), ct.c_double(0)
    _check(load().bapipe_measure_peaks(stream, ct.byref(tf), ct.byref(gb)))
    return tf.value, gb.value


def bapipe_measure_lds(stream=0):
    """(TB/s all compute units read LDS with ds_read_b128, with ds_read_b64_tr_b16) on the current device."""
    a, b = ct.c_double(0), ct.c_double(0)
    _check(load().bapipe_measure_lds(stream, ct.byref(a), ct.byref(b)))
    return a.value, b.value


def bapipe_stage_destroy(h):
    load().bapipe_stage_destroy(h)


def make_opts(stage, io_layout=NHWC, stream=0, allocator=None, loss_scale=0.0, schedule=None):
    """StageOpts from a workload description (stage_inputs.configs)."""
    o = StageOpts()
    o.dtype = stage["dtype"]
    o.in_c, o.in_h, o.in_w = stage["in_c"], stage["in_h"], stage["in_w"]
    o.io_layout = io_layout
    o.stage_index, o.n_stages = stage["stage_index"], stage["n_stages"]
    o.schedule = stage.get("schedule", SCHED_1F1B) if schedule is None else schedule
    o.need_input_grad = stage["need_input_grad"]
    o.loss_scale = loss_scale
    o.hip_stream = stream
    if allocator is not None:
        o.mem = allocator.struct()
    return o


# ---------------------------------------------------------------- planner (include/bapipe_plan.h)
class ScheduleCost(ct.Structure):
    _fields_ = [("minibatch_time", ct.c_double), ("bubble_fraction", ct.c_double), ("features_memory", ct.c_double),
                ("weights_memory", ct.c_double), ("bandwidth_demand", ct.c_double), ("in_flight", ct.c_int)]


class PlanInput(ct.Structure):
    _fields_ = [("n_layers", ct.c_int), ("n_acc", ct.c_int), ("fwd_ms", ct.POINTER(ct.c_double)),
                ("bwd_ms", ct.POINTER(ct.c_double)), ("out_bytes", ct.POINTER(ct.c_double)),
                ("weight_bytes", ct.POINTER(ct.c_double)), ("stash_bytes", ct.POINTER(ct.c_double)),
                ("mem_capacity", ct.POINTER(ct.c_double)), ("link_bytes_per_ms", ct.c_double),
                ("n_micro", ct.c_int), ("schedule", ct.c_int)]


class PlanReport(ct.Structure):
    _fields_ = [("ideal_stage_ms", ct.c_double), ("seed_bottleneck_ms", ct.c_double), ("bottleneck_ms", ct.c_double),
                ("a_th_bytes", ct.c_double), ("comm_bottleneck", ct.c_int), ("memory_tuned", ct.c_int)]


def bapipe_schedule_cost(schedule, M, N, i, F, B, SR, a, w):
    out = ScheduleCost()
    _check(load().bapipe_schedule_cost(int(schedule), int(M), int(N), int(i), ct.c_double(F), ct.c_double(B),
                                       ct.c_double(SR), ct.c_double(a), ct.c_double(w), ct.byref(out)))
    return {k: getattr(out, k) for k, _ in ScheduleCost._fields_}


class ScheduleCandidate(ct.Structure):
    _fields_ = [("schedule", ct.c_int), ("n_micro", ct.c_int), ("F", ct.c_double), ("B", ct.c_double),
                ("SR", ct.c_double), ("a", ct.POINTER(ct.c_double))]


def bapipe_schedule_choose(candidates, w, capacity=None):
    """candidates: dicts with schedule, n_micro, F, B, SR, a (per-stage list).  Returns (index, cost of stage 1)."""
    N = len(w)
    keep = [_darr(c["a"]) for c in candidates]
    arr = (ScheduleCandidate * len(candidates))(*[
        ScheduleCandidate(int(c["schedule"]), int(c["n_micro"]), float(c["F"]), float(c["B"]), float(c["SR"]), k)
        for c, k in zip(candidates, keep)])
    best, cost = ct.c_int(-1), ScheduleCost()
    _check(load().bapipe_schedule_choose(arr, len(candidates), N, _darr(w), _darr(capacity) if capacity is not None else None,
                                         ct.byref(best), ct.byref(cost)))
    return best.value, {k: getattr(cost, k) for k, _ in ScheduleCost._fields_}


def _darr(values):
    values = [float(v) for v in values]
    return (ct.c_double * len(values))(*values)


def bapipe_partition(fwd_ms, bwd_ms, out_bytes, weight_bytes, stash_bytes, mem_capacity=None, link_bytes_per_ms=0.0,
                     n_micro=1, schedule=PLAN_1F1B_SO):
    """fwd_ms / bwd_ms: one row of per-layer times per accelerator.  Returns (stage_begin, report);
    raises BapipeError (status E_UNSUPPORTED: nothing satisfies the constraints)."""
    n_acc, n_layers = len(fwd_ms), len(fwd_ms[0])
    keep = [_darr([v for row in fwd_ms for v in row]), _darr([v for row in bwd_ms for v in row]), _darr(out_bytes),
            _darr(weight_bytes), _darr(stash_bytes), _darr(mem_capacity) if mem_capacity is not None else None]
    inp = PlanInput(n_layers, n_acc, keep[0], keep[1], keep[2], keep[3], keep[4],
                    keep[5] if keep[5] is not None else ct.POINTER(ct.c_double)(), float(link_bytes_per_ms),
                    int(n_micro), int(schedule))
    sb = (ct.c_int * (n_acc + 1))()
    rep = PlanReport()
    status = load().bapipe_partition(ct.byref(inp), sb, ct.byref(rep))
    report = {k: getattr(rep, k) for k, _ in PlanReport._fields_}
    if status != OK:
        err = BapipeError(status, "no partition satisfies the constraints" if status == E_UNSUPPORTED else "bad planner input")
        err.report = report
        raise err
    return list(sb), report
