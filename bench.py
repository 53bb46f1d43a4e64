#!/usr/bin/env python3
"""Stage fwd+bwd throughput of one pipeline stage on one MI355X.

A "step" is one mini-batch of the workload: M forward and M backward passes in 1F1B order
(depth warm-up forwards, alternate B/F, drain) followed by the weight update, all enqueued
through the C ABI without waiting in between - forward passes and the update on one HIP stream,
backward passes on a second one and their weight-gradient kernels on a third (--streams 3, the
default; the library orders them with events), so that independent kernels share the chip; inputs and upstream gradients of
all M micro-batches are seeded synthetic tensors resident in HBM before the timed region.

Prints ONE JSON line for the headline workload (default: VGG-16 stage 1): samples/s (value), ms per
step (mean of the K timed steps and the median of their per-step event times), TFLOP/s, and
  roofline       - the dominant kernel class, timed live with HIP events on the stage's stream (the
                   library's tap brackets every launch of the class) over extra steps run right after
                   the timed ones, on ONE stream (the tap's events cost a few per cent and kernels of
                   two streams sharing the chip cannot be timed one by one, so the headline runs
                   with the tap off), against MI355X's published peak and against the peaks measured
                   on this very GPU (register-resident MFMA loop, streaming copy)
  per_config     - the other configurations of the benchmark suite, each timed the same way for a
                   few steps in the same process: ms per step, samples/s, TFLOP/s, dominant class
  measured_peaks - what bapipe_measure_peaks and bapipe_measure_lds return on this GPU
  cpu_baseline   - the CPU oracle timed on the host cores on a bounded sample of the workload
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from stage_inputs import configs as C  # noqa: E402
from stage_inputs import gen  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PEAK_FP32_VALU_TFLOPS = 157.3
SUITE = ["tiny", "vgg16_stage1", "vgg16_deep", "vgg16_classifier", "resnet50_stage"]   # the five configurations


def one_f_one_b(M, depth):
    W = min(M, depth)
    order = [("F", m) for m in range(W)]
    for m in range(M - W):
        order += [("B", m), ("F", m + W)]
    order += [("B", m) for m in range(M - W, M)]
    return order


def cpu_baseline(stage, sample):
    """Oracle fwd+bwd on `sample` samples (same seeded inputs), timed: the first `sample` samples of micro-batch 0,
    or whole micro-batches 0, 1, ... when `sample` is a multiple of the micro-batch size."""
    from oracle import ops
    from oracle.stage import OracleStage
    mb = stage["micro_batch"]
    n_mb = max(1, sample // mb)
    per = sample if n_mb == 1 else mb
    sub = dict(stage, micro_batch=per, n_micro=n_mb)
    params = gen.all_params(stage)
    loss = gen.ends_in_loss(stage)
    xs = [gen.stage_input(stage, m)[:per] for m in range(n_mb)]
    gs = [(gen.labels(stage, m) if loss else gen.upstream_grad(stage, m))[:per] for m in range(n_mb)]
    orc = OracleStage(sub, params, depth=1)
    t0 = time.time()
    for m in range(n_mb):
        orc.forward(m, xs[m])
        orc.backward(m, gs[m])
    dt = time.time() - t0
    what = "%d samples of micro-batch 0" % per if n_mb == 1 else "micro-batches 0..%d (%d samples)" % (n_mb - 1, per * n_mb)
    return dict(value=per * n_mb / dt, unit="samples/s", cores=int(ops.num_threads()), kind="oracle",
                sample="%s, fwd+bwd, %.1f s" % (what, dt))


class Workload:
    """One stage created through the C ABI with its seeded inputs resident in HBM."""

    def __init__(self, name, torch, B, dev="cuda:0", streams=3, **shape):
        self.name, self.torch, self.B = name, torch, B
        self.stage = stage = C.FULL[name](**shape)
        self.M, self.mb = stage["n_micro"], stage["micro_batch"]
        tdt = torch.bfloat16 if stage["dtype"] == C.BF16 else torch.float32
        is_loss = gen.ends_in_loss(stage)

        def up(x):
            t = torch.from_numpy(x).to(dev)
            if t.dim() == 4:
                t = t.permute(0, 2, 3, 1)
            return t.contiguous().to(tdt)

        self.xs = [up(gen.stage_input(stage, m)) for m in range(self.M)]
        if is_loss:
            self.gs = [torch.from_numpy(gen.labels(stage, m)).to(dev) for m in range(self.M)]
        else:
            self.gs = [up(gen.upstream_grad(stage, m)) for m in range(self.M)]
        oshape = (self.mb,) + tuple(C.infer_shapes(stage)[-1])
        self.y = torch.empty(int(np.prod(oshape)), dtype=torch.float32 if is_loss else tdt, device=dev)
        self.dx = torch.empty(self.xs[0].numel(), dtype=tdt, device=dev) if stage["need_input_grad"] else None
        self.stream = torch.cuda.Stream(device=dev)
        self.alloc = B.TorchAllocator(dev)
        opts = B.make_opts(stage, io_layout=B.NHWC, stream=self.stream.cuda_stream, allocator=self.alloc)
        self.h = B.bapipe_stage_create(stage["layers"], self.mb, self.M, opts)
        for i, (w, b) in enumerate(gen.all_params(stage)):
            if w is not None:
                B.bapipe_stage_set_params(self.h, i, w, b)
        self.per_mb, self.depth = B.bapipe_stage_stash_bytes(self.h)
        self.order = one_f_one_b(self.M, self.depth)
        # backward passes on a stream of their own, beside the forward passes of later micro-batches; a ring of
        # depth 1 leaves nothing to overlap
        self.bstream = torch.cuda.Stream(device=dev) if streams >= 2 and self.depth >= 2 else None
        self.wstream = torch.cuda.Stream(device=dev) if streams >= 3 and self.bstream is not None else None
        self.streams = 1 + (self.bstream is not None) + (self.wstream is not None)
        self.set_streams(True)

    def set_streams(self, on):
        bs = self.bstream.cuda_stream if on and self.bstream is not None else None
        ws = self.wstream.cuda_stream if on and self.wstream is not None else None
        self.B.bapipe_stage_set_streams(self.h, bs, ws)

    def step(self, lr=0.01):
        B, h = self.B, self.h
        dxp = None if self.dx is None else self.dx.data_ptr()
        for t, m in self.order:
            if t == "F":
                B.bapipe_stage_forward(h, m, self.xs[m].data_ptr(), self.y.data_ptr())
            else:
                B.bapipe_stage_backward(h, m, self.gs[m].data_ptr(), dxp)
        B.bapipe_stage_step(h, lr)

    def timed(self, steps, warmup):
        """K steps bracketed by events on the stage's stream (tap off): total ms, per-step ms list, host seconds."""
        torch = self.torch
        self.B.bapipe_stage_kernel_timing(self.h, -1)
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.time()
        ev[0].record(self.stream)
        for k in range(steps):
            self.step()
            ev[k + 1].record(self.stream)
        torch.cuda.synchronize()
        wall = time.time() - t0
        return ev[0].elapsed_time(ev[steps]), [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)], wall

    def roofline(self, tap, tap_steps, peaks):
        """The dominant kernel class (or the named one) under the library's event tap for tap_steps steps."""
        torch, B, h = self.torch, self.B, self.h
        # one stream for these steps: with kernels of two streams sharing the chip the event pair around a launch
        # would time both
        torch.cuda.synchronize()
        self.set_streams(False)
        names = dict(gather=B.KC_CONV_GATHER_MFMA, wgrad=B.KC_CONV_WGRAD_MFMA, direct=B.KC_CONV_DIRECT,
                     pool=B.KC_POOL, bn=B.KC_BATCHNORM, eltwise=B.KC_ELEMENTWISE)
        if tap == "auto":      # one untimed step per candidate, pick the class with the largest share
            best, best_ms = None, -1.0
            for name, kc in names.items():
                B.bapipe_stage_kernel_timing(h, kc)
                self.step()
                r = B.bapipe_stage_kernel_timing_read(h)
                if r["total_ms"] > best_ms:
                    best, best_ms = name, r["total_ms"]
            tap = best
        B.bapipe_stage_kernel_timing(h, names[tap])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(self.stream)
        for _ in range(tap_steps):
            self.step()
        e1.record(self.stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        r = B.bapipe_stage_kernel_timing_read(h)
        B.bapipe_stage_kernel_timing(h, -1)
        self.set_streams(self.streams > 1)
        sec = r["total_ms"] * 1e-3
        mfma_meas, copy_meas = peaks
        other = None
        if tap in ("gather", "wgrad", "direct"):
            ach = r["flop"] / sec / 1e12 if sec > 0 else 0.0
            bound, unit = ("alu", "TFLOP/s") if tap == "direct" else ("mfma", "TFLOP/s")
            peak = PEAK_FP32_VALU_TFLOPS if tap == "direct" else PEAK_BF16_TFLOPS
            meas = None if tap == "direct" else mfma_meas
            # a contraction with little reuse (weight streaming of the linear layers, one-step recurrent products)
            # sits on the HBM roof instead: report the roof the launches are closer to, keep the other beside it
            gbs = r["bytes"] / sec / 1e9 if sec > 0 else 0.0
            if tap != "direct" and gbs / PEAK_HBM_GBS > ach / peak:
                other = dict(bound=bound, achieved=round(ach, 2), peak=peak, unit=unit, frac=round(ach / peak, 4))
                ach, bound, unit, peak, meas = gbs, "hbm", "GB/s", PEAK_HBM_GBS, copy_meas
            else:
                other = dict(bound="hbm", achieved=round(gbs, 2), peak=PEAK_HBM_GBS, unit="GB/s",
                             frac=round(gbs / PEAK_HBM_GBS, 4))
        else:
            ach = r["bytes"] / sec / 1e9 if sec > 0 else 0.0
            bound, unit, peak, meas = "hbm", "GB/s", PEAK_HBM_GBS, copy_meas
        # HBM bytes per launch of this class as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
        # (profiles/<workload>_traffic.json); null if absent
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "%s_traffic.json" % self.name)
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("per_class", {}).get(tap)
        roof = dict(bound=bound, kernel_class=tap, achieved=round(ach, 2), peak=peak, unit=unit,
                    frac=round(ach / peak, 4), traffic=None if traffic is None else round(traffic),
                    launches=int(r["launches"]), avg_launch_ms=round(r["total_ms"] / max(1, r["launches"]), 5),
                    share_of_step=round(r["total_ms"] / ms, 4) if ms > 0 else None,
                    measured_peak=None if not meas else round(meas, 1),
                    frac_of_measured_peak=None if not meas else round(ach / meas, 4))
        if other is not None:
            roof["other_roof"] = other
        return roof

    def summary(self, total_ms, per_step, steps):
        ms_per_step = total_ms / steps
        flop = C.flops_per_minibatch(self.stage)
        tflops = flop / (ms_per_step * 1e-3) / 1e12
        return dict(ms_per_step=round(ms_per_step, 4), ms_per_step_median=round(statistics.median(per_step), 4),
                    samples_per_s=round(self.mb * self.M / (ms_per_step * 1e-3), 2), tflops=round(tflops, 2),
                    frac_of_bf16_mfma_peak=round(tflops / PEAK_BF16_TFLOPS, 4))

    def close(self):
        self.B.bapipe_stage_destroy(self.h)
        self.h = None
        self.xs = self.gs = self.y = self.dx = None
        self.alloc = None
        self.torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg16_stage1", choices=sorted(C.FULL))
    ap.add_argument("--tap", default="auto", help="kernel class for the roofline tap: auto|gather|wgrad|direct|pool|bn|eltwise")
    ap.add_argument("--tap-steps", type=int, default=3, help="extra steps run under the event tap for the roofline object")
    ap.add_argument("--streams", type=int, default=3, choices=[1, 2, 3],
                    help="2: backward passes on their own stream beside later forward passes (where the ring is deeper "
                         "than 1); 3: also their weight-gradient kernels on a stream of their own")
    ap.add_argument("--micro-batch", type=int, default=0, help="override the workload's micro-batch size (a different workload: say so)")
    ap.add_argument("--n-micro", type=int, default=0, help="override the workload's number of micro-batches per mini-batch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="time only the headline workload")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured-peak microbenchmarks")
    ap.add_argument("--cpu-sample", type=int, default=0)
    ap.add_argument("--profile-layers", action="store_true", help="also print the per-layer profile (stderr)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus %d is not supported "
              "(no collectives or sharding exist here)" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2012_12544_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.load()
    dev = "cuda:0"
    torch.cuda.init()
    peaks, lds = (None, None), (None, None)
    if not a.no_peaks:
        peaks = B.bapipe_measure_peaks(torch.cuda.current_stream().cuda_stream)
        lds = B.bapipe_measure_lds(torch.cuda.current_stream().cuda_stream)

    shape = {}
    if a.micro_batch:
        shape["micro_batch"] = a.micro_batch
    if a.n_micro:
        shape["n_micro"] = a.n_micro
    w = Workload(a.workload, torch, B, dev, a.streams, **shape)
    stage = w.stage

    if a.profile_layers:
        prof = B.bapipe_profile_layers(w.h, 2, 5, len(stage["layers"]))
        for i, p in enumerate(prof):
            print("layer %2d %-12s fwd %8.3f ms  bwd %8.3f ms  w %10d B  out %11d B  stash %11d B" % (
                i, C.KIND_NAMES[stage["layers"][i]["kind"]], p["fwd_ms"], p["bwd_ms"], p["weight_bytes"],
                p["out_feature_bytes"], p["stash_bytes"]), file=sys.stderr)

    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)                                     # one element-wise read+write pass
        torch.cuda.synchronize()
        del src, dst

    total_ms, per_step, wall = w.timed(a.steps, a.warmup)
    head = w.summary(total_ms, per_step, a.steps)
    roof = w.roofline(a.tap, max(1, a.tap_steps), peaks)

    out = {
        "metric": "stage fwd+bwd samples/s (1F1B mini-batch incl. weight update)",
        "value": head["samples_per_s"], "unit": "samples/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if stage["dtype"] == C.BF16 else "f32", "data": "synthetic",
        "config": {"workload": a.workload, "micro_batch": w.mb, "n_micro": w.M, "stash_depth": w.depth,
                   "stash_bytes_per_micro_batch": w.per_mb, "schedule": "1F1B", "io_layout": "NHWC", "streams": w.streams},
        "ms_per_step_median": head["ms_per_step_median"],
        "tflops": head["tflops"], "frac_of_bf16_mfma_peak": head["frac_of_bf16_mfma_peak"],
        "host_wall_s": round(wall, 3),
        "roofline": roof,
    }
    if peaks[0]:
        out["measured_peaks"] = {"mfma_bf16_tflops": round(peaks[0], 1), "copy_gbs": round(peaks[1], 1),
                                 "frac_of_measured_mfma_peak": round(head["tflops"] / peaks[0], 4),
                                 "lds_read_b128_tbs": round(lds[0], 1), "lds_read_b64_tr_tbs": round(lds[1], 1)}
    w.close()

    if not a.no_per_config:
        # the other configurations of the suite, a few steps each (the headline's figures are repeated for reference)
        per = {a.workload: dict(head, dominant_class=roof["kernel_class"], class_bound=roof["bound"], class_frac=roof["frac"])}
        for name in SUITE:
            if name == a.workload:
                continue
            wl = Workload(name, torch, B, dev, a.streams)
            steps = 5
            t_ms, t_steps, _ = wl.timed(steps, 2)
            if wl.bstream is not None:
                # both ways: a stage whose kernels are a few microseconds long can lose more to the event hand-overs
                # between the streams than the overlap returns
                torch.cuda.synchronize()
                wl.set_streams(False)
                o_ms, o_steps, _ = wl.timed(steps, 1)
                one = round(o_ms / steps, 4)
                if o_ms < t_ms:
                    t_ms, t_steps, wl.streams = o_ms, o_steps, 1
                else:
                    wl.set_streams(True)
            rec = wl.summary(t_ms, t_steps, steps)
            if wl.bstream is not None:
                rec["ms_per_step_one_stream"] = one
            rf = wl.roofline("auto", 2, peaks)
            rec.update(streams=wl.streams, dominant_class=rf["kernel_class"], class_bound=rf["bound"], class_frac=rf["frac"],
                       class_achieved=rf["achieved"], class_unit=rf["unit"], steps=steps)
            per[name] = rec
            wl.close()
        out["per_config"] = per

    if not a.no_cpu_baseline:
        # about 10-30 s of oracle work on the 16 host threads of the GPU machine
        default_sample = {"tiny": 16, "vgg16_stage1": 64, "vgg16_deep": 32, "vgg16_classifier": 64,
                          "resnet50_stage": 32, "vgg16_conv3": 32, "resnet50_stem": 32, "resnet50_tail": 32,
                          "vgg16_full": 16, "resnet50_full": 32, "gnmt_lstm_stage": 64}[a.workload]
        sample = min(w.mb * w.M, a.cpu_sample or default_sample)
        if sample > w.mb:
            sample -= sample % w.mb                       # whole micro-batches
        out["cpu_baseline"] = cpu_baseline(stage, sample)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
