#!/usr/bin/env python3
"""Stage fwd+bwd throughput of one pipeline stage on one MI355X.

A "step" is one mini-batch of the workload: M forward and M backward passes in 1F1B order
(depth warm-up forwards, alternate B/F, drain) followed by the weight update, all enqueued on
one HIP stream through the C ABI; inputs and upstream gradients of all M micro-batches are
seeded synthetic tensors resident in HBM before the timed region.

Prints ONE JSON line: samples/s (value), ms per step, TFLOP/s, and two objects:
  roofline     - the dominant kernel class, timed live with HIP events on the stage's stream
                 (library tap) over the same timed steps, against MI355X's published peak
  cpu_baseline - the CPU oracle timed on the host cores on a bounded sample of the workload
"""
import argparse
import json
import os
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


def one_f_one_b(M, depth):
    W = min(M, depth)
    order = [("F", m) for m in range(W)]
    for m in range(M - W):
        order += [("B", m), ("F", m + W)]
    order += [("B", m) for m in range(M - W, M)]
    return order


def cpu_baseline(stage, sample):
    """Oracle fwd+bwd on `sample` samples of micro-batch 0 (same seeded inputs), timed."""
    from oracle import ops
    from oracle.stage import OracleStage
    sub = dict(stage, micro_batch=sample, n_micro=1)
    params = gen.all_params(stage)
    x = gen.stage_input(stage, 0)[:sample]
    g = gen.labels(stage, 0)[:sample] if gen.ends_in_loss(stage) else gen.upstream_grad(stage, 0)[:sample]
    orc = OracleStage(sub, params, depth=1)
    t0 = time.time()
    orc.forward(0, x)
    orc.backward(0, g)
    dt = time.time() - t0
    return dict(value=sample / dt, unit="samples/s", cores=int(ops.num_threads()), kind="oracle",
                sample="%d samples of micro-batch 0, fwd+bwd, %.1f s" % (sample, dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg16_stage1", choices=sorted(C.FULL))
    ap.add_argument("--tap", default="auto", help="kernel class for the roofline tap: auto|gather|wgrad|direct|pool|bn|eltwise")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    stage = C.FULL[a.workload]()
    M, mb = stage["n_micro"], stage["micro_batch"]
    tdt = torch.bfloat16 if stage["dtype"] == C.BF16 else torch.float32
    is_loss = gen.ends_in_loss(stage)

    def up(x):
        t = torch.from_numpy(x).to(dev)
        if t.dim() == 4:
            t = t.permute(0, 2, 3, 1)
        return t.contiguous().to(tdt)

    xs = [up(gen.stage_input(stage, m)) for m in range(M)]
    if is_loss:
        gs = [torch.from_numpy(gen.labels(stage, m)).to(dev) for m in range(M)]
    else:
        gs = [up(gen.upstream_grad(stage, m)) for m in range(M)]
    oshape = (mb,) + tuple(C.infer_shapes(stage)[-1])
    y = torch.empty(int(np.prod(oshape)), dtype=torch.float32 if is_loss else tdt, device=dev)
    dx = torch.empty(xs[0].numel(), dtype=tdt, device=dev) if stage["need_input_grad"] else None

    stream = torch.cuda.Stream(device=dev)
    alloc = B.TorchAllocator(dev)
    opts = B.make_opts(stage, io_layout=B.NHWC, stream=stream.cuda_stream, allocator=alloc)
    h = B.bapipe_stage_create(stage["layers"], mb, M, opts)
    for i, (w, b) in enumerate(gen.all_params(stage)):
        if w is not None:
            B.bapipe_stage_set_params(h, i, w, b)
    per_mb, depth = B.bapipe_stage_stash_bytes(h)
    order = one_f_one_b(M, depth)
    lr = 0.01

    def step():
        for t, m in order:
            if t == "F":
                B.bapipe_stage_forward(h, m, xs[m].data_ptr(), y.data_ptr())
            else:
                B.bapipe_stage_backward(h, m, gs[m].data_ptr(), None if dx is None else dx.data_ptr())
        B.bapipe_stage_step(h, lr)

    if a.profile_layers:
        prof = B.bapipe_profile_layers(h, 2, 5, len(stage["layers"]))
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

    torch.cuda.synchronize()
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()

    tap_names = dict(gather=B.KC_CONV_GATHER_MFMA, wgrad=B.KC_CONV_WGRAD_MFMA, direct=B.KC_CONV_DIRECT,
                     pool=B.KC_POOL, bn=B.KC_BATCHNORM, eltwise=B.KC_ELEMENTWISE)
    if a.tap == "auto":
        # dominant class of this workload: one untimed step per candidate, pick the largest share
        best, best_ms = None, -1.0
        for name, kc in tap_names.items():
            B.bapipe_stage_kernel_timing(h, kc)
            step()
            r = B.bapipe_stage_kernel_timing_read(h)
            if r["total_ms"] > best_ms:
                best, best_ms = name, r["total_ms"]
        tap = best
    else:
        tap = a.tap
    B.bapipe_stage_kernel_timing(h, tap_names[tap])

    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.time()
    e0.record(stream)
    for _ in range(a.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.time() - t0
    ms = e0.elapsed_time(e1)
    r = B.bapipe_stage_kernel_timing_read(h)
    B.bapipe_stage_kernel_timing(h, -1)

    ms_per_step = ms / a.steps
    samples_per_s = mb * M / (ms_per_step * 1e-3)
    flop = C.flops_per_minibatch(stage)
    tflops = flop / (ms_per_step * 1e-3) / 1e12

    other = None
    if tap in ("gather", "wgrad", "direct"):
        ach = r["flop"] / (r["total_ms"] * 1e-3) / 1e12 if r["total_ms"] > 0 else 0.0
        bound, unit = ("alu", "TFLOP/s") if tap == "direct" else ("mfma", "TFLOP/s")
        peak = PEAK_FP32_VALU_TFLOPS if tap == "direct" else PEAK_BF16_TFLOPS
        # a contraction with little reuse (weight streaming of the linear layers, one-step recurrent products)
        # sits on the HBM roof instead: report the roof the launches are closer to, keep the other beside it
        gbs = r["bytes"] / (r["total_ms"] * 1e-3) / 1e9 if r["total_ms"] > 0 else 0.0
        if tap != "direct" and gbs / PEAK_HBM_GBS > ach / peak:
            other = dict(bound=bound, achieved=round(ach, 2), peak=peak, unit=unit, frac=round(ach / peak, 4))
            ach, bound, unit, peak = gbs, "hbm", "GB/s", PEAK_HBM_GBS
        else:
            other = dict(bound="hbm", achieved=round(gbs, 2), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(gbs / PEAK_HBM_GBS, 4))
    else:
        ach = r["bytes"] / (r["total_ms"] * 1e-3) / 1e9 if r["total_ms"] > 0 else 0.0
        bound, unit, peak = "hbm", "GB/s", PEAK_HBM_GBS
    # HBM bytes per launch of this class as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    # (profiles/<workload>_traffic.json); null if absent
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "%s_traffic.json" % a.workload)
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("per_class", {}).get(tap)
    roof = dict(bound=bound, kernel_class=tap, achieved=round(ach, 2), peak=peak, unit=unit,
                frac=round(ach / peak, 4), traffic=None if traffic is None else round(traffic),
                launches=int(r["launches"]),
                avg_launch_ms=round(r["total_ms"] / max(1, r["launches"]), 5),
                share_of_step=round(r["total_ms"] / ms, 4))
    if other is not None:
        roof["other_roof"] = other

    out = {
        "metric": "stage fwd+bwd samples/s (1F1B mini-batch incl. weight update)",
        "value": round(samples_per_s, 2), "unit": "samples/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if stage["dtype"] == C.BF16 else "f32", "data": "synthetic",
        "config": {"workload": a.workload, "micro_batch": mb, "n_micro": M, "stash_depth": depth,
                   "stash_bytes_per_micro_batch": per_mb, "schedule": "1F1B", "io_layout": "NHWC"},
        "tflops": round(tflops, 2), "frac_of_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "host_wall_s": round(wall, 3),
        "roofline": roof,
    }
    if not a.no_cpu_baseline:
        # about 10-30 s of oracle work on the 16 host threads of the GPU machine
        default_sample = {"tiny": 16, "vgg16_stage1": 32, "vgg16_deep": 32, "vgg16_classifier": 64,
                          "resnet50_stage": 32, "vgg16_conv3": 32, "resnet50_stem": 32, "resnet50_tail": 32,
                          "vgg16_full": 16, "resnet50_full": 32, "gnmt_lstm_stage": 64}[a.workload]
        sample = min(mb * M if a.workload == "tiny" else mb, a.cpu_sample or default_sample)
        sample = min(sample, mb)
        out["cpu_baseline"] = cpu_baseline(stage, sample)
    B.bapipe_stage_destroy(h)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
