#!/usr/bin/env python3
"""Benchmark of the merged-operator hot path on one MI355X.

A "step" is one merged forward pass of the workload over one batch of synthetic inputs that are
already resident in HBM (one sequence / image per model).  Reported: merged inferences/s
(= M / mean step time), the same kernels launched once per model (M separate launches), a
per-kernel roofline from HIP events, and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-graph] [--quick]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
MFMA_BF16_PEAK = 2.5e15    # FLOP/s dense bf16
FP32_VALU_PEAK = 157.3e12

WORKLOADS = {
    # name: (kind, M, params)
    "encoder12_m32_s128": ("encoder", 32, dict(layers=12, seq=128, cfg=5)),
    "encoder12_m32_s512": ("encoder", 32, dict(layers=12, seq=512, cfg=5)),
    "encoder1_m8_s128": ("encoder", 8, dict(layers=1, seq=128, cfg=2)),
    "resnet50_m32": ("resnet", 32, dict(card=1, bw=64, cfg=3)),
    "resnext50_32x4d_m16": ("resnet", 16, dict(card=32, bw=4, cfg=4)),
}
HEADLINE = "encoder12_m32_s128"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------------------------------
class OpTimer:
    """Wraps the binding's entry points with HIP events (on the stream the kernels run on) and
    accumulates, per op tag, launches, time, algorithmic flops and algorithmic bytes (every operand
    read once, the output written once)."""

    def __init__(self, nf, torch):
        self.nf, self.torch = nf, torch
        self.records = []          # (tag, start, stop, flops, bytes)
        self.saved = {}

    def _wrap(self, name, describe):
        orig = getattr(self.nf, name)
        self.saved[name] = orig
        torch = self.torch

        def wrapped(*a, **kw):
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            out = orig(*a, **kw)
            e.record()
            tag, fl, by = describe(out, *a, **kw)
            self.records.append((tag, s, e, fl, by))
            return out
        setattr(self.nf, name, wrapped)

    def __enter__(self):
        def d_linear(y_, X, W, bias=None, residual=None, act=0, **kw):
            M, N, K = X.shape
            No = W.shape[2]
            e = X.element_size()
            by = e * (X.numel() + W.numel() + y_.numel() * (2 if residual is not None else 1)) + (4 * M * No if bias is not None else 0)
            return "linear_%dx%dx%d" % (N, K, No), 2.0 * M * N * K * No, by

        def d_conv(y_, x, w, M, g=1, bias=None, scale=None, shift=None, residual=None, stride=1, pad=0, **kw):
            e = x.element_size()
            fl = 2.0 * y_.numel() * w.shape[1] * w.shape[2] * w.shape[3]
            by = e * (x.numel() + w.numel() + y_.numel() * (2 if residual is not None else 1)) + (8 * w.shape[0] if scale is not None else 0)
            tag = "conv%dx%d_s%d_g%d_%d->%d@%d" % (w.shape[2], w.shape[3], stride, g, x.shape[1] // M, w.shape[0] // M, x.shape[2])
            return tag, fl, by

        def d_attn(y_, QKV, B, S, heads, **kw):
            M, N, th = QKV.shape
            return "attention_S%d" % S, 4.0 * M * B * heads * S * S * (th // 3 // heads), QKV.element_size() * (QKV.numel() + y_.numel())

        def d_ln(y_, x, gamma, beta, M, residual=None, **kw):
            by = x.element_size() * x.numel() * (3 if residual is not None else 2) + 8 * gamma.numel()
            return "layernorm_H%d" % (gamma.numel() // M), 8.0 * x.numel(), by

        def d_pool(tag):
            def d(y_, x, *a, **kw):
                return tag, float(x.numel()), x.element_size() * (x.numel() + y_.numel())
            return d

        self._wrap("linear", d_linear)
        self._wrap("conv2d", d_conv)
        self._wrap("attention_packed", d_attn)
        self._wrap("layernorm", d_ln)
        self._wrap("maxpool2d", d_pool("maxpool"))
        self._wrap("avgpool_global", d_pool("avgpool"))
        return self

    def __exit__(self, *exc):
        for k, v in self.saved.items():
            setattr(self.nf, k, v)

    def empty_pairs(self, n=64):
        """Event pairs around nothing, recorded in the middle of the same stream of work: what a
        start/stop pair measures by itself (subtracted from every bracketed launch)."""
        torch = self.torch
        self.empty = []
        for _ in range(n):
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            e.record()
            self.empty.append((s, e))

    def summary(self):
        self.torch.cuda.synchronize()
        self.overhead_ms = 0.0
        if getattr(self, "empty", None):
            vals = sorted(s.elapsed_time(e) for s, e in self.empty)
            self.overhead_ms = vals[0]            # the smallest: never over-corrects
        agg = {}
        for tag, s, e, fl, by in self.records:
            a = agg.setdefault(tag, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
            a["launches"] += 1
            a["ms"] += max(s.elapsed_time(e) - self.overhead_ms, 1e-4)
            a["flops"] += fl
            a["bytes"] += by
        return agg


def group_family(tag):
    """Kernel family of an op tag: every convolution shape runs in the same two kernel templates
    (gemm_mfma_kernel / conv_patch_kernel), every matmul in gemm_dma_kernel / gemm_mfma_kernel."""
    head = tag.split("_")[0]
    return "conv" if head.startswith("conv") else head


def roofline_for(agg):
    """Roofline of the kernel family that takes the most time; bound = the larger of the HBM and the
    MFMA lower bounds for its algorithmic bytes and flops."""
    fam = {}
    for tag, a in agg.items():
        f = fam.setdefault(group_family(tag), dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
        for k in f:
            f[k] += a[k]
    name, a = max(fam.items(), key=lambda kv: kv[1]["ms"])
    sec = a["ms"] * 1e-3
    t_hbm, t_mfma = a["bytes"] / HBM_PEAK, a["flops"] / MFMA_BF16_PEAK
    contraction = name in ("linear", "attention") or name.startswith("conv")
    out = dict(kernel=name, launches=a["launches"], avg_us=1e3 * a["ms"] / a["launches"],
               bytes_per_launch=a["bytes"] / a["launches"], flops_per_launch=a["flops"] / a["launches"],
               achieved_GBps=a["bytes"] / sec / 1e9, achieved_TFLOPs=a["flops"] / sec / 1e12,
               frac_hbm=a["bytes"] / sec / HBM_PEAK, frac_mfma=a["flops"] / sec / MFMA_BF16_PEAK,
               frac_of_min_roof=max(t_hbm, t_mfma) / sec, traffic=None)
    if contraction and t_mfma > t_hbm:
        out.update(bound="mfma", achieved=out["achieved_TFLOPs"], peak=MFMA_BF16_PEAK / 1e12, unit="TFLOP/s",
                   frac=out["frac_mfma"])
    else:
        out.update(bound="hbm", achieved=out["achieved_GBps"], peak=HBM_PEAK / 1e9, unit="GB/s",
                   frac=out["frac_hbm"])
    return out


# ------------------------------------------------------------------------------------------
def build_workload(name, torch):
    import netfuse_inputs as NI
    from netfuse_inputs.device import encoder_stack_device, resnet_params_device
    from paper_2009_13062_amd.workloads import EncoderStack, ResNetForward
    kind, M, p = WORKLOADS[name]
    if kind == "encoder":
        shape = NI.EncoderShape(layers=p["layers"], seq=p["seq"])
        inp = encoder_stack_device(M, shape, cfg=p["cfg"])
        net = EncoderStack(inp["layers"], M, 1, shape.seq, shape.heads)
        x = inp["X"]
        cfg = dict(workload=name, M=M, layers=shape.layers, seq_len=shape.seq, hidden=shape.hidden,
                   heads=shape.heads, ffn=shape.ffn, batch_per_model=1)
        singles = [(one, x[m:m + 1]) for m, one in enumerate(net.per_model())]
    else:
        spec = NI.resnet_spec(cardinality=p["card"], base_width=p["bw"])
        inp = resnet_params_device(spec, M, cfg=p["cfg"])
        net = ResNetForward(spec, inp["params"], M)
        x = inp["x"]
        cfg = dict(workload=name, M=M, image=spec.image, convs=len(spec.convs()),
                   merged_groups_3x3=M * p["card"], batch_per_model=1)
        singles = [(one, net.slice_input(x, m)) for m, one in enumerate(net.per_model())]
    return net, x, singles, cfg, M


def timed(torch, fn, steps, warmup):
    """W untimed steps, then exactly K steps between synchronisations; wall clock and HIP events."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    s.record()
    for _ in range(steps):
        fn()
    e.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, s.elapsed_time(e) / steps


def make_graph(torch, fn):
    """Capture one step into a HIP graph (the forward allocates nothing and uses no memset)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g.replay


def load_traffic(name):
    """HBM bytes per launch of the dominant kernel, measured offline with rocprofv3 --pmc (FETCH_SIZE,
    WRITE_SIZE, calibrated against --calibrate-copy) and recorded under profiles/; None if not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f).get(name)


def calibrate_copy(torch, nf):
    """A plain copy of known size (netfuse_merge_transpose with M = 1 is src -> dst), for scaling the
    FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run."""
    rows, H = 65536, 2048                                   # 256 MiB of bf16 in, 256 MiB out
    src = torch.empty((1, rows, H), dtype=torch.bfloat16, device="cuda").normal_()
    dst = torch.empty((rows, H), dtype=torch.bfloat16, device="cuda")
    for _ in range(5):
        nf.merge_transpose(src, 1, True, out=dst)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy": {"kernel": "merge_transpose_kernel", "launches": 5,
                                         "bytes_read_per_launch": src.numel() * 2,
                                         "bytes_written_per_launch": dst.numel() * 2}}))


def run_workload(name, steps, warmup, use_graph, torch, nf, sep_steps=None, separate_too=True):
    net, x, singles, cfg, M = build_workload(name, torch)
    merged = lambda: net.forward(x)

    def separate():
        for one, xm in singles:
            one.forward(xm)

    res = dict(config=cfg)
    wall, ev = timed(torch, merged, steps, warmup)
    res["eager_ms"], res["eager_event_ms"] = wall, ev
    best = wall
    if use_graph:
        try:
            replay = make_graph(torch, merged)
            gw, ge = timed(torch, replay, steps, warmup)
            res["graph_ms"], res["graph_event_ms"] = gw, ge
            best = min(best, gw)
        except Exception as ex:                       # report, keep the eager number
            res["graph_error"] = repr(ex)[:200]
    res["ms_per_step"] = best
    res["inferences_per_s"] = M / (best * 1e-3)
    if separate_too:
        ss = sep_steps or max(2, steps // 4)
        sw, se = timed(torch, separate, ss, max(1, warmup // 2))
        sep_best = sw
        res["separate_eager_ms"] = sw
        if use_graph:
            try:
                replay_s = make_graph(torch, separate)
                sgw, _ = timed(torch, replay_s, ss, max(1, warmup // 2))
                res["separate_graph_ms"] = sgw
                sep_best = min(sep_best, sgw)
            except Exception as ex:
                res["separate_graph_error"] = repr(ex)[:200]
        res["separate_ms"] = sep_best
        res["separate_inferences_per_s"] = M / (sep_best * 1e-3)
        res["speedup_vs_separate"] = sep_best / best
    else:
        res["separate_ms"] = res["separate_inferences_per_s"] = res["speedup_vs_separate"] = None
    # per-kernel pass: the same steps, un-graphed, HIP events around every launch
    with OpTimer(nf, torch) as ot:
        npass = max(3, min(steps, 10))
        for i in range(npass):
            merged()
            if i == npass // 2:
                ot.empty_pairs()
        agg = ot.summary()
    res["event_pair_overhead_us"] = 1e3 * ot.overhead_ms
    res["kernels"] = {k: dict(launches=v["launches"], avg_us=1e3 * v["ms"] / v["launches"],
                              GBps=v["bytes"] / (v["ms"] * 1e-3) / 1e9, TFLOPs=v["flops"] / (v["ms"] * 1e-3) / 1e12)
                      for k, v in sorted(agg.items(), key=lambda kv: -kv[1]["ms"])}
    res["roofline"] = roofline_for(agg)
    res["roofline"]["traffic"] = load_traffic(name)
    total_fl = sum(v["flops"] for v in agg.values()) / max(3, min(steps, 10))
    res["model_TFLOPs"] = total_fl / (best * 1e-3) / 1e12
    return res


def cpu_baseline(name):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    import numpy as np
    import netfuse_inputs as NI
    import oracle
    from oracle import models as OM
    kind, M, p = WORKLOADS[name]
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    threads = int(os.environ.get("OMP_NUM_THREADS", cores))
    oracle.build()
    if kind == "encoder":
        # about 10 s including input generation: every model through 1 layer (seq 128), 4 models through 1 layer (seq 512)
        ms, nl = (min(M, 32), 1) if p["seq"] <= 128 else (min(M, 4), 1)
        shape = NI.EncoderShape(layers=nl, seq=p["seq"])
        inp = NI.encoder_stack(ms, shape, cfg=p["cfg"], bf16=True)
        t0 = time.perf_counter()
        OM.encoder_stack(inp, ms, 1, shape.seq, shape.heads, out_bf16=True)
        dt = time.perf_counter() - t0
        per_inference = dt / ms / nl * p["layers"]
        sample = "%d of %d models x %d of %d layers (seq %d), scaled by the layer count" % (ms, M, nl, p["layers"], p["seq"])
    else:
        spec = NI.resnet_spec(cardinality=p["card"], base_width=p["bw"])
        inp = NI.resnet_params(spec, 1, cfg=p["cfg"], bf16=True)
        t0 = time.perf_counter()
        OM.resnet_forward(inp, spec, 1, out_bf16=True)
        dt = time.perf_counter() - t0
        per_inference = dt
        sample = "1 of %d models, whole forward" % M
    return dict(value=1.0 / per_inference, unit="inferences/s", cores=min(threads, cores), kind="oracle",
                sample=sample, seconds=dt)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(WORKLOADS))
    ap.add_argument("--others", default="encoder12_m32_s512,resnet50_m32,resnext50_32x4d_m16,encoder1_m8_s128",
                    help="comma list of further workloads reported under 'other_workloads' ('' = none)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="headline workload only, no CPU baseline")
    ap.add_argument("--no-separate", action="store_true", help="skip the M-separate-launches leg (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true", help="only run a plain copy of known size and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (models are independent: sharding M over GPUs needs no "
                 "collective and is not part of this build); run with --gpus 1")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import paper_2009_13062_amd as nf
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        calibrate_copy(torch, nf)
        return
    t_start = time.time()
    head = run_workload(args.workload, args.steps, args.warmup, not args.no_graph, torch, nf,
                        separate_too=not args.no_separate)
    log("[bench] %s: %.3f ms/step, %.1f inf/s, %sx vs separate (%.1f s)" % (
        args.workload, head["ms_per_step"], head["inferences_per_s"],
        "%.2f" % head["speedup_vs_separate"] if head["speedup_vs_separate"] else "-", time.time() - t_start))
    others = {}
    if not args.quick and args.others:
        for name in [n for n in args.others.split(",") if n and n != args.workload]:
            t1 = time.time()
            try:
                torch.cuda.empty_cache()
                r = run_workload(name, max(5, args.steps // 5), max(2, args.warmup // 2), not args.no_graph, torch, nf)
                others[name] = dict(ms_per_step=r["ms_per_step"], inferences_per_s=r["inferences_per_s"],
                                    separate_ms=r["separate_ms"], speedup_vs_separate=r["speedup_vs_separate"],
                                    model_TFLOPs=r["model_TFLOPs"], roofline=r["roofline"],
                                    kernels=dict(list(r["kernels"].items())[:8]))
                log("[bench] %s: %.3f ms/step, %.2fx vs separate (%.1f s)" % (
                    name, r["ms_per_step"], r["speedup_vs_separate"], time.time() - t1))
            except Exception as ex:
                others[name] = dict(error=repr(ex)[:300])
                log("[bench] %s failed: %r" % (name, ex))
    cpu = None
    if not (args.quick or args.no_cpu_baseline):
        cpu = cpu_baseline(args.workload)
        log("[bench] cpu oracle: %.4f inf/s on %d cores" % (cpu["value"], cpu["cores"]))

    kind, M, _ = WORKLOADS[args.workload]
    rf = head["roofline"]
    line = {
        "metric": "merged inferences/sec at M=%d (one %s per model), vs M separate launches" % (
            M, "sequence" if kind == "encoder" else "image"),
        "value": head["inferences_per_s"], "unit": "inferences/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": head["config"],
        "separate_launches": {"ms_per_step": head["separate_ms"], "inferences_per_s": head["separate_inferences_per_s"]},
        "speedup_vs_separate": head["speedup_vs_separate"],
        "launch": {k: head[k] for k in ("eager_ms", "graph_ms", "separate_eager_ms", "separate_graph_ms", "graph_error") if k in head},
        "model_TFLOPs": head["model_TFLOPs"],
        "event_pair_overhead_us": head["event_pair_overhead_us"],
        "roofline": {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel", "launches",
                                        "avg_us", "bytes_per_launch", "flops_per_launch", "frac_hbm", "frac_mfma",
                                        "frac_of_min_roof")},
        "kernels": head["kernels"],
        "cpu_baseline": cpu,
        "other_workloads": others,
        "paper_context": "NetFuse reports up to 3.6x (V100) / 3.0x (TITAN Xp) over its best baseline at 32 instances, fp32, bs 1",
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
