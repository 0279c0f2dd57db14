#!/usr/bin/env python3
"""Benchmark of the merged-operator hot path on one MI355X.

A "step" is one merged forward pass of the workload over one batch of synthetic inputs that are
already resident in HBM.  Reported in ONE JSON line: merged inferences/s (= M x batch / mean step
time) with the standard deviation over the timed steps, the same kernels launched once per model
(M separate launches, the paper's Sequential baseline), a per-kernel roofline whose durations are
the kernels' own begin/end timestamps on the device (netfuse_time_next_launch), a sweep over the
number of merged models and over the batch size per model (the paper's two experiments), achieved
HBM GB/s of the normalisation and pooling kernels, and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--quick] ...
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
MFMA_BF16_PEAK = 2.5e15    # FLOP/s dense bf16

WORKLOADS = {
    # name: (kind, M, params)
    "encoder12_m32_s128": ("encoder", 32, dict(layers=12, seq=128, cfg=5)),
    "encoder12_m32_s512": ("encoder", 32, dict(layers=12, seq=512, cfg=5)),
    # 113 MB of weights would stay in the 256 MB memory-side cache: three weight copies are rotated
    "encoder1_m8_s128": ("encoder", 8, dict(layers=1, seq=128, cfg=2, rotate=3)),
    # XLNet-shaped: the same stack with relative-position attention (one more matmul and a position term per layer)
    "xlnet12_m32_s128": ("encoder", 32, dict(layers=12, seq=128, cfg=6, rel=True)),
    "resnet50_m32": ("resnet", 32, dict(card=1, bw=64, cfg=3)),
    "resnext50_32x4d_m16": ("resnet", 16, dict(card=32, bw=4, cfg=4)),
}
HEADLINE = "encoder12_m32_s128"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------------------------------
class HipEvents:
    """Raw hipEvent_t handles from the HIP runtime this process already loaded (torch's events are
    created lazily and do not expose a handle before they are recorded)."""

    def __init__(self):
        path = None
        with open("/proc/self/maps") as f:
            for line in f:
                m = re.search(r"(/\S*libamdhip64\.so\S*)", line)
                if m:
                    path = m.group(1)
                    break
        self.hip = ctypes.CDLL(path or "libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.free, self.all = [], []

    def get(self):
        if self.free:
            return self.free.pop()
        e = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(e)) != 0:
            raise RuntimeError("hipEventCreate failed")
        self.all.append(e)
        return e

    def ms(self, a, b):
        f = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(f), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed (%d)" % rc)
        return f.value

    def release(self, *ev):
        self.free.extend(ev)


class OpTimer:
    """Wraps the binding's entry points: before each call the library is armed (netfuse_time_next_launch)
    so that the ONE kernel the call launches records its own begin and end on the device.  No host-side
    event pair is involved, so nothing is subtracted.  Accumulates, per op tag, launches, kernel time,
    algorithmic flops and algorithmic bytes (every operand read once, the output written once)."""

    def __init__(self, nf, torch, events):
        self.nf, self.torch, self.ev = nf, torch, events
        self.records = []          # (tag, start, stop, flops, bytes)
        self.saved = {}

    def _wrap(self, name, describe):
        orig = getattr(self.nf, name)
        self.saved[name] = orig

        def wrapped(*a, **kw):
            s, e = self.ev.get(), self.ev.get()
            self.nf.time_next_launch(s, e)
            out = orig(*a, **kw)
            tag, fl, by = describe(out, *a, **kw)
            self.records.append((tag, s, e, fl, by))
            return out
        setattr(self.nf, name, wrapped)

    def __enter__(self):
        def d_linear(y_, X, W, bias=None, residual=None, act=0, **kw):
            M, N, K = X.shape
            No = W.shape[2]
            # per model: activations in, weights, activations out (2 bytes each)
            return "linear_%dx%dx%d" % (N, K, No), 2.0 * M * N * K * No, X.element_size() * (X.numel() + W.numel() + y_.numel())

        def d_linear_packed(y_, X, Wp, **kw):
            return d_linear(y_, X, Wp, **kw)

        def d_conv(y_, x, w, M, g=1, bias=None, scale=None, shift=None, residual=None, stride=1, pad=0, **kw):
            fl = 2.0 * y_.numel() * w.shape[1] * w.shape[2] * w.shape[3]
            by = x.element_size() * (x.numel() + w.numel() + y_.numel())
            tag = "conv%dx%d_s%d_g%d_%d->%d@%d" % (w.shape[2], w.shape[3], stride, g, x.shape[1] // M, w.shape[0] // M, x.shape[2])
            return tag, fl, by

        def d_attn(y_, QKV, B, S, heads, **kw):
            M, N, th = QKV.shape
            return "attention_S%d" % S, 4.0 * M * B * heads * S * S * (th // 3 // heads), QKV.element_size() * (QKV.numel() + y_.numel())

        def d_attn_rel(y_, QKV, Kr, B, S, heads, **kw):
            M, N, th = QKV.shape
            return ("attention_relpos_S%d" % S, 6.0 * M * B * heads * S * S * (th // 3 // heads),
                    QKV.element_size() * (QKV.numel() + Kr.numel() + y_.numel()))

        def d_ln(y_, x, gamma, beta, M, residual=None, **kw):
            return "layernorm_H%d" % (gamma.numel() // M), 8.0 * x.numel(), x.element_size() * x.numel() * 2 + 8 * gamma.numel()

        def d_pool(tag):
            def d(y_, x, *a, **kw):
                return tag, float(x.numel()), x.element_size() * (x.numel() + y_.numel())
            return d

        self._wrap("linear", d_linear)
        self._wrap("linear_packed", d_linear_packed)
        self._wrap("conv2d", d_conv)
        self._wrap("attention_packed", d_attn)
        self._wrap("attention_relpos_packed", d_attn_rel)
        self._wrap("layernorm", d_ln)
        self._wrap("maxpool2d", d_pool("maxpool"))
        self._wrap("avgpool_global", d_pool("avgpool"))
        return self

    def __exit__(self, *exc):
        for k, v in self.saved.items():
            setattr(self.nf, k, v)
        self.nf.time_next_launch(None, None)

    def keep_only(self, lo, hi):
        """Forget the records outside [lo, hi) (their events go back to the pool after the next synchronisation)."""
        self.dropped = getattr(self, "dropped", []) + self.records[:lo] + self.records[hi:]
        self.records = self.records[lo:hi]

    def summary(self):
        self.torch.cuda.synchronize()
        for _, s, e, _, _ in getattr(self, "dropped", []):
            self.ev.release(s, e)
        self.dropped = []
        agg = {}
        for tag, s, e, fl, by in self.records:
            a = agg.setdefault(tag, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0, max_ms=0.0))
            t = self.ev.ms(s, e)
            a["launches"] += 1
            a["ms"] += t
            a["max_ms"] = max(a["max_ms"], t)
            a["flops"] += fl
            a["bytes"] += by
            self.ev.release(s, e)
        self.records = []
        return agg


def group_family(tag):
    """Kernel family of an op tag: all matmul shapes form `linear`, all convolution shapes `conv`."""
    head = tag.split("_")[0]
    return "conv" if head.startswith("conv") else head


def roofline_for(agg):
    """Roofline of the kernel family that takes the most kernel time.  achieved = algorithmic bytes (or
    flops) per launch / the family's average kernel duration; bound = the larger of the HBM and the MFMA
    lower bounds for those bytes and flops."""
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
               frac_of_min_roof=max(t_hbm, t_mfma) / sec, traffic=None,
               timing="kernel begin/end timestamps on the device (hipExtLaunchKernel events), eager launches")
    if contraction and t_mfma > t_hbm:
        out.update(bound="mfma", achieved=out["achieved_TFLOPs"], peak=MFMA_BF16_PEAK / 1e12, unit="TFLOP/s",
                   frac=out["frac_mfma"])
    else:
        out.update(bound="hbm", achieved=out["achieved_GBps"], peak=HBM_PEAK / 1e9, unit="GB/s",
                   frac=out["frac_hbm"])
    return out


# ------------------------------------------------------------------------------------------
CONCURRENT_STREAMS = 4    # streams of the Concurrent stand-in (the box exposes 4 hardware queues per process)
PACKED_WEIGHTS = True     # encoder matmuls on weights packed once by netfuse_linear_pack_weight (--unpacked: off)


def build_workload(name, torch, M=None, batch=1):
    """-> (merged forward(), all models one after the other(), config, M, inferences per step, [model m alone()])."""
    import netfuse_inputs as NI
    from netfuse_inputs.device import encoder_stack_device, resnet_params_device
    from paper_2009_13062_amd.workloads import EncoderStack, ResNetForward
    kind, M0, p = WORKLOADS[name]
    M = M or M0
    if kind == "encoder":
        shape = NI.EncoderShape(layers=p["layers"], seq=p["seq"], batch=batch)
        rot = p.get("rotate", 1)
        nets, x = [], None
        for r in range(rot):
            inp = encoder_stack_device(M, shape, cfg=p["cfg"] + 100 * r, rel=p.get("rel", False))
            nets.append(EncoderStack(inp["layers"], M, batch, shape.seq, shape.heads,
                                     buffers=nets[0].buf if nets else None, R=inp.get("R"), packed=PACKED_WEIGHTS))
            x = inp["X"] if x is None else x
        cfg = dict(workload=name, M=M, layers=shape.layers, seq_len=shape.seq, hidden=shape.hidden,
                   heads=shape.heads, ffn=shape.ffn, batch_per_model=batch, weight_copies_rotated=rot,
                   packed_weights=PACKED_WEIGHTS)

        def merged():
            for n in nets:
                n.forward(x)
        per = [n.per_model() for n in nets]

        def separate():
            for pm in per:
                for m, one in enumerate(pm):
                    one.forward(x[m:m + 1])

        def alone(m):
            def run():
                for pm in per:
                    pm[m].forward(x[m:m + 1])
            return run
        return merged, separate, cfg, M, rot, [alone(m) for m in range(M)]
    spec = NI.resnet_spec(cardinality=p["card"], base_width=p["bw"])
    inp = resnet_params_device(spec, M, cfg=p["cfg"], batch=batch)
    net = ResNetForward(spec, inp["params"], M, batch=batch)
    x = inp["x"]
    cfg = dict(workload=name, M=M, image=spec.image, convs=len(spec.convs()),
               merged_groups_3x3=M * p["card"], batch_per_model=batch, weight_copies_rotated=1)
    singles = [(one, net.slice_input(x, m)) for m, one in enumerate(net.per_model())]

    def separate():
        for one, xm in singles:
            one.forward(xm)
    return (lambda: net.forward(x)), separate, cfg, M, 1, [(lambda one=one, xm=xm: one.forward(xm)) for one, xm in singles]


def timed(torch, fn, steps, warmup):
    """W untimed steps, then exactly K steps between synchronisations: mean from the wall clock around the
    K steps; standard deviation from one torch event per step boundary on the launch stream (they add no
    synchronisation)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        fn()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    per = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    return wall, (statistics.pstdev(per) if steps > 1 else 0.0), statistics.mean(per)


def concurrent_streams(torch, singles, nstreams):
    """The models dealt over `nstreams` streams of the default priority, each model's launches in order on its
    stream: a single-process stand-in for the paper's Concurrent baseline (Section 5.1: one process per model
    on the same GPU).  Fork from and join into the current stream."""
    streams = [torch.cuda.Stream() for _ in range(nstreams)]

    def run():
        cur = torch.cuda.current_stream()
        for st in streams:
            st.wait_stream(cur)
        for i, f in enumerate(singles):
            with torch.cuda.stream(streams[i % nstreams]):
                f()
        for st in streams:
            cur.wait_stream(st)
    return run


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


def best_of(torch, fn, steps, warmup, use_graph, res, prefix):
    """Eager and (optionally) graph-replayed timing of fn; the faster is the step time."""
    wall, sd, ev = timed(torch, fn, steps, warmup)
    res[prefix + "eager_ms"] = wall
    best, best_sd = wall, sd
    if use_graph:
        try:
            replay = make_graph(torch, fn)
            gw, gsd, _ = timed(torch, replay, steps, warmup)
            res[prefix + "graph_ms"] = gw
            if gw < best:
                best, best_sd = gw, gsd
        except Exception as ex:                       # report, keep the eager number
            res[prefix + "graph_error"] = repr(ex)[:200]
    return best, best_sd


def load_traffic(name):
    """HBM bytes per launch of the dominant kernel family, measured offline with rocprofv3 --pmc (FETCH_SIZE,
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


def kernel_pass(torch, nf, events, fn, npass, lead=None):
    """npass eager steps with every launch timed by its own device timestamps, inside one uninterrupted run of
    launches: `lead` passes before them and one behind are launched the same way and their records dropped.
    The passes in front carry the first-use costs of the timed launch path (events, the extended launch call per
    kernel function) and bring the device to the state it has in a sustained run -- measured from idle, the
    matrix-bound kernels of the 512-token workload read 3 - 4 % shorter than in the timed loop of steps and in a
    rocprofv3 trace of the same command.  The pass behind is there because the last launches before the closing
    synchronisation have read 0.4 - 2 ms on one workload (a 23 us kernel, the same launch every time) with
    nothing to match in the step times (30 steps of 0.828 +- 0.002 ms)."""
    lead = max(2, npass) if lead is None else lead
    with OpTimer(nf, torch, events) as ot:
        for _ in range(lead):
            fn()
        skip = len(ot.records)
        for _ in range(npass):
            fn()
        keep = len(ot.records)
        fn()
        ot.keep_only(skip, keep)
        return ot.summary()


def run_workload(name, steps, warmup, use_graph, torch, nf, events, separate_too=True, M=None, batch=1,
                 sep_steps=None, kernels=True, concurrent=0):
    merged, separate, cfg, M, per_step, singles = build_workload(name, torch, M=M, batch=batch)
    res = dict(config=cfg)
    best, sd = best_of(torch, merged, steps, warmup, use_graph, res, "")
    res["ms_per_step"] = best / per_step
    res["ms_per_step_std"] = sd / per_step
    res["inferences_per_s"] = M * batch / (res["ms_per_step"] * 1e-3)
    if separate_too:
        ss = sep_steps or steps
        sbest, ssd = best_of(torch, separate, ss, max(1, warmup // 2), use_graph, res, "separate_")
        res["separate_ms"], res["separate_ms_std"] = sbest / per_step, ssd / per_step
        res["separate_inferences_per_s"] = M * batch / (res["separate_ms"] * 1e-3)
        res["speedup_vs_separate"] = sbest / best
    else:
        res["separate_ms"] = res["separate_inferences_per_s"] = res["speedup_vs_separate"] = None
    if concurrent and separate_too:
        ss = sep_steps or steps
        cres = {}
        cw, csd = best_of(torch, concurrent_streams(torch, singles, concurrent), ss, max(1, warmup // 2), use_graph, cres, "")
        res["concurrent"] = dict(streams=concurrent, ms_per_step=cw / per_step, ms_per_step_std=csd / per_step,
                                 inferences_per_s=M * batch / (cw / per_step * 1e-3), steps=ss,
                                 speedup_vs_concurrent=cw / best, **cres,
                                 note="the M single-model forwards dealt over this many streams of one process; "
                                      "eager launches are bound by the host's launch rate, the captured graph is not")
    if kernels:
        npass = max(3, min(steps, 10))
        agg = kernel_pass(torch, nf, events, merged, npass)
        res["kernels"] = {k: dict(launches=v["launches"], avg_us=1e3 * v["ms"] / v["launches"], max_us=1e3 * v["max_ms"],
                                  GBps=v["bytes"] / (v["ms"] * 1e-3) / 1e9, TFLOPs=v["flops"] / (v["ms"] * 1e-3) / 1e12)
                          for k, v in sorted(agg.items(), key=lambda kv: -kv[1]["ms"])}
        res["roofline"] = roofline_for(agg)
        res["roofline"]["traffic"] = load_traffic(name) if (M, batch) == (WORKLOADS[name][1], 1) else None
        res["kernel_time_ms_per_step"] = sum(v["ms"] for v in agg.values()) / npass / per_step
        res["model_TFLOPs"] = sum(v["flops"] for v in agg.values()) / npass / per_step / (res["ms_per_step"] * 1e-3) / 1e12
    return res


def m_sweep(name, steps, warmup, use_graph, torch, nf, events, head):
    """Merged vs M separate launches for 1 ... 32 models (the paper's first experiment)."""
    out = {}
    M0 = WORKLOADS[name][1]
    for M in (1, 2, 8, 16, 32):
        if M > M0:
            continue
        if M == M0:
            r = head
        else:
            torch.cuda.empty_cache()
            r = run_workload(name, steps, warmup, use_graph, torch, nf, events, M=M, kernels=False)
        out[str(M)] = dict(merged_ms=r["ms_per_step"], merged_ms_std=r["ms_per_step_std"], separate_ms=r["separate_ms"],
                           separate_ms_std=r.get("separate_ms_std"), speedup_vs_separate=r["speedup_vs_separate"],
                           inferences_per_s=r["inferences_per_s"])
        log("[bench]   M=%2d: merged %.3f ms, separate %.3f ms, %.2fx" % (M, r["ms_per_step"], r["separate_ms"], r["speedup_vs_separate"]))
    return out


def batch_sweep(name, steps, warmup, use_graph, torch, nf, events, head):
    """Merged vs separate for 1 ... 8 sequences (images) per model (the paper's batch-size experiment), with
    the matmul family's share of the bf16 MFMA peak per batch size; `crossover_batch` = the first batch size
    at which merging no longer pays (None if it pays everywhere)."""
    out, cross = {}, None
    for B in (1, 2, 4, 8):
        if B == 1:
            r = head
        else:
            torch.cuda.empty_cache()
            r = run_workload(name, steps, warmup, use_graph, torch, nf, events, batch=B)
        fam = r["roofline"]
        out[str(B)] = dict(merged_ms=r["ms_per_step"], separate_ms=r["separate_ms"], speedup_vs_separate=r["speedup_vs_separate"],
                           inferences_per_s=r["inferences_per_s"], dominant_family=fam["kernel"],
                           family_frac_mfma=fam["frac_mfma"], family_frac_hbm=fam["frac_hbm"], family_avg_us=fam["avg_us"])
        if cross is None and r["speedup_vs_separate"] < 1.0:
            cross = B
        log("[bench]   batch %d: merged %.3f ms, separate %.3f ms, %.2fx, %s at %.1f%% of MFMA peak" % (
            B, r["ms_per_step"], r["separate_ms"], r["speedup_vs_separate"], fam["kernel"], 100 * fam["frac_mfma"]))
    out["crossover_batch"] = cross
    return out


def micro_norms(torch, nf, events):
    """Achieved HBM GB/s (bytes in + out over the kernel's own duration) of the normalisation and pooling
    kernels at the shapes of the workloads, 32 models, bf16."""
    bf = torch.bfloat16
    rnd = lambda *s: torch.empty(s, dtype=bf, device="cuda").normal_()
    f32 = lambda n, mean=0.0: torch.empty(n, dtype=torch.float32, device="cuda").normal_(mean, 0.1)
    cases = {}
    for rows, tag in ((128, "layernorm_4096x768"), (512, "layernorm_16384x768")):
        x, r, y = rnd(32, rows, 768), rnd(32, rows, 768), rnd(32, rows, 768)
        g, b = f32(32 * 768, 1.0), f32(32 * 768)
        cases[tag] = (lambda x=x, g=g, b=b, y=y: nf.layernorm(x, g, b, 32, out=y), 2 * x.numel() * 2)
        cases[tag + "+residual"] = (lambda x=x, r=r, g=g, b=b, y=y: nf.layernorm(x, g, b, 32, residual=r, out=y), 3 * x.numel() * 2)
    for C, hw, tag in ((64, 112, "batchnorm_64ch_112x112"), (256, 56, "batchnorm_256ch_56x56"), (2048, 7, "batchnorm_2048ch_7x7")):
        x, y = rnd(1, 32 * C, hw, hw), rnd(1, 32 * C, hw, hw)
        g, b, mu = f32(32 * C, 1.0), f32(32 * C), f32(32 * C)
        var = torch.empty(32 * C, dtype=torch.float32, device="cuda").uniform_(0.5, 1.5)
        cases[tag] = (lambda x=x, g=g, b=b, mu=mu, var=var, y=y: nf.batchnorm(x, g, b, mu, var, 32, act=nf.ACT_RELU, out=y), 2 * x.numel() * 2)
    x = rnd(1, 32 * 64, 112, 112)
    y = rnd(1, 32 * 64, 56, 56)
    cases["maxpool3x3s2_64ch_112x112"] = (lambda x=x, y=y: nf.maxpool2d(x, 3, 2, 1, out=y), (x.numel() + y.numel()) * 2)
    x = rnd(1, 32 * 2048, 7, 7)
    y = rnd(1, 32 * 2048)
    cases["avgpool_2048ch_7x7"] = (lambda x=x, y=y: nf.avgpool_global(x, out=y), (x.numel() + y.numel()) * 2)
    out = {}
    for tag, (fn, nbytes) in cases.items():
        for _ in range(3):
            fn()
        pairs = []
        for _ in range(20):
            s, e = events.get(), events.get()
            nf.time_next_launch(s, e)
            fn()
            pairs.append((s, e))
        torch.cuda.synchronize()
        us = sorted(1e3 * events.ms(s, e) for s, e in pairs)
        for s, e in pairs:
            events.release(s, e)
        med = us[len(us) // 2]
        out[tag] = dict(us=med, GBps=nbytes / med / 1e3, frac_hbm=nbytes / (med * 1e-6) / HBM_PEAK, MB=nbytes / 1e6)
    return out


def measured_peaks(torch, nf, events):
    """What this device reaches on the two roofs, measured like the operators (kernel begin/end timestamps): the
    issue rate of the bf16 matrix instruction from registers, a read-only stream over 2 GiB, and a plain copy."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    out = {}

    def best_us(fn, reps=7):
        us = []
        for _ in range(reps):
            s, e = events.get(), events.get()
            nf.time_next_launch(s, e)
            fn()
            torch.cuda.synchronize()
            us.append(1e3 * events.ms(s, e))
            events.release(s, e)
        return min(us[1:])
    box = {}
    us = best_us(lambda: box.__setitem__("fl", nf.probe_mfma(sink, 4000)))
    out["mfma_bf16_TFLOPs"] = box["fl"] / (us * 1e-6) / 1e12
    buf = torch.empty(1 << 30, dtype=torch.int16, device="cuda").zero_()          # 2 GiB: eight times the memory-side cache
    us = best_us(lambda: box.__setitem__("by", nf.probe_hbm_read(buf, sink)))
    out["hbm_read_GBps"] = box["by"] / (us * 1e-6) / 1e9
    src = buf[: 1 << 29].view(1, 1 << 18, 2048).view(torch.bfloat16)
    dst = buf[1 << 29:].view(1 << 18, 2048).view(torch.bfloat16)
    us = best_us(lambda: nf.merge_transpose(src, 1, True, out=dst))
    out["hbm_copy_GBps"] = 2 * src.numel() * 2 / (us * 1e-6) / 1e9                # bytes read + bytes written
    out["datasheet"] = {"mfma_bf16_TFLOPs": MFMA_BF16_PEAK / 1e12, "hbm_GBps": HBM_PEAK / 1e9}
    return out


def cpu_baseline(name):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    import netfuse_inputs as NI
    import oracle
    from oracle import models as OM
    kind, M, p = WORKLOADS[name]
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    threads = int(os.environ.get("OMP_NUM_THREADS", cores))
    oracle.build()
    if kind == "encoder":
        # about 10 s of oracle time: every model through 3 layers (seq 128), 8 models through 1 layer (seq 512)
        ms, nl = (min(M, 32), min(3, p["layers"])) if p["seq"] <= 128 else (min(M, 8), 1)
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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(WORKLOADS))
    ap.add_argument("--others", default="encoder12_m32_s512,xlnet12_m32_s128,resnet50_m32,resnext50_32x4d_m16,encoder1_m8_s128",
                    help="comma list of further workloads reported under 'other_workloads' ('' = none)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--unpacked", action="store_true", help="encoder matmuls on the row-major weights (netfuse_linear) instead of the packed ones")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweeps", action="store_true", help="skip the model-count and batch-size sweeps")
    ap.add_argument("--quick", action="store_true", help="headline workload only: no sweeps, no other workloads, no CPU baseline")
    ap.add_argument("--no-separate", action="store_true", help="skip the M-separate-launches leg (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true", help="only run a plain copy of known size and exit")
    ap.add_argument("--micro", default="", choices=["", "norms", "peaks"], help="only the named micro-benchmark leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (models are independent: sharding M over GPUs needs no "
                 "collective and is not part of this build); run with --gpus 1")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import paper_2009_13062_amd as nf
    torch.cuda.set_device(0)
    events = HipEvents()
    global PACKED_WEIGHTS
    PACKED_WEIGHTS = not args.unpacked

    if args.calibrate_copy:
        calibrate_copy(torch, nf)
        return
    if args.micro == "norms":
        print(json.dumps({"norm_kernels": micro_norms(torch, nf, events)}))
        return
    if args.micro == "peaks":
        print(json.dumps({"measured_peaks": measured_peaks(torch, nf, events)}))
        return
    use_graph = not args.no_graph
    sweep_steps = max(5, min(args.steps, 30))
    t_start = time.time()
    head = run_workload(args.workload, args.steps, args.warmup, use_graph, torch, nf, events,
                        separate_too=not args.no_separate, sep_steps=sweep_steps,
                        concurrent=0 if args.quick else CONCURRENT_STREAMS)
    if head.get("concurrent"):
        log("[bench] %s: the models on %d streams %.3f ms/step (%.2fx)" % (
            args.workload, head["concurrent"]["streams"], head["concurrent"]["ms_per_step"],
            head["concurrent"]["speedup_vs_concurrent"]))
    log("[bench] %s: %.3f +- %.3f ms/step, %.1f inf/s, %sx vs separate (%.1f s)" % (
        args.workload, head["ms_per_step"], head["ms_per_step_std"], head["inferences_per_s"],
        "%.2f" % head["speedup_vs_separate"] if head["speedup_vs_separate"] else "-", time.time() - t_start))
    sweeps = {}
    if not (args.quick or args.no_sweeps or args.no_separate):
        t1 = time.time()
        sweeps["m_sweep"] = m_sweep(args.workload, sweep_steps, args.warmup, use_graph, torch, nf, events, head)
        sweeps["batch_sweep"] = batch_sweep(args.workload, sweep_steps, args.warmup, use_graph, torch, nf, events, head)
        log("[bench] sweeps done (%.1f s)" % (time.time() - t1))
    others = {}
    if not args.quick and args.others:
        for name in [n for n in args.others.split(",") if n and n != args.workload]:
            t1 = time.time()
            try:
                torch.cuda.empty_cache()
                r = run_workload(name, args.steps, args.warmup, use_graph, torch, nf, events, sep_steps=sweep_steps)
                others[name] = dict(ms_per_step=r["ms_per_step"], ms_per_step_std=r["ms_per_step_std"],
                                    inferences_per_s=r["inferences_per_s"], steps=args.steps,
                                    separate_ms=r["separate_ms"], speedup_vs_separate=r["speedup_vs_separate"],
                                    model_TFLOPs=r["model_TFLOPs"], kernel_time_ms_per_step=r["kernel_time_ms_per_step"],
                                    weight_copies_rotated=r["config"]["weight_copies_rotated"],
                                    roofline=r["roofline"], kernels=dict(list(r["kernels"].items())[:8]))
                log("[bench] %s: %.3f +- %.3f ms/step, %.2fx vs separate (%.1f s)" % (
                    name, r["ms_per_step"], r["ms_per_step_std"], r["speedup_vs_separate"], time.time() - t1))
            except Exception as ex:
                others[name] = dict(error=repr(ex)[:300])
                log("[bench] %s failed: %r" % (name, ex))
    norms = peaks = None
    if not args.quick:
        torch.cuda.empty_cache()
        norms = micro_norms(torch, nf, events)
        peaks = measured_peaks(torch, nf, events)
        torch.cuda.empty_cache()
    cpu = None
    if not (args.quick or args.no_cpu_baseline):
        cpu = cpu_baseline(args.workload)
        log("[bench] cpu oracle: %.4f inf/s on %d cores" % (cpu["value"], cpu["cores"]))

    kind, M, _ = WORKLOADS[args.workload]
    rf = head["roofline"]
    rf = dict(rf)
    if peaks:
        # beside the fractions of the datasheet peaks: the same against what this device measures on a pure
        # matrix-instruction loop and on a pure read stream
        rf["frac_of_measured_hbm_read"] = rf["frac_hbm"] * HBM_PEAK / 1e9 / peaks["hbm_read_GBps"]
        rf["frac_of_measured_mfma"] = rf["frac_mfma"] * MFMA_BF16_PEAK / 1e12 / peaks["mfma_bf16_TFLOPs"]
    line = {
        "metric": "merged inferences/sec at M=%d (one %s per model), vs M separate launches" % (
            M, "sequence" if kind == "encoder" else "image"),
        "value": head["inferences_per_s"], "unit": "inferences/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "ms_per_step_std": head["ms_per_step_std"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": head["config"],
        "separate_launches": {"ms_per_step": head["separate_ms"], "inferences_per_s": head["separate_inferences_per_s"],
                              "steps": sweep_steps},
        "speedup_vs_separate": head["speedup_vs_separate"],
        "concurrent_streams": head.get("concurrent"),
        "launch": {k: head[k] for k in ("eager_ms", "graph_ms", "separate_eager_ms", "separate_graph_ms", "graph_error") if k in head},
        "model_TFLOPs": head["model_TFLOPs"],
        "kernel_time_ms_per_step": head["kernel_time_ms_per_step"],
        "roofline": {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel", "launches",
                                        "avg_us", "bytes_per_launch", "flops_per_launch", "frac_hbm", "frac_mfma",
                                        "frac_of_min_roof", "frac_of_measured_hbm_read", "frac_of_measured_mfma",
                                        "timing") if k in rf},
        "kernels": head["kernels"],
        "cpu_baseline": cpu,
        **sweeps,
        "norm_kernels": norms,
        "measured_peaks": peaks,
        "other_workloads": others,
        "paper_context": "NetFuse reports up to 3.6x (V100) / 3.0x (TITAN Xp) over its best baseline at 32 instances, fp32, bs 1",
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
