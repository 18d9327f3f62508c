#!/usr/bin/env python3
"""Throughput of one GPU's share of a layer-separated training iteration (paper Sec. 3.2) on MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
  CONV worker forward (all conv + pool layers)  ->  FC worker step over the n = K*B rows of features
  (this worker's B rows plus filler rows standing for the other K-1 workers)  ->  CONV worker backward
  ->  aggregation of K gradient shards + momentum-SGD update of the conv parameters.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
`value` comes from K steps run as a caller runs them (nothing between the calls); the per-call times and the roofline come from the
same K steps run once more with a HIP event pair around every entry-point call on the launch stream.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16|alexnet|resnet50|resnet50bn|resnet152|resnet152bn|inception3|vgg19|mlp|tiny]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak


class SclkSampler:
    """Reads the driver's shader-clock table (sysfs, no GPU call) from a thread while the timed steps run: the published MFMA
    peaks assume 2.4 GHz, and under a matrix-heavy load the clock the GPU actually sustains is lower."""

    def __init__(self, period_s=0.004):
        import glob
        import threading
        paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.path = paths[0] if paths else None
        self.period = period_s
        self.samples = []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        try:
            with open(self.path) as f:
                for line in f:
                    if "*" in line:
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            return None
        return None

    def _run(self):
        while not self._stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            self._stop.wait(self.period)

    def __enter__(self):
        if self.path:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self.path:
            self._thread.join()

    def summary(self):
        if not self.samples:
            return None
        v = sorted(self.samples)
        return {"mean": sum(v) / len(v), "median": v[len(v) // 2], "min": v[0], "max": v[-1], "samples": len(v)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"], help="conv-stack storage type (accumulation is always f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="per-call timing table on stderr")
    ap.add_argument("--one-stream", action="store_true",
                    help="issue every call of the CONV worker on the caller's stream, instead of spreading independent calls (a layer's "
                         "filter gradient beside its data gradient, the branches of a module) over several streams; the per-call pass "
                         "always runs this way")
    ap.add_argument("--dropout", type=float, default=0.0, help="seeded dropout after the FC worker's hidden layers (0: none)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step as one HIP graph in the timed region (launch-bound workloads); the per-call breakdown "
                         "and the roofline figures then come from the eager warm-up steps")
    ap.add_argument("--only", default=None, choices=["ps"],
                    help="ps: run only the K = 16 aggregation of BASELINE.json's config 5 (conv set and FC set) and print its figures; "
                         "with --calibrate the known-size launch that scales the profiler's HBM counters runs first")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch one stanza_add_relu_fwd over 3 x 1 GiB (2 GiB read, 1 GiB written): the known-size "
                         "kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the iteration; run with --gpus 1 "
              "(no collectives or multi-GPU paths exist here)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as W
    from paper_1812_10624_amd import api
    from paper_1812_10624_amd.netrun import Aggregator, ConvWorker, FcWorker

    api.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    if args.only == "ps":
        if args.calibrate:
            ca, cb, cc = (torch.ones(1 << 28, device=dev) for _ in range(3))
            api.stanza_add_relu_fwd(ca, cb, cc)
            torch.cuda.synchronize()
            del ca, cb, cc
            torch.cuda.empty_cache()
        print(json.dumps({"ps_aggregate_k16": ps_config5(torch, api, W, dev, iters=args.steps)}))
        return
    wl = W.get_workload(args.workload)
    K, B, n = wl.K, wl.B, wl.n
    seed = 0
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- inputs, resident before timing
    images = to_dev(W.gen_images(wl, seed, 0))
    labels = to_dev(W.gen_labels(wl, seed))
    cp = {nm: (to_dev(w), None if b is None else to_dev(b)) for nm, (w, b) in W.gen_conv_params(wl, seed).items()}
    cm = {nm: (torch.zeros_like(w), None if b is None else torch.zeros_like(b)) for nm, (w, b) in cp.items()}
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    fp, fm = [], []
    for o, i in W.fc_param_shapes(wl):   # drawn on the device: the FC set is up to 495 MB
        fp.append((torch.randn((o, i), device=dev, generator=gen) * (2.0 / i) ** 0.5,
                   (torch.rand(o, device=dev, generator=gen) * 2 - 1) / i ** 0.5))
        fm.append((torch.zeros((o, i), device=dev), torch.zeros(o, device=dev)))
    feats = torch.randn((n, wl.fc_dims[0]), device=dev, generator=gen).clamp_(min=0)   # filler rows of the other workers
    worker = ConvWorker(wl.ops, wl.image, B, cp, dtype=api.BF16 if args.dtype == "bf16" else api.F32, feat_out=feats[:B])
    fcw = FcWorker(wl.fc_dims, n, fp, fm, wl.lr, wl.momentum, wl.weight_decay, dropout=(args.dropout, seed) if args.dropout > 0 else None,
                   dtype=api.BF16 if (args.dtype == "bf16" and all(d % 8 == 0 for d in wl.fc_dims[:-1])) else api.F32)
    worker.multi_stream = not args.one_stream
    joined_ops = sorted(worker.joined)           # ops that run with the residual join fused into their epilogue
    shard0 = W.flat_tensors(worker.grads)
    shards = [shard0] + [[torch.randn(t.shape, device=dev, generator=gen) * 1e-3 for t in shard0] for _ in range(K - 1)]
    agg = Aggregator(W.flat_tensors(cp), W.flat_tensors(cm), shards)
    worker.buf["x0"].copy_(images)

    # ---- per-call instrumentation (HIP events on the stream the kernels are launched on)
    records = []     # (tag, start_event, end_event)

    call_reads = {}  # entry point -> per call (reads y as gate, reads the x mask, reads dx to accumulate), in issue order
    pool = []        # event pairs, reused by every step: a step's times are read before the next step records into them again

    recording = [True]

    def timed(tag, fn, *a, **kw):
        if not recording[0]:
            return fn(*a, **kw)
        if len(records) == len(pool):
            pool.append((torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)))
        s, e = pool[len(records)]
        s.record()
        fn(*a, **kw)
        e.record()
        records.append((tag, s, e))
        # which optional tensors this call reads (they count in its algorithmic bytes): the forward output that gates dy, the
        # layer input that gates dx, the previous dx of an accumulating call
        if tag == "stanza_conv_bwd_weight":
            call_reads.setdefault(tag, []).append((a[3] is not None, False, False))
        elif tag == "stanza_conv_bwd_data":
            call_reads.setdefault(tag, []).append((a[2] is not None, a[4] is not None, bool(a[0].flags & api.CONV_ACCUM)))

    real = {k: getattr(api, k) for k in ("stanza_conv_fwd", "stanza_conv_bwd_data", "stanza_conv_bwd_weight",
                                         "stanza_pool_relu_fwd", "stanza_pool_relu_bwd", "stanza_add_relu_fwd",
                                         "stanza_add_relu_bwd", "stanza_gap_fwd", "stanza_gap_bwd", "stanza_bn_fwd", "stanza_bn_bwd", "stanza_avgpool_fwd",
                                         "stanza_avgpool_bwd", "stanza_copy_channels", "stanza_cast_f32_to_bf16",
                                         "stanza_cast_bf16_to_f32")}
    import paper_1812_10624_amd.netrun as netrun

    class _Tap:
        """Same call surface as the api module, with an event pair around every call."""
        def __getattr__(self, k):
            if k in real:
                return lambda *a, **kw: timed(k, real[k], *a, **kw)
            if k == "stanza_conv_fwd_res":      # a forward convolution with the residual join in its epilogue: counted with the others
                return lambda *a, **kw: timed("stanza_conv_fwd", api.stanza_conv_fwd_res, *a, **kw)
            if k == "stanza_bn_fwd_res":        # likewise a normalisation layer with the join fused in
                return lambda *a, **kw: timed("stanza_bn_fwd", api.stanza_bn_fwd_res, *a, **kw)
            if k == "stanza_conv_fwd_stats":    # a forward convolution that leaves its output's column sums behind
                return lambda *a, **kw: timed("stanza_conv_fwd", api.stanza_conv_fwd_stats, *a, **kw)
            if k == "stanza_bn_fwd_stats":      # the normalisation layer that takes them (no statistics pass of its own)
                return lambda *a, **kw: timed("stanza_bn_fwd", api.stanza_bn_fwd_stats, *a, **kw)
            return getattr(api, k)
    tap = _Tap()

    def step():
        worker.forward()                                        # hand-off: written straight into this worker's rows of the FC input
        fcw.step(feats, labels)
        worker.backward(fcw.dfeats[:B])                         # hand-back: this worker's slice of the gradient
        agg.step(1.0, wl.lr, wl.momentum, wl.weight_decay)

    def step_instrumented():
        worker.forward()
        timed("stanza_fc_step", fcw.step, feats, labels)
        worker.backward(fcw.dfeats[:B])
        timed("stanza_ps_aggregate", agg.step, 1.0, wl.lr, wl.momentum, wl.weight_decay)

    if args.calibrate:
        ca, cb, cc = (torch.ones(1 << 28, device=dev) for _ in range(3))
        api.stanza_add_relu_fwd(ca, cb, cc)
        torch.cuda.synchronize()
        del ca, cb, cc
    # warm-up steps are issued exactly like the timed ones, the event mark after each step included (the first timing event that
    # a process records is not free, and it belongs here, not in the first timed step)
    warm_marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.warmup + 1)]
    warm_marks[0].record()
    for i in range(args.warmup):
        step()
        warm_marks[i + 1].record()
    # The interpreter's cyclic garbage collector is emptied here and what exists now is taken out of its reach: a full collection
    # walks every object of the process (torch's modules included) and takes some 40 ms; when its allocation count happened to come
    # up in the first timed step -- the one step that the host does not issue a whole step ahead of the GPU -- the GPU sat idle for
    # those 40 ms (seen as a first step of 85-95 ms against 47.6; which step it hits depends on how many objects were allocated
    # before, so it came and went with unrelated changes).  Collections still run afterwards, over the few objects made since.
    import gc
    gc.collect()
    gc.freeze()
    torch.cuda.synchronize()
    # ---- the timed region: K steps as a caller runs them, nothing between the calls.  (An event pair around every call keeps each
    # kernel from starting before the previous call's end event has been written: 1 % of a VGG-16-shaped step, 8 % of a
    # ResNet-50-shaped one, 20 % of an Inception-V3-shaped one.)
    if args.graph:
        graph = netrun.StepGraph(step, warmup=0)
        graph.replay()
        torch.cuda.synchronize()
        run_step = graph.replay
    else:
        run_step = step
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        run_step()
        marks[i + 1].record()
        if i == 0:
            loss_first = fcw.loss.clone()      # one 4-byte device copy inside the timed region
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # The timed data is live: every step is a real SGD step on the same batch, so the loss is finite and moves, and the features
    # this worker hands over keep about half of their units active (a stack whose activations had died would time faster).
    import math
    live = {"loss_after_first_timed_step": float(loss_first.item()), "loss_after_last_timed_step": float(fcw.loss.item()),
            "handed_over_features_nonzero_fraction": float((feats[:B] != 0).float().mean().item()),
            "fc_gradient_handed_back_abs_max": float(fcw.dfeats[:B].abs().max().item())}
    assert all(math.isfinite(v) for v in live.values()), live
    assert (args.steps < 2 or live["loss_after_first_timed_step"] != live["loss_after_last_timed_step"]) \
        and live["handed_over_features_nonzero_fraction"] > 0.01, live
    # ---- a few steps with every call on one stream (what the per-call pass below and the committed kernel traces measure), so that
    # the line shows what issuing independent calls on several streams is worth
    worker.multi_stream = False
    n_one = min(args.steps, 5)
    if args.one_stream or args.graph:
        ms_per_step_one_stream = None if args.graph else (t1 - t0) * 1e3 / args.steps      # the timed steps were such steps
    else:
        one_a, one_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        step()
        one_a.record()
        for _ in range(n_one):
            step()
        one_b.record()
        torch.cuda.synchronize()
        ms_per_step_one_stream = one_a.elapsed_time(one_b) / n_one
    # ---- the driver's shader clock while such steps run, read in a pass of its own, so that the sampling thread (it takes the
    # interpreter's lock every 4 ms) stays out of every timed pass
    with SclkSampler() as sclk:
        for _ in range(n_one):
            step()
        torch.cuda.synchronize()
    # ---- the same K steps again, eager, with an event pair around every entry-point call: per-call times, roofline
    # (still one stream: a call's event pair then brackets that call's kernels alone)
    netrun.api = tap
    plan = getattr(worker, "cast_plan", None)          # the one-launch cast of all bf16 filter copies is a method of its plan object
    if plan is not None:
        plan_run = plan.run
        plan.run = lambda: timed("stanza_cast_f32_to_bf16", plan_run)
    n_timed_eager = args.steps
    # The host must stay ahead of the GPU here, or the time the GPU waits for the next launch lands inside an event pair (a
    # bf16 AlexNet-shaped step is 2.7 ms of GPU work behind some sixty calls, each now with two event records).  So every
    # instrumented step is queued behind untimed work that keeps the GPU busy a little longer than the host needs to issue the
    # whole step: all of the step is queued before its first kernel starts.  That work is the worker's own forward pass, repeated
    # as often as needed, and not a spin kernel: behind a spin of one wavefront the driver drops the shader clock, and the forward
    # convolutions, first in the step, then ran 8 to 26 % slower than in the timed steps (16.9 against 15.0 ms for the
    # VGG-16-shaped stack), which understated every figure taken from this pass.  The blocker is outside every event pair.
    def blocker(times):
        recording[0] = False
        for _ in range(times):
            worker.forward()
        recording[0] = True

    blocker(1)
    t_issue = time.perf_counter()
    step_instrumented()
    t_issue = time.perf_counter() - t_issue              # host time to issue one instrumented step (the GPU may still be running)
    torch.cuda.synchronize()
    records.clear()
    ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev_a.record()
    blocker(1)
    ev_b.record()
    torch.cuda.synchronize()
    n_block = int(min(max(1.0, np.ceil(1.5 * t_issue * 1e3 / max(ev_a.elapsed_time(ev_b), 1e-3))), 64))
    inst_marks = []
    per = {}         # entry point -> its calls' times in issue order, step after step
    for i in range(args.steps):
        blocker(n_block)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step_instrumented()
        b.record()
        inst_marks.append((a, b))
        torch.cuda.synchronize()
        for tag, s, e in records:
            per.setdefault(tag, []).append(s.elapsed_time(e))
        records.clear()
    ms_per_step_instrumented = sum(a.elapsed_time(b) for a, b in inst_marks) / args.steps      # GPU time of a step, blocker excluded
    netrun.api = api
    if plan is not None:
        plan.run = plan_run
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    step_ms_in_order = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    step_ms = sorted(step_ms_in_order)     # each step between events on the stream
    props = torch.cuda.get_device_properties(0)

    tot = {k: sum(v) / n_timed_eager for k, v in per.items()}      # ms per step per entry point
    conv_ms = sum(tot.get(k, 0.0) for k in ("stanza_conv_fwd", "stanza_conv_bwd_data", "stanza_conv_bwd_weight"))
    conv_worker_ms = sum(v for k, v in tot.items() if k not in ("stanza_fc_step", "stanza_ps_aggregate"))
    fwd_f, bwd_f = W.conv_flops(wl)
    conv_tflops = (fwd_f + bwd_f) / (conv_ms * 1e-3) / 1e12
    gemm_flops = fwd_f + bwd_f + W.fc_flops(wl)
    gemm_ms = conv_ms + tot["stanza_fc_step"]
    gemm_tflops = gemm_flops / (gemm_ms * 1e-3) / 1e12
    conv_params, fc_params = W.count_params(wl)
    ps_bytes = (K + 4) * 4 * conv_params
    ps_gbs = ps_bytes / (tot["stanza_ps_aggregate"] * 1e-3) / 1e9

    # ---- per layer and direction: flops, algorithmic bytes (input, filter and output each moved once; the forward output too where
    # the backward pass gates on it), time.  Layers at or below the ridge of the roofline (peak flops / peak bytes) are bound by HBM,
    # not by the matrix pipes: they are also reported against the HBM peak.
    esz_c = 2 if args.dtype == "bf16" else 4
    ridge = (MFMA_BF16_PEAK_TFLOPS if args.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS) * 1e12 / (HBM_PEAK_GBS * 1e9)
    conv_ops = [(i, op) for i, op in enumerate(wl.ops) if op["op"] == "conv"]
    shapes = W.shape_pass(wl)
    layer_rows = []
    for kind in ("stanza_conv_fwd", "stanza_conv_bwd_weight", "stanza_conv_bwd_data"):
        v = per.get(kind, [])
        calls = len(v) // n_timed_eager
        ops_k = conv_ops if kind == "stanza_conv_fwd" else list(reversed(conv_ops))
        if kind == "stanza_conv_bwd_data":
            ops_k = [(i, op) for i, op in ops_k if op["src"] != "x0"]
        if calls != len(ops_k):
            continue
        for ci, (oi, op) in enumerate(ops_k):
            ms = float(np.median(v[ci::calls]))          # median over the steps: one stalled call must not set a layer's figure
            nn, ho, wo, kk = shapes[op["dst"]]
            _, hi, wi, c = shapes[op["src"]]
            fl = 2.0 * nn * ho * wo * kk * c * op["R"] * op["S"]
            n_in, n_out, n_w = float(nn * hi * wi * c), float(nn * ho * wo * kk), float(kk * op["R"] * op["S"] * c)
            reads_y, reads_mask, reads_dx = call_reads[kind][ci] if kind in call_reads else (False, False, False)
            if kind == "stanza_conv_fwd":
                by = esz_c * (n_in + n_w + n_out) + (esz_c * n_out if oi in worker.joined else 0.0)      # a fused join reads the other addend
            elif kind == "stanza_conv_bwd_data":
                by = esz_c * (n_out + n_w + n_in) + esz_c * (n_out * reads_y + n_in * reads_mask + n_in * reads_dx)
            else:
                by = esz_c * (n_in + n_out) + 4.0 * n_w + esz_c * n_out * reads_y                        # the filter gradient is float32
            layer_rows.append({"kind": kind[7:], "layer": op["name"], "in": f"{hi}x{wi}x{c}", "K": kk, "R": op["R"], "S": op["S"],
                               "stride": op["stride"], "ms": ms, "flops": fl, "bytes": by})
    low = [r for r in layer_rows if r["flops"] / r["bytes"] <= ridge]
    conv_at_ridge = None
    if low:
        lb, lms, lf = sum(r["bytes"] for r in low), sum(r["ms"] for r in low), sum(r["flops"] for r in low)
        conv_at_ridge = {"ridge_flop_per_byte": ridge, "calls_per_step": len(low), "algorithmic_bytes_per_step": lb, "ms_per_step": lms,
                         "GBps": lb / (lms * 1e-3) / 1e9, "frac_hbm": lb / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "TFLOPs": lf / (lms * 1e-3) / 1e12, "share_of_conv_ms": lms / conv_ms}
    if args.detail:
        print(f"per entry point, ms/step: " + ", ".join(f"{k}={v:.3f}" for k, v in sorted(tot.items())), file=sys.stderr)
        for k, v in sorted(per.items()):          # step by step: a pass that runs slower in some steps than in others shows here
            c = len(v) // n_timed_eager
            print(f"  {k} per instrumented step: " + " ".join(f"{sum(v[i * c:(i + 1) * c]):.3f}" for i in range(n_timed_eager)), file=sys.stderr)
        for r in layer_rows:
            print(f"  {r['kind']:16s} {r['layer']:8s} {r['in']:>12s} K{r['K']:<4d} R{r['R']} S{r['S']} s{r['stride']}  {r['ms']:8.3f} ms  "
                  f"{r['flops'] / r['ms'] / 1e9:7.1f} TFLOP/s  {r['flops'] / r['bytes']:7.1f} flop/B  {r['bytes'] / r['ms'] / 1e6:7.0f} GB/s",
                  file=sys.stderr)

    # HBM-bound kernels of the CONV worker: algorithmic bytes (every tensor moved once) over the measured time
    esz = 2 if args.dtype == "bf16" else 4
    shapes_all = W.shape_pass(wl)
    pool_f = pool_b = 0.0
    for op in wl.ops:
        if op["op"] == "pool":
            n_in = float(np.prod(shapes_all[op["src"]])); n_out = float(np.prod(shapes_all[op["dst"]]))
            pool_f += esz * n_in + esz * n_out + n_out                       # x read, y and argmax written
            pool_b += esz * n_out + n_out + (esz * n_out if op["relu"] else 0) + esz * n_in   # dy, argmax, y (gate) read, dx written
    # normalisation layers: forward reads x twice (statistics, then apply) and writes y; backward reads x and dy twice, writes dx.
    # A layer that takes its statistics from the producing convolution's epilogue reads x once.
    bn_elems = sum(float(np.prod(shapes_all[op["src"]])) for op in wl.ops if op["op"] == "bn")
    bn_fused_elems = sum(float(np.prod(shapes_all[wl.ops[i]["src"]])) for i in getattr(worker, "stats_bn", ()))
    # (a layer with the residual join fused in also reads the shortcut's tensor)
    bn_join_elems = sum(float(np.prod(shapes_all[wl.ops[i]["src"]])) for i in joined_ops if wl.ops[i]["op"] == "bn")
    hbm_kernels = {}
    for tag, by in (("stanza_pool_relu_fwd", pool_f), ("stanza_pool_relu_bwd", pool_b),
                    ("stanza_bn_fwd", 3 * esz * bn_elems - esz * bn_fused_elems + esz * bn_join_elems), ("stanza_bn_bwd", 5 * esz * bn_elems)):
        if tag in tot and by > 0:
            gbs = by / (tot[tag] * 1e-3) / 1e9
            hbm_kernels[tag] = {"algorithmic_bytes_per_step": by, "ms_per_step": tot[tag], "GBps": gbs, "frac_hbm": gbs / HBM_PEAK_GBS}

    out = {
        "metric": "conv_worker_train_images_per_sec_per_gpu",
        "value": B / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "conv_worker_streams": 1 if (args.one_stream or args.graph) else worker.n_streams,   # independent calls side by side
        "ms_per_step_one_stream": ms_per_step_one_stream,          # eager, every call on the caller's stream
        "ms_per_step_instrumented": ms_per_step_instrumented,      # the per-call pass, one stream, an event pair around every call
        "per_entry_point_ms": {k: round(v, 4) for k, v in sorted(tot.items())},      # of that pass, per step
        # untimed forward passes that the instrumented pass queues ahead of its steps (they are in a profiler's trace of this run)
        "blocker_forward_passes": 2 + n_block * args.steps,
        "step_ms_in_order": [round(v, 3) for v in step_ms_in_order],
        "step_ms_median": step_ms[len(step_ms) // 2], "step_ms_min": step_ms[0], "step_ms_max": step_ms[-1],
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "sclk_mhz_during_steps": sclk.summary(),
                   "note": "clocks and power state as the box provides them (not set by this run); sclk is the driver's own figure "
                           "(pp_dpm_sclk, sampled every 4 ms while a few further, untimed steps run); the roofline peaks assume 2400 MHz; cycle counters "
                           "read inside the GEMM kernels show lower effective clocks than the driver reports (bf16 launches 1.5-1.9 GHz)"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic", "launch": "hip_graph_replay" if args.graph else "eager",
        "config": {"workload": f"{wl.name}_shaped_conv_worker_B{B}_fc_worker_n{n}_K{K}_" + ("fp32" if args.dtype == "f32" else "bf16in_fp32acc"),
                   "per_worker_batch": B, "conv_workers_K": K, "fc_rows": n, "fc_dropout": args.dropout},
        "timed_data_is_live": live,
        "conv_worker_images_per_s": B / (conv_worker_ms * 1e-3),
        "conv_worker_ms": conv_worker_ms,
        "fc_worker_samples_per_s": n / (tot["stanza_fc_step"] * 1e-3),
        "fc_step_ms": tot["stanza_fc_step"],
        "fc_tflops": W.fc_flops(wl) / (tot["stanza_fc_step"] * 1e-3) / 1e12,
        "ps_aggregate_ms": tot["stanza_ps_aggregate"], "ps_aggregate_GBps": ps_gbs, "ps_aggregate_frac_hbm": ps_gbs / HBM_PEAK_GBS,
        "hbm_kernels": hbm_kernels,
        "conv_layers_at_or_below_ridge": conv_at_ridge,            # convolution calls that HBM bounds, not the matrix pipes
        "roofline": {"bound": "mfma", "kernel": "stanza::igemm_kernel (all launches of a step: conv fwd / bwd_data / bwd_weight "
                                                 "and the FC worker's GEMMs)",
                     "achieved": gemm_tflops, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / MFMA_F32_PEAK_TFLOPS, "traffic": traffic_from_profile(wl.name) if args.dtype == "f32" else None,
                     "algorithmic_gflop_per_step": gemm_flops / 1e9, "kernel_ms_per_step": gemm_ms,
                     "conv_only": {"achieved": conv_tflops, "frac": conv_tflops / MFMA_F32_PEAK_TFLOPS,
                                   "algorithmic_gflop_per_step": (fwd_f + bwd_f) / 1e9, "kernel_ms_per_step": conv_ms}},
    }

    # the paper's performance model (Sec. 4.2) fed with the times measured above
    mp = api.ModelParams(conv_worker_ms * 1e-3, tot["stanza_fc_step"] * 1e-3 / K, float(wl.fc_dims[0]), float(B), float(conv_params), 10e9)
    model = {"T_c_s": mp.T_c, "T_f_s_per_conv_worker": mp.T_f, "A": mp.A, "K_per_node_batch": mp.K, "P_c": mp.P_c}
    for tag, bw in (("ethernet_10Gb", 10e9), ("xgmi_link_153GBps", 153e9 * 8)):
        mp.bandwidth_bits = bw
        nc, nf, th = api.stanza_model_assign(mp, 9)
        model[tag] = {"t_iteration_s_at_K_conv_1_fc": api.stanza_model_stanza_time(mp, K, 1),
                      "throughput_samples_per_s_at_K_conv_1_fc": api.stanza_model_stanza_throughput(mp, K, 1),
                      "best_split_of_9_nodes": [nc, nf], "best_throughput_samples_per_s": th}
    out["stanza_model"] = model
    del worker, fcw, agg, shards, feats
    torch.cuda.empty_cache()
    out["ps_aggregate_k16"] = ps_config5(torch, api, W, dev)
    if args.dtype == "bf16":
        # the conv GEMMs run on the bf16 matrix pipe (the 3-channel first layer and the FC worker stay f32)
        out["roofline"] = {"bound": "mfma", "kernel": "stanza::igemm_bf16_kernel (conv fwd / bwd_data / bwd_weight launches of the conv stack)",
                           "achieved": conv_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": conv_tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                           "algorithmic_gflop_per_step": (fwd_f + bwd_f) / 1e9, "kernel_ms_per_step": conv_ms}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, seed)
    print(json.dumps(out))


def traffic_from_profile(workload):
    """HBM-side bytes per step of the igemm launches, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and written
    into profiles/ (bench.py cannot profile itself); None when no measurement of this workload is on file."""
    import re
    path = os.path.join(ROOT, "profiles", f"igemm_{workload}_b64_hbm_traffic.md")
    try:
        m = re.search(r"traffic_bytes_per_step:\s*(\d+)", open(path).read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


def ps_config5(torch, api, W, dev, iters=20):
    """Benchmark config 5: K = 16 gradient shards over the VGG-16-shaped conv parameter set (26 tensors) and
    over the FC set (6 tensors); one launch each, timed with HIP events, three buffer sets rotated for the conv
    set so that w and v do not stay in the 256 MB Infinity Cache between repetitions."""
    wl = W.get_workload("vgg16")
    K, res = 16, {}
    for which, nsets in (("conv", 3), ("fc", 1)):
        numels, _ = W.param_tensor_numels(wl, which)
        sets = []
        for _ in range(nsets):
            w = [torch.randn(n, device=dev) * 0.05 for n in numels]
            v = [torch.zeros(n, device=dev) for n in numels]
            g = [[torch.randn(n, device=dev) * 1e-3 for n in numels] for _ in range(K)]
            ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device=dev)
            sets.append((ws, api.stanza_ps_plan(w, v, g, ws), w, v, g))
        for i in range(3):
            api.stanza_ps_aggregate_planned(sets[i % nsets][1], 1.0, 0.01, 0.9, 5e-4, sets[i % nsets][0])
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for i in range(iters):
            api.stanza_ps_aggregate_planned(sets[i % nsets][1], 1.0, 0.01, 0.9, 5e-4, sets[i % nsets][0])
        e.record()
        torch.cuda.synchronize()
        us = s.elapsed_time(e) * 1e3 / iters
        by = (K + 4) * 4 * sum(numels)
        res[which] = {"params": sum(numels), "tensors": len(numels), "us": us, "GBps": by / us / 1e3,
                      "frac_hbm": by / us / 1e3 / HBM_PEAK_GBS, "algorithmic_bytes": by}
        del sets
        torch.cuda.empty_cache()
    return res


def cpu_baseline(wl, seed):
    """The CPU checker as it stands, timed on a bounded sample of the same workload: the same step with
    a few images per CONV worker (conv stack forward + backward, FC step over K times as many rows,
    aggregation of K shards over the full conv parameter set)."""
    import copy

    import numpy as np

    import oracle
    import workloads as W
    from oracle import network as onet

    o = oracle.lib("f32")
    K = wl.K
    b1 = 4      # images per CONV worker in the sample (about 15 s of checker time on 16 cores)
    img = W.gen_images(wl, seed, 0, b1)
    cp = W.gen_conv_params(wl, seed)
    rng = np.random.default_rng(seed)
    fp = [((rng.standard_normal((oo, ii), dtype=np.float32) * np.float32((2.0 / ii) ** 0.5)), np.zeros(oo, np.float32))
          for oo, ii in W.fc_param_shapes(wl)]
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    labels = W.gen_labels(wl, seed, K * b1)
    t0 = time.perf_counter()
    bufs = onet.conv_stack_forward(o, wl.ops, img, cp)
    feats = np.concatenate([bufs["feat"].reshape(b1, -1)] + [np.maximum(rng.standard_normal((b1, wl.fc_dims[0]), dtype=np.float32), 0)
                                                              for _ in range(K - 1)], 0)
    fc = onet.fc_step(o, feats, labels, fp, fm, wl.lr, wl.momentum, wl.weight_decay)
    pg, _ = onet.conv_stack_backward(o, wl.ops, bufs, cp, fc["dfeats"][:b1])
    for nm, (w, b) in cp.items():
        shards_w = [np.ascontiguousarray(pg[nm][0]).reshape(-1)] * K
        o.ps_aggregate(w.reshape(-1), np.zeros(w.size, np.float32), shards_w, 1.0, wl.lr, wl.momentum, wl.weight_decay)
        if b is not None:
            o.ps_aggregate(b, np.zeros_like(b), [pg[nm][1]] * K, 1.0, wl.lr, wl.momentum, wl.weight_decay)
    dt = time.perf_counter() - t0
    return {"value": b1 / dt, "unit": "images/s", "cores": o.threads(),
            "kind": "oracle", "seconds": dt,
            "sample": f"same step at {b1} images per CONV worker: conv stack fwd+bwd on {b1} images, FC step over {K * b1} rows, "
                      f"aggregation of {K} shards over the full conv parameter set"}


if __name__ == "__main__":
    main()
