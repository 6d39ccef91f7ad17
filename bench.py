#!/usr/bin/env python3
"""Benchmark of the PAB attention hot path on one MI355X.

A "step" is one denoising step of the named synthetic workload: every
(block, kind) attention call of the video DiT goes through ``pab_attention``,
which computes or reuses according to the broadcast schedule (paper Sec. 2.3,
Eq. 1).  ``--steps`` defaults to one whole video.  Inputs are synthetic (seeded,
bf16 N(0,1), shapes of the workload) and resident in HBM before timing starts;
a pool of input sets larger than the last-level cache is rotated so that HBM
numbers are not cache hits.

Prints ONE JSON line: whole-job computed attention TFLOP/s under the PAB
schedule, per-video latency with and without PAB, the roofline of the dominant
kernel (spatial attention, bf16 MFMA) measured with stream events inside the
timed region, per-kind rates, and the CPU oracle timed on a bounded sample.
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# HBM bytes per launch, from the rocprofv3 --pmc runs summarised in
# profiles/attn_kernels_<workload>_hbm_traffic.txt (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the scales
# a 1 GiB copy gives), keyed by (workload, kind).  Not measured live: counters need the profiler.
# None where no profile exists.
PROFILED_TRAFFIC_BYTES = {("opensora_480p", 0): 413.9e6, ("opensora_480p", 1): 234.7e6, ("opensora_480p", 2): 122.1e6}
SPATIAL_KERNEL = "attn_tile16_kernel (spatial)"
CROSS_KERNEL = "attn_cross_kernel"
OTHER_WORKLOADS = ("latte_512", "osp_512_long", "stress_720p")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="denoising steps to time (default: one video)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first (default: one video)")
    ap.add_argument("--workload", default="opensora_480p")
    ap.add_argument("--pool", type=int, default=8, help="rotating input sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-module", action="store_true", help="skip the module-level section")
    ap.add_argument("--no-mfma-reference", action="store_true",
                    help="skip the library GEMM that shows what the matrix core sustains on this box")
    ap.add_argument("--videos", type=int, default=1, help="timed videos when --steps is not given (steps = videos x the workload's steps)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--kind-reps", type=int, default=40, help="launches per kind in the per-kind section")
    ap.add_argument("--repeats", type=int, default=5, help="repeats of the timed K-step region (PAB and no-PAB alternating); medians are reported")
    ap.add_argument("--latency-videos", type=int, default=5, help="whole videos timed per schedule after one warm-up video")
    ap.add_argument("--no-workloads", action="store_true", help="skip the compact section on the other configurations")
    ap.add_argument("--profile-kind", default=None, choices=["spatial", "temporal", "cross"],
                    help="counter-collection mode: one 1 GiB device copy (calibration), then --kind-reps launches "
                         "of this kind over the rotating pool; prints no result line")
    ap.add_argument("--input-scale", type=float, default=1.0,
                    help="profile mode only: multiply the inputs by this (0 = all-zero operands, the same "
                         "instruction stream with no data toggling: shows how far the clock follows the data)")
    return ap.parse_args()


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def _stats(xs, digits=4):
    return {"median": round(_median(xs), digits), "min": round(min(xs), digits), "max": round(max(xs), digits), "n": len(xs)}


class Harness:
    """Device-resident synthetic inputs of one workload and the loops that play its denoising steps through
    pab_attention.  Inputs rotate over a pool larger than the last-level cache; outputs go to the cache slots."""

    def __init__(self, wl, dev, pool_n, input_scale=1.0):
        import torch
        from paper_2408_12588_amd import workloads as W
        self.wl, self.dev, self.pool_n = wl, dev, pool_n
        self.torch, self.W = torch, W
        self.stream = torch.cuda.current_stream()
        gen = torch.Generator(device=dev)
        gen.manual_seed(wl.seed)
        self.full = (wl.T, wl.S, wl.heads, wl.head_dim)
        dt = wl.torch_dtype

        def randn(shape):
            return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * input_scale).to(dt)

        self.pool = [tuple(randn(self.full) for _ in range(3)) for _ in range(pool_n)]
        if wl.peaked_frac > 0:
            rows = torch.from_numpy(W.peaked_rows(wl)).to(dev)
            for q, _, _ in self.pool:
                q.view(wl.tokens, wl.heads, wl.head_dim)[rows] *= wl.peaked_scale
        self.kv_cross = [tuple(randn((wl.L, wl.heads, wl.head_dim)) for _ in range(2)) for _ in range(pool_n)] \
            if wl.intervals[W.CROSS] > 0 else None
        self.calls = wl.calls_per_step()

    def inputs(self, i, kind):
        q, k, v = self.pool[i % self.pool_n]
        if kind == self.W.CROSS:
            k, v = self.kv_cross[i % self.pool_n]
        return q, k, v

    def run_steps(self, ctx, first_step, n, marks=None, events=None):
        """Queue n denoising steps asynchronously; returns computed FLOPs and launches per kind.  marks collects one
        stream event at the start of every video and one after the last step; events (a list per kind) collects
        an event pair around every computed call."""
        from paper_2408_12588_amd import pab
        torch, wl = self.torch, self.wl
        flops, launches = [0.0, 0.0, 0.0], [0, 0, 0]
        i = first_step * len(self.calls)
        for s in range(first_step, first_step + n):
            step = s % wl.n_steps
            if step == 0:
                ctx.pab_reset()
                if marks is not None:
                    marks.append(torch.cuda.Event(enable_timing=True))
                    marks[-1].record(self.stream)
            for block, kind in self.calls:
                q, k, v = self.inputs(i, kind)
                i += 1
                if events is not None and pab.pab_schedule(kind, step, wl.lo, wl.hi, ctx.cfg.interval[kind]) == pab.COMPUTE:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(self.stream)
                    dec, _ = ctx.pab_attention(block, kind, step, q, k, v)
                    e1.record(self.stream)
                    events[kind].append((e0, e1))
                else:
                    dec, _ = ctx.pab_attention(block, kind, step, q, k, v)
                if dec == pab.COMPUTE:
                    flops[kind] += wl.flops(kind)
                    launches[kind] += 1
        if marks is not None:
            marks.append(torch.cuda.Event(enable_timing=True))
            marks[-1].record(self.stream)
        return flops, launches

    def region(self, ctx, n):
        """n steps from step 0, bracketed by synchronisation: (seconds, flops per kind, launches per kind)."""
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        flops, launches = self.run_steps(ctx, 0, n)
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0, flops, launches

    def videos(self, ctx, n_videos):
        """Latencies (ms) of n whole videos played back to back, from stream events at the video boundaries."""
        marks = []
        self.run_steps(ctx, 0, n_videos * self.wl.n_steps, marks=marks)
        self.torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:])]

    def traced_video(self, ctx):
        """One video with a stream-event pair around every computed call: per kind, the launch durations (ms) as
        they are inside the loop, neighbours of other kinds in between and every output going to its own slot."""
        events = [[], [], []]
        self.run_steps(ctx, 0, self.wl.n_steps, events=events)
        self.torch.cuda.synchronize()
        return [[a.elapsed_time(b) for a, b in ev] for ev in events]

    def back_to_back(self, ctx, kind, reps):
        """reps launches of one kind in a row, inputs rotating over the pool, outputs over the cache slots."""
        from paper_2408_12588_amd import pab
        torch = self.torch
        slots = [ctx.slot_tensor(b, kind) for b, k in self.calls if k == kind]
        for i in range(3):
            pab.pab_attention_compute(kind, *self.inputs(i, kind), out=slots[i % len(slots)])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        for i in range(reps):
            pab.pab_attention_compute(kind, *self.inputs(i, kind), out=slots[i % len(slots)])
        e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps


def kind_report(wl, kind, ms_list):
    """Rates and roofline fractions of one kind from a list of launch durations (ms)."""
    ms = sum(ms_list) / len(ms_list)
    tf = wl.flops(kind) / (ms * 1e-3) / 1e12
    gbs = wl.bytes(kind) / (ms * 1e-3) / 1e9
    return {"avg_launch_ms": round(ms, 4), "min_launch_ms": round(min(ms_list), 4), "max_launch_ms": round(max(ms_list), 4),
            "launches": len(ms_list), "tflops": round(tf, 2), "gbs": round(gbs, 1),
            "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}


def cross_roofline(wl, ms_list):
    """Cross attention runs one of two kernels: up to 128 text tokens the op is a stream of q and o rows against a
    resident K/V (HBM-bound); with more keys per query it is bound by the matrix core like the spatial kernel."""
    from paper_2408_12588_amd import workloads as W
    if wl.L <= 128:
        return hbm_roofline(wl, W.CROSS, CROSS_KERNEL, ms_list)
    ms = sum(ms_list) / len(ms_list)
    tf = wl.flops(W.CROSS) / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "kernel": "attn_cross_long_kernel" if wl.L <= 512 else SPATIAL_KERNEL,
            "achieved": round(tf, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4),
            "traffic": None, "algorithmic_bytes": wl.bytes(W.CROSS), "flops_per_launch": wl.flops(W.CROSS),
            "avg_launch_ms": round(ms, 4), "median_launch_ms": round(sorted(ms_list)[len(ms_list) // 2], 4),
            "launches": len(ms_list),
            "where": "stream events around every computed call inside one video, outputs to the cache slots"}


def hbm_roofline(wl, kind, kernel, ms_list):
    ms = sum(ms_list) / len(ms_list)
    gbs = wl.bytes(kind) / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "kernel": kernel, "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": PROFILED_TRAFFIC_BYTES.get((wl.name, kind)),
            "algorithmic_bytes": wl.bytes(kind), "avg_launch_ms": round(ms, 4),
            "median_launch_ms": round(sorted(ms_list)[len(ms_list) // 2], 4), "launches": len(ms_list),
            "where": "stream events around every computed call inside one video, outputs to the cache slots"}


def other_workload(name, args, dev):
    """One more configuration, compactly: a video with and without broadcasting, and the in-loop launch time of
    every kind from one traced video."""
    import torch
    from paper_2408_12588_amd import pab, workloads as W
    wl = W.BY_NAME[name]
    h = Harness(wl, dev, min(args.pool, 4))
    ctx = pab.PabContext(pab.config_of(wl), dev)
    ctx0 = pab.PabContext(pab.config_of(wl, (1, 1, 1)), dev, workspace=ctx.workspace)
    h.run_steps(ctx, 0, max(2, wl.lo + 1))                      # warm-up: a few steps
    ms_pab = h.videos(ctx, 1)[0]
    ms_all = h.videos(ctx0, 1)[0]
    traced = h.traced_video(ctx)
    flops = flops0 = 0.0
    for kind in range(3):
        if wl.intervals[kind] == 0:
            continue
        blocks = sum(1 for b, k in h.calls if k == kind)
        computed = sum(pab.pab_schedule(kind, s, wl.lo, wl.hi, wl.intervals[kind]) == pab.COMPUTE for s in range(wl.n_steps))
        flops += wl.flops(kind) * blocks * computed
        flops0 += wl.flops(kind) * blocks * wl.n_steps
    res = {"video_ms": {"pab": round(ms_pab, 3), "no_pab": round(ms_all, 3)},
           "time_reduction": round(1.0 - ms_pab / ms_all, 4), "skipped_flop_fraction": round(1.0 - flops / flops0, 4),
           "value_tflops": round(flops / (ms_pab * 1e-3) / 1e12, 2),
           "kinds_in_loop": {W.KIND_NAMES[k]: kind_report(wl, k, traced[k]) for k in range(3) if traced[k]}}
    ctx.pab_destroy()
    ctx0.pab_destroy()
    del h, ctx, ctx0
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2408_12588_amd import build as pab_build
    pab_build.ensure_built()                   # loads what is built; builds only if nothing is
    from paper_2408_12588_amd import pab, workloads as W

    wl = W.BY_NAME[args.workload]
    K = args.steps if args.steps is not None else wl.n_steps * max(1, args.videos)
    Wm = args.warmup if args.warmup is not None else wl.n_steps
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ---- inputs: seeded, on device, before any timing ----
    h = Harness(wl, dev, args.pool, args.input_scale if args.profile_kind else 1.0)

    if args.profile_kind:
        kind = W.KIND_NAMES.index(args.profile_kind)
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)   # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a)                                  # reads 1 GiB, writes 1 GiB: scale for FETCH_SIZE / WRITE_SIZE
        outs = [torch.empty(h.full, device=dev, dtype=wl.torch_dtype) for _ in range(4)]
        for i in range(args.kind_reps):
            pab.pab_attention_compute(kind, *h.inputs(i, kind), out=outs[i % 4])
        torch.cuda.synchronize()
        print("profiled %d launches of %s on %s" % (args.kind_reps, args.profile_kind, wl.name))
        return

    # ---- the timed region: K steps under the PAB schedule and K steps with ranges 1/1/1 (the same library),
    #      repeated and alternating, nothing but pab_attention calls inside ----
    ctx = pab.PabContext(pab.config_of(wl), dev)
    ctx0 = pab.PabContext(pab.config_of(wl, (1, 1, 1)), dev, workspace=ctx.workspace)
    h.run_steps(ctx, 0, Wm)
    secs, secs0 = [], []
    for _ in range(max(1, args.repeats)):
        sec, flops, launches = h.region(ctx, K)
        secs.append(sec)
        sec0, flops0, launches0 = h.region(ctx0, K)
        secs0.append(sec0)
    sec, sec0 = _median(secs), _median(secs0)
    total_flops = sum(flops)

    # ---- whole videos: one warm-up video, then --latency-videos timed ones, per schedule ----
    vids = h.videos(ctx, 1 + args.latency_videos)[1:]
    vids0 = h.videos(ctx0, 1 + args.latency_videos)[1:]

    # ---- launch durations inside the loop: a separate traced video (events around every computed call) ----
    traced = h.traced_video(ctx)
    in_loop = {W.KIND_NAMES[k]: kind_report(wl, k, traced[k]) for k in range(3) if traced[k]}
    sp = traced[W.SPATIAL]
    if sp:
        avg_ms = sum(sp) / len(sp)
        achieved = wl.flops(W.SPATIAL) / (avg_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": SPATIAL_KERNEL, "achieved": round(achieved, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": PROFILED_TRAFFIC_BYTES.get((wl.name, W.SPATIAL)),
                    "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, see profiles/)",
                    "algorithmic_bytes": wl.bytes(W.SPATIAL), "avg_launch_ms": round(avg_ms, 4), "launches": len(sp),
                    "flops_per_launch": wl.flops(W.SPATIAL),
                    "where": "stream events around every computed spatial call inside one video"}
    else:
        roofline = None
    roofline_hbm = {}
    if traced[W.TEMPORAL]:
        roofline_hbm["temporal"] = hbm_roofline(wl, W.TEMPORAL, "attn_temporal_kernel", traced[W.TEMPORAL])
    if traced[W.CROSS]:
        roofline_hbm["cross"] = cross_roofline(wl, traced[W.CROSS])

    # ---- per-kind section: back-to-back computes of one kind, inputs over the pool, outputs over the slots ----
    kinds = {}
    for kind in (W.SPATIAL, W.TEMPORAL, W.CROSS):
        if wl.intervals[kind] == 0:
            continue
        ms = h.back_to_back(ctx, kind, args.kind_reps)
        tf = wl.flops(kind) / (ms * 1e-3) / 1e12
        gbs = wl.bytes(kind) / (ms * 1e-3) / 1e9
        kinds[W.KIND_NAMES[kind]] = {
            "ms_per_call": round(ms, 4), "tflops": round(tf, 2), "gbs": round(gbs, 1),
            "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}
    ctx.pab_destroy()
    ctx0.pab_destroy()

    # ---- schedule accounting ----
    skipped_flop_fraction = 1.0 - total_flops / sum(flops0) if sum(flops0) else 0.0
    time_reduction = 1.0 - sec / sec0
    # what the in-loop launch times predict (reuse is free, so a kind's time scales with its launches)
    ms_of = [in_loop.get(n, {}).get("avg_launch_ms", 0.0) for n in W.KIND_NAMES]
    t_pab = sum(l * m for l, m in zip(launches, ms_of))
    t_all = sum(l * m for l, m in zip(launches0, ms_of))
    time_weighted_prediction = 1.0 - t_pab / t_all if t_all else 0.0
    vid_red = 1.0 - _median(vids) / _median(vids0)

    result = {
        "metric": "attention TFLOP/s + %roofline; per-video attention latency PAB vs no-PAB",
        "value": round(total_flops / sec / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(sec * 1e3 / K, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "blocks": wl.n_blocks, "T": wl.T, "S": wl.S, "L": wl.L,
                   "heads": wl.heads, "head_dim": wl.head_dim, "video_steps": wl.n_steps,
                   "intervals": list(wl.intervals), "window": [wl.lo, wl.hi], "input_pool": args.pool},
        "value_definition": "attention FLOPs actually computed under the PAB schedule in K steps / median wall time of "
                            "the K-step region over the repeats",
        "timed_region": {"repeats": len(secs), "pab_ms": _stats([x * 1e3 for x in secs], 3),
                         "no_pab_ms": _stats([x * 1e3 for x in secs0], 3)},
        "roofline": roofline,
        "roofline_hbm": roofline_hbm,
        "latency_ms": {"pab": round(sec * 1e3, 3), "no_pab": round(sec0 * 1e3, 3), "steps": K,
                       "videos_pab": {"per_video": [round(x, 3) for x in vids], **_stats(vids, 3)},
                       "videos_no_pab": {"per_video": [round(x, 3) for x in vids0], **_stats(vids0, 3)},
                       "video_time_reduction": round(vid_red, 4)},
        "pab": {"time_reduction": round(time_reduction, 4), "skipped_flop_fraction": round(skipped_flop_fraction, 4),
                "gap_abs": round(time_reduction - skipped_flop_fraction, 4),
                "gap_rel": round((time_reduction - skipped_flop_fraction) / skipped_flop_fraction, 4) if skipped_flop_fraction else None,
                "time_weighted_prediction": round(time_weighted_prediction, 4),
                "skipped_launch_fraction": [round(1.0 - a / b, 4) if b else None for a, b in zip(launches, launches0)],
                "launches_pab": launches, "launches_no_pab": launches0,
                "effective_tflops": round(sum(flops0) / sec / 1e12, 3)},
        "kinds_in_loop": in_loop,
        "kinds": kinds,
    }
    if not args.no_workloads:
        del h
        torch.cuda.empty_cache()
        result["workloads"] = {n: other_workload(n, args, dev) for n in OTHER_WORKLOADS if n != wl.name}
        h = Harness(wl, dev, args.pool)
    if not args.no_mfma_reference and wl.dtype == "bf16":
        result["mfma_reference"] = mfma_reference(dev)
        result["hbm_reference"] = hbm_reference(dev, wl)
    if not args.no_module and wl.dtype == "bf16":
        result["module"] = module_section(wl, h.pool, args, dev)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds)
    print(json.dumps(result), flush=True)


def mfma_reference(dev, n=8192, reps=20):
    """Context for the roofline fraction, not part of the path: the vendor library's plain bf16 GEMM
    (torch.matmul, n x n x n) on this machine, on N(0,1) operands and on all-zero ones.  The published peak
    assumes the full shader clock; under its power limit the chip does not hold it on real data, and
    this is the rate a dense contraction with no softmax in it sustains here."""
    import torch
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    stream = torch.cuda.current_stream()
    res = {"what": "torch.matmul bf16 %d^3 (vendor library), %d back-to-back calls" % (n, reps), "unit": "TFLOP/s"}
    for name, scale in (("normal", 1.0), ("zeros", 0.0)):
        a = [(torch.randn((n, n), generator=gen, device=dev) * scale).to(torch.bfloat16) for _ in range(2)]
        b = [(torch.randn((n, n), generator=gen, device=dev) * scale).to(torch.bfloat16) for _ in range(2)]
        c = torch.empty((n, n), device=dev, dtype=torch.bfloat16)
        for i in range(3):
            torch.matmul(a[i % 2], b[i % 2], out=c)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(reps):
            torch.matmul(a[i % 2], b[i % 2], out=c)
        e1.record(stream)
        torch.cuda.synchronize()
        tf = 2.0 * n ** 3 * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12
        res[name] = round(tf, 1)
        res[name + "_frac_of_peak"] = round(tf / PEAK_BF16_TFLOPS, 4)
    return res


def hbm_reference(dev, wl, n=1 << 29, reps=10):
    """Context for the HBM roofline fractions, not part of the path: what contiguous streams sustain on this machine, with
    torch's own elementwise kernels: a device copy (one read, one write) and q + k * v (three reads, one write: the
    traffic mix of an attention call), on 1 GiB bf16 tensors and, for the second, on tensors of the workload's own
    size (eight rotating sets, so that nothing is found in the last-level cache; launches this short carry their
    ramp-up and drain like the attention kernels do)."""
    import torch
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    stream = torch.cuda.current_stream()

    def rate(fn, nbytes, calls):
        for i in range(2):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(calls):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        return nbytes * calls / (e0.elapsed_time(e1) * 1e-3) / 1e9

    q, k, v = (torch.randn(n, generator=gen, device=dev, dtype=torch.bfloat16) for _ in range(3))
    o = torch.empty_like(q)
    res = {"what": "torch copy_ and addcmul on %d MiB bf16 tensors (%d back-to-back calls) and on [T,S,H,D] tensors of "
                   "the workload (8 rotating sets, 40 calls)" % (n * 2 >> 20, reps), "unit": "GB/s"}
    res["copy"] = round(rate(lambda i: o.copy_(q), 2 * n * 2, reps), 1)
    res["three_reads_one_write"] = round(rate(lambda i: torch.addcmul(q, k, v, out=o), 4 * n * 2, reps), 1)
    del q, k, v, o
    m = wl.T * wl.S * wl.heads * wl.head_dim
    sets = [[torch.randn(m, generator=gen, device=dev, dtype=torch.bfloat16) for _ in range(4)] for _ in range(8)]
    res["three_reads_one_write_workload_size"] = round(
        rate(lambda i: torch.addcmul(sets[i % 8][0], sets[i % 8][1], sets[i % 8][2], out=sets[(i + 3) % 8][3]), 4 * m * 2, 40), 1)
    for key in ("copy", "three_reads_one_write", "three_reads_one_write_workload_size"):
        res[key + "_frac_of_peak"] = round(res[key] / PEAK_HBM_GBS, 4)
    return res


def module_section(wl, pool, args, dev):
    """The same video with the whole attention module as the broadcast object (paper App. B.5 / B.6):
    layernorm + modulate, qkv projection, q/k layernorm (+ rotary), attention, output projection per
    computed call; reuse still costs nothing.  One weight set per (block, kind), random init."""
    import math
    import torch
    from paper_2408_12588_amd import pab, workloads as W
    T, S, H, D = wl.T, wl.S, wl.heads, wl.head_dim
    C, L, tok = H * D, max(wl.L, 1), wl.T * wl.S
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed + 1)

    def rn(shape, scale=1.0, offset=0.0):
        return (torch.randn(shape, generator=gen, device=dev) * scale + offset).to(torch.bfloat16)

    def weights(kind):
        if kind == W.CROSS:
            return pab.module_weights(w_qkv=rn((C, C), 1 / math.sqrt(C)), b_qkv=rn((C,), 0.1),
                                      w_kv=rn((2 * C, C), 1 / math.sqrt(C)), b_kv=rn((2 * C,), 0.1),
                                      w_o=rn((C, C), 1 / math.sqrt(C)), b_o=rn((C,), 0.1))
        return pab.module_weights(shift=rn((C,), 0.3), scale=rn((C,), 0.3), w_qkv=rn((3 * C, C), 1 / math.sqrt(C)),
                                  b_qkv=rn((3 * C,), 0.1), gamma_q=rn((D,), 0.2, 1.0), beta_q=rn((D,), 0.2),
                                  gamma_k=rn((D,), 0.2, 1.0), beta_k=rn((D,), 0.2),
                                  w_o=rn((C, C), 1 / math.sqrt(C)), b_o=rn((C,), 0.1))

    calls = wl.calls_per_step()
    wts = {(b, k): weights(k) for b, k in calls}
    text = rn((L, C))
    scratch = pab.module_scratch(T, S, wl.L, H, D, dev)
    xs = [p[0].view(T, S, C) for p in pool]

    def module_flops(kind):
        if kind == W.CROSS:
            return wl.flops(kind) + 2.0 * tok * C * C * 2 + 2.0 * L * C * 2 * C
        return wl.flops(kind) + 2.0 * tok * C * 3 * C + 2.0 * tok * C * C

    def video(intervals):
        ctx = pab.PabContext(pab.config_of(wl, intervals), dev)
        flops, launches = 0.0, [0, 0, 0]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        i = 0
        for step in range(wl.n_steps):
            for block, kind in calls:
                dec, _ = ctx.pab_module_attention(block, kind, step, xs[i % len(xs)], text if kind == W.CROSS else None,
                                                  wts[(block, kind)], scratch)
                i += 1
                if dec == pab.COMPUTE:
                    flops += module_flops(kind)
                    launches[kind] += 1
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        ctx.pab_destroy()
        return sec, flops, launches

    video(None)                                   # warm-up: one video under the PAB schedule
    sec, flops, launches = video(None)
    sec0, flops0, launches0 = video((1, 1, 1))
    per_kind = {}
    out = torch.empty((T, S, C), device=dev, dtype=torch.bfloat16)
    for kind in (W.SPATIAL, W.TEMPORAL, W.CROSS):
        if wl.intervals[kind] == 0:
            continue
        blocks = [b for b, k in calls if k == kind]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(8, args.kind_reps // 2)
        for timed in (False, True):
            if timed:
                e0.record(stream)
            for i in range(reps if timed else 2):
                pab.pab_module_compute(kind, xs[i % len(xs)], text if kind == W.CROSS else None,
                                       wts[(blocks[i % len(blocks)], kind)], H, scratch=scratch, out=out)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        per_kind[W.KIND_NAMES[kind]] = {"ms_per_call": round(ms, 4),
                                        "tflops": round(module_flops(kind) / (ms * 1e-3) / 1e12, 2)}
    # the MLP module of a block, the other object the paper broadcasts (App. A.2.2 MLP table): per-call rate only,
    # its schedule (three starting steps, blocks 0-4, range 2) skips 15 of 840 calls of this video
    inner = 4 * C
    mw = [pab.mlp_weights(shift=rn((C,), 0.3), scale=rn((C,), 0.3), w1=rn((inner, C), 1 / math.sqrt(C)), b1=rn((inner,), 0.1),
                          w2=rn((C, inner), 1 / math.sqrt(inner)), b2=rn((C,), 0.1)) for _ in range(4)]
    mscratch = pab.mlp_scratch(tok, C, inner, dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(8, args.kind_reps // 2)
    for timed in (False, True):
        if timed:
            e0.record(stream)
        for i in range(reps if timed else 2):
            pab.pab_mlp_compute(xs[i % len(xs)], mw[i % 4], inner, scratch=mscratch, out=out)
    e1.record(stream)
    torch.cuda.synchronize()
    mlp_ms = e0.elapsed_time(e1) / reps
    per_kind["mlp"] = {"ms_per_call": round(mlp_ms, 4), "tflops": round(4.0 * tok * C * inner / (mlp_ms * 1e-3) / 1e12, 2)}
    return {"object": "output of the attention module (layernorm+modulate, qkv proj, q/k layernorm, rotary, attention, o proj)",
            "value": round(flops / sec / 1e12, 3), "unit": "TFLOP/s",
            "latency_ms": {"pab": round(sec * 1e3, 3), "no_pab": round(sec0 * 1e3, 3), "steps": wl.n_steps},
            "time_reduction": round(1.0 - sec / sec0, 4),
            "skipped_flop_fraction": round(1.0 - flops / flops0, 4),
            "launches_pab": launches, "launches_no_pab": launches0, "kinds": per_kind}


def cpu_baseline(wl, target_seconds):
    """The fp64 oracle as it stands, timed on the host cores over a bounded sample of the same workload:
    whole frames of spatial attention (about 70 % of the budget, sized from a one-frame probe), then
    whole temporal and cross calls.  The per-video figures are extrapolations: seconds per call of each
    kind times the calls that kind computes in a video, with the broadcast schedule and without."""
    import numpy as np
    from oracle import pab_oracle as orc
    from paper_2408_12588_amd import workloads as W
    g = np.random.default_rng(wl.seed)
    H, D, S, T = wl.heads, wl.head_dim, wl.S, wl.T
    sec_per_call, samples, threads, total_fl, total_sec = {}, [], 1, 0.0, 0.0

    full = tuple(g.standard_normal((T, S, H, D)) for _ in range(3))

    def frames(n):
        return tuple(a[:n] for a in full)

    if wl.intervals[W.SPATIAL] > 0:
        q, k, v = frames(1)
        t0 = time.perf_counter()
        _, threads = orc.attention(q, k, v, return_threads=True)
        t1 = time.perf_counter() - t0
        budget = 0.7 * target_seconds
        n = int(max(1, min(T, budget / max(t1, 1e-3))))
        reps = int(max(1, budget / max(t1 * n, 1e-3)))
        q, k, v = frames(n)
        t0 = time.perf_counter()
        for _ in range(reps):
            orc.attention(q, k, v)
        sec = time.perf_counter() - t0
        sec_per_call[W.SPATIAL] = sec / reps * T / n
        total_fl += wl.flops(W.SPATIAL) * n / T * reps
        total_sec += sec
        samples.append("%d of %d frames of one spatial call x %d (%.1f s)" % (n, T, reps, sec))
    for kind in (W.TEMPORAL, W.CROSS):
        if wl.intervals[kind] == 0:
            continue
        q, k, v = frames(T)
        if kind == W.CROSS:
            k, v = (g.standard_normal((wl.L, H, D)) for _ in range(2))
        budget, reps, sec = 0.15 * target_seconds, 0, 0.0
        t0 = time.perf_counter()
        while reps == 0 or sec < budget:
            orc.kind_attention(kind, q, k, v)
            reps += 1
            sec = time.perf_counter() - t0
        sec_per_call[kind] = sec / reps
        total_fl += wl.flops(kind) * reps
        total_sec += sec
        samples.append("%d whole %s calls (%.1f s)" % (reps, W.KIND_NAMES[kind], sec))

    # calls each kind computes in one video, from the oracle's own schedule (Eq. 1)
    video = {}
    for name, ivals in (("pab", wl.intervals), ("no_pab", (1, 1, 1))):
        sec_v, fl_v = 0.0, 0.0
        for kind, sc in sec_per_call.items():
            per_block = sum(orc.schedule(st, wl.lo, wl.hi, ivals[kind]) == orc.COMPUTE for st in range(wl.n_steps))
            n_calls = per_block * sum(1 for b in range(wl.n_blocks) if kind in wl.kinds_of_block(b))
            sec_v += sc * n_calls
            fl_v += wl.flops(kind) * n_calls
        video[name] = (sec_v, fl_v)
    return {"value": round(video["pab"][1] / video["pab"][0] / 1e12, 6), "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle",
            "sample": "%s; fp64; %s; value = computed FLOPs of one video under the schedule / its extrapolated time"
                      % (wl.name, "; ".join(samples)),
            "seconds": round(total_sec, 2), "sample_tflops": round(total_fl / total_sec / 1e12, 6),
            "sec_per_call": {W.KIND_NAMES[kd]: round(sc, 6) for kd, sc in sec_per_call.items()},
            "video_seconds_extrapolated": {"pab": round(video["pab"][0], 3), "no_pab": round(video["no_pab"][0], 3)}}


if __name__ == "__main__":
    main()
