#!/usr/bin/env python3
"""Benchmark of the five-stage hot path on one MI355X.

One *step* runs every stage once at its benchmark configuration (hb_fir1d 256x256/8 taps,
hb_sepblur 4096x4096/16-tap Gaussian, hb_sat2d 4096x4096, hb_conv3x3 1x1024x1024x64->64,
hb_pyr_level 8192x8192) on seeded synthetic inputs that are already resident in HBM.
Buffers rotate between launches so that no input is reused before more than the 256 MB
memory-side cache has gone past (the outputs are written with streaming stores).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--variant mfma|valu] [--no-cpu] [--no-extra]

prints ONE JSON line:
  value / ms_per_step   wall clock over exactly K timed steps (after W warm-up steps);
  step_stats            median / min / max over five more batches of K steps (HIP events);
  stages                per stage: median / min / max per launch over five batches of 50 back-to-back
                        launches between one pair of HIP events (rotating buffers), its roofline
                        fraction from the median, and the HBM traffic measured for it (profiles/);
  roofline              the stage that takes the longest: HIP events around its launch inside the
                        timed steps (and the batched figure next to it);
  supplementary         the tuned fp16 -> fp32 copy as the practical ceiling, the stacked FIR, a graph
                        replay of the step, and the paper's other case studies, each with its own
                        roofline object;
  cpu_baseline          the fp64 oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense f16 MFMA
MFMA_F32_PEAK_TFLOPS = 157.3   # fp32 on the matrix units

STAGES = ["fir1d", "sepblur", "sat2d", "conv3x3", "pyr_level"]
BATCHES, PER_BATCH = 5, 50
MIB = 1 << 20


def measured_traffic(fname):
    """HBM bytes per launch {name: (read, written)} from a counter summary under profiles/ (lines
    `traffic <name> read_MiB <r> write_MiB <w>`, written by the FETCH_SIZE / WRITE_SIZE runs whose
    commands the file states).  Empty when the file is absent: the figure is then reported as null."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", fname)) as f:
            for line in f:
                m = re.match(r"traffic\s+(\S+)\s+read_MiB\s+([0-9.]+)\s+write_MiB\s+([0-9.]+)", line)
                if m:
                    out[m.group(1)] = (float(m.group(2)) * MIB, float(m.group(3)) * MIB)
    except OSError:
        pass
    return out


def stage_work(cfg):
    """pixels, algorithmic bytes, algorithmic flops per launch (input + output sizes, true MACs)."""
    from paper_2512_02371_amd.synth import CONFIGS as C
    px = {
        "fir1d": C["fir1d"]["H"] * C["fir1d"]["W"],
        "sepblur": C["sepblur"]["H"] * C["sepblur"]["W"],
        "sat2d": C["sat2d"]["H"] * C["sat2d"]["W"],
        "conv3x3": C["conv3x3"]["N"] * C["conv3x3"]["H"] * C["conv3x3"]["W"],
        "pyr_level": C["pyr_level"]["H"] * C["pyr_level"]["W"],
    }[cfg]
    if cfg == "conv3x3":
        nbytes = px * 64 * 2 * 2 + 9 * 64 * 64 * 2
        flops = px * 2 * 9 * 64 * 64
    else:
        nbytes = px * 6
        flops = px * {"fir1d": 16, "sepblur": 64, "sat2d": 2, "pyr_level": 17}[cfg]
    return px, nbytes, flops


def stats(v):
    v = sorted(v)
    return {"median": float(np.median(v)), "min": float(v[0]), "max": float(v[-1])}


def roofline_object(ms, nbytes, flops, mfma_peak=MFMA_F16_PEAK_TFLOPS, traffic=None, force=None):
    """The roofline that binds at the peaks: memory time against matrix time of the ALGORITHMIC work
    (`force` names it for the five stages, whose governing roofline the benchmark definition fixes:
    the conv stage sits at the ridge, 30.9 us of products against 33.6 us of traffic, and counts as
    a matrix-unit stage)."""
    t_mem, t_mat = nbytes / (HBM_PEAK_GBS * 1e9), flops / (mfma_peak * 1e12)
    if force == "mfma" or (force is None and t_mat > t_mem):
        ach = flops / ms / 1e9
        o = {"bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s", "frac": ach / mfma_peak}
    else:
        ach = nbytes / ms / 1e6
        o = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS}
    o["algorithmic_bytes"] = int(nbytes)
    o["algorithmic_flops"] = int(flops)
    o["traffic"] = None if traffic is None else int(traffic[0] + traffic[1])
    return o


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--variant", choices=["mfma", "valu"], default="mfma")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the supplementary runs")
    ap.add_argument("--counter-run", action="store_true",
                    help="for hardware-counter runs under rocprofv3: one batch of two launches wherever batches are timed")
    ap.add_argument("--only-row", default=None,
                    help="for counter runs: launch the calibration copy and ONE supplementary row (matrix-unit path), "
                         "skip the five-stage step; prints that row")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; every box of this pool has one. Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_02371_amd import hb, synth
    hb.load()                                   # raises if libhb.so is missing: no fallback
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    C = synth.CONFIGS
    sfx = "" if args.variant == "mfma" else "_valu"
    traffic5 = measured_traffic("bench_five_stages_hbm_traffic.txt") if sfx == "" else {}
    traffic_x = measured_traffic("bench_supplementary_hbm_traffic.txt") if sfx == "" else {}

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).to(dev)

    def event():
        return torch.cuda.Event(enable_timing=True)

    def batched(fn, nsets, per_batch=PER_BATCH, batches=BATCHES, warm=10):
        """ms per launch: `batches` times `per_batch` back-to-back launches between two HIP events."""
        if args.counter_run:
            per_batch, batches, warm = 2, 1, 1
        for i in range(warm):
            fn(i % nsets)
        torch.cuda.synchronize()
        ms = []
        for b in range(batches):
            e0, e1 = event(), event()
            e0.record()
            for i in range(per_batch):
                fn((b * per_batch + i) % nsets)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1) / per_batch)
        return stats(ms)

    # ---- seeded inputs, several buffer sets per stage (rotated per launch) -----------------
    fir_taps = synth.random_taps_f16(C["fir1d"]["seed_taps"], 8)
    gau_taps = synth.gaussian_taps_f16(16, 3.0)
    host = {
        "fir1d": synth.uniform01_f16(C["fir1d"]["seed_img"], (256, 256)),
        "sepblur": synth.uniform01_f16(C["sepblur"]["seed_img"], (4096, 4096)),
        "sat2d": synth.uniform01_f16(C["sat2d"]["seed_img"], (4096, 4096)),
        "conv3x3": synth.uniform_pm1_f16(C["conv3x3"]["seed_img"], (1, 1024, 1024, 64)),
        "conv3x3_w": synth.normal_f16(C["conv3x3"]["seed_w"], (3, 3, 64, 64), 1.0 / 24.0),
        "pyr_level": synth.uniform01_f16(C["pyr_level"]["seed_img"], (8192, 8192)),
    }
    # inputs of one stage alone exceed the 256 MB memory-side cache between two uses of a buffer
    nsets = {"fir1d": 4, "sepblur": 10, "sat2d": 10, "conv3x3": 3, "pyr_level": 3}
    ins, outs = {}, {}
    for st in STAGES:
        base = up(host[st])
        ins[st] = [base] + [base.clone() for _ in range(nsets[st] - 1)]
        odt = torch.float16 if st == "conv3x3" else torch.float32
        outs[st] = [torch.empty(base.shape, dtype=odt, device=dev) for _ in range(nsets[st])]
    w_dev = up(host["conv3x3_w"])
    sat_ws = torch.empty(hb.hb_sat2d_workspace_size(4096, 4096), dtype=torch.uint8, device=dev)

    calls = {
        "fir1d": lambda i: getattr(hb, "hb_fir1d" + sfx)(ins["fir1d"][i], outs["fir1d"][i], fir_taps, 3),
        "sepblur": lambda i: getattr(hb, "hb_sepblur" + sfx)(ins["sepblur"][i], outs["sepblur"][i],
                                                             gau_taps, 7, gau_taps, 7),
        "sat2d": lambda i: getattr(hb, "hb_sat2d" + sfx)(ins["sat2d"][i], outs["sat2d"][i], sat_ws),
        "conv3x3": lambda i: getattr(hb, "hb_conv3x3" + sfx)(ins["conv3x3"][i], w_dev, outs["conv3x3"][i]),
        "pyr_level": lambda i: getattr(hb, "hb_pyr_level" + sfx)(ins["pyr_level"][i], outs["pyr_level"][i], None),
    }

    def step(k, ev=None, only=None):
        for st in STAGES:
            if ev is not None and only == st:
                ev[0].record()
            calls[st](k % nsets[st])
            if ev is not None and only == st:
                ev[1].record()

    # One plain copy of known size (32 MiB read, 64 MiB written), untimed: a counter run of this
    # program reads its own scale for FETCH_SIZE / WRITE_SIZE from this dispatch.
    hb.hb_copy_f16_f32(ins["sepblur"][0], outs["sepblur"][0])
    # no collector pauses between launches: a collection during a batch shows up as tens of milliseconds
    # of GPU idle time in that batch
    gc.collect()
    gc.disable()
    if args.only_row:
        sup = supplementary(args, hb, synth, torch, dev, up, batched, step, ins, outs, host, fir_taps, 0, 0.0, sfx, traffic_x,
                            calls, nsets)
        print(json.dumps({"row": args.only_row, "result": sup.get(args.only_row)}))
        return
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    # ---- per stage: batches of back-to-back launches (before the timed steps, untimed region) ----
    per_batch = PER_BATCH if sfx == "" else 10
    stage_ms = {st: batched(calls[st], nsets[st], per_batch=per_batch) for st in STAGES}
    dom = max(STAGES, key=lambda s: stage_ms[s]["median"])

    # ---- the timed region: exactly K steps, wall clock; HIP events around the longest stage only ----
    evs = [(event(), event()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k, evs[k], only=dom)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    dom_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))      # inside the timed steps
    total_px = sum(stage_work(st)[0] for st in STAGES)

    # ---- five more batches of K steps for the spread ----
    step_ms = []
    for b in range(BATCHES):
        e0, e1 = event(), event()
        e0.record()
        for k in range(args.steps):
            step(b * args.steps + k)
        e1.record()
        torch.cuda.synchronize()
        step_ms.append(e0.elapsed_time(e1) / args.steps)

    stages = {}
    for st in STAGES:
        px, nbytes, flops = stage_work(st)
        ms = stage_ms[st]["median"]
        r = roofline_object(ms, nbytes, flops, traffic=traffic5.get(st), force="mfma" if st == "conv3x3" else "hbm")
        stages[st] = dict({"gpixels_per_s": px / ms / 1e6, "ms": ms, "ms_min": stage_ms[st]["min"],
                           "ms_max": stage_ms[st]["max"], "launches_per_batch": per_batch, "batches": BATCHES}, **r)
    _, dbytes, dflops = stage_work(dom)
    roofline = roofline_object(dom_ms, dbytes, dflops, traffic=traffic5.get(dom), force="mfma" if dom == "conv3x3" else "hbm")
    roofline.update({"kernel": "hb_" + dom + sfx, "ms": dom_ms, "ms_batched_median": stage_ms[dom]["median"],
                     "timing": "HIP events around the launch inside the timed steps (mean over the steps)"})

    out = {
        "metric": "Gpixels/s per stage (fp16 in, fp32 acc) + % of HBM / MFMA roofline",
        "value": total_px / ms_per_step / 1e6,
        "unit": "Gpixels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 operands, f32 accumulate",
        "data": "synthetic (seeded hash; values on the fp16 grid), inputs resident in HBM, buffers rotated",
        "config": {"workload": "one step = all five stages at their benchmark configurations: "
                               "fir1d 256x256 T8, sepblur 4096x4096 T16 sigma3, sat2d 4096x4096, "
                               "conv3x3 1x1024x1024x64->64, pyr_level 8192x8192",
                   "variant": args.variant, "pixels_per_step": total_px},
        "step_stats": dict(stats(step_ms), unit="ms", batches=BATCHES, steps_per_batch=args.steps),
        "stages": stages,
        "roofline": roofline,
    }

    if not args.no_extra:
        out["supplementary"] = supplementary(args, hb, synth, torch, dev, up, batched, step, ins, outs, host,
                                             fir_taps, total_px, ms_per_step, sfx, traffic_x, calls, nsets)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(host, fir_taps, gau_taps, total_px)
    print(json.dumps(out))


def supplementary(args, hb, synth, torch, dev, up, batched, step, ins, outs, host, fir_taps, total_px,
                  ms_per_step, sfx, traffic_x, calls=None, nsets=None):
    """Outside the timed step: the copy ceiling, the stacked FIR, the step from a graph, and the paper's other
    case studies (matrix-unit kernel and vector-ALU twin), each with a roofline object of its ALGORITHMIC work
    (input + output bytes once, the definition's multiply-adds; Sec. V-A's accounting)."""
    sup = {}
    lx, lo = ins["sepblur"], outs["sepblur"]
    ns = len(lx)
    npx = 4096 * 4096

    only = args.only_row

    def pair(name, mfn, vfn, nsets, nbytes, flops, px, mfma_peak=MFMA_F16_PEAK_TFLOPS, extra=None):
        if only and name != only:
            return
        m = batched(mfn, nsets, per_batch=20)
        if only:
            sup[name] = {"mfma_ms": m["median"]}
            return
        v = batched(vfn, nsets, per_batch=5, batches=3, warm=2)
        row = {"mfma_ms": m["median"], "mfma_ms_min": m["min"], "mfma_ms_max": m["max"], "valu_ms": v["median"],
               "mfma_gpixels_per_s": px / m["median"] / 1e6, "valu_gpixels_per_s": px / v["median"] / 1e6,
               "mfma_over_valu": v["median"] / m["median"],
               "roofline": roofline_object(m["median"], nbytes, flops, mfma_peak, traffic_x.get(name))}
        if extra:
            row.update(extra)
        sup[name] = row

    # the practical ceiling of a 2 B in + 4 B out stream: the tuned copy at both image sizes
    for size, bufs_in, bufs_out in ((4096, lx, lo), (8192, ins["pyr_level"], outs["pyr_level"])):
        if only:
            break
        n = size * size
        m = batched(lambda i: hb.hb_copy_f16_f32(bufs_in[i], bufs_out[i]), len(bufs_in))
        sup["copy_ceiling_%dx%d" % (size, size)] = {
            "ms": m["median"], "ms_min": m["min"], "ms_max": m["max"], "achieved": 6.0 * n / m["median"] / 1e6,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": 6.0 * n / m["median"] / 1e6 / HBM_PEAK_GBS}

    # the same step replayed from a HIP graph (the library allocates nothing, synchronises nothing and issues
    # no memset, so its launches can be captured)
    # the same step with its independent stages on TWO streams (the pyramid on one, the other four on the other;
    # no stage waits for another, each stream keeps its order): the tail of one kernel overlaps the start of the
    # next.  Not the headline figure: kernels that share the chip cannot be timed one by one, so `value`,
    # `stages` and `roofline` come from the single-stream step.  (Three or more streams put the two longest
    # kernels on the chip together and measured 2-3x SLOWER.)
    if not only and calls is not None:
        s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
        others = [st for st in STAGES if st != "pyr_level"]

        def step2(k):
            with torch.cuda.stream(s_a):
                calls["pyr_level"](k % nsets["pyr_level"])
            with torch.cuda.stream(s_b):
                for st in others:
                    calls[st](k % nsets[st])
        for k in range(args.warmup):
            step2(k)
        torch.cuda.synchronize()
        ms2 = []
        for b in range(BATCHES):
            t0 = time.perf_counter()
            for k in range(args.steps):
                step2(b * args.steps + k)
            torch.cuda.synchronize()
            ms2.append((time.perf_counter() - t0) * 1e3 / args.steps)
        st2 = stats(ms2)
        sup["five_stage_step_two_streams"] = {
            "ms_per_step": st2["median"], "ms_min": st2["min"], "ms_max": st2["max"],
            "gpixels_per_s": total_px / st2["median"] / 1e6, "one_stream_over_two": ms_per_step / st2["median"],
            "streams": "pyr_level | fir1d, sepblur, sat2d, conv3x3", "batches": BATCHES, "steps_per_batch": args.steps}
    if not only:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for k in range(4):
                step(k)
        graph.replay()
        torch.cuda.synchronize()
        nrep = max(1, args.steps // 4)
        t0 = time.perf_counter()
        for _ in range(nrep):
            graph.replay()
        torch.cuda.synchronize()
        gms = (time.perf_counter() - t0) * 1e3 / (4 * nrep)
        sup["five_stage_step_graph_replay"] = {"ms_per_step": gms, "gpixels_per_s": total_px / gms / 1e6,
                                               "steps_per_graph": 4, "eager_over_graph": ms_per_step / gms}
        del graph
    del ins["pyr_level"], outs["pyr_level"], ins["conv3x3"], outs["conv3x3"]
    torch.cuda.empty_cache()

    # the FIR stage on 1024 of its 256 x 256 images stacked into one 262144 x 256 image, where its launch
    # latency no longer hides its bandwidth
    Hs = 256 * 1024
    if not only or only == "fir1d_stacked_262144x256":
        sx = [up(host["fir1d"]).repeat(1024, 1) for _ in range(3)]
        so = [torch.empty((Hs, 256), dtype=torch.float32, device=dev) for _ in range(3)]
        fir = getattr(hb, "hb_fir1d" + sfx)
        m = batched(lambda i: fir(sx[i], so[i], fir_taps, 3), 3, per_batch=10)
        sup["fir1d_stacked_262144x256"] = dict(
            {"ms": m["median"], "ms_min": m["min"], "ms_max": m["max"], "gpixels_per_s": Hs * 256 / m["median"] / 1e6},
            **roofline_object(m["median"], Hs * 256 * 6, Hs * 256 * 16, traffic=traffic_x.get("fir1d_stacked_262144x256")))
        del sx, so
        torch.cuda.empty_cache()

    # the large-tap regime of the paper's 1-D study (Sec. V-A)
    for ntaps in (64, 128, 256):
        t = synth.random_taps_f16(2000 + ntaps, ntaps)
        pair("fir1d_%dtaps_4096x4096" % ntaps,
             lambda i: hb.hb_fir1d(lx[i], lo[i], t, (ntaps - 1) // 2),
             lambda i: hb.hb_fir1d_valu(lx[i], lo[i], t, (ntaps - 1) // 2),
             ns, 6 * npx, 2 * ntaps * npx, npx)
    # the 2-D study (Sec. V-A): non-separable k x k kernels
    for k in (16, 32):
        k2d = synth.random_kernel2d_f16(2300 + k, k, k)
        pair("conv2d_%dx%d_4096x4096" % (k, k),
             lambda i: hb.hb_conv2d(lx[i], lo[i], k2d, k // 2, k // 2),
             lambda i: hb.hb_conv2d_valu(lx[i], lo[i], k2d, k // 2, k // 2),
             ns, 6 * npx, 2 * k * k * npx, npx)
    # the resampling study (Sec. V-B): 2x down (4096^2 -> 2048^2) and 2x up (2048^2 -> 4096^2); pixels are counted
    # on the larger image
    half_out = [torch.empty((2048, 2048), dtype=torch.float32, device=dev) for _ in range(ns)]
    half_in = [t[:2048, :2048] for t in lx]               # row pitch 4096
    for k in (16, 32):
        k2d = synth.random_kernel2d_f16(2400 + k, k, k)
        pair("down2_%dx%d_4096x4096" % (k, k),
             lambda i: hb.hb_down2(lx[i], half_out[i], k2d, k // 2, k // 2),
             lambda i: hb.hb_down2_valu(lx[i], half_out[i], k2d, k // 2, k // 2),
             ns, 2 * npx + 4 * npx // 4, 2 * k * k * (npx // 4), npx)
        pair("up2_%dx%d_4096x4096" % (k, k),
             lambda i: hb.hb_up2(half_in[i], lo[i], k2d, k // 4, k // 4),
             lambda i: hb.hb_up2_valu(half_in[i], lo[i], k2d, k // 4, k // 4),
             ns, 2 * npx // 4 + 4 * npx, 2 * (k // 2) * (k // 2) * npx, npx)
    del half_out, half_in
    # the non-integer resize (Sec. V-C, Table II): a 2048 x 2048 RGB image down to 143 / 245 / 450 / 921 squared
    rgb = [torch.rand((3, 2048, 2048), device=dev).half() for _ in range(12)]
    for n in (143, 245, 450, 921):
        st_h, cf_h = hb.hb_lanczos3_matrix(2048, n)
        st_d = torch.from_numpy(st_h).to(dev)
        cf_d = torch.from_numpy(cf_h.view(np.int16)).to(dev).view(torch.float16)
        ro = torch.empty((3, n, n), dtype=torch.float32, device=dev)
        rws = torch.empty(hb.hb_resize_workspace_size(3, 2048, n), dtype=torch.uint8, device=dev)
        band = int(cf_h.shape[1])
        pair("resize_lanczos3_3x2048x2048_to_%d" % n,
             lambda i: hb.hb_resize(rgb[i], ro, rws, st_d, cf_d, st_d, cf_d),
             lambda i: hb.hb_resize_valu(rgb[i], ro, rws, st_d, cf_d, st_d, cf_d),
             12, 3 * (2 * 2048 * 2048 + 4 * n * n), 3 * 2 * band * (2048 * n + n * n), 3 * 2048 * 2048,
             extra={"band": band})
    del rgb
    # the recursive filter (Sec. V-D): 2^21 stereo samples, a resonant second-order filter
    T = 1 << 21
    aud = [(torch.rand((2, T), device=dev) * 2 - 1).half() for _ in range(4)]
    aout = [torch.empty((2, T), dtype=torch.float32, device=dev) for _ in range(4)]
    aws = torch.empty(hb.hb_iir2_workspace_size(2, T), dtype=torch.uint8, device=dev)
    pair("iir2_2x2097152",
         lambda i: hb.hb_iir2(aud[i], aout[i], 1.6, -0.8, aws),
         lambda i: hb.hb_iir2_valu(aud[i], aout[i], 1.6, -0.8, aws),
         4, 6 * 2 * T, 4 * 2 * T, 2 * T)
    if "iir2_2x2097152" in sup:
        sup["iir2_2x2097152"]["mfma_gsamples_per_s"] = 2 * T / sup["iir2_2x2097152"]["mfma_ms"] / 1e6
    del aud, aout
    # DCT-domain denoising (Sec. V-E): a one-megapixel three-channel image; fp32 products on the matrix units
    dimg = [torch.rand((3, 1024, 1024), device=dev).half() for _ in range(4)]
    dout = [torch.empty((3, 1024, 1024), dtype=torch.float32, device=dev) for _ in range(4)]
    dws = torch.empty(hb.hb_dct_denoise_workspace_size(3, 1024, 1024), dtype=torch.uint8, device=dev)
    ntile = 3 * 127 * 127
    pair("dct_denoise_3x1024x1024",
         lambda i: hb.hb_dct_denoise(dimg[i], dout[i], 0.05, dws),
         lambda i: hb.hb_dct_denoise_valu(dimg[i], dout[i], 0.05, dws),
         4, 6 * 3 * 1024 * 1024, ntile * 4 * 2 * 16 ** 3, 3 * 1024 * 1024, mfma_peak=MFMA_F32_PEAK_TFLOPS)
    return sup


def cpu_baseline(host, fir_taps, gau_taps, total_px):
    """The fp64 oracle, as it stands, on the host cores: every stage on a bounded sample of its
    benchmark input; the step rate is projected from the per-stage rates."""
    import oracle
    oracle.build()
    ncores = oracle.num_threads()
    rates = {}

    def timed(fn):
        t = time.perf_counter()
        fn()
        return time.perf_counter() - t

    s = timed(lambda: oracle.fir1d(host["fir1d"], fir_taps, 3))
    rates["fir1d"] = 256 * 256 / s
    s = timed(lambda: oracle.sepblur(host["sepblur"], gau_taps, 7, gau_taps, 7))
    rates["sepblur"] = 4096 * 4096 / s
    s = timed(lambda: oracle.sat2d(host["sat2d"]))
    rates["sat2d"] = 4096 * 4096 / s
    band = 512                                   # half the image: ~20 G fp64 multiply-adds
    s = timed(lambda: oracle.conv3x3_rows(host["conv3x3"], host["conv3x3_w"], 256, 256 + band))
    rates["conv3x3"] = band * 1024 / s
    s = timed(lambda: oracle.pyr_level(host["pyr_level"]))
    rates["pyr_level"] = 8192 * 8192 / s
    step_s = sum(stage_work(st)[0] / rates[st] for st in STAGES)
    return {
        "value": total_px / step_s / 1e9, "unit": "Gpixels/s", "cores": ncores, "kind": "oracle",
        "sample": "every stage once on its whole benchmark input, except conv3x3: rows 256..767 of "
                  "1024x1024x64 (half the image); step rate from the per-stage rates",
        "stages_gpixels_per_s": {k: v / 1e9 for k, v in rates.items()},
    }


if __name__ == "__main__":
    main()
