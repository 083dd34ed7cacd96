#!/usr/bin/env python3
"""Benchmark of the five-stage hot path on one MI355X.

One *step* runs every stage once at its benchmark configuration (hb_fir1d 256x256/8 taps,
hb_sepblur 4096x4096/16-tap Gaussian, hb_sat2d 4096x4096, hb_conv3x3 1x1024x1024x64->64,
hb_pyr_level 8192x8192) on seeded synthetic inputs that are already resident in HBM.
Buffers rotate between steps so that no input or output is reused before more than the
256 MB memory-side cache has gone past.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--variant mfma|valu] [--no-cpu] [--no-extra]

prints ONE JSON line: aggregate Gpixels/s of the step (wall clock over the K timed steps), per-stage
Gpixels/s with each stage's roofline fraction (HIP events around every stage, in an instrumented
pass before the timed steps), the roofline object of the stage that takes the longest (HIP events
around that stage inside the timed steps), and the fp64 oracle timed on the host cores
(cpu_baseline).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense f16 MFMA

STAGES = ["fir1d", "sepblur", "sat2d", "conv3x3", "pyr_level"]

# HBM bytes per launch (read + written) of the MFMA kernels at the benchmark configurations, from
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this program scaled by its calibration copy (the
# summaries and commands are under profiles/).
MIB = 1 << 20
MEASURED_TRAFFIC_BYTES = {
    "pyr_level": int((143.47 + 256.27) * MIB),
    "conv3x3": int((138.18 + 128.00) * MIB),
    "sepblur": int((33.75 + 64.00) * MIB),
}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--variant", choices=["mfma", "valu"], default="mfma")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the supplementary runs (stacked FIR, long-tap FIR, 2-D convolution, 2x resampling, Lanczos resize, recursive filter, DCT denoise)")
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

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).to(dev)

    # ---- seeded inputs, several buffer sets per stage (rotated per step) -----------------
    t0 = time.time()
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
    nsets = {"fir1d": 4, "sepblur": 4, "sat2d": 4, "conv3x3": 2, "pyr_level": 2}
    ins, outs = {}, {}
    for st in STAGES:
        base = up(host[st])
        ins[st] = [base] + [base.clone() for _ in range(nsets[st] - 1)]
        odt = torch.float16 if st == "conv3x3" else torch.float32
        oshape = base.shape
        outs[st] = [torch.empty(oshape, dtype=odt, device=dev) for _ in range(nsets[st])]
    w_dev = up(host["conv3x3_w"])
    sat_ws = torch.empty(hb.hb_sat2d_workspace_size(4096, 4096), dtype=torch.uint8, device=dev)
    gen_s = time.time() - t0

    calls = {
        "fir1d": lambda i: getattr(hb, "hb_fir1d" + sfx)(ins["fir1d"][i], outs["fir1d"][i], fir_taps, 3),
        "sepblur": lambda i: getattr(hb, "hb_sepblur" + sfx)(ins["sepblur"][i], outs["sepblur"][i],
                                                             gau_taps, 7, gau_taps, 7),
        "sat2d": lambda i: getattr(hb, "hb_sat2d" + sfx)(ins["sat2d"][i], outs["sat2d"][i], sat_ws),
        "conv3x3": lambda i: getattr(hb, "hb_conv3x3" + sfx)(ins["conv3x3"][i], w_dev, outs["conv3x3"][i]),
        "pyr_level": lambda i: getattr(hb, "hb_pyr_level" + sfx)(ins["pyr_level"][i], outs["pyr_level"][i], None),
    }

    def step(k, events=None, only=None):
        for st in STAGES:
            i = k % nsets[st]
            rec = events is not None and (only is None or only == st)
            if rec:
                events[st][0].record()
            calls[st](i)
            if rec:
                events[st][1].record()

    def new_events(n):
        return [{st: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for st in STAGES}
                for _ in range(n)]

    # One plain copy of known size (32 MiB read, 64 MiB written), untimed: a counter run of this
    # program reads its own scale for FETCH_SIZE / WRITE_SIZE from this dispatch.
    hb.hb_copy_f16_f32(ins["sepblur"][0], outs["sepblur"][0])
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    # Instrumented pass (untimed): HIP events around every stage.  Event records cost about 3 us of
    # GPU idle time each, so the timed steps below carry them around the longest stage only.
    nprobe = max(1, min(args.steps, 10))
    evp = new_events(nprobe)
    for k in range(nprobe):
        step(args.warmup + k, evp[k])
    torch.cuda.synchronize()
    stage_ms = {st: float(np.mean([e[st][0].elapsed_time(e[st][1]) for e in evp])) for st in STAGES}
    dom = max(STAGES, key=lambda s: stage_ms[s])

    ev = new_events(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + nprobe + k, ev[k], only=dom)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    dom_ms = float(np.mean([e[dom][0].elapsed_time(e[dom][1]) for e in ev]))   # inside the timed steps
    total_px = sum(stage_work(st)[0] for st in STAGES)

    stages = {}
    for st in STAGES:
        px, nbytes, flops = stage_work(st)
        ms = stage_ms[st]
        gbs = nbytes / ms / 1e6
        tfl = flops / ms / 1e9
        bound = "mfma" if st == "conv3x3" else "hbm"
        stages[st] = {
            "gpixels_per_s": px / ms / 1e6, "ms": ms, "bound": bound,
            "achieved": tfl if bound == "mfma" else gbs,
            "peak": MFMA_F16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
            "frac": (tfl / MFMA_F16_PEAK_TFLOPS) if bound == "mfma" else (gbs / HBM_PEAK_GBS),
        }
    # roofline of the longest stage, from its HIP-event time inside the timed steps
    _, dbytes, dflops = stage_work(dom)
    dbound = stages[dom]["bound"]
    dach = (dflops / dom_ms / 1e9) if dbound == "mfma" else (dbytes / dom_ms / 1e6)
    roofline = {"bound": dbound, "achieved": dach, "peak": stages[dom]["peak"], "unit": stages[dom]["unit"],
                "frac": dach / stages[dom]["peak"], "kernel": "hb_" + dom + sfx, "ms": dom_ms,
                "traffic": MEASURED_TRAFFIC_BYTES.get(dom) if sfx == "" else None}

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
        "stages": stages,
        "roofline": roofline,
    }

    if not args.no_extra:
        # Supplementary (outside the timed step).  First the same step replayed from a HIP graph (four
        # steps per graph, so that the buffer sets rotate as in the timed loop): what the launch gaps
        # between the seven kernels of a step cost.  The library allocates nothing, synchronises
        # nothing and issues no memset, so its launches can be captured.
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
        graph_line = {
            "ms_per_step": gms, "gpixels_per_s": total_px / gms / 1e6, "steps_per_graph": 4,
            "eager_over_graph": ms_per_step / gms}
        del graph
        # The FIR stage on 1024 of its 256 x 256 images stacked into one 262144 x 256 image, where its
        # launch latency no longer hides its bandwidth.
        del ins["pyr_level"], outs["pyr_level"], ins["conv3x3"], outs["conv3x3"]
        torch.cuda.empty_cache()
        Hs = 256 * 1024
        sx = [up(host["fir1d"]).repeat(1024, 1) for _ in range(2)]
        so = [torch.empty((Hs, 256), dtype=torch.float32, device=dev) for _ in range(2)]
        fir = getattr(hb, "hb_fir1d" + sfx)
        for i in range(4):
            fir(sx[i % 2], so[i % 2], fir_taps, 3)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(10):
            fir(sx[i % 2], so[i % 2], fir_taps, 3)
        e1.record()
        torch.cuda.synchronize()
        sms = e0.elapsed_time(e1) / 10
        out["supplementary"] = {"fir1d_stacked_262144x256": {
            "ms": sms, "gpixels_per_s": Hs * 256 / sms / 1e6, "achieved": Hs * 256 * 6 / sms / 1e6,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": Hs * 256 * 6 / sms / 1e6 / HBM_PEAK_GBS}}
        out["supplementary"]["five_stage_step_graph_replay"] = graph_line
        # ... and the large-tap regime of the paper's 1-D study (Sec. V-A): 64, 128 and 256 taps on the
        # blur stage's 4096 x 4096 image, matrix-unit kernel and vector-ALU twin.
        del sx, so
        torch.cuda.empty_cache()
        lx, lo = ins["sepblur"], outs["sepblur"]
        npx = 4096 * 4096
        for ntaps in (64, 128, 256):
            long_taps = synth.random_taps_f16(2000 + ntaps, ntaps)

            def timed(fn, iters):
                for i in range(2):
                    fn(lx[i % 4], lo[i % 4], long_taps, (ntaps - 1) // 2)
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                for i in range(iters):
                    fn(lx[i % 4], lo[i % 4], long_taps, (ntaps - 1) // 2)
                a1.record()
                torch.cuda.synchronize()
                return a0.elapsed_time(a1) / iters
            m_ms, v_ms = timed(hb.hb_fir1d, 10), timed(hb.hb_fir1d_valu, 3)
            out["supplementary"]["fir1d_%dtaps_4096x4096" % ntaps] = {
                "mfma_ms": m_ms, "valu_ms": v_ms, "mfma_gpixels_per_s": npx / m_ms / 1e6,
                "valu_gpixels_per_s": npx / v_ms / 1e6, "mfma_over_valu": v_ms / m_ms}
        # ... and the paper's 2-D study (Sec. V-A): non-separable k x k kernels, k = 16 and 32, on
        # the same image.  tflops counts the definition's 2 k^2 flops per pixel, not the Toeplitz zeros.
        for k in (16, 32):
            k2d = synth.random_kernel2d_f16(2300 + k, k, k)

            def timed2(fn, iters):
                for i in range(2):
                    fn(lx[i % 4], lo[i % 4], k2d, k // 2, k // 2)
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                for i in range(iters):
                    fn(lx[i % 4], lo[i % 4], k2d, k // 2, k // 2)
                a1.record()
                torch.cuda.synchronize()
                return a0.elapsed_time(a1) / iters
            m_ms, v_ms = timed2(hb.hb_conv2d, 10), timed2(hb.hb_conv2d_valu, 3)
            out["supplementary"]["conv2d_%dx%d_4096x4096" % (k, k)] = {
                "mfma_ms": m_ms, "valu_ms": v_ms, "mfma_gpixels_per_s": npx / m_ms / 1e6,
                "valu_gpixels_per_s": npx / v_ms / 1e6, "mfma_over_valu": v_ms / m_ms,
                "mfma_tflops": 2.0 * k * k * npx / m_ms / 1e9}
        # ... and the paper's resampling study (Sec. V-B): 2x down (4096^2 -> 2048^2) and 2x up
        # (2048^2 -> 4096^2) with k x k kernels.  Pixels are counted on the larger image.
        half_out = [torch.empty((2048, 2048), dtype=torch.float32, device=dev) for _ in range(4)]
        half_in = [t[:2048, :2048] for t in lx]              # row pitch 4096
        for k in (16, 32):
            k2d = synth.random_kernel2d_f16(2400 + k, k, k)
            for name, src, dst, anc in (("down2", lx, half_out, k // 2), ("up2", half_in, lo, k // 4)):
                def timed3(fn, iters):
                    for i in range(2):
                        fn(src[i % 4], dst[i % 4], k2d, anc, anc)
                    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a0.record()
                    for i in range(iters):
                        fn(src[i % 4], dst[i % 4], k2d, anc, anc)
                    a1.record()
                    torch.cuda.synchronize()
                    return a0.elapsed_time(a1) / iters
                m_ms, v_ms = timed3(getattr(hb, "hb_" + name), 10), timed3(getattr(hb, "hb_" + name + "_valu"), 3)
                out["supplementary"]["%s_%dx%d_4096x4096" % (name, k, k)] = {
                    "mfma_ms": m_ms, "valu_ms": v_ms, "mfma_gpixels_per_s": npx / m_ms / 1e6,
                    "valu_gpixels_per_s": npx / v_ms / 1e6, "mfma_over_valu": v_ms / m_ms}
        # ... and the paper's non-integer resize (Sec. V-C, Table II): a 2048 x 2048 RGB image (three
        # planes) down to 143 / 245 / 450 / 921 squared with Lanczos-3 matrices built by the library.
        del half_out, half_in
        rgb = (torch.rand((3, 2048, 2048), device=dev)).half()
        for n in (143, 245, 450, 921):
            st_h, cf_h = hb.hb_lanczos3_matrix(2048, n)
            st_d = torch.from_numpy(st_h).to(dev)
            cf_d = torch.from_numpy(cf_h.view(np.int16)).to(dev).view(torch.float16)
            ro = torch.empty((3, n, n), dtype=torch.float32, device=dev)
            rws = torch.empty(hb.hb_resize_workspace_size(3, 2048, n), dtype=torch.uint8, device=dev)

            def timed4(fn, iters):
                for i in range(2):
                    fn(rgb, ro, rws, st_d, cf_d, st_d, cf_d)
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                for i in range(iters):
                    fn(rgb, ro, rws, st_d, cf_d, st_d, cf_d)
                a1.record()
                torch.cuda.synchronize()
                return a0.elapsed_time(a1) / iters
            m_ms, v_ms = timed4(hb.hb_resize, 10), timed4(hb.hb_resize_valu, 3)
            out["supplementary"]["resize_lanczos3_3x2048x2048_to_%d" % n] = {
                "mfma_ms": m_ms, "valu_ms": v_ms, "band": int(cf_h.shape[1]),
                "mfma_input_gpixels_per_s": 3 * 2048 * 2048 / m_ms / 1e6, "mfma_over_valu": v_ms / m_ms}
        # ... and the paper's recursive filter (Sec. V-D): 2^21 stereo samples, a resonant second-order filter.
        del rgb
        aud = (torch.rand((2, 1 << 21), device=dev) * 2 - 1).half()
        aout = torch.empty((2, 1 << 21), dtype=torch.float32, device=dev)
        aws = torch.empty(hb.hb_iir2_workspace_size(2, 1 << 21), dtype=torch.uint8, device=dev)

        def timed5(fn, iters):
            for i in range(2):
                fn(aud, aout, 1.6, -0.8, aws)
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for i in range(iters):
                fn(aud, aout, 1.6, -0.8, aws)
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / iters
        m_ms, v_ms = timed5(hb.hb_iir2, 10), timed5(hb.hb_iir2_valu, 3)
        out["supplementary"]["iir2_2x2097152"] = {
            "mfma_ms": m_ms, "valu_ms": v_ms, "mfma_gsamples_per_s": 2 * (1 << 21) / m_ms / 1e6,
            "mfma_over_valu": v_ms / m_ms}
        # ... and the paper's DCT-domain denoising (Sec. V-E): a one-megapixel three-channel image.
        del aud, aout
        dimg = torch.rand((3, 1024, 1024), device=dev).half()
        dout = torch.empty((3, 1024, 1024), dtype=torch.float32, device=dev)
        dws = torch.empty(hb.hb_dct_denoise_workspace_size(3, 1024, 1024), dtype=torch.uint8, device=dev)

        def timed6(fn, iters):
            for i in range(2):
                fn(dimg, dout, 0.05, dws)
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for i in range(iters):
                fn(dimg, dout, 0.05, dws)
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / iters
        m_ms, v_ms = timed6(hb.hb_dct_denoise, 10), timed6(hb.hb_dct_denoise_valu, 3)
        out["supplementary"]["dct_denoise_3x1024x1024"] = {
            "mfma_ms": m_ms, "valu_ms": v_ms, "mfma_gpixels_per_s": 3 * 1024 * 1024 / m_ms / 1e6,
            "mfma_over_valu": v_ms / m_ms}

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(host, fir_taps, gau_taps, total_px)
    print(json.dumps(out))


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
