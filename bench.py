#!/usr/bin/env python3
"""Throughput of the binary-convolution hot path on one MI355X.

One step = one pass of the whole hot path over the five synthetic layer shapes:
for each shape, sign+pack of the real-valued NCHW input (bcnn_pack), then the
binary convolution (int32 sums for shapes 1-2, fused threshold/sign/repack for
3-5, shape 5 being a chain of four layers with packed hand-off).  Weights are
packed once, outside the timed region, as at inference.  All inputs are
resident in HBM before the clock starts.

Prints ONE JSON line.  `value` is total binary ops per step / step time
(1 binary multiply-accumulate = 2 binary ops, padded taps counted).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# VALU xor+popcount peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-ops/s;
# one v_xor_b32 + one v_bcnt_u32_b32 (2 lane-ops) do 32 multiply-accumulates
# = 64 binary ops  ->  39.3e12 / 2 * 64 = 1258 T binary ops/s.
VALU_PEAK_TBOPS = 256 * 64 * 2.4e9 * 32 / 1e12
HBM_PEAK_GBS = 8000.0
MFMA_FP4_PEAK_TFLOPS = 10100.0  # dense fp4 matrix rate of MI355X


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--variant", default="auto", choices=["auto", "valu", "mfma_i8", "mfma_fp4", "mfma_fp4_t4", "mfma_fp4_t7", "mfma_fp4_p6", "mfma_fp4_p7", "mfma_fp4_p5", "mfma_fp4_p68"])
    ap.add_argument("--shapes", default="1,2,3,4,5",
                    help="comma list of layer shapes in the step (default all five; a subset is for profiling)")
    ap.add_argument("--eager", action="store_true", help="time eagerly enqueued steps instead of graph replays")
    ap.add_argument("--branch-per-shape", action="store_true",
                    help="capture every layer shape on a stream of its own (a graph branch per shape) "
                         "instead of one chain of launches; measured 2.5 %% faster per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-aux", action="store_true", help="skip the stand-alone kernel measurements")
    ap.add_argument("--probes", action="store_true",
                    help="launch the copy, xor+popcount and matrix-core probes once before the steps (for "
                         "profiler runs: they calibrate the counters of paper_2010_00704_amd.rocprof_summary)")
    ap.add_argument("--no-sustained", action="store_true",
                    help="skip the two-second replays with power and clock sampling (e.g. under a profiler)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (images shard over the batch "
                 "dimension with no exchange; no multi-GPU figure is produced). Use --gpus 1.")
    import numpy as np
    import torch

    from paper_2010_00704_amd import binding as B
    from paper_2010_00704_amd import workloads as W

    B.lib()  # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    variant = {"auto": B.BCNN_VARIANT_AUTO, "valu": B.BCNN_VARIANT_VALU,
               "mfma_i8": B.BCNN_VARIANT_MFMA_I8, "mfma_fp4": B.BCNN_VARIANT_MFMA_FP4,
               "mfma_fp4_t4": B.BCNN_VARIANT_MFMA_FP4_T4, "mfma_fp4_t7": B.BCNN_VARIANT_MFMA_FP4_T7,
               "mfma_fp4_p6": B.BCNN_VARIANT_MFMA_FP4_P6, "mfma_fp4_p7": B.BCNN_VARIANT_MFMA_FP4_P7,
               "mfma_fp4_p5": B.BCNN_VARIANT_MFMA_FP4_P5, "mfma_fp4_p68": B.BCNN_VARIANT_MFMA_FP4_P68}[args.variant]

    # ---------------------------------------------------------------- inputs
    work = []
    shapes = sorted(set(int(v) for v in args.shapes.split(",")))
    for index in shapes:
        cfg, x, ws, ts = W.make_inputs(index)
        x_real = torch.from_numpy(W.real_with_sign(W.seeds(index)[0], x)).to(dev)
        del x
        wps = [B.pack_nchw(torch.from_numpy(w).to(dev)) for w in ws]
        thr = [torch.from_numpy(t).to(dev) if t is not None else None for t in ts]
        ho, wo = W.out_hw(cfg)
        cw = (cfg.c_in + 31) // 32
        cwo = (cfg.c_out + 31) // 32
        xp = torch.empty((cfg.n, cfg.h * cfg.w, cw), dtype=torch.int32, device=dev)
        descs, outs = [], []
        c, h, w_ = cfg.c_in, cfg.h, cfg.w
        for _ in range(cfg.layers):
            d = B.conv_desc(cfg.n, c, h, w_, cfg.c_out, cfg.k, cfg.stride, cfg.pad)
            descs.append(d)
            h, w_ = B.out_shape(d)
            c = cfg.c_out
            if cfg.fused:
                outs.append(torch.empty((cfg.n, h * w_, cwo), dtype=torch.int32, device=dev))
            else:
                outs.append(torch.empty((cfg.n, h, w_, cfg.c_out), dtype=torch.int32, device=dev))
        work.append(dict(cfg=cfg, x_real=x_real, xp=xp, wps=wps, thr=thr, descs=descs, outs=outs,
                         ev=None, pack_ms=0.0, conv_ms=0.0))
    torch.cuda.synchronize()

    def run_config(wk, timed):
        cfg = wk["cfg"]
        if timed:
            wk["ev"][0].record()
        B.check(B.bcnn_pack(wk["x_real"], B.BCNN_F32, cfg.n, cfg.c_in, cfg.h * cfg.w, wk["xp"]), "pack")
        if timed:
            wk["ev"][1].record()
        cur = wk["xp"]
        for d, wp, t, out in zip(wk["descs"], wk["wps"], wk["thr"], wk["outs"]):
            B.check(B.bcnn_conv2d_binary_variant(d, cur, wp, t, out, variant), "conv")
            cur = out
        if timed:
            wk["ev"][2].record()

    def step(timed):
        for wk in work:
            run_config(wk, timed)

    if args.probes:
        words = (64 << 20) // 4
        src = torch.randint(-2**31, 2**31 - 1, (words,), dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            B.check(B.bcnn_diag_copy_u32(src, dst, words), "copy probe")
        sink = torch.empty(4096 * 256, dtype=torch.int32, device=dev)
        B.check(B.bcnn_diag_valu_peak(sink, 4096, 400), "xor+popcount probe")
        fsink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
        for mblocks in (256, 224):
            B.check(B.bcnn_diag_mfma_fp4_peak(fsink, mblocks, 400), "matrix-core probe")
        torch.cuda.synchronize()
        del src, dst, sink, fsink

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()

    # ------------------------------------------------------------ timed region
    # The 13 launches of a step are short (3-55 us each), so the step is
    # captured once into a HIP graph and the timed region is K replays of it
    # between two synchronisations, timed by the wall clock.  (--eager times K
    # eagerly enqueued steps instead.)  The graph holds kernel nodes only.
    # Its results are checked against the eager results before timing.
    launch = "eager"
    graph = None
    if not args.eager:
        try:
            ref = [wk["outs"][-1].clone() for wk in work]
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step(False)                      # warm the capture stream
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            if not args.branch_per_shape or len(work) == 1:
                with torch.cuda.graph(graph, stream=side):
                    step(False)
            else:
                # The layer shapes of a step do not depend on one another, so each is captured on a
                # stream of its own (default priority) forked from and joined to the capture stream:
                # the graph then has one branch per shape and the GPU may overlap them (the HBM-bound
                # packs under the matrix-core-bound chain of shape 5).  Longest branch first.
                branch_streams = [torch.cuda.Stream() for _ in work]
                order = sorted(range(len(work)), key=lambda i: -W.binary_ops(work[i]["cfg"]))
                with torch.cuda.graph(graph, stream=side):
                    for i in order:
                        branch_streams[i].wait_stream(side)
                        with torch.cuda.stream(branch_streams[i]):
                            run_config(work[i], False)
                    for i in order:
                        side.wait_stream(branch_streams[i])
                launch = "hip_graph_branch_per_shape"
            for _ in range(3):                   # replays with eager work and syncs in between
                for wk in work:
                    wk["outs"][-1].zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                for wk, r in zip(work, ref):
                    assert torch.equal(wk["outs"][-1], r), "graph replay differs from the eager result"
            launch = "hip_graph" if launch == "eager" else launch
        except Exception as e:  # capture unavailable: time the eager path and say so
            sys.stderr.write("bench.py: graph capture failed (%s); timing eager launches\n" % (e,))
            graph = None
            launch = "eager"
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        for k in range(args.steps):
            graph.replay()
    else:
        for k in range(args.steps):
            step(False)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # Per-part breakdown and the dominant kernel's launch duration: the same K
    # steps again, enqueued eagerly with HIP events (on torch's current stream,
    # which is the stream every kernel is launched on) around the pack and the
    # convolution part of every shape; read after the region ends.
    evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in work]
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        for wk, ev in zip(work, evs[k]):
            wk["ev"] = ev
        step(True)
    torch.cuda.synchronize()
    ms_per_step_evented = (time.perf_counter() - t0) * 1e3 / args.steps
    for k in range(args.steps):
        for wk, ev in zip(work, evs[k]):
            wk["pack_ms"] += ev[0].elapsed_time(ev[1])
            wk["conv_ms"] += ev[1].elapsed_time(ev[2])

    total_bops = sum(W.binary_ops(wk["cfg"]) for wk in work)
    value = total_bops / (ms_per_step * 1e-3) / 1e12

    per_config = []
    for wk in work:
        cfg = wk["cfg"]
        conv_ms = wk["conv_ms"] / args.steps
        pack_ms = wk["pack_ms"] / args.steps
        bops = W.binary_ops(cfg)
        src_bytes = wk["x_real"].numel() * 4 + wk["xp"].numel() * 4
        tb = bops / (conv_ms * 1e-3) / 1e12
        per_config.append({
            "name": cfg.name, "conv_ms": round(conv_ms, 4), "launches": cfg.layers,
            "tbops": round(tb, 1), "frac_valu_peak": round(tb / VALU_PEAK_TBOPS, 4),
            "pack_ms": round(pack_ms, 4),
            "pack_gbs": round(src_bytes / (pack_ms * 1e-3) / 1e9, 1),
            # against the published 8 TB/s; event-timed inside the step, launch gap included
            "pack_frac_hbm": round(src_bytes / (pack_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        })

    # ---------------------------------------------------------------- roofline
    # Dominant kernel: the 3x3 convolution of shape 5 (four launches per step,
    # > 60 % of the step).  Algorithmic work per launch = 2*M*N*K binary ops.
    dom = work[-1] if 5 in shapes else max(work, key=lambda wk: wk["conv_ms"])
    dom_ms = dom["conv_ms"] / args.steps / dom["cfg"].layers
    dom_bops = W.binary_ops(dom["cfg"]) / dom["cfg"].layers
    achieved = dom_bops / (dom_ms * 1e-3) / 1e12
    on_mfma = args.variant.startswith("mfma_fp4") or args.variant == "auto"
    if on_mfma:
        # fp4 matrix-core path: one binary multiply-accumulate is one fp4 FMA = 2 FLOP.  The kernel
        # the library launches for the dominant shape under each variant (shape 5: AUTO takes the
        # position-major kernel with two-wave workgroups)
        pos = {"mfma_fp4_p5": "<5, 8, 2>", "mfma_fp4_p68": "<6, 8, 2>", "mfma_fp4_p6": "<6, 7, 4>", "mfma_fp4_p7": "<7, 7, 4>"}
        if args.variant in pos:
            kernel = "conv_mfma_fp4_pos_kernel" + pos[args.variant]
        elif args.variant in ("auto", "mfma_fp4") and dom["cfg"].name.startswith("cfg5"):
            kernel = "conv_mfma_fp4_pos_kernel<5, 8, 2>"
        else:
            kernel = "conv_mfma_fp4_kernel"
        # share of the filter taps that lie inside the image: the position-major kernel does not walk
        # the others (it adds their closed form), the algorithmic count above includes them
        cfg = dom["cfg"]
        ho, wo = W.out_hw(cfg)
        inside = sum(sum(0 <= o * cfg.stride - cfg.pad + u < cfg.h for u in range(cfg.k)) for o in range(ho)) * \
            sum(sum(0 <= o * cfg.stride - cfg.pad + v < cfg.w for v in range(cfg.k)) for o in range(wo))
        roofline = {
            "kernel": kernel + " on " + dom["cfg"].name + " (per launch)",
            "taps_inside_image": round(inside / float(ho * wo * cfg.k * cfg.k), 4),
            "bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_FP4_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": round(achieved / MFMA_FP4_PEAK_TFLOPS, 4),
            "avg_launch_ms": round(dom_ms, 4),
        }
        # HBM bytes per launch: not measurable from inside this script; taken from the table that
        # `python -m paper_2010_00704_amd.rocprof_summary pmc ...` wrote from the FETCH_SIZE / WRITE_SIZE
        # counter runs of this same command (null if that summary is not there)
        roofline.update(traffic_from_profile(dom["cfg"]))
    elif args.variant == "mfma_i8":
        roofline = {
            "kernel": "conv_mfma_i8_kernel on " + dom["cfg"].name + " (per launch)",
            "bound": "mfma", "achieved": round(achieved, 1), "peak": 5000.0,   # dense int8 matrix rate, TOP/s
            "unit": "TOP/s", "frac": round(achieved / 5000.0, 4),
            "avg_launch_ms": round(dom_ms, 4), "traffic": None,
        }
    else:
        roofline = {
            "kernel": "conv_valu_kernel on " + dom["cfg"].name + " (per launch)",
            "bound": "alu", "achieved": round(achieved, 1), "peak": round(VALU_PEAK_TBOPS, 1),
            "unit": "TBOP/s", "frac": round(achieved / VALU_PEAK_TBOPS, 4),
            "avg_launch_ms": round(dom_ms, 4), "traffic": None,
        }

    aux = {}
    if not args.no_aux and shapes == [1, 2, 3, 4, 5]:
        aux = aux_measurements(torch, B, dev, work, sustained=not args.no_sustained)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(np, W, shapes)

    line = {
        "metric": "binary conv TBOPS (and % of VALU popcount peak) per layer shape, 1 MI355X",
        "value": round(value, 2), "unit": "TBOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        # the arithmetic the convolution runs in: +-1 as 4-bit floats on the matrix cores (fp32 accumulate,
        # every sum an exact integer), bytes on the int8 arm, packed 32-bit words on the vector ALUs
        "dtype": "fp4" if on_mfma else ("int8" if args.variant == "mfma_i8" else "u32"),
        "data": "synthetic",
        "config": {"workload": ("all five layer shapes per step: pack + binary conv "
                                "(cfg1-2 int32 sums, cfg3-4 fused sign-pack, cfg5 4-layer chain)")
                   if shapes == [1, 2, 3, 4, 5] else "SUBSET of the layer shapes (profiling run): %s" % shapes,
                   "variant": args.variant},
        "frac_valu_peak": round(value / VALU_PEAK_TBOPS, 4),
        "launch": launch, "ms_per_step_eager_with_events": round(ms_per_step_evented, 4),
        "per_config": per_config,
        "roofline": roofline,
        "aux": aux,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def traffic_from_profile(cfg):
    """{"traffic": HBM bytes per launch of the convolution of `cfg`, "traffic_source": file and run,
    "traffic_over_algorithmic": ratio to the compulsory bytes (packed input + packed weights + thresholds
    + packed output)} from profiles/bench_hbm_traffic_pmc.md, or traffic = None."""
    path = os.path.join(ROOT, "profiles", "bench_hbm_traffic_pmc.md")
    out = {"traffic": None}
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == cfg.name:
                    cw, cwo = (cfg.c_in + 31) // 32, (cfg.c_out + 31) // 32
                    ho = (cfg.h + 2 * cfg.pad - cfg.k) // cfg.stride + 1
                    wo = (cfg.w + 2 * cfg.pad - cfg.k) // cfg.stride + 1
                    # a layer of the chain reads the previous layer's output: same size as the input here
                    algorithmic = 4 * (cfg.n * cfg.h * cfg.w * cw + cfg.c_out * cfg.k * cfg.k * cw + cfg.c_out +
                                       cfg.n * ho * wo * (cwo if cfg.fused else cfg.c_out))
                    out = {"traffic": float(parts[2]), "traffic_source": "profiles/bench_hbm_traffic_pmc.md",
                           "traffic_over_algorithmic": round(float(parts[2]) / algorithmic, 2)}
    except OSError:
        pass
    return out


def _gpu_sensors():
    """(power sensor path, shader clock table path) of the first amdgpu card, or None."""
    import glob
    power = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                   glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
    sclk = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
    if not power or not sclk:
        return None
    return power[0], sclk[0]


def sustained_load(torch, B, dev, work, seconds=2.0):
    """Replays 20-launch HIP graphs of one kernel for `seconds` each and samples the board's
    power and shader clock meanwhile.  Returns a list of {"what", "us_per_launch", "watts",
    "sclk_mhz"}; the sensor fields are None where the sensors cannot be read."""
    import threading
    import time

    wk = next((w for w in work if w["cfg"].name.startswith("cfg5")), work[-1])
    cfg, d = wk["cfg"], wk["descs"][0]
    x_rand = torch.randint(-2**31, 2**31 - 1, wk["xp"].shape, dtype=torch.int32, device=dev)
    w_rand, thr, y = wk["wps"][0], wk["thr"][0], wk["outs"][0]
    x_zero, w_zero = torch.zeros_like(x_rand), torch.zeros_like(w_rand)
    fsink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
    cases = [
        ("%s conv, AUTO, random bits" % cfg.name,
         lambda: B.check(B.bcnn_conv2d_binary_variant(d, x_rand, w_rand, thr, y, B.BCNN_VARIANT_AUTO), "conv")),
        ("%s conv, AUTO, all-zero words" % cfg.name,
         lambda: B.check(B.bcnn_conv2d_binary_variant(d, x_zero, w_zero, thr, y, B.BCNN_VARIANT_AUTO), "conv")),
        ("fp4 matrix-core probe, 256 blocks x 400 rounds",
         lambda: B.check(B.bcnn_diag_mfma_fp4_peak(fsink, 256, 400), "probe")),
    ]
    sens = _gpu_sensors()
    res = []
    for what, launch in cases:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            launch()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(20):
                launch()
        samples, stop = [], threading.Event()

        def sampler():
            while not stop.is_set():
                try:
                    watts = float(open(sens[0]).read()) / 1e6
                    cur = [l for l in open(sens[1]).read().splitlines() if l.rstrip().endswith("*")][0]
                    samples.append((watts, float(cur.split(":")[1].lower().replace("mhz", "").replace("*", ""))))
                except (OSError, ValueError, IndexError):
                    pass
                time.sleep(0.05)

        th = threading.Thread(target=sampler) if sens else None
        if th:
            th.start()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n, t0 = 0, time.time()
        a.record()
        while time.time() - t0 < seconds:
            for _ in range(20):
                g.replay()
            n += 400
            torch.cuda.synchronize()
        b.record()
        b.synchronize()
        stop.set()
        if th:
            th.join()
        tail = samples[len(samples) // 3:]          # after the sensors' averaging has settled
        res.append({"what": what, "us_per_launch": round(a.elapsed_time(b) * 1e3 / n, 2),
                    "watts": round(sum(p for p, _ in tail) / len(tail), 0) if tail else None,
                    "sclk_mhz": round(sum(c for _, c in tail) / len(tail), 0) if tail else None})
    return res



def aux_measurements(torch, B, dev, work, sustained=True):
    """Stand-alone figures outside the timed steps: the measured xor+popcount
    issue rate, and HBM rates of the pack and epilogue kernels on rotating
    buffers larger than the last-level cache."""
    out = {}
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731

    def graph_ms(launch, reps):
        """Average time of one launch(r), r = 0..reps-1, replayed from a HIP graph
        (kernel nodes only), so that the host's launch cost is not in the figure."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            launch(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for r in range(reps):
                launch(r)
        g.replay()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        g.replay()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    def eager_ms(launch, reps):
        """Average time of one launch(r), r = 0..reps-1, enqueued back to back between two
        events (kernels of 15 us and more: the host keeps ahead of the GPU, and a graph
        launch's own start-up cost would be 5 % of such a short replay)."""
        launch(0)
        a, b = ev(), ev()
        a.record()
        for r in range(reps):
            launch(r)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    # VALU issue-rate probe: blocks*256 lanes * iters * 64 pairs * 64 binary ops
    blocks, iters = 256 * 16, 4000
    sink = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
    B.check(B.bcnn_diag_valu_peak(sink, blocks, 10), "peak")
    a, b = ev(), ev()
    a.record()
    B.check(B.bcnn_diag_valu_peak(sink, blocks, iters), "peak")
    b.record()
    b.synchronize()
    ms = a.elapsed_time(b)
    tbops = blocks * 256 * iters * 64 * 64 / (ms * 1e-3) / 1e12
    out["valu_probe_tbops"] = round(tbops, 1)
    out["valu_probe_implied_ghz"] = round(tbops / (256 * 64 * 32) * 1e3, 3)

    # matrix-core issue-rate probe: blocks*4 waves * iters * 8 MFMAs * 2*32*32*64 FLOP, random +-1 fp4
    # operands in registers: what the matrix cores sustain on this kind of data (clock under load included)
    for tag, mblocks in (("mfma_fp4_probe_tflops", 256), ("mfma_fp4_probe_224cu_tflops", 224)):
        fsink = torch.empty(mblocks * 256, dtype=torch.float32, device=dev)
        B.check(B.bcnn_diag_mfma_fp4_peak(fsink, mblocks, 50), "mfma peak")
        a, b = ev(), ev()
        a.record()
        B.check(B.bcnn_diag_mfma_fp4_peak(fsink, mblocks, 4000), "mfma peak")
        b.record()
        b.synchronize()
        out[tag] = round(mblocks * 4 * 4000 * 8 * 2.0 * 32 * 32 * 64 / (a.elapsed_time(b) * 1e-3) / 1e12, 1)

    # Clock and board power while the dominant kernel is replayed back to back for about two
    # seconds (the amdgpu driver's sysfs sensors, read by a thread every 50 ms): once on random
    # operands, once on all-zero words (constant operands), and the matrix-core probe.  The
    # constant-operand launch shows the kernel's time at the full clock; the difference to the
    # random-operand launch is what the board's power limit costs.
    # (measured last, below: it holds the chip at its power limit for seconds, which would bias
    # whatever is timed right after it)

    # pack kernel on the largest input (shape 4, 205 MB fp32), 4 rotating copies
    wk = work[3]
    cfg = wk["cfg"]
    srcs = [wk["x_real"]] + [wk["x_real"].clone() for _ in range(3)]
    reps = 12
    for s in srcs:
        B.check(B.bcnn_pack(s, B.BCNN_F32, cfg.n, cfg.c_in, cfg.h * cfg.w, wk["xp"]), "pack")
    ms = eager_ms(lambda r: B.check(B.bcnn_pack(srcs[r % 4], B.BCNN_F32, cfg.n, cfg.c_in, cfg.h * cfg.w, wk["xp"]),
                                    "pack"), reps)
    nbytes = srcs[0].numel() * 4 + wk["xp"].numel() * 4
    out["pack_f32_gbs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    out["pack_f32_frac_hbm"] = round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    del srcs

    # stand-alone epilogue on shape 4's int32 sums (102.8 MB), 4 rotating copies
    rows, c_out = cfg.n * 28 * 28, cfg.c_out
    ys = [torch.randint(-300, 300, (rows, c_out), dtype=torch.int32, device=dev) for _ in range(4)]
    yp = torch.empty((rows, c_out // 32), dtype=torch.int32, device=dev)
    thr = wk["thr"][0]
    for y in ys:
        B.check(B.bcnn_threshold_sign_pack(y, thr, rows, c_out, yp), "thr")
    ms = eager_ms(lambda r: B.check(B.bcnn_threshold_sign_pack(ys[r % 4], thr, rows, c_out, yp), "thr"), reps)
    nbytes = ys[0].numel() * 4 + yp.numel() * 4
    out["epilogue_gbs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    out["epilogue_frac_hbm"] = round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)

    # plain copy of the same size for reference (what a streaming kernel reaches here)
    dst = torch.empty_like(ys[0])
    B.check(B.bcnn_diag_copy_u32(ys[0], dst, ys[0].numel()), "copy")
    ms = eager_ms(lambda r: B.check(B.bcnn_diag_copy_u32(ys[r % 4], dst, ys[0].numel()), "copy"), reps)
    out["copy_gbs_read_plus_write"] = round(2 * ys[0].numel() * 4 / (ms * 1e-3) / 1e9, 1)
    # one-sided ceilings on the same 102.8 MB: a pure store (what bounds the int32 convolution of shape 2)
    # and a pure read (what bounds pack and the stand-alone epilogue), 16-byte non-temporal accesses
    dsts = [dst] + [torch.empty_like(dst) for _ in range(3)]
    words = dst.numel()
    for d4 in dsts:
        B.check(B.bcnn_diag_store_u32(d4, words), "store")
    ms = eager_ms(lambda r: B.check(B.bcnn_diag_store_u32(dsts[r % 4], words), "store"), reps)
    out["store_only_gbs"] = round(words * 4 / (ms * 1e-3) / 1e9, 1)
    rsink = torch.empty(((words // 4 + 2047) // 2048) * 256, dtype=torch.int32, device=dev)
    B.check(B.bcnn_diag_read_u32(ys[0], words, rsink), "read")
    ms = eager_ms(lambda r: B.check(B.bcnn_diag_read_u32(ys[r % 4], words, rsink), "read"), reps)
    out["read_only_gbs"] = round(words * 4 / (ms * 1e-3) / 1e9, 1)
    del ys, dst, dsts, rsink

    # pack with a per-channel bias before the sign, same input as the pack figure above
    from paper_2010_00704_amd import workloads as W
    bias_c = torch.from_numpy(W.uniform_f32(4100, (cfg.c_in,), -0.75, 0.75)).to(dev)
    srcs = [wk["x_real"]] + [wk["x_real"].clone() for _ in range(3)]
    B.check(B.bcnn_pack_bias(srcs[0], B.BCNN_F32, cfg.n, cfg.c_in, cfg.h * cfg.w, bias_c, wk["xp"]), "pack_bias")
    ms = eager_ms(lambda r: B.check(B.bcnn_pack_bias(srcs[r % 4], B.BCNN_F32, cfg.n, cfg.c_in, cfg.h * cfg.w, bias_c,
                                                     wk["xp"]), "pack_bias"), reps)
    nbytes = srcs[0].numel() * 4 + wk["xp"].numel() * 4
    out["pack_bias_f32_gbs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    del srcs

    # branch convolution (F*F shifted 1x1 branches, per-branch real scales, per-branch pad words,
    # fused sign-pack) on the 3x3 shapes.  These shapes run on the matrix cores (C_in a multiple of 256);
    # the fraction quoted is against the xor+popcount peak of the vector ALUs, the arm every shape can use
    out["branches"] = []
    for wk in work[2:5]:
        cfg = wk["cfg"]
        d = wk["descs"][0]
        taps = cfg.k * cfg.k
        cw = (cfg.c_in + 31) // 32
        scale = torch.from_numpy(W.uniform_f32(4200, (taps, cfg.c_out), -1.5, 1.5)).to(dev)
        hb = torch.from_numpy(W.uniform_f32(4300, (cfg.c_out,), -40.0, 40.0)).to(dev)
        padw = torch.randint(-2**31, 2**31 - 1, (taps, cw), dtype=torch.int32, device=dev)
        zp = torch.empty_like(wk["outs"][0])
        for _ in range(2):
            B.check(B.bcnn_conv2d_binary_branches_sign_pack(d, taps, wk["xp"], 0, wk["wps"][0], padw, B.BCNN_PAD_WORDS,
                                                            scale, hb, zp), "branches")
        ms = graph_ms(lambda r: B.check(B.bcnn_conv2d_binary_branches_sign_pack(
            d, taps, wk["xp"], 0, wk["wps"][0], padw, B.BCNN_PAD_WORDS, scale, hb, zp), "branches"), reps)
        tb = W.binary_ops(cfg) / cfg.layers / (ms * 1e-3) / 1e12
        out["branches"].append({"name": cfg.name, "ms": round(ms, 4), "tbops": round(tb, 1),
                                "frac_valu_peak": round(tb / VALU_PEAK_TBOPS, 4)})

    # convolution module (1x1 binary convolution + batch norm + identity + PReLU -> real stream in place,
    # + next bias, sign, pack) on the 1x1 shape; HBM bound: real stream read + written per element
    wk = work[1]
    cfg, d = wk["cfg"], wk["descs"][0]
    m_rows = cfg.n * cfg.h * cfg.w
    par = [torch.from_numpy(W.uniform_f32(4400 + k, (cfg.c_out,), lo, hi)).to(dev)
           for k, (lo, hi) in enumerate([(-1.5, 1.5), (-30.0, 30.0), (0.05, 0.5), (-10.0, 10.0)])]
    xn = torch.empty((cfg.n, cfg.h * cfg.w, cfg.c_out // 32), dtype=torch.int32, device=dev)
    out["module_1x1"] = []
    for name, tdt, code, esz in (("f32", torch.float32, B.BCNN_F32, 4), ("f16", torch.float16, B.BCNN_F16, 2)):
        streams = [(torch.rand((m_rows, cfg.c_out), device=dev) * 80 - 40).to(tdt) for _ in range(4)]
        for st in streams:
            B.check(B.bcnn_conv2d_binary_module(d, wk["xp"], wk["wps"][0], par[0], par[1], st, par[2], par[3],
                                                code, st, xn), "module")
        ms = graph_ms(lambda r: B.check(B.bcnn_conv2d_binary_module(
            d, wk["xp"], wk["wps"][0], par[0], par[1], streams[r % 4], par[2], par[3], code, streams[r % 4], xn),
            "module"), reps)
        nbytes = 2 * m_rows * cfg.c_out * esz + wk["xp"].numel() * 4 + xn.numel() * 4
        out["module_1x1"].append({"real": name, "ms": round(ms, 4), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                  "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                  "tbops": round(W.binary_ops(cfg) / (ms * 1e-3) / 1e12, 1)})
        del streams

    # the 1x1 modules of the paper's network (its Table 1), batch 32, fp16 real stream updated in place
    out["table1_modules_n32_f16"] = []
    for name, ch, side in W.TABLE1_MODULES:
        nb = 32
        d = B.conv_desc(nb, ch, side, side, ch, 1, 1, 0)
        rows = nb * side * side
        cw = (ch + 31) // 32
        xp = torch.randint(-2**31, 2**31 - 1, (rows, cw), dtype=torch.int32, device=dev)
        wp = torch.randint(-2**31, 2**31 - 1, (ch, cw), dtype=torch.int32, device=dev)
        par = [torch.from_numpy(W.uniform_f32(4500 + k, (ch,), lo, hi)).to(dev)
               for k, (lo, hi) in enumerate([(-1.5, 1.5), (-30.0, 30.0), (0.05, 0.5), (-10.0, 10.0)])]
        nbuf = 4 if rows * ch * 2 > (64 << 20) else 1
        streams = [(torch.rand((rows, ch), device=dev) * 80 - 40).to(torch.float16) for _ in range(nbuf)]
        xn = torch.empty((rows, cw), dtype=torch.int32, device=dev)
        for st in streams:
            B.check(B.bcnn_conv2d_binary_module(d, xp, wp, par[0], par[1], st, par[2], par[3], B.BCNN_F16, st, xn),
                    "module")
        ms = graph_ms(lambda r: B.check(B.bcnn_conv2d_binary_module(
            d, xp, wp, par[0], par[1], streams[r % nbuf], par[2], par[3], B.BCNN_F16, streams[r % nbuf], xn),
            "module"), reps)
        nbytes = 2 * rows * ch * 2 + 2 * rows * cw * 4
        out["table1_modules_n32_f16"].append({
            "level": name, "c": ch, "side": side, "ms": round(ms, 4),
            "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "tbops": round(2.0 * rows * ch * ch / (ms * 1e-3) / 1e12, 1)})
        del streams

    # down-sampling identity path: 2x2/2 average pooling of the real stream + bias + sign + pack in one pass
    # (4 elements read, 1 written per output element); a 205 MB fp32 map on rotating buffers and the level-1
    # map of Table 1 at batch 32 in fp16
    out["avgpool_bias_sign_pack"] = []
    for name, tdt, code, esz, shape in (("f32", torch.float32, B.BCNN_F32, 4, (64, 56, 56, 256)),
                                        ("f16", torch.float16, B.BCNN_F16, 2, (32, 112, 112, 64))):
        nb, hh, ww, ch = shape
        nbuf = 4
        maps = [(torch.rand(shape, device=dev) * 80 - 40).to(tdt) for _ in range(nbuf)]
        pooled = torch.empty((nb, hh // 2, ww // 2, ch), dtype=tdt, device=dev)
        bits = torch.empty((nb, (hh // 2) * (ww // 2), (ch + 31) // 32), dtype=torch.int32, device=dev)
        pbias = torch.from_numpy(W.uniform_f32(4600, (ch,), -10.0, 10.0)).to(dev)
        for mp in maps:
            B.check(B.bcnn_avgpool_bias_sign_pack(mp, code, nb, hh, ww, ch, 2, pbias, pooled, bits), "avgpool")
        ms = graph_ms(lambda r: B.check(B.bcnn_avgpool_bias_sign_pack(
            maps[r % nbuf], code, nb, hh, ww, ch, 2, pbias, pooled, bits), "avgpool"), reps)
        nbytes = maps[0].numel() * esz + pooled.numel() * esz + bits.numel() * 4
        out["avgpool_bias_sign_pack"].append({
            "real": name, "shape": list(shape), "ms": round(ms, 4), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
        del maps
    if sustained:
        out["sustained"] = sustained_load(torch, B, dev, work)
    return out


def cpu_baseline(np, W, shapes):
    """The CPU oracle, as it stands, on one whole step of the same workload:
    for every layer shape the full batch goes through sign -> (conv ->
    threshold -> channel packing) per layer, on the host's threads.  Input
    generation is outside the clock.  About 25 s of CPU work on 16 threads."""
    import oracle
    c1, x1, w1, _ = W.make_inputs(1)
    oracle.conv2d_pm1(x1, w1[0], c1.stride, c1.pad)  # load the library, start the thread pool
    seconds, bops = 0.0, 0
    for index in shapes:
        cfg, x, ws, ts = W.make_inputs(index)
        x_real = W.real_with_sign(W.seeds(index)[0], x)
        del x
        t0 = time.perf_counter()
        cur = oracle.sign_f32(x_real)
        for w, t in zip(ws, ts):
            y = oracle.conv2d_pm1(cur, w, cfg.stride, cfg.pad)
            if t is None:
                break
            s = oracle.threshold_sign(y, t)
            n, ho, wo, o = s.shape
            cur = np.ascontiguousarray(s.transpose(0, 3, 1, 2))
            oracle.pack_channels(cur.reshape(n, o, ho * wo))
        seconds += time.perf_counter() - t0
        bops += W.binary_ops(cfg)
        del x_real, cur, y
    return {"value": round(bops / seconds / 1e12, 6), "unit": "TBOPS", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(seconds, 2),
            "sample": "one whole step: layer shapes %s at full batch, every layer (sign, conv, threshold, "
                      "channel packing) through the oracle" % (shapes,)}


if __name__ == "__main__":
    main()
