#!/usr/bin/env python3
"""Benchmark of the incremental-inference hot path on one MI355X.

A step = one evconv_step_frame call: increment builder, every layer's increment kernel, output
integration and list compaction, on one frame of a synthetic event-voxel stream that is already
resident in HBM.  Workload: the UNet depth network on 5x256x352 at 2 % changed pixels per step,
fp32 weights (headline); the fp32-through-bf16-parts and bf16-weight variants are reported beside it.

Prints ONE JSON line.  `value` is 1000 / the median of the per-step durations of the K timed steps,
each measured with HIP events on the library's stream (`step_time_ms` gives median, min, max and
the wall-clock mean of the same K steps).  Extra keys:
  roofline            dominant kernel family (matrix-core conv): algorithmic FLOPs of its timed launches
                      over their HIP-event durations; `traffic` is read from the committed rocprofv3
                      counter summary under profiles/
  roofline_hbm        the gather/scatter-bound kernels (increment builder, narrow first-layer conv,
                      1x1 prediction head, list compaction): algorithmic bytes over HIP-event
                      durations against 8 TB/s, with one stream and with 16 streams in one net
  dense_recompute     the same frames as regular forward passes through the same kernels
  auto_mode           the same frames with EVCONV_MODE_AUTO
  cpu_baseline        the CPU oracle on a bounded sample of the same frames (all cores and one
                      thread), with its executed-operation counters (the paper's MFLOPs metric)
  f32_split_variant, bf16_variant, hip_graph_replay, multi_stream, single_object_stream,
  sparsified_variant (threshold sweep on a stream with small-valued increments),
  recurrent_variant (a ConvLSTM cell), density_sweep (workload 5, ten densities, short), drift, layers.

`--sweep` / `--drift` run the long forms of the density sweep and the drift study instead (one
JSON line each).
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAKS = {  # MI355X published dense peaks
    "conv_mfma_f32": ("mfma", 157.3, "TFLOP/s"),
    "conv_mfma_bf16": ("mfma", 2500.0, "TFLOP/s"),
    # three bf16 MFMAs per fp32 product: executed flops = 3 x algorithmic, priced against the bf16 peak
    "conv_mfma_f32_split_bf16x3": ("mfma", 2500.0, "TFLOP/s"),
    # vector ALU fp32: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2 (packed) x 2.4 GHz
    "conv_valu_f32": ("alu", 157.3, "TFLOP/s"),
    "conv_narrow_mfma_f32": ("mfma", 157.3, "TFLOP/s"),
    "conv_pointwise_f32": ("hbm", 8000.0, "GB/s"),
}
PROFILE_FILES = {"conv_mfma_f32": "unet_depth_f32_incremental_kernels.md",
                 "conv_mfma_f32_split_bf16x3": "unet_depth_f32_split_incremental_kernels.md",
                 "conv_mfma_bf16": "unet_depth_bf16_incremental_kernels.md"}


def traffic_from_profile(family):
    """HBM bytes per launch of a kernel family as the committed rocprofv3 counter summary states
    them (FETCH_SIZE and WRITE_SIZE scaled by a copy kernel of known size); None if the summary
    holds no such line."""
    name = PROFILE_FILES.get(family)
    if not name:
        return None
    try:
        text = open(os.path.join(ROOT, "profiles", name)).read()
    except OSError:
        return None
    m = re.search(r"scaled HBM\s+traffic\s+([0-9.]+)\s*MB per launch", text)
    return float(m.group(1)) * 1e6 if m else None


def timed_steps(torch, g, dframes, first, count):
    """Runs steps first .. first+count-1 with one HIP event per step boundary on the net's stream.
    Returns (per-step milliseconds from the events, wall-clock seconds of the whole region)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(count + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for j in range(count):
        g.step_frame(dframes[first + j])
        ev[j + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return [ev[j].elapsed_time(ev[j + 1]) for j in range(count)], wall


def step_stats(per_step, wall):
    med = statistics.median(per_step)
    return med, {"median": med, "min": min(per_step), "max": max(per_step), "wall_clock_mean": wall / len(per_step) * 1e3}


def make_net(wl, variant, **kw):
    net = wl.net_unet_depth(1003, bf16=(variant == "bf16"), **kw)
    if variant == "f32_split":
        net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
    return net


def hbm_rows(np, ev, wl, g, net, n_streams):
    """Algorithmic HBM bytes per launch (stream 0's counts x streams) of the gather/scatter-bound
    kernels over their HIP-event time.  Byte counts: builder = frame read + cached frame read and
    write + increment write + the occupancy words it clears; narrow conv and 1x1 head = per touched
    output site c_in x 4 x halo factor read + c_out x 12 (old z, new z, increment) [+ c_out x 8 for
    the public y / dy of an output head]; list compaction = 8 bytes per tile read + 4 bytes per
    listed site + counts and bitmaps."""
    rows = []
    shapes = [g.shape(i) for i in range(len(net.nodes))]

    def row(name, node, nbytes):
        ms, n = g.node_time(node)
        if n == 0 or ms <= 0:
            return
        us = ms / n * 1e3
        gbs = nbytes * n_streams / (us * 1e-6) / 1e9
        rows.append(dict(kernel=name, node=node, streams=n_streams, bytes_per_launch=nbytes * n_streams, avg_launch_us=us,
                         achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS))
    c, h, w = net.in_c, net.in_h, net.in_w
    tiles_all = sum(-(-s[1] // 8) * -(-s[2] // 8) for s in shapes)
    row("builder_kernel", -1, 4 * c * h * w * 4 + 2 * tiles_all * 8 + -(-h // 8) * -(-w // 8) * 8)
    listed = 0
    for i, nd in enumerate(net.nodes):
        name = g.kernel_name(i)
        if name.startswith("fused_into_conv_g") or name.startswith("fused_into_conv_w") or name.startswith("fused_into_concat"):
            continue
        st = g.stats(i)
        listed += st.n_active
        if name in ("conv_narrow_mfma_f32", "conv_pointwise_f32"):
            halo = ((8 - 1) * nd.stride + nd.k) ** 2 / 64.0
            per_site = nd.c_in * 4 * halo + nd.c_out * 12 + (nd.c_out * 8 if nd.is_output else 0)
            row(name, i, per_site * st.n_touched + nd.k * nd.k * nd.c_in * nd.c_out * 4)
    listed += int(g.state(-1, ev.STATE_COUNT)[0])
    n_sets = len(net.nodes) + 1
    row("build_lists_kernel", len(net.nodes), (tiles_all + -(-h // 8) * -(-w // 8)) * 8 + listed * 4 + n_sets * 4 + (tiles_all // 64 + n_sets) * 8)
    return rows


def run_variant(args, np, torch, ev, wl, variant, dframes, with_dense, with_layers):
    net = make_net(wl, variant)
    n_frames = args.warmup + args.steps

    def fresh(mode):
        g = ev.EvConvNet(net, device="cuda:0")
        g.set_mode(mode)
        g.reset(dframes[0])
        for i in range(1, args.warmup + 1):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        return g

    # pass 1: the K timed steps, one HIP event per step boundary -> value
    g = fresh(ev.MODE_INCREMENTAL)
    per_step, wall = timed_steps(torch, g, dframes, args.warmup + 1, args.steps)
    g.destroy()
    med, stats = step_stats(per_step, wall)
    # pass 2: the same K steps with a HIP event pair around every node's launches -> per-kernel
    # durations for the rooflines (the events themselves cost a few microseconds per launch)
    g = fresh(ev.MODE_INCREMENTAL)
    g.profile_begin(args.steps * (len(net.nodes) + 2))
    t0 = time.perf_counter()
    for i in range(args.warmup + 1, n_frames + 1):
        g.step_frame(dframes[i])
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t0
    g.profile_end()
    fam, layers = {}, []
    for i, nd in enumerate(net.nodes):
        ms, n = g.node_time(i)
        name = g.kernel_name(i)
        st = g.stats(i)
        per_site = 2.0 * nd.k * nd.k * nd.c_in * nd.c_out if nd.op in (wl.OP_CONV2D, wl.OP_LINEAR) else 0.0
        flops = per_site * st.n_touched            # algorithmic: touched output sites of the last step
        # Executed: a 5 x 5 conv reading a x2 up-sampling that the library folded into its weights
        # runs 4 x 4 taps on the output tiles over stored tiles whose sites all lie 2 or more from
        # the border of the stored tensor (the other tiles run all 25 taps)
        executed = flops
        if nd.op == wl.OP_CONV2D and nd.in0 >= 0 and g.kernel_name(nd.in0) == "fused_into_conv_weights":
            c, h, w = g.shape(i)
            words = g.state(i, ev.STATE_OCC_TOUCHED).reshape(-(-h // 8), -(-w // 8))
            inner = lambda t, n_sites: (8 * t >= 2) & (8 * t + 7 <= n_sites - 3)
            ty, tx = np.indices(words.shape)
            folded_tiles = inner(ty // 2, h // 2) & inner(tx // 2, w // 2)
            pop = np.array([bin(int(x)).count("1") for x in words.ravel()]).reshape(words.shape)
            executed = per_site * (pop[~folded_tiles].sum() + pop[folded_tiles].sum() * 16.0 / 25.0)
        f = fam.setdefault(name, dict(ms=0.0, launches=0, flops=0.0, executed=0.0))
        f["ms"] += ms
        f["launches"] += n
        f["flops"] += flops * n
        f["executed"] += executed * n
        layers.append(dict(node=i, kernel=name, ms_avg=ms / max(n, 1), touched=st.n_touched, sites=st.n_sites,
                           active=st.n_active, touched_tiles=st.n_touched_tiles, tiles=st.n_tiles,
                           gflop_alg=flops / 1e9))
    dom = max((k for k in fam if k.startswith("conv")), key=lambda k: fam[k]["ms"])
    bound, peak, unit = PEAKS[dom]
    achieved = fam[dom]["flops"] / (fam[dom]["ms"] * 1e-3) / 1e12 if fam[dom]["ms"] > 0 else 0.0
    executed = fam[dom]["executed"] / (fam[dom]["ms"] * 1e-3) / 1e12 if fam[dom]["ms"] > 0 else 0.0
    roofline = dict(kernel=dom, bound=bound, achieved=achieved, peak=peak, unit=unit, frac=achieved / peak,
                    executed=executed, executed_frac=executed / peak,
                    traffic=traffic_from_profile(dom), traffic_source="profiles/" + PROFILE_FILES.get(dom, "-"),
                    avg_launch_ms=fam[dom]["ms"] / max(fam[dom]["launches"], 1),
                    launches=fam[dom]["launches"], share_of_step=fam[dom]["ms"] / (dt_prof * 1e3),
                    event_pass_ms_per_step=dt_prof / args.steps * 1e3)
    res = dict(value=1e3 / med, ms_per_step=med, step_time_ms=stats, roofline=roofline)
    if with_layers:
        res["roofline_hbm"] = hbm_rows(np, ev, wl, g, net, 1)
    g.destroy()
    if with_dense:
        g2 = fresh(ev.MODE_DENSE_RECOMPUTE)
        per2, wall2 = timed_steps(torch, g2, dframes, args.warmup + 1, args.steps)
        g2.destroy()
        med2, stats2 = step_stats(per2, wall2)
        res["dense_recompute"] = {"value": 1e3 / med2, "unit": "steps/s", "ms_per_step": med2, "step_time_ms": stats2,
                                  "incremental_speedup": med2 / med}
        if with_layers:
            g2 = fresh(ev.MODE_DENSE_RECOMPUTE)
            g2.profile_begin(args.steps * (len(net.nodes) + 2))
            for i in range(args.warmup + 1, n_frames + 1):
                g2.step_frame(dframes[i])
            g2.profile_end()
            for i, l in enumerate(layers):
                ms, n = g2.node_time(i)
                l["dense_ms_avg"] = ms / max(n, 1)
            g2.destroy()
            # AUTO: probes both modes, then holds the faster one
            g3 = fresh(ev.MODE_AUTO)
            for i in range(args.warmup + 1, args.warmup + 13):   # both probe windows, then the decision
                g3.step_frame(dframes[min(i, n_frames)])
            torch.cuda.synchronize()
            g3.step_frame(dframes[n_frames])
            torch.cuda.synchronize()
            chosen = g3.current_mode()
            per3, wall3 = timed_steps(torch, g3, dframes, args.warmup + 1, args.steps)
            g3.destroy()
            med3, stats3 = step_stats(per3, wall3)
            res["auto_mode"] = {"value": 1e3 / med3, "unit": "steps/s", "ms_per_step": med3, "step_time_ms": stats3,
                                "holds": "incremental" if chosen == ev.MODE_INCREMENTAL else "dense_recompute"}
    if with_layers:
        res["layers"] = layers
    return net, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--density", type=float, default=0.02, help="changed pixels per step of the synthetic event stream")
    ap.add_argument("--variant", choices=["f32", "bf16", "f32_split"], default="f32",
                    help="contraction of the headline run: fp32 MFMA, bf16 weights, or fp32 through bf16 high/low parts")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the timed CPU oracle leg")
    ap.add_argument("--cpu-steps", type=int, default=20, help="frames of the stream the CPU oracle is timed on (all cores)")
    ap.add_argument("--cpu-steps-1t", type=int, default=3, help="frames the CPU oracle is timed on with one thread")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-recompute and AUTO legs")
    ap.add_argument("--no-second-variant", action="store_true", help="skip the other contraction modes")
    ap.add_argument("--no-sparsified", action="store_true", help="skip the sparsification-layer leg")
    ap.add_argument("--phase-times", action="store_true",
                    help="per-phase times of the matrix-core conv workgroups on the headline workload, from the library "
                         "built with `python -m paper_2303_04670_amd.build --phase-stamps`; prints tables and exits")
    ap.add_argument("--chip-probes", action="store_true",
                    help="run the library's timing probes of the chip (evconv_debug_chip_probes), print them as a table and exit")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--no-recurrent", action="store_true", help="skip the ConvLSTM leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the single-object, short density-sweep and drift legs")
    ap.add_argument("--streams", type=int, default=16,
                    help="independent event streams per net in the multi_stream leg (0: skip the leg)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run plain device-to-device copies of this size (for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings against a kernel of known traffic)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run: optical-flow encoder-decoder (4x256x256), incremental "
                         "vs dense recompute at 10 increment densities 0.1 %% .. 20 %%; prints one JSON line")
    ap.add_argument("--sweep-steps", type=int, default=100)
    ap.add_argument("--drift", action="store_true",
                    help="instead of the headline run: drift of the fp32 running sums over --drift-steps steps of "
                         "the UNet stream, without refresh and with a refresh every --refresh-period steps, measured "
                         "against a regular forward pass of the same frame; prints one JSON line")
    ap.add_argument("--drift-steps", type=int, default=1000)
    ap.add_argument("--refresh-period", type=int, default=100)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (one event stream per device, no collectives); "
                 "--gpus must be 1")

    import numpy as np
    import torch
    from paper_2303_04670_amd import evconv as ev
    from paper_2303_04670_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.chip_probes:
        print(chip_probe_table(ev.chip_probes()))
        return
    if args.phase_times:
        from paper_2303_04670_amd import build as evbuild
        ev.use_library(evbuild.PHASE_LIB_PATH)
        print(phase_time_tables(args, np, torch, ev, wl, dev))
        return
    if args.sweep:
        out = {"metric": "density sweep: incremental vs dense recompute (flow encoder-decoder 4x256x256 and its "
                         "delayed-integration variant)",
               "unit": "ms/step", "n_gpus": 1, "steps_per_density": args.sweep_steps, "dtype": "f32", "data": "synthetic"}
        out.update(density_sweep(args, np, torch, ev, wl, dev, args.sweep_steps))
        print(json.dumps(out), flush=True)
        return
    if args.drift:
        rows, deep = drift_study(args, np, torch, ev, wl, dev, args.drift_steps)
        print(json.dumps({"metric": "drift of the fp32 incremental state against a regular forward pass (UNet depth net)",
                          "unit": "max-abs error (deepest wide conv's accumulated tensor relative to its max; output absolute)",
                          "n_gpus": 1, "steps": args.drift_steps, "dtype": "f32", "data": "synthetic",
                          "node": deep, "rows": rows}), flush=True)
        return
    H, W = 256, 352
    n_frames = args.warmup + args.steps
    frames = list(wl.stream_voxel(1003, H, W, n_frames, args.density))
    dens = float(np.mean([wl.changed_fraction(frames[i], frames[i + 1]) for i in range(args.warmup, n_frames)]))
    dframes = [torch.from_numpy(f).to(dev) for f in frames]
    torch.cuda.synchronize()
    if args.calib_copy_mb:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()

    net, res = run_variant(args, np, torch, ev, wl, args.variant, dframes, not args.no_dense, True)
    out = {
        "metric": "incremental steps/sec at 2% density (UNet depth net)",
        "value": res["value"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.variant, "data": "synthetic",
        "config": {"workload": f"unet_depth_5x{H}x{W}_voxel_stream", "changed_pixel_fraction": round(dens, 5),
                   "weights": args.variant, "mode": "incremental", "batch": 1},
        "step_time_ms": res["step_time_ms"],
        "roofline": res["roofline"],
        "roofline_hbm": res["roofline_hbm"],
    }
    for key in ("dense_recompute", "auto_mode"):
        if key in res:
            out[key] = res[key]
    if not args.no_second_variant:
        for other in ("f32", "f32_split", "bf16"):
            if other == args.variant:
                continue
            _, r2 = run_variant(args, np, torch, ev, wl, other, dframes, not args.no_dense, False)
            r2["unit"] = "steps/s"
            r2["weights"] = other
            r2["parity_bar"] = "2e-2 relative (Frobenius)" if other == "bf16" else "1e-4 max-abs"
            out[f"{other}_variant"] = r2
    if not args.no_graph:
        out["hip_graph_replay"] = graph_leg(args, np, torch, ev, wl, dframes)
    if args.streams > 1:
        out["multi_stream"] = multi_stream_leg(args, np, torch, ev, wl, dev)
        out["roofline_hbm"] += out["multi_stream"].pop("roofline_hbm", [])
    if not args.no_sparsified:
        out["sparsified_variant"] = sparsified_leg(args, np, torch, ev, wl, dev)
    if not args.no_recurrent:
        out["recurrent_variant"] = recurrent_leg(args, np, torch, ev, wl, dframes)
    if not args.no_extras:
        out["single_object_stream"] = single_object_leg(args, np, torch, ev, wl, dev)
        out["density_sweep"] = dict(steps_per_density=10, **density_sweep(args, np, torch, ev, wl, dev, 10))
        rows, deep = drift_study(args, np, torch, ev, wl, dev, 300, quiet=True)
        out["drift"] = {"node": deep, "refresh_period": args.refresh_period, "rows": rows}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args, np, net, frames)
    out["layers"] = res["layers"]
    print(json.dumps(out), flush=True)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(args, np, net, frames):
    """The oracle as it stands on the host cores: all cores, then one thread (fewer frames), plus
    its operation counters averaged over the all-core sample: the paper's MFLOPs metric (2 x
    multiply-accumulates per inference) for a regular pass and for the incremental step at site and
    at 8 x 8 tile granularity."""
    import ctypes
    from oracle.oracle import Oracle
    omp = ctypes.CDLL("libgomp.so.1")
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    ora = Oracle(net)
    ora.reset(frames[0])
    k = min(args.cpu_steps, len(frames) - 1)
    conv = [i for i, nd in enumerate(net.nodes) if nd.op in (0, 6)]
    site = tile = 0.0
    t0 = time.perf_counter()
    for i in range(1, k + 1):
        ora.step_frame(frames[i])
        for j in conv:
            m = ora.macs(j)
            site += m["site"]
            tile += m["tile"]
    cdt = time.perf_counter() - t0
    dense = sum(ora.macs(j)["dense"] for j in conv)
    k1 = min(args.cpu_steps_1t, len(frames) - 1 - k)
    omp.omp_set_num_threads(1)
    t0 = time.perf_counter()
    for i in range(k + 1, k + 1 + k1):
        ora.step_frame(frames[i])
    cdt1 = time.perf_counter() - t0
    omp.omp_set_num_threads(cores)
    return {"value": k / cdt, "unit": "steps/s", "cores": cores, "kind": "oracle", "cpu": cpu_model(),
            "sample": f"frames 1..{k} of the same stream on {cores} threads (fp64, OpenMP); one thread: the next {k1} frames",
            "single_thread": {"value": k1 / cdt1 if k1 else None, "unit": "steps/s", "cores": 1},
            "mflops_per_inference": {"regular_forward_pass": 2 * dense / 1e6, "incremental_site_level": 2 * site / k / 1e6,
                                     "incremental_tile_level": 2 * tile / k / 1e6,
                                     "reduction_site_level": 1 - site / k / dense, "reduction_tile_level": 1 - tile / k / dense,
                                     "rule": "2 x multiply-accumulates of the conv layers; a tap on a zero-padding or inactive site costs nothing at site level"}}


def phase_time_tables(args, np, torch, ev, wl, dev):
    """One step of the headline workload per weight type on the library with phase stamps: per
    conv layer the mean time a workgroup spends in each phase (field names: PhaseField in
    csrc/conv_mfma_impl.h), the workgroup's life and the span of the launch."""
    frames = [torch.from_numpy(f).to(dev) for f in wl.stream_voxel(1003, 256, 352, 10, args.density)]
    order = [0, 1, 2, 3, 4, 5, 6, 10, 7, 14, 8, 11, 12, 13, 9]   # the stamps in program order
    names = ["occupancy words", "bit rows", "touched set, old z, gather predicates", "first requests",
             "first patch in LDS", "chunk loop", "fused operands requested", "partial sums reduced", "operands arrived",
             "epilogue passes", "flag ballots", "flags to LDS", "barrier", "tile words"]
    out = []
    for variant, mode in (("f32", 0), ("f32_split", 2), ("bf16", 1)):
        net = make_net(wl, variant)
        g = ev.EvConvNet(net, device="cuda:0")
        g.reset(frames[0])
        for i in range(1, 9):
            g.step_frame(frames[i])
        torch.cuda.synchronize()
        ev.phase_stamps(mode, reset=True, max_records=0)
        g.step_frame(frames[9])
        torch.cuda.synchronize()
        rec, n = ev.phase_stamps(mode)
        g.destroy()
        rec = rec.astype(np.int64)
        out.append(f"## {variant}: {n} workgroups of the matrix-core conv in one step\n")
        out.append("Mean microseconds per workgroup that ran the chunk loop.\n")
        out.append("| layer (out rows, c_in, k, c_out) | workgroups (active) | launch span | life | " + " | ".join(names) +
                   " | inside contraction loops | between them |")
        out.append("|" + "---|" * (len(names) + 6))
        layers = []
        for key in rec[:, 27]:
            if key not in layers:
                layers.append(key)
        for key in layers:
            r = rec[rec[:, 27] == key]
            full = r[r[:, 6] > 0]
            if len(full) == 0:
                continue
            d = np.diff(full[:, order], axis=1) / 100.0
            life = (full[:, 9] - full[:, 0]) / 100.0
            span = (r[:, [0, 9]].max() - r[:, 0].min()) / 100.0
            desc = f"{key & 0xffff}, {(key >> 16) & 0xffff}, {(key >> 32) & 0xff}, {key >> 40}"
            out.append(f"| {desc} | {len(r)} ({len(full)}) | {span:.1f} | {life.mean():.1f} | " +
                       " | ".join(f"{d[:, i].mean():.2f}" for i in range(len(names))) +
                       f" | {full[:, 20].mean() / 100:.2f} | {full[:, 21].mean() / 100:.2f} |")
        out.append("")
    return "\n".join(out)


def chip_probe_table(v):
    """The values of evconv_debug_chip_probes as a markdown table (layout: include/evconv.h)."""
    rows = [("one wave per SIMD, per iteration one fp32 MFMA (64 cycles of the pipeline) + k independent vector instructions",
             "cycles / iteration for k = 0, 4, 16, 32", f"{v[0]:.0f}, {v[1]:.0f}, {v[2]:.0f}, {v[3]:.0f}"),
            ("two waves per SIMD: vector loop | fp32 MFMA chain", "us alone", f"{v[4]:.0f} | {v[5]:.0f}"),
            ("", "us side by side", f"{v[6]:.0f} | {v[7]:.0f}"),
            ("two waves per SIMD: vector loop | bf16 MFMA chain", "us alone", f"{v[4]:.0f} | {v[8]:.0f}"),
            ("", "us side by side", f"{v[9]:.0f} | {v[10]:.0f}"),
            ("chain of 100 dependent global loads, one wave per SIMD", "us alone / beside three fp32 MFMA chain waves per SIMD",
             f"{v[11]:.0f} / {v[12]:.0f}"),
            ("chain of 1000 dependent LDS reads", "us alone / beside them", f"{v[13]:.0f} / {v[14]:.0f}"),
            ("LDS atomic OR, 64 lanes", "ns per instruction: one word / 64 words", f"{v[15]:.0f} / {v[16]:.0f}"),
            ("20000 16-byte LDS reads of one wave per SIMD", "us alone / beside one-word atomics / beside 64-word atomics",
             f"{v[17]:.0f} / {v[18]:.0f} / {v[19]:.0f}"),
            ("fp32 MFMA chain with a 16-cycle s_nop after every MFMA", "us alone (chain without: %.0f)" % v[5], f"{v[20]:.0f}"),
            ("the two dependent chains beside three such waves per SIMD", "us global loads / LDS reads", f"{v[21]:.0f} / {v[22]:.0f}")]
    out = ["| Probe | Quantity | Measured |", "|---|---|---|"]
    out += [f"| {a} | {b} | {c} |" for a, b, c in rows]
    return "\n".join(out)


def graph_leg(args, np, torch, ev, wl, dframes):
    """One step captured in a HIP graph by the caller (the library only launches kernels on the
    given stream) and replayed per frame; the frame is copied into the captured input buffer on
    the same stream before each replay.  Same frames and step count as the headline."""
    n_frames = args.warmup + args.steps
    res = {"unit": "steps/s"}
    side = torch.cuda.Stream()
    for variant in ("f32", "f32_split", "bf16"):
        net = make_net(wl, variant)
        with torch.cuda.stream(side):
            g = ev.EvConvNet(net, device="cuda:0", stream=side)
            static_in = dframes[0].clone()
            g.reset(static_in)
            static_in.copy_(dframes[1])
            g.step_frame(static_in)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            g.step_frame(static_in)
        with torch.cuda.stream(side):
            for i in range(2, args.warmup + 1):
                static_in.copy_(dframes[i])
                graph.replay()
            side.synchronize()
            t0 = time.perf_counter()
            for i in range(args.warmup + 1, n_frames + 1):
                static_in.copy_(dframes[i])
                graph.replay()
            side.synchronize()
            dt = time.perf_counter() - t0
        del graph
        g.destroy()
        res[variant] = {"value": args.steps / dt, "ms_per_step": dt / args.steps * 1e3}
    return res


def multi_stream_leg(args, np, torch, ev, wl, dev):
    """The chip-filling shape: n independent event streams (cameras) in one net, sharing the
    weights and stepped by one call.  Reported as stream-steps per second; not the headline (the
    headline is one stream, batch 1)."""
    H, W, n = 256, 352, args.streams
    steps = max(10, args.steps // 4)
    n_frames = 3 + steps
    gens = [wl.stream_voxel(2000 + s, H, W, n_frames, args.density) for s in range(n)]
    frames = []
    for t in range(n_frames + 1):
        frames.append(torch.from_numpy(np.stack([next(g) for g in gens])).to(dev))
    res = {"streams": n, "unit": "stream-steps/s", "steps": steps}
    for variant in ("f32", "f32_split", "bf16"):
        net = make_net(wl, variant)

        def run(mode, profile=False):
            g = ev.EvConvNet(net, device="cuda:0", n_streams=n)
            g.set_mode(mode)
            g.reset(frames[0])
            for t in range(1, 4):
                g.step_frame(frames[t])
            torch.cuda.synchronize()
            if profile:
                g.profile_begin(steps * (len(net.nodes) + 2))
            t0 = time.perf_counter()
            for t in range(4, n_frames + 1):
                g.step_frame(frames[t])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            if profile:
                g.profile_end()
            return g, dt
        g, dt = run(ev.MODE_INCREMENTAL)
        conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
        flops = sum(2.0 * net.nodes[i].k ** 2 * net.nodes[i].c_in * net.nodes[i].c_out * g.stats(i).n_touched for i in conv)
        g.destroy()
        res[variant] = {"value": n * steps / dt, "ms_per_call": dt / steps * 1e3,
                        "conv_tflops_alg": flops * n * steps / dt / 1e12}
        if variant == "f32":
            g, _ = run(ev.MODE_INCREMENTAL, profile=True)
            res["roofline_hbm"] = hbm_rows(np, ev, wl, g, net, n)
            g.destroy()
        if not args.no_dense:   # the same frames as regular forward passes through the same kernels
            g, dt2 = run(ev.MODE_DENSE_RECOMPUTE)
            g.destroy()
            res[variant]["dense_recompute_ms_per_call"] = dt2 / steps * 1e3
            res[variant]["incremental_speedup"] = dt2 / dt
    return res


def mode_pair(torch, ev, net, dfr, warm, steps, **kw):
    """Median step time (ms) in incremental and in dense-recompute mode on the same frames, plus
    the tile-level fraction of a regular pass's conv operations the incremental steps executed."""
    t = {}
    frac = None
    for mode in (ev.MODE_INCREMENTAL, ev.MODE_DENSE_RECOMPUTE):
        g = ev.EvConvNet(net, device="cuda:0", **kw)
        g.set_mode(mode)
        g.reset(dfr[0])
        for i in range(1, warm + 1):
            g.step_frame(dfr[i])
        per, wall = timed_steps(torch, g, dfr, warm + 1, steps)
        t[mode] = statistics.median(per)
        if mode == ev.MODE_INCREMENTAL:
            ex = sum(g.stats(i).flops_executed for i in range(len(net.nodes)))
            de = sum(g.stats(i).flops_dense for i in range(len(net.nodes)))
            frac = ex / de
        g.destroy()
    return t[ev.MODE_INCREMENTAL], t[ev.MODE_DENSE_RECOMPUTE], frac


def single_object_leg(args, np, torch, ev, wl, dev):
    """Locality instead of uniform density: the UNet on a stream in which a single object moves
    (0.1 % changed pixels, all in one region of the frame), incremental against dense recompute."""
    H, W, n = 256, 352, 45
    net = wl.net_unet_depth(1003, h=H, w=W)
    rows = []
    for dens in (0.001, 0.0003):
        frames = list(wl.stream_voxel(77, H, W, n, dens, n_prim=1))
        real = float(np.mean([wl.changed_fraction(frames[i], frames[i + 1]) for i in range(5, n)]))
        dfr = [torch.from_numpy(f).to(dev) for f in frames]
        inc, dense, frac = mode_pair(torch, ev, net, dfr, 5, n - 5)
        rows.append(dict(changed_pixel_fraction=real, incremental_ms=inc, dense_ms=dense, speedup=dense / inc,
                         tile_flop_fraction=frac))
    return {"net": "UNet depth net 5x256x352, one moving primitive", "unit": "ms/step", "rows": rows}


def sparsified_leg(args, np, torch, ev, wl, dev):
    """What the sparsification layer (Eq.3-8) is for: a stream whose increments are dense but mostly
    tiny (a slowly drifting smooth background under the event voxel grid: every pixel changes a
    little at every step, event pixels change by order one).  Lossless incremental inference sees
    every site active; with a layer ahead of every convolution, including the first, the small
    changes stay in the residuals until they add up to half a rounding step.  Threshold sweep of the
    paper's sensitivity study, t_p in {0.01, 0.05, 0.1, 0.3}, at two drift rates: step time against
    the lossless incremental step and against dense recompute, touched-site and touched-tile
    fractions, tile-level operation fraction, deviation of the output from the lossless run.

    Measured in the steady state: the residuals start at zero at the reset and the drift is
    coherent, so nothing but events is emitted until the first residuals reach half a rounding
    step (50 steps and more at t_p = 0.3); timing that quiet stretch would flatter the layer.  The
    warm-up is 300 steps, longer than the first crossing at every threshold of the sweep."""
    H, W = 256, 352
    warm, steps = 300, max(20, args.steps // 2)
    base = list(wl.stream_voxel(1003, H, W, warm + steps, args.density))
    res = {"unit": "ms/step", "warmup_steps": warm, "timed_steps": steps, "streams": []}
    for drift in (1e-3, 2e-4):
        dfr = [torch.from_numpy(f).to(dev)
               for f in wl.drifting_background(base, amplitude=0.5, drift=drift, event_scale=0.05)]
        plain = wl.net_unet_depth(1003, h=H, w=W)
        inc, dense, frac = mode_pair(torch, ev, plain, dfr, warm, steps)
        leg = {"stream": f"0.05 x event voxel grid + smooth background of amplitude 0.5 drifting by at most {drift:g} per step at every pixel",
               "lossless_incremental_ms": inc, "dense_recompute_ms": dense, "lossless_tile_flop_fraction": frac, "rows": []}
        # lossless output for the deviation column
        g = ev.EvConvNet(plain, device="cuda:0")
        g.reset(dfr[0])
        for i in range(1, warm + steps + 1):
            g.step_frame(dfr[i])
        torch.cuda.synchronize()
        y_ref = g.outputs()[0]["y"].clone()
        g.destroy()
        for tp in (0.01, 0.05, 0.1, 0.3):
            net = wl.net_unet_depth(1003, h=H, w=W, sparsify=True, sparsify_input=True)
            net.sparsify_tp = tp
            g = ev.EvConvNet(net, device="cuda:0")
            g.reset(dfr[0])
            for i in range(1, warm + 1):
                g.step_frame(dfr[i])
            per, wall = timed_steps(torch, g, dfr, warm + 1, steps)
            conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
            st = [g.stats(i) for i in conv]
            dev_out = float((g.outputs()[0]["y"] - y_ref).abs().max())
            g.destroy()
            med = statistics.median(per)
            leg["rows"].append(dict(t_p=tp, ms_per_step=med, speedup_vs_lossless=inc / med, speedup_vs_dense=dense / med,
                                    touched_site_fraction=sum(x.n_touched for x in st) / sum(x.n_sites for x in st),
                                    touched_tile_fraction=sum(x.n_touched_tiles for x in st) / sum(x.n_tiles for x in st),
                                    tile_flop_fraction=sum(x.flops_executed for x in st) / sum(x.flops_dense for x in st),
                                    max_abs_output_deviation_from_lossless=dev_out))
        res["streams"].append(leg)
        del dfr
    return res


def recurrent_leg(args, np, torch, ev, wl, dframes):
    """The same frames through a ConvLSTM cell (64 hidden channels at full resolution, two
    recurrent states as DELAY nodes) with a 1 x 1 head.  A recurrent state moves at every step, so
    everything behind it is dense; reported beside a dense recompute of the same frames and AUTO
    mode, which settles on the faster of the two."""
    # (the gate convs read 5 + 64 = 69 channels)
    net = wl.net_convlstm(1008, in_c=5, h=256, w=352, hidden=64, out_c=1)
    steps = max(10, args.steps // 4)
    dframes = dframes[:16 + steps]
    res = {}
    for mode, key in ((ev.MODE_INCREMENTAL, "incremental"), (ev.MODE_DENSE_RECOMPUTE, "dense_recompute"), (ev.MODE_AUTO, "auto")):
        g = ev.EvConvNet(net, device="cuda:0")
        g.set_mode(mode)
        g.reset(dframes[0])
        for i in range(1, 15):
            g.step_frame(dframes[i])
            if i % 4 == 0:
                torch.cuda.synchronize()   # (lets AUTO pick its probe timings up)
        per, wall = timed_steps(torch, g, dframes, 15, steps)
        conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
        res[key] = dict(ms_per_step=statistics.median(per),
                        touched_site_fraction=sum(g.stats(i).n_touched for i in conv) / sum(g.stats(i).n_sites for i in conv))
        if mode == ev.MODE_AUTO:
            res[key]["holds"] = "incremental" if g.current_mode() == ev.MODE_INCREMENTAL else "dense_recompute"
        g.destroy()
    return {"net": "ConvLSTM 5->64 hidden, 3x3 gates, 256x352, 1x1 head", "unit": "steps/s", "steps": steps,
            "value": 1e3 / res["incremental"]["ms_per_step"], "ms_per_step": res["incremental"]["ms_per_step"],
            "touched_site_fraction": res["incremental"]["touched_site_fraction"],
            "dense_recompute_ms_per_step": res["dense_recompute"]["ms_per_step"],
            "auto_ms_per_step": res["auto"]["ms_per_step"], "auto_holds": res["auto"]["holds"]}


def drift_study(args, np, torch, ev, wl, dev, n_steps, quiet=False):
    """"Drift Errors": the accumulated tensors are fp32 running sums, so their difference from a
    regular forward pass of the current frame grows with the number of steps since the last
    refresh.  Three nets see the same frames: no refresh, a refresh every N steps, and a reference
    that is reset (regular forward pass) at every checkpoint."""
    H, W = 256, 352
    net = wl.net_unet_depth(1003, h=H, w=W)
    deep = max(i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D and nd.c_out > 1)
    free, pol, ref = (ev.EvConvNet(net, device="cuda:0") for _ in range(3))
    pol.set_refresh_period(args.refresh_period)
    gen = wl.stream_voxel(1003, H, W, n_steps, args.density)
    x0 = torch.from_numpy(next(gen)).to(dev)
    for g in (free, pol):
        g.reset(x0)
    checks = sorted({c for c in (1, 10, 99, 100, 101, 199, 300, 500, 999, 1000, 2000, 5000, 10000)
                     if c <= n_steps} | {n_steps})
    rows = []
    t0 = time.perf_counter()
    for t, f in enumerate(gen, 1):
        x = torch.from_numpy(f).to(dev)
        free.step_frame(x)
        pol.step_frame(x)
        if t in checks:
            ref.reset(x)
            torch.cuda.synchronize()
            zr = ref.state(deep, ev.STATE_Z).astype(np.float64)
            yr = ref.outputs()[0]["y"].double()
            row = {"step": t}
            for name, g in (("no_refresh", free), ("refresh_every_%d" % args.refresh_period, pol)):
                z = g.state(deep, ev.STATE_Z).astype(np.float64)
                row[name] = {"max_abs_z_error_rel": float(np.abs(z - zr).max() / np.abs(zr).max()),
                             "max_abs_output_error": float((g.outputs()[0]["y"].double() - yr).abs().max())}
            rows.append(row)
            if not quiet:
                print(f"# step {t} ({time.perf_counter() - t0:.0f} s)", file=sys.stderr, flush=True)
    for g in (free, pol, ref):
        g.destroy()
    return rows, deep


def density_sweep(args, np, torch, ev, wl, dev, steps):
    """Workload 5: where does incremental inference beat a dense recompute built from the same
    kernels?  One stream per density so that every timed step runs at that density."""
    out = {}
    for key, net in (("rows", wl.net_flow(1005)), ("rows_delayed_integration", wl.net_flow_delayed(1006))):
        rows = []
        for dens in np.geomspace(0.001, 0.2, 10):
            n = 5 + steps
            frames = list(wl.stream_count_timestamp(1005, 256, 256, densities=[float(dens)], steps_per=n))
            real = float(np.mean([wl.changed_fraction(frames[i], frames[i + 1]) for i in range(5, n)]))
            dfr = [torch.from_numpy(f).to(dev) for f in frames]
            inc, dense, frac = mode_pair(torch, ev, net, dfr, 5, n - 5)
            rows.append(dict(density=real, incremental_ms=inc, dense_ms=dense, speedup=dense / inc, tile_flop_fraction=frac))
        out[key] = rows
    return out


if __name__ == "__main__":
    main()
