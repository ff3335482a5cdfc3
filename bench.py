#!/usr/bin/env python3
"""Benchmark of the incremental-inference hot path on one MI355X.

A step = one evconv_step_frame call: increment builder, every layer's increment kernel, output
integration and list compaction, on one frame of a synthetic event-voxel stream that is already
resident in HBM.  Workload: the UNet depth network on 5x256x352 at 2 % changed pixels per step,
fp32 weights (headline) and the bf16-weight variant (reported beside it).

Prints ONE JSON line.  Extra keys: `dense_recompute` (the same frames run as regular forward
passes through the same kernels), `roofline` (dominant kernel family, timed with HIP events on the
library's stream inside the timed region; `achieved` counts the operator's algorithmic FLOPs, `executed`
the FLOPs of the taps that were run: the library folds a x2 up-sampling into 4 x 4-tap weights on most
tiles of the 5 x 5 convs that read one), `cpu_baseline` (the CPU oracle on a bounded sample of
the same frames), `f32_split_variant`, `bf16_variant`, `hip_graph_replay`, `multi_stream` (16 streams
in one net), `sparsified_variant`, `recurrent_variant` (a ConvLSTM cell), `layers`.

`--sweep` runs the density sweep of the optical-flow encoder-decoder instead (one JSON line).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

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

# HBM bytes per launch of the dominant kernel family, from the committed rocprofv3 counter runs
# (profiles/unet_depth_f32_incremental_kernels.md: FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00)
TRAFFIC_FROM_PROFILE = {"conv_mfma_f32": 28.0e6, "conv_mfma_f32_split_bf16x3": 28.0e6}


def run_variant(args, np, torch, ev, wl, variant, frames, dframes, with_dense, with_layers):
    H, W = 256, 352
    net = wl.net_unet_depth(1003, h=H, w=W, bf16=(variant == "bf16"))
    if variant == "f32_split":
        net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
    n_frames = args.warmup + args.steps

    def timed_run(mode, profile):
        g = ev.EvConvNet(net, device="cuda:0")
        g.set_mode(mode)
        g.reset(dframes[0])
        for i in range(1, args.warmup + 1):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        if profile:
            g.profile_begin(args.steps * len(net.nodes))
        t0 = time.perf_counter()
        for i in range(args.warmup + 1, n_frames + 1):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if profile:
            g.profile_end()
        return g, dt

    # pass 1: the K timed steps with nothing but the library's own launches on the stream -> value
    g, dt = timed_run(ev.MODE_INCREMENTAL, False)
    g.destroy()
    # pass 2: the same K steps with a HIP event pair around every node's launches -> per-kernel
    # durations for the roofline (the events themselves cost ~1 us each and stretch this pass)
    g, dt_prof = timed_run(ev.MODE_INCREMENTAL, True)
    # per kernel family: accumulated event time, launches, algorithmic flops of the timed launches
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
                    traffic=TRAFFIC_FROM_PROFILE.get(dom), avg_launch_ms=fam[dom]["ms"] / max(fam[dom]["launches"], 1),
                    launches=fam[dom]["launches"], share_of_step=fam[dom]["ms"] / (dt_prof * 1e3),
                    event_pass_ms_per_step=dt_prof / args.steps * 1e3)
    g.destroy()
    res = dict(value=args.steps / dt, ms_per_step=dt / args.steps * 1e3, roofline=roofline)
    if with_dense:
        g2, dt2 = timed_run(ev.MODE_DENSE_RECOMPUTE, False)
        g2.destroy()
        g2, _ = timed_run(ev.MODE_DENSE_RECOMPUTE, True)
        for i, l in enumerate(layers):
            ms, n = g2.node_time(i)
            l["dense_ms_avg"] = ms / max(n, 1)
        g2.destroy()
        res["dense_recompute"] = {"value": args.steps / dt2, "unit": "steps/s", "ms_per_step": dt2 / args.steps * 1e3,
                                  "incremental_speedup": dt2 / dt}
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
    ap.add_argument("--cpu-steps", type=int, default=20, help="frames of the stream the CPU oracle is timed on")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-recompute legs")
    ap.add_argument("--no-second-variant", action="store_true", help="skip the other contraction modes")
    ap.add_argument("--no-sparsified", action="store_true", help="skip the sparsification-layer leg")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--no-recurrent", action="store_true", help="skip the ConvLSTM leg")
    ap.add_argument("--streams", type=int, default=16,
                    help="independent event streams per net in the multi_stream leg (0: skip the leg)")
    ap.add_argument("--sparsify-tp", type=float, default=0.1, help="threshold parameter t_p of the sparsification-layer leg")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run plain device-to-device copies of this size (for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings against a kernel of known traffic)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run: optical-flow encoder-decoder (4x256x256), incremental "
                         "vs dense recompute at 10 increment densities 0.1 %% .. 20 %%; prints one JSON line")
    ap.add_argument("--sweep-steps", type=int, default=30)
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
    if args.sweep:
        return density_sweep(args, np, torch, ev, wl, dev)
    if args.drift:
        return drift_study(args, np, torch, ev, wl, dev)
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

    net, res = run_variant(args, np, torch, ev, wl, args.variant, frames, dframes, not args.no_dense, True)
    out = {
        "metric": "incremental steps/sec at 2% density (UNet depth net)",
        "value": res["value"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.variant, "data": "synthetic",
        "config": {"workload": f"unet_depth_5x{H}x{W}_voxel_stream", "changed_pixel_fraction": round(dens, 5),
                   "weights": args.variant, "mode": "incremental", "batch": 1},
        "roofline": res["roofline"],
    }
    if "dense_recompute" in res:
        out["dense_recompute"] = res["dense_recompute"]
    if not args.no_second_variant:
        for other in ("f32", "f32_split", "bf16"):
            if other == args.variant:
                continue
            _, r2 = run_variant(args, np, torch, ev, wl, other, frames, dframes, not args.no_dense, False)
            r2["unit"] = "steps/s"
            r2["weights"] = other
            r2["parity_bar"] = "2e-2 relative (Frobenius)" if other == "bf16" else "1e-4 max-abs"
            out[f"{other}_variant"] = r2
    if not args.no_graph:
        out["hip_graph_replay"] = graph_leg(args, np, torch, ev, wl, dframes)
    if args.streams > 1:
        out["multi_stream"] = multi_stream_leg(args, np, torch, ev, wl, dev)
    if not args.no_sparsified:
        out["sparsified_variant"] = sparsified_leg(args, np, torch, ev, wl, dframes)
    if not args.no_recurrent:
        out["recurrent_variant"] = recurrent_leg(args, np, torch, ev, wl, dframes)
    if not args.no_cpu_baseline:
        from oracle.oracle import Oracle
        ora = Oracle(net)
        ora.reset(frames[0])
        k = min(args.cpu_steps, n_frames)
        t0 = time.perf_counter()
        for i in range(1, k + 1):
            ora.step_frame(frames[i])
        cdt = time.perf_counter() - t0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": k / cdt, "unit": "steps/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {k} frames of the same stream, fp64, OpenMP"}
    out["layers"] = res["layers"]
    print(json.dumps(out), flush=True)


def graph_leg(args, np, torch, ev, wl, dframes):
    """One step captured in a HIP graph by the caller (the library only launches kernels on the
    given stream) and replayed per frame; the frame is copied into the captured input buffer on
    the same stream before each replay.  Same frames and step count as the headline."""
    H, W = 256, 352
    n_frames = args.warmup + args.steps
    res = {"unit": "steps/s"}
    side = torch.cuda.Stream()
    for variant in ("f32", "f32_split", "bf16"):
        net = wl.net_unet_depth(1003, h=H, w=W, bf16=(variant == "bf16"))
        if variant == "f32_split":
            net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
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
        net = wl.net_unet_depth(1003, h=H, w=W, bf16=(variant == "bf16"))
        if variant == "f32_split":
            net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
        def run(mode):
            g = ev.EvConvNet(net, device="cuda:0", n_streams=n)
            g.set_mode(mode)
            g.reset(frames[0])
            for t in range(1, 4):
                g.step_frame(frames[t])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for t in range(4, n_frames + 1):
                g.step_frame(frames[t])
            torch.cuda.synchronize()
            return g, time.perf_counter() - t0
        g, dt = run(ev.MODE_INCREMENTAL)
        conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
        flops = sum(2.0 * net.nodes[i].k ** 2 * net.nodes[i].c_in * net.nodes[i].c_out * g.stats(i).n_touched for i in conv)
        g.destroy()
        res[variant] = {"value": n * steps / dt, "ms_per_call": dt / steps * 1e3,
                        "conv_tflops_alg": flops * n * steps / dt / 1e12}
        if not args.no_dense:   # the same frames as regular forward passes through the same kernels
            g, dt2 = run(ev.MODE_DENSE_RECOMPUTE)
            g.destroy()
            res[variant]["dense_recompute_ms_per_call"] = dt2 / steps * 1e3
            res[variant]["incremental_speedup"] = dt2 / dt
    return res


def sparsified_leg(args, np, torch, ev, wl, dframes):
    """The same frames through the UNet with a sparsification layer ahead of every convolution
    that reads a layer output (Eq.3-8; threshold parameter t_p, default 0.1, the paper's quoted
    operating point).  Lossy: reports how far the output moved from the lossless run, and how
    many convolution output sites were touched compared with it."""
    H, W = 256, 352
    n_frames = args.warmup + args.steps
    res = {}
    ys = {}
    for tp in (0.0, args.sparsify_tp):
        net = wl.net_unet_depth(1003, h=H, w=W, sparsify=True)
        net.sparsify_tp = tp
        g = ev.EvConvNet(net, device="cuda:0")
        g.reset(dframes[0])
        for i in range(1, args.warmup + 1):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.warmup + 1, n_frames + 1):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
        touched = sum(g.stats(i).n_touched for i in conv)
        sites = sum(g.stats(i).n_sites for i in conv)
        ex = sum(g.stats(i).flops_executed for i in conv)
        de = sum(g.stats(i).flops_dense for i in conv)
        ys[tp] = g.outputs()[0]["y"].clone()
        g.destroy()
        res[tp] = dict(value=args.steps / dt, ms_per_step=dt / args.steps * 1e3, touched_site_fraction=touched / sites,
                       tile_flop_fraction=ex / de)
    a, b = res[0.0], res[args.sparsify_tp]
    dev_out = float((ys[0.0] - ys[args.sparsify_tp]).abs().max())
    return {"t_p": args.sparsify_tp, "value": b["value"], "unit": "steps/s", "ms_per_step": b["ms_per_step"],
            "touched_site_fraction": b["touched_site_fraction"], "tile_flop_fraction": b["tile_flop_fraction"],
            "with_t_p_0": a, "max_abs_output_deviation_from_lossless": dev_out,
            "note": "random weights and unit-size input increments: few elements fall under k, see the text"}


def recurrent_leg(args, np, torch, ev, wl, dframes):
    """The same frames through a ConvLSTM cell (64 hidden channels at full resolution, two
    recurrent states as DELAY nodes) with a 1 x 1 head.  A recurrent state moves at every step, so
    everything behind it is dense; reported beside a dense recompute of the same frames."""
    # (the gate convs read 5 + 64 = 69 channels)
    net = wl.net_convlstm(1008, in_c=5, h=256, w=352, hidden=64, out_c=1)
    dframes = dframes[:5 + max(10, args.steps // 4)]
    steps = max(10, args.steps // 4)
    res = {}
    for mode, key in ((ev.MODE_INCREMENTAL, "incremental"), (ev.MODE_DENSE_RECOMPUTE, "dense_recompute")):
        g = ev.EvConvNet(net, device="cuda:0")
        g.set_mode(mode)
        g.reset(dframes[0])
        for i in range(1, 4):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(4, 4 + steps):
            g.step_frame(dframes[i])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        conv = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D]
        res[key] = dict(value=steps / dt, ms_per_step=dt / steps * 1e3,
                        touched_site_fraction=sum(g.stats(i).n_touched for i in conv) / sum(g.stats(i).n_sites for i in conv))
        g.destroy()
    return {"net": "ConvLSTM 5->64 hidden, 3x3 gates, 256x352, 1x1 head", "unit": "steps/s", "steps": steps,
            "value": res["incremental"]["value"], "ms_per_step": res["incremental"]["ms_per_step"],
            "touched_site_fraction": res["incremental"]["touched_site_fraction"],
            "dense_recompute_ms_per_step": res["dense_recompute"]["ms_per_step"]}


def drift_study(args, np, torch, ev, wl, dev):
    """"Drift Errors": the accumulated tensors are fp32 running sums, so their difference from a
    regular forward pass of the current frame grows with the number of steps since the last
    refresh.  Three nets see the same frames: no refresh, a refresh every N steps, and a reference
    that is reset (regular forward pass) at every checkpoint."""
    H, W = 256, 352
    net = wl.net_unet_depth(1003, h=H, w=W)
    deep = max(i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D and nd.c_out > 1)
    free, pol, ref = (ev.EvConvNet(net, device="cuda:0") for _ in range(3))
    pol.set_refresh_period(args.refresh_period)
    gen = wl.stream_voxel(1003, H, W, args.drift_steps, args.density)
    x0 = torch.from_numpy(next(gen)).to(dev)
    for g in (free, pol):
        g.reset(x0)
    checks = sorted({c for c in (1, 3, 10, 30, 99, 100, 101, 199, 300, 500, 999, 1000, 2000, 5000, 10000)
                     if c <= args.drift_steps} | {args.drift_steps})
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
            print(f"# step {t} ({time.perf_counter() - t0:.0f} s)", file=sys.stderr, flush=True)
    for g in (free, pol, ref):
        g.destroy()
    print(json.dumps({"metric": "drift of the fp32 incremental state against a regular forward pass (UNet depth net)",
                      "unit": "max-abs error (deepest wide conv's accumulated tensor relative to its max; output absolute)",
                      "n_gpus": 1, "steps": args.drift_steps, "dtype": "f32", "data": "synthetic",
                      "node": deep, "rows": rows}), flush=True)


def density_sweep(args, np, torch, ev, wl, dev):
    """Workload 5: where does incremental inference beat a dense recompute built from the same
    kernels?  One stream per density so that every timed step runs at that density."""
    out = {"metric": "density sweep: incremental vs dense recompute (flow encoder-decoder 4x256x256 and its "
                     "delayed-integration variant)",
           "unit": "ms/step", "n_gpus": 1, "steps_per_density": args.sweep_steps, "dtype": "f32", "data": "synthetic"}
    for key, net in (("rows", wl.net_flow(1005)), ("rows_delayed_integration", wl.net_flow_delayed(1006))):
        out[key] = sweep_one(args, np, torch, ev, wl, dev, net)
    print(json.dumps(out), flush=True)


def sweep_one(args, np, torch, ev, wl, dev, net):
    rows = []
    for dens in np.geomspace(0.001, 0.2, 10):
        n = 5 + args.sweep_steps
        frames = list(wl.stream_count_timestamp(1005, 256, 256, densities=[float(dens)], steps_per=n))
        real = float(np.mean([wl.changed_fraction(frames[i], frames[i + 1]) for i in range(5, n)]))
        dfr = [torch.from_numpy(f).to(dev) for f in frames]
        t = {}
        for mode in (ev.MODE_INCREMENTAL, ev.MODE_DENSE_RECOMPUTE):
            g = ev.EvConvNet(net, device="cuda:0")
            g.set_mode(mode)
            g.reset(dfr[0])
            for i in range(1, 6):
                g.step_frame(dfr[i])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(6, n + 1):
                g.step_frame(dfr[i])
            torch.cuda.synchronize()
            t[mode] = (time.perf_counter() - t0) / (n - 5) * 1e3
            if mode == ev.MODE_INCREMENTAL:
                ex = sum(g.stats(i).flops_executed for i in range(len(net.nodes)))
                de = sum(g.stats(i).flops_dense for i in range(len(net.nodes)))
            g.destroy()
        rows.append(dict(density=real, incremental_ms=t[ev.MODE_INCREMENTAL], dense_ms=t[ev.MODE_DENSE_RECOMPUTE],
                         speedup=t[ev.MODE_DENSE_RECOMPUTE] / t[ev.MODE_INCREMENTAL],
                         tile_flop_fraction=ex / de))
    return rows


if __name__ == "__main__":
    main()
