#!/usr/bin/env python3
"""Benchmark of the module-parallel local step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic mini-batch, all K modules:
[AuxNet forward if the config has one] + module forward + local loss / terminal adjoint + module-local
backward + [multiplier update for augmented-Lagrangian configs].  Default workload: the WideResNet-28-10-shaped
configuration (batch 128, bf16 storage / fp32 accumulate, K=4, augmented Lagrangian), which is the one the
conv-TFLOP/s target is quoted on.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}     # dense MFMA, MI355X data sheet
PEAK_HBM_GBS = 8000.0
N_CUS = 256


def build_state(net, seed_noise=True):
    """Device state for timing: seeded parameters / image / labels; auxiliary variables = the device's own
    serial forward states + N(0, sigma^2) (the CPU oracle cannot run the full-size forward in bench time)."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_2112_05387_amd import LocalStep
    ls = LocalStep(net)
    for k in range(net.K):
        ls.set_params(k, wl.make_params(net, k))
    ls.set_x(0, wl.make_image(net))
    ls.set_labels(wl.make_labels(net))
    if net.aux is not None:
        for j in range(net.K - 1):
            ls.set_aux_params(j, wl.make_aux_params(net, j))
        ls.auxnet_forward()
    else:
        g = torch.Generator(device="cuda")
        g.manual_seed(net.seed)
        for k in range(net.K - 1):
            ls.module_forward(mask=1 << k)
            noise = torch.randn(ls.y[k].shape, generator=g, device="cuda", dtype=torch.float32) * net.noise_sigma
            ls.x[k + 1].copy_((ls.y[k].float() + noise).to(ls.tdtype))
    if net.al:
        g = torch.Generator(device="cuda")
        g.manual_seed(net.seed + 1000)
        ls.lam = [(torch.randn(s, generator=g, device="cuda", dtype=torch.float32) * net.lam_sigma).to(ls.tdtype)
                  for s in ls.y_shapes]
    torch.cuda.synchronize()
    return ls


SEPARATE_CALLS = False


def time_graph_replays(ls, net, steps):
    """The same step captured once into a HIP graph (stream lanes included) and replayed `steps` times: wall time per
    replay.  What it takes away is the host's launch work, which bounds the small networks."""
    import torch
    if SEPARATE_CALLS:
        raise SystemExit("--graph captures the one-call step; it does not combine with --separate-calls")
    g = ls.capture_step(net.rho, 1.0, mult_step=(net.step if net.al else None), with_aux=(net.aux is not None))
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def one_step(ls, net):
    if not SEPARATE_CALLS:
        ls.step(net.rho, 1.0, mult_step=(net.step if net.al else None), with_aux=(net.aux is not None))
        return
    if net.aux is not None:
        ls.auxnet_forward()
    ls.module_forward()
    ls.local_loss_grad(net.rho, 1.0)
    ls.module_backward()
    if net.al and ls.lam is not None:
        ls.al_multiplier_update(net.step)


def speedup_terms(name, batch, reps):
    """One-GPU measurement of the terms of the paper's speed-up model (Sec. 4.3): the layer-serial network
    (K = 1) gives T_f and T_b; the K-module network, one module at a time, gives what each of K devices would
    run; the interface work gives t_psi and the AuxNet work t_f^lambda, t_b^lambda.  Data loading T_d is not
    modelled (0): the result is the model's upper bound for this network on this device."""
    import torch
    import workloads as wl
    from workloads.configs import AuxDesc

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    net = wl.make_config(name, batch=batch)
    nblocks = sum(len(m.blocks) for m in net.modules)
    serial = wl.make_config(name, batch=batch, split=[nblocks])
    ls = build_state(serial)
    T_f = timed(lambda: ls.module_forward())
    # a backward pass consumes its forward pass: time both and subtract
    T_b = timed(lambda: (ls.module_forward(), ls.local_loss_grad(serial.rho, 1.0), ls.module_backward())) - T_f
    T_u = timed(lambda: ls.sgd_update(0.0))
    ls.close()
    del ls
    if net.aux is None:
        m0 = net.modules[0]
        net.aux = [AuxDesc(cin=m0.C, cout=m.C, stride=m0.H // m.H, relu=False) for m in net.modules[1:]]
    ls = build_state(net)
    K = net.K
    f = [timed(lambda k=k: ls.module_forward(mask=1 << k)) for k in range(K)]
    ls.local_loss_grad(net.rho, 1.0)
    b = [timed(lambda k=k: (ls.module_forward(mask=1 << k), ls.module_backward(mask=1 << k))) - f[k]
         for k in range(K - 1)]                                                              # interface loss: in t_psi
    last = 1 << (K - 1)
    b.append(timed(lambda: (ls.module_forward(mask=last), ls.local_loss_grad(net.rho, 1.0, mask=last),
                            ls.module_backward(mask=last))) - f[K - 1])
    t_loss = timed(lambda: ls.local_loss_grad(net.rho, 1.0, mask=(1 << (K - 1)) - 1))
    x_keep = [t.clone() for t in ls.x]
    t_corr = timed(lambda: ls.aux_variable_update(net.rho, 1.0, 0.0))
    t_mult = timed(lambda: ls.al_multiplier_update(0.0)) if net.al else 0.0
    t_lf = timed(lambda: ls.auxnet_forward())
    for t, keep in zip(ls.x, x_keep):
        t.copy_(keep)
    t_lb = timed(lambda: ls.auxnet_distill_grad(1.0))
    ls.close()
    t_psi = t_loss + t_corr + t_mult
    over = t_psi + t_lf + t_lb
    model = 1.0 / ((T_f + T_b) / K / (T_f + T_b) + over / (T_f + T_b))
    slowest = max(fk + bk for fk, bk in zip(f, b))
    return {"workload": f"{name}, batch {net.modules[0].N}, K={K}", "ms": {
                "T_f": T_f, "T_b": T_b, "T_update": T_u, "module_forward": f, "module_backward": b,
                "t_psi": t_psi, "t_psi_parts": {"loss_adjoint": t_loss, "aux_variable_update": t_corr, "multiplier_update": t_mult},
                "t_f_lambda": t_lf, "t_b_lambda": t_lb},
            "speedup_model_T_d_0": model,
            "speedup_with_measured_module_balance": (T_f + T_b) / (slowest + over),
            "note": "every term measured on ONE GPU; the K devices of the model are not run"}


def measure_peak():
    """What the matrix cores of this device sustain under their own power management: MFMA-only and MFMA + LDS
    operand reads (the convolution kernels' wave tile), one workgroup per CU and two, with the shader clock each ran at."""
    import torch
    from paper_2112_05387_amd import binding as B
    dev = torch.device("cuda:0")
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    out = {}
    stream = torch.cuda.current_stream().cuda_stream
    for mode, name in ((0, "mfma_only"), (1, "mfma_plus_lds_reads")):
        for blocks in (256, 512):
            iters = 4000
            clk = torch.zeros(2 * blocks, dtype=torch.int64, device=dev)
            B.lp_debug_mfma_peak(stream, mode, blocks, 200, clk.data_ptr(), sink.data_ptr())      # warm-up
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                B.lp_debug_mfma_peak(stream, mode, blocks, iters, clk.data_ptr(), sink.data_ptr())
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 3
            c = clk.cpu().numpy().reshape(blocks, 2).astype("float64")
            ghz = float((c[:, 0] / c[:, 1]).mean()) * 0.1           # cycles per tick of the 100 MHz counter
            flops = blocks * 8.0 * iters * 40 * 32768
            out[f"{name}_{blocks}_workgroups"] = {"TFLOP/s": flops / (ms * 1e-3) / 1e12, "shader_clock_GHz": ghz, "ms": ms}
    return out


def measure_step_clock(ls, net, steps=12):
    """The shader clock while the local step runs: one workgroup of the synthetic MFMA kernel (it records shader-clock
    cycles and ticks of the constant 100 MHz counter) on a stream of its own beside the steps, about 1.5 ms long; the
    compute unit it takes is 1/256 of the chip."""
    import torch
    from paper_2112_05387_amd import binding as B
    dev = torch.device("cuda:0")
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    side = torch.cuda.Stream()
    probes = [torch.zeros(2, dtype=torch.int64, device=dev) for _ in range(steps)]
    B.lp_debug_mfma_peak(side.cuda_stream, 0, 1, 200, probes[0].data_ptr(), sink.data_ptr())
    torch.cuda.synchronize()
    for i in range(steps):
        one_step(ls, net)
        B.lp_debug_mfma_peak(side.cuda_stream, 0, 1, 2500, probes[i].data_ptr(), sink.data_ptr())
    torch.cuda.synchronize()
    ghz = [float(p[0].item()) / float(p[1].item()) * 0.1 for p in probes[2:]]
    B.lp_debug_mfma_peak(side.cuda_stream, 0, 1, 2500, probes[0].data_ptr(), sink.data_ptr())     # the same probe on an idle chip
    torch.cuda.synchronize()
    idle = float(probes[0][0].item()) / float(probes[0][1].item()) * 0.1
    return {"shader_clock_GHz_during_steps": sum(ghz) / len(ghz), "min": min(ghz), "max": max(ghz),
            "shader_clock_GHz_probe_alone": idle, "probes": len(ghz)}


def cpu_baseline(net_name, target_seconds=60.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: one local step of the same network, at
    the configuration's own mini-batch when the plain loops finish it within about a minute on the host's cores (the
    headline configuration does), else at a reduced one (the network, K and every layer shape are the configuration's)."""
    import workloads as wl
    from oracle import lpref
    from workloads import configs as cfg
    full = wl.make_config(net_name)
    # the plain double loops reach roughly 4 GFLOP/s per thread on the GPU machine's host; size the sample from that
    per_sample = cfg.conv_flops_step(full) / full.modules[0].N
    guess_rate = 4.0e9 * lpref.num_threads()
    batch = int(max(1, min(full.modules[0].N, target_seconds * guess_rate / per_sample)))
    if batch * 10 >= full.modules[0].N * 9:
        batch = full.modules[0].N
    net = wl.make_config(net_name, batch=batch)
    params = [wl.make_params(net, k) for k in range(net.K)]
    image, labels = wl.make_image(net), wl.make_labels(net)
    # auxiliary variables with the module-input shapes (values do not change the cost)
    xs = [image] + [wl.normal(net.seed, f"cpu_x{k}", (m.N, m.H, m.W, m.C)) for k, m in enumerate(net.modules) if k > 0]
    lams = None
    if net.al:
        lams = [wl.normal(net.seed, f"cpu_lam{k}", xs[k + 1].shape, net.lam_sigma) for k in range(net.K - 1)]
    t0 = time.perf_counter()
    if net.aux is not None:
        for j in range(net.K - 1):
            lpref.auxnet_forward(net.aux[j], image, wl.make_aux_params(net, j), net.bn_eps)
    out = lpref.local_step(net, xs, params, labels, lams, 1.0)
    if lams is not None:
        for k in range(net.K - 1):
            lpref.multiplier_update(lams[k], out["y"][k], xs[k + 1], net.step)
    dt = time.perf_counter() - t0
    return {"value": batch / dt, "unit": "samples/s", "cores": lpref.num_threads(), "kind": "oracle",
            "sample": f"one local step of {net_name} (all K={net.K} modules, every layer at its real width) at "
                      + (f"the configuration's mini-batch {batch}" if batch == full.modules[0].N else
                         f"mini-batch {batch} instead of {full.modules[0].N}") + f", float64 plain loops, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="wrn28_10")
    ap.add_argument("--batch", type=int, default=None, help="override the mini-batch (the result is then not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--steps-only", action="store_true",
                    help="skip what follows the timed steps (parameter-update timings): for rocprofv3 runs, whose summaries\n"
                         "then hold the kernels of the warm-up and timed steps alone")
    ap.add_argument("--kernel-table", action="store_true", help="print the per-kernel breakdown to stderr")
    ap.add_argument("--dump-launches", action="store_true", help="print every launch of the last timed step to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run three plain 256 MiB device copies (a known-size kernel that scales "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--lanes", default="default",
                    help="default: the library's concurrent stream lanes; single: every module on one stream; serial: the "
                         "launches of the default lanes (same grouping, same tile variants) issued one after another on "
                         "one stream, warm-up included (what the per-kernel rocprofv3 summaries are taken with); or one "
                         "digit 0..3 per module, e.g. 1200 (in all these cases the result is not the headline)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step into a HIP graph and time its replays (reported beside the eager step)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="run the step as lp_module_forward / lp_local_loss_grad / lp_module_backward / "
                         "lp_al_multiplier_update instead of the one lp_local_step call")
    ap.add_argument("--order", choices=["post", "pre"], default="post",
                    help="block order: post = conv-BN-ReLU (the headline configuration), pre = BN-ReLU-conv (Fig. 2)")
    ap.add_argument("--measure-peak", action="store_true",
                    help="also run the synthetic MFMA kernels (register operands only / with the kernels' LDS operand reads) "
                         "and report what the matrix cores of this device sustain, with the shader clock they ran at")
    ap.add_argument("--speedup-terms", action="store_true",
                    help="also time the terms of the paper's speed-up model (K = 1 network, single modules, interface "
                         "and AuxNet work) and add them to the JSON line")
    args = ap.parse_args()
    global SEPARATE_CALLS
    SEPARATE_CALLS = args.separate_calls
    if args.gpus != 1:
        print("bench.py: this build runs the local step of all K modules on ONE GPU; --gpus must be 1 "
              "(no multi-GPU figure is produced).", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2112_05387_amd import binding as B
    from workloads import configs as cfg

    net = wl.make_config(args.config, batch=args.batch)
    if args.order == "pre":
        cfg.with_order(net, "pre")
    N = net.modules[0].N
    ls = build_state(net)
    if args.lanes not in ("default", "serial"):
        ls.set_stream_lanes(None if args.lanes == "single" else [int(c) for c in args.lanes])
    if args.lanes == "serial":
        B.lp_profile_enable(ls.net, 2)
    for _ in range(args.warmup):
        one_step(ls, net)
    torch.cuda.synchronize()


    def timed_steps(profile):
        # EXACTLY --steps steps; profile 1: every grouped launch is bracketed by hipEvents on its own stream; profile 2:
        # the launches of all stream lanes are issued one after another on the caller's stream (durations alone)
        B.lp_profile_enable(ls.net, profile)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(args.steps):
            one_step(ls, net)
        ev1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        recs = B.lp_profile_fetch(ls.net) if profile else []
        B.lp_profile_enable(ls.net, 0)
        return wall, ev0.elapsed_time(ev1), recs

    # The timed region: the step as the library runs it (modules on concurrent stream lanes, no events between launches).
    # Kernels of different lanes overlap there, so a kernel's own duration is measured in a second pass over the same
    # steps: the SAME launches (same grouping per lane, same tile variants as in the timed region), enqueued one after
    # another on the caller's stream, each bracketed by hipEvents on that stream (lp_profile_enable(net, 2)).
    graph_ms = None
    if args.lanes == "serial":
        B.lp_profile_fetch(ls.net)                       # drop the warm-up's records
        wall_ms, gpu_ms, recs = timed_steps(2)
        iso_wall, gpu_iso = wall_ms, gpu_ms
    elif args.lanes == "single":
        wall_ms, gpu_ms, recs = timed_steps(1)           # one stream: the timed region itself carries the events
        iso_wall, gpu_iso = wall_ms, gpu_ms
        if args.graph:
            graph_ms = time_graph_replays(ls, net, args.steps)
    else:
        wall_ms, gpu_ms, _ = timed_steps(0)
        if args.graph:
            graph_ms = time_graph_replays(ls, net, args.steps)
        one_step(ls, net)
        iso_wall, gpu_iso, recs = timed_steps(2)
    ms_per_step = wall_ms / args.steps
    iso_ms_per_step = iso_wall / args.steps

    # per-kernel aggregation (kind, tile configuration)
    agg = {}
    for r in recs:
        a = agg.setdefault((r["kind"], r["cfg"]), {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0, "blocks": 0, "cu_ms": 0.0})
        a["ms"] += r["ms"]; a["flops"] += r["flops"]; a["bytes"] += r["bytes"]; a["launches"] += 1; a["blocks"] += r["blocks"]
        a["cu_ms"] += r["ms"] * min(1.0, r["blocks"] / N_CUS)
    conv_ms = sum(a["ms"] for (k, _), a in agg.items() if k in (2, 10))
    conv_flops = sum(a["flops"] for (k, _), a in agg.items() if k in (2, 10))
    (dk, dcfg), dom = max(agg.items(), key=lambda kv: kv[1]["ms"])
    peak = PEAK_TFLOPS[net.dtype]
    # a convolution whose algorithmic intensity lies under the ridge of its dtype (peak flop/s over peak bytes/s: 312 flop/B
    # in bf16, 20 in fp32) is bounded by HBM, like the elementwise passes: the 16- and 32-channel layers of ResNet-20 / -56
    ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)
    if dk in (2, 10) and dom["flops"] >= ridge * dom["bytes"]:
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak}
        if dom["cu_ms"] > 0 and dcfg >= 8:       # the direct-to-LDS kernels: one workgroup per compute unit
            # a lane's launch is sized to share the chip with the other lanes: workgroups per launch, and the rate per
            # compute unit it occupies (one workgroup per CU) against a CU's share of the peak
            roof["workgroups_per_launch"] = dom["blocks"] / dom["launches"]
            roof["frac_on_occupied_cus"] = dom["flops"] / (dom["cu_ms"] * 1e-3) / 1e12 / peak
            # ... and what all convolutions of the step reach in the timed region itself, where the lanes' launches fill the
            # chip together (every other kernel of the step included in the time)
            roof["frac_all_convs_over_timed_step"] = cfg.conv_flops_step(net) / (ms_per_step * 1e-3) / 1e12 / peak
    else:
        achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS}
    roof.update({"traffic": None, "kernel": f"{B.KIND_NAMES[dk]} cfg{dcfg}", "launches_per_step": dom["launches"] / args.steps,
                 "avg_launch_ms": dom["ms"] / dom["launches"], "share_of_gpu_time": dom["ms"] / max(gpu_iso, 1e-9),
                 "measured": "hipEvents around every launch in a second pass over the same steps: the launches of the timed "
                             "region (same grouping per stream lane, same tile variants), one after another on one stream"})
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            roof["traffic"] = json.load(f).get(f"{args.config}:{B.KIND_NAMES[dk]} cfg{dcfg}")
    if args.dump_launches:
        per = len(recs) // args.steps
        for r in recs[-per:]:
            tf = r["flops"] / (r["ms"] * 1e-3) / 1e12 if r["ms"] > 0 else 0.0
            print(f"    {B.KIND_NAMES[r['kind']]:24s} cfg{r['cfg']} nprob {r['nprob']:2d}  {r['ms'] * 1e3:9.1f} us  {r['flops'] / 1e9:9.2f} GFLOP  {tf:8.1f} TFLOP/s"
                  f"  {r['bytes'] / 1e6:9.2f} MB(alg)", file=sys.stderr)
    if args.kernel_table:
        for (k, c), a in sorted(agg.items(), key=lambda kv: -kv[1]["ms"]):
            tf = a["flops"] / (a["ms"] * 1e-3) / 1e12 if a["ms"] > 0 else 0.0
            gb = a["bytes"] / (a["ms"] * 1e-3) / 1e9 if a["ms"] > 0 else 0.0
            print(f"  {B.KIND_NAMES[k]:24s} cfg{c} launches/step {a['launches'] / args.steps:6.1f}  ms/step {a['ms'] / args.steps:8.3f}"
                  f"  TFLOP/s {tf:8.1f}  GB/s(alg) {gb:8.1f}", file=sys.stderr)
        print(f"  one stream: GPU time/step by events {gpu_iso / args.steps:.3f} ms; timed region ({args.lanes} lanes): "
              f"{gpu_ms / args.steps:.3f} ms by events, wall {ms_per_step:.3f} ms", file=sys.stderr)

    out = {
        "metric": "module-parallel local-step samples/s (all K modules); conv TFLOP/s vs MFMA peak",
        "value": N / (ms_per_step * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": net.dtype, "data": "synthetic",
        "config": {"workload": f"{net.name} local step, K={net.K} modules, batch {N}, "
                               f"{'augmented Lagrangian' if net.al else 'penalty'}, rho={net.rho}"
                               f"{', AuxNet forward included' if net.aux is not None else ''}"
                               f"{', pre-activation block order' if args.order == 'pre' else ''}"},
        "conv_tflops": conv_flops / (conv_ms * 1e-3) / 1e12 if conv_ms > 0 else None,
        "conv_frac_of_mfma_peak": (conv_flops / (conv_ms * 1e-3) / 1e12) / peak if conv_ms > 0 else None,
        "conv_tflop_per_step": cfg.conv_flops_step(net) / 1e12,
        "gpu_ms_per_step_events": gpu_ms / args.steps,
        "stream_lanes": args.lanes, "ms_per_step_one_stream_with_events": iso_ms_per_step,
        "step_conv_tflops": cfg.conv_flops_step(net) / (ms_per_step * 1e-3) / 1e12,
        "roofline": roof,
    }
    if not args.steps_only:
        # the parameter update that follows a step (not part of `value`): momentum form, fp32 velocity, timed by events
        vel = [torch.zeros_like(d) for d in ls.dparams]
        ls.sgd_update(0.0, 0.9, 5e-4, velocity=vel)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            ls.sgd_update(0.0, 0.9, 5e-4, velocity=vel)
        e1.record()
        torch.cuda.synchronize()
        sgd_ms = e0.elapsed_time(e1) / 10
        sgd_bytes = sum(int(t.numel) * ((4 if t.dtype == B.LP_BF16 else 8) + 12) for tab in ls.tables for t in tab)
        if graph_ms is not None:
            out["hip_graph"] = {"ms_per_step": graph_ms, "samples/s": N / (graph_ms * 1e-3),
                                "note": "the step captured once (stream lanes included) and replayed; `value` is the eager step"}
        out["sgd_update"] = {"ms": sgd_ms, "GB/s(alg)": sgd_bytes / (sgd_ms * 1e-3) / 1e9, "form": "momentum 0.9, weight decay 5e-4"}
        # the same update inside the backward pass (epilogues of the filter-gradient kernels), lr = 0 so that the parameters
        # stay what they are: K steps with it against K steps followed by the pass above
        ls.set_fused_update(True, 0.0, 0.9, 5e-4, velocity=vel)
        one_step(ls, net)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step(ls, net)
        torch.cuda.synchronize()
        inside_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ls.set_fused_update(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step(ls, net)
            ls.sgd_update(0.0, 0.9, 5e-4, velocity=vel)
        torch.cuda.synchronize()
        behind_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["step_with_update"] = {"inside_backward_ms": inside_ms, "as_a_pass_behind_the_step_ms": behind_ms,
                                   "note": "not part of `value` (the metric is the local step); same box, same run"}
    if args.measure_peak:
        out["step_clock"] = measure_step_clock(ls, net)
    ls.close()
    if args.measure_peak:
        out["measured_mfma_peak"] = measure_peak()
    if args.speedup_terms:
        out["speedup_model"] = speedup_terms(args.config, args.batch, max(3, args.steps // 2))
    if args.calibrate_copy:
        src = torch.full((64 << 20,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
