#!/usr/bin/env python3
"""Benchmark of the SpeCa sampling step on one MI355X.

Workload (configuration 3): DiT-XL/2-shaped class-conditional model, bf16, 28 blocks,
hidden 1152, 16 heads, 256 tokens, batch 8 with classifier-free guidance 1.5 (16 rows),
DDIM, Taylor order 2, forced interval 5, thresholds tau0 = 0.1 decaying geometrically to
0.02; seed-generated N(0, 0.02^2) weights and N(0,1) latents (synthetic).

A "step" is one denoising step of the whole batch through speca_sample: schedule,
speculative attempt (forecast + verify block + Eq. 4), fallback full step with cache
refresh, solver update.  --steps K times exactly one K-step trajectory (default 50, the
paper's setting), after one untimed W-step trajectory.  Inputs are resident in HBM before
the timed region.

Prints ONE JSON line.  `roofline` describes the dominant kernel class of the timed
trajectory, measured with HIP events on the library's stream in a second, identical
trajectory (event pairs around every launch would perturb the throughput figure);
`cpu_baseline` times the NumPy oracle on a bounded sample of the same workload."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E


# L2 <-> fabric bytes per launch from rocprofv3 counter runs of these same workloads
# (2 x FETCH_SIZE + WRITE_SIZE in bytes, the factor 2 from a plain copy of known size under the
# same counters; summed over the kernels of the class and divided by the number of GEMMs the library was asked
# for, which is what `launches` counts: the fc1 GEMM of configuration 3 runs as two kernels).  Counters cannot be read from
# inside the process, so the figures are carried here; profiles/hbm_counters.txt holds the runs.
MEASURED_TRAFFIC = {
    ("dit_xl2", "gemm"): 106.7e6,                 # ring layout of the cache (the default)
    ("dit_xl2", "gemm", "differences"): 134.1e6,
    ("forecast", "forecast"): 528.5e6,
}


def cpu_baseline(shape, weights, seconds_budget=30.0):
    """The oracle as it stands, on the host cores: one full-compute step of one guided
    sample (2 of the 16 rows), scaled to the 16-row batch step."""
    from oracle import dit as odit
    import speca_inputs as si
    om = odit.DiTOracle(shape, weights)
    x = si.make_latents(1, shape.in_channels, shape.latent_hw, 0)
    xr = np.repeat(x, 2, axis=0)
    t0 = time.time()
    om.forward(xr, 980.0, [1, shape.num_classes])
    dt = time.time() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": 1.0 / (8.0 * dt), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one full-compute step of one guided sample (2 of 16 rows, float64 NumPy) took {dt:.2f} s; "
                      "scaled x8 to the 16-row batch step; speculative steps are not timed on the CPU"}


def bench_forecast(args):
    """Configuration 2: the HBM-bound kernels in isolation.  Cache of 28 slots x 8 rows x 256
    tokens x 1152 hidden in bf16, order 2, built from 3 reference steps (0, 4, 8) of a seeded
    quadratic-in-step trajectory plus noise; a step = materialised forecast of every slot at
    k = 1 + Eq. 4 verification of the last slot against a seeded perturbed target."""
    import torch
    import speca_inputs as si
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    slots, B, T, D, m = 28, 8, 256, 1152, 2
    ctx = sp.Context(sp.cache_only_desc(slots, T, D, bd.BF16))
    ctx.init_cache(sp.make_cfg(order=m, interval=4, layout=_layout(args)), B)
    rows = list(range(B))
    for s_, f in zip([0, 4, 8], si.feature_trajectory(slots, B, T, D, [0, 4, 8], seed=0, dtype="bf16")):
        ctx.refresh(s_, rows, torch.from_numpy(f).cuda().bfloat16())
    out = torch.empty((slots, B, T, D), dtype=torch.bfloat16, device="cuda")
    ctx.forecast(9, rows, out)
    pred = out[slots - 1].float().cpu().numpy()
    truth = torch.from_numpy(si.perturbed_target(pred, si.VERIFY_DELTAS, seed=0, dtype="bf16")).cuda().bfloat16()
    last = out[slots - 1]

    def step():
        ctx.forecast(9, rows, out)
        return ctx.verify(last, truth, tau=0.05)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        err, acc = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile_begin()
    for _ in range(args.steps):
        step()
    prof = ctx.profile_end()
    p = prof["forecast"]
    ach = p["bytes"] / (p["ms"] * 1e-3) / 1e9
    v = prof["verify"]
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import speca_core as core
        feats = si.feature_trajectory(1, 1, T, D, [0, 4, 8], seed=0, dtype="bf16")
        c = core.make_cache(args.layout, 1, m, "taylor", "bf16")
        for s_, f in zip([0, 4, 8], feats):
            c.refresh(s_, [f[0, 0]])
        t1 = time.perf_counter()
        n = 0
        while time.perf_counter() - t1 < 10.0:
            core.bf16_round(c.forecast(9, 0)); n += 1
        dtc = (time.perf_counter() - t1) / n
        cpu = {"value": 1.0 / (dtc * slots * B), "unit": "steps/s", "cores": 1, "kind": "oracle",
               "sample": f"forecast of one (slot,row) tensor of {T * D} elements took {dtc * 1e3:.2f} ms (float64 NumPy, single thread); "
                         f"scaled x{slots * B} to all slots and rows"}
    out_json = {
        "metric": "forecast_verify_steps_per_s", "value": args.steps / dt, "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 2: forecast + verify in isolation, 28 slots x 8 rows x 256 tokens x 1152 hidden, bf16, order 2",
                   "slots": slots, "rows": B, "tokens": T, "hidden": D, "order": m},
        "roofline": {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBPS,
                     "traffic": MEASURED_TRAFFIC[("forecast", "forecast")], "kernel": "forecast", "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / p["launches"],
                     "bytes_per_launch": p["bytes"] / p["launches"]},
        "cpu_baseline": cpu,
        "extras": {"accepted": [bool(a) for a in acc], "errors": [float(e) for e in err],
                   "verify_avg_launch_us": 1e3 * v["ms"] / max(v["launches"], 1), "verify_bytes_per_launch": v["bytes"] / max(v["launches"], 1)},
    }
    print(json.dumps(out_json))


def bench_copy(args):
    """A plain device copy of known size (512 MiB read + 512 MiB written per step): the
    calibration run for the FETCH_SIZE / WRITE_SIZE counters and a measured HBM ceiling."""
    import torch
    n = 512 * 1024 * 1024 // 2
    a = torch.empty(n, dtype=torch.bfloat16, device="cuda").normal_()
    b = torch.empty_like(a)
    for _ in range(max(args.warmup, 1)):
        b.copy_(a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        b.copy_(a)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    gbps = 2 * n * 2 / dt / 1e9
    print(json.dumps({"metric": "copy_GBps", "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
                      "data": "synthetic", "config": {"workload": "plain copy, 512 MiB in + 512 MiB out"},
                      "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS, "traffic": 2.0 * n * 2},
                      "cpu_baseline": None}))


def device_mmdit_weights(shape, seed=0, std=0.02):
    """Full-size MMDiT weights drawn on the device (12 G parameters do not fit a host-side
    NumPy draw in reasonable time): N(0, std^2) in bf16 from a seeded device generator, RMS-norm
    scales 1 + N(0, std^2), rotary tables from the shared input module."""
    import torch
    import speca_inputs as si
    g = torch.Generator(device="cuda").manual_seed(seed)
    out = {}
    for name, shp in si.mmdit_param_shapes(shape).items():
        t = torch.randn(shp, generator=g, device="cuda", dtype=torch.float32) * std
        if name.endswith("norm"):
            t = t + 1.0
        out[name] = t.to(torch.bfloat16).contiguous()
        del t
    c, sn = si.rope_tables(shape)
    out["rope_cos"] = torch.from_numpy(c).cuda().contiguous()
    out["rope_sin"] = torch.from_numpy(sn).cuda().contiguous()
    return out


def bench_mmdit(args, which):
    """Configurations 4 / 5: FLUX-shaped (4096 image + 512 text tokens) or HunyuanVideo-shaped
    (27030 video + 256 text tokens) rectified-flow MMDiT, bf16, batch 1, Euler steps, Taylor
    order 2, interval 5.  Weights are seeded random on the device; there is no CPU oracle at this
    size (parity is tested on reduced shapes), so the run is checked through properties only:
    finite latents, tau = 0 gives an all-full schedule, tau = inf the fixed pattern."""
    import torch
    import speca_inputs as si
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    shape = si.mmdit_flux() if which == "flux" else si.mmdit_hunyuan()
    w = device_mmdit_weights(shape)
    print(f"bench.py: {which} weights on the device", file=sys.stderr, flush=True)
    ctx = sp.Context(sp.mmdit_desc(shape), w)
    order = 2
    ctx.init_cache(sp.make_cfg(order=order, interval=args.interval, layout=_layout(args)), 1)
    lat = si.make_video_latents(1, shape, 0)
    txt, vec = si.make_text(1, shape, 0)
    td, vd = torch.from_numpy(txt).cuda().bfloat16(), torch.from_numpy(vec).cuda().bfloat16()

    def run(steps, tau, profile=False):
        ts, sg = si.flow_tables(steps)
        x = torch.from_numpy(lat).cuda()
        torch.cuda.synchronize()
        if profile:
            ctx.profile_begin()
        t0 = time.perf_counter()
        tr = ctx.sample(x, ts, sg, tau, solver_kind=bd.SOLVER_FLOW, txt=td, pooled=vd)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = ctx.profile_end() if profile else None
        assert bool(torch.isfinite(x).all()), "non-finite latents"
        print(f"bench.py: {which} trajectory of {steps} steps done in {dt:.1f} s", file=sys.stderr, flush=True)
        return dt, tr, prof, x

    K = args.steps
    tau = bd.tau_geometric(args.tau0, args.tau_end / args.tau0, K)
    if args.warmup > 0:
        run(args.warmup, bd.tau_geometric(args.tau0, args.tau_end / args.tau0, args.warmup))
    dt, tr, _, x_timed = run(K, tau)
    _, _, prof, x_prof = run(K, tau, profile=True)
    assert torch.equal(x_timed, x_prof), "the same trajectory gave different bits on a second run"
    dt_plain, tr_plain, _, _ = run(K, np.zeros(K, np.float32))
    dt_acc, tr_acc, _, _ = run(K, np.full(K, np.inf, np.float32))
    assert tr_plain["n_spec"] == 0 and tr_acc["kind"][0].tolist() == [0 if i % args.interval == 0 else 1 for i in range(K)]
    dom = max(("gemm", "attention", "forecast", "verify", "other"), key=lambda k: prof[k]["ms"])
    p = prof[dom]
    ach = p["flops"] / (p["ms"] * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
            "kernel": dom, "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / max(p["launches"], 1),
            "flops_per_launch": p["flops"] / max(p["launches"], 1)}

    def cls(name, peak, key, scale):
        q = prof[name]
        if not q["launches"]:
            return None
        a = q[key] / (q["ms"] * 1e-3) / scale
        return {"launches": q["launches"], "ms": q["ms"], "achieved": a, "frac": a / peak}

    out = {
        "metric": "denoising_steps_per_s", "value": K / dt, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": ("config 4: FLUX-shaped MMDiT 1024x1024" if which == "flux" else "config 5: HunyuanVideo-shaped MMDiT 480p 2s")
                   + ", bf16, batch 1, Euler, Taylor order 2", "tokens": shape.tokens, "hidden": shape.hidden,
                   "blocks": [shape.depth_dual, shape.depth_single], "order": order, "interval": args.interval, "tau0": args.tau0,
                   "tau_end": args.tau_end, "cache_layout": args.layout, "parallelism": "single GPU"},
        "roofline": roof, "cpu_baseline": None,
        "extras": {"images_per_s": 1.0 / dt, "accept_rate": tr["n_spec"] / float(K), "n_full": tr["n_full"], "n_spec": tr["n_spec"],
                   "n_reject": tr["n_reject"], "errors": [None if np.isnan(e) else float(e) for e in tr["err"][0, :, 0]],
                   "plain_sampling_steps_per_s": K / dt_plain, "all_accepted_steps_per_s": K / dt_acc,
                   "all_accepted_accept_rate": tr_acc["n_spec"] / float(K),
                   "gemm_mfma_TFLOPs": cls("gemm", PEAK_BF16_TFLOPS, "flops", 1e12),
                   "attention_mfma_TFLOPs": cls("attention", PEAK_BF16_TFLOPS, "flops", 1e12),
                   "forecast_hbm_GBps": cls("forecast", PEAK_HBM_GBPS, "bytes", 1e9),
                   "verify_hbm_GBps": cls("verify", PEAK_HBM_GBPS, "bytes", 1e9), "other_ms": prof["other"]["ms"]},
    }
    print(json.dumps(out))


def _layout(args):
    from paper_2509_11628_amd import binding as bd
    return bd.CACHE_RING if args.layout == "ring" else bd.CACHE_DIFFERENCES


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", choices=["dit_xl2", "forecast", "copy", "flux", "hunyuan"], default="dit_xl2")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tau0", type=float, default=0.1)
    ap.add_argument("--tau-end", type=float, default=0.02)
    ap.add_argument("--interval", type=int, default=5)
    ap.add_argument("--layout", choices=["differences", "ring"], default="ring",
                    help="what the cache planes hold: the differences of Eq. 3, or the raw features of the last m+1 full steps")
    ap.add_argument("--lanes", type=int, default=4, help="row groups of a step that run side by side (1 = serial)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import speca_inputs as si
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.workload == "forecast":
        return bench_forecast(args)
    if args.workload == "copy":
        return bench_copy(args)
    if args.workload in ("flux", "hunyuan"):
        return bench_mmdit(args, args.workload)

    shape = si.dit_xl2("bf16")
    B, cfg_scale, order = 8, 1.5, 2
    weights = si.make_dit_weights(shape, 0)
    ctx = sp.Context(sp.dit_desc(shape), sp.to_device(weights, bd.BF16))
    ctx.init_cache(sp.make_cfg(order=order, interval=args.interval, layout=_layout(args)), 2 * B)
    ctx.set_lanes(args.lanes)          # the event-profiled pass below always runs serially (clean per-kernel times)
    lat = si.make_latents(B, shape.in_channels, shape.latent_hw, 0)
    lab = si.make_labels(B, shape.num_classes, 0)

    def run(steps, tau=None, profile=False):
        ts, ab = si.ddim_tables(steps)
        if tau is None:
            tau = bd.tau_geometric(args.tau0, args.tau_end / args.tau0, steps)
        x = torch.from_numpy(lat).cuda()
        torch.cuda.synchronize()
        if profile:
            ctx.profile_begin()
        t0 = time.perf_counter()
        tr = ctx.sample(x, ts, ab, tau, cfg_scale=cfg_scale, labels=lab)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = ctx.profile_end() if profile else None
        return dt, tr, prof, x

    if args.warmup > 0:
        run(args.warmup)
    K = args.steps
    dt, tr, _, x_timed = run(K)
    _, _, prof, x_prof = run(K, profile=True)
    # the profiled pass runs the row groups serially, the timed one side by side: same bits required
    assert torch.equal(x_timed, x_prof), "lanes changed the result"
    # the same trajectory without speculation (tau = 0: plain sampling) and with every attempt accepted
    dt_plain, _, _, _ = run(K, tau=np.zeros(K, np.float32))
    dt_acc, tr_acc, _, _ = run(K, tau=np.full(K, np.inf, np.float32))

    dom = max(("gemm", "attention", "forecast", "verify", "other"), key=lambda k: prof[k]["ms"])
    p = prof[dom]
    if dom in ("gemm", "attention"):
        ach = p["flops"] / (p["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                "traffic": None}
    else:
        ach = p["bytes"] / (p["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBPS, "traffic": None}
    roof["traffic"] = MEASURED_TRAFFIC.get(("dit_xl2", dom, args.layout), MEASURED_TRAFFIC.get(("dit_xl2", dom)) if args.layout == "ring" else None)
    roof["measured_on"] = "same trajectory, row groups run serially on one stream (per-kernel event times need no overlap); value is timed with lanes"
    roof.update({"kernel": dom, "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / max(p["launches"], 1),
                 "flops_per_launch": p["flops"] / max(p["launches"], 1), "bytes_per_launch": p["bytes"] / max(p["launches"], 1)})

    def cls(name, peak, key, scale):
        q = prof[name]
        if not q["launches"]:
            return None
        a = q[key] / (q["ms"] * 1e-3) / scale
        return {"launches": q["launches"], "ms": q["ms"], "achieved": a, "frac": a / peak}

    extras = {
        "images_per_s": B * (K / dt) / K,
        "accept_rate": tr["n_spec"] / float(B * K), "n_full": tr["n_full"], "n_spec": tr["n_spec"], "n_reject": tr["n_reject"],
        "plain_sampling_steps_per_s": K / dt_plain,
        "all_accepted_steps_per_s": K / dt_acc, "all_accepted_accept_rate": tr_acc["n_spec"] / float(B * K),
        "gemm_mfma_TFLOPs": cls("gemm", PEAK_BF16_TFLOPS, "flops", 1e12),
        "attention_mfma_TFLOPs": cls("attention", PEAK_BF16_TFLOPS, "flops", 1e12),
        "forecast_hbm_GBps": cls("forecast", PEAK_HBM_GBPS, "bytes", 1e9),
        "verify_hbm_GBps": cls("verify", PEAK_HBM_GBPS, "bytes", 1e9),
        "other_ms": prof["other"]["ms"],
    }
    # Speed-up model of the paper's complexity analysis, S = 1 / (1 - alpha (1 - gamma - overhead)), beside
    # what was measured: alpha from the all-accepted run, gamma = 1 / blocks nominal; the measured cost of an
    # accepted speculative step relative to a full one (verify block + forecast + everything else) replaces
    # gamma + overhead in the second prediction.
    t_full = dt_plain / K
    n_spec_steps = tr_acc["n_spec"] / float(B)
    n_full_steps = K - n_spec_steps
    t_spec = (dt_acc - n_full_steps * t_full) / max(n_spec_steps, 1.0)
    alpha = n_spec_steps / K
    gamma = 1.0 / shape.depth
    extras["speedup_model"] = {
        "alpha": alpha, "gamma_nominal": gamma, "predicted_nominal": 1.0 / (1.0 - alpha * (1.0 - gamma)),
        "spec_step_cost_ratio_measured": t_spec / t_full,
        "predicted_with_measured_cost": 1.0 / (1.0 - alpha * (1.0 - t_spec / t_full)),
        "measured_vs_plain": dt_plain / dt_acc,
    }
    out = {
        "metric": "denoising_steps_per_s", "value": K / dt, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 3: DiT-XL/2-shaped bf16, batch 8 x CFG 1.5 (16 rows), 256 tokens, DDIM, Taylor order 2",
                   "global_batch": B, "rows": 2 * B, "tokens": shape.tokens, "hidden": shape.hidden, "blocks": shape.depth,
                   "order": order, "interval": args.interval, "tau0": args.tau0, "tau_end": args.tau_end, "lanes": args.lanes,
                   "cache_layout": args.layout, "parallelism": "single GPU"},
        "roofline": roof,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(shape, weights),
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
