#!/usr/bin/env python3
"""Benchmark of the SpeCa sampling step on one MI355X.

Headline workload (configuration 3): DiT-XL/2-shaped class-conditional model, bf16, 28 blocks,
hidden 1152, 16 heads, 256 tokens, batch 8 with classifier-free guidance 1.5 (16 rows), DDIM,
Taylor order 2, forced interval 5, thresholds tau0 = 0.1 decaying geometrically to 0.02;
seed-generated N(0, 0.02^2) weights and N(0,1) latents (synthetic).

A "step" is one denoising step of the whole batch through speca_sample: schedule, speculative
attempt (forecast + verify block + Eq. 4), fallback full step with cache refresh, solver update.
--steps K times exactly one K-step trajectory, after one untimed W-step trajectory.  Inputs are
resident in HBM before the timed region.

Prints ONE JSON line.  `roofline` describes the dominant kernel class of the timed trajectory,
measured with HIP events on the library's stream in a second, identical trajectory (event pairs
around every launch would perturb the throughput figure); `cpu_baseline` times the NumPy oracle on
a bounded sample of the same workload.  `extras` carries, from the same process: the 50-step
images/s figure, the plain / all-accepted / calibrated-threshold / mixed-row runs of configuration 3
with the speed-up model (rejected attempts included), configuration 2's forecast kernel and the
256 MB verification stress shape, the GEMMs at the sub-batch sizes per-sample rejection produces,
and short runs of configurations 4 and 5 (FLUX- and HunyuanVideo-shaped) with their own property
checks.  --no-extras skips everything beyond configuration 3 itself (profiling runs)."""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E


def _log(msg):
    print(f"bench.py: {msg}", file=sys.stderr, flush=True)


# ---- counter-measured traffic -----------------------------------------------------------------------
# L2 <-> fabric bytes per launch cannot be read from inside the process: they come from rocprofv3 counter runs of
# this same file (2 x FETCH_SIZE + WRITE_SIZE, the factor 2 from a plain copy of known size under the same
# counters), whose summary profiles/hbm_counters.txt records them in lines
#   "# roofline.traffic <workload> <class> <layout> = <bytes> ; kernel sources <hash>"
# together with the hash of the kernel sources they were measured on.  A figure measured on other sources is
# not reported (traffic: null, with a note).


def kernel_sources_hash() -> str:
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2509_11628_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, cls: str, layout: str):
    """-> (bytes per launch or None, note)."""
    path = os.path.join(ROOT, "profiles", "hbm_counters.txt")
    try:
        txt = open(path).read()
    except OSError:
        return None, "profiles/hbm_counters.txt is missing"
    m = re.search(r"# roofline\.traffic %s %s %s = ([0-9.eE+]+) ; kernel sources ([0-9a-f]+)" % (workload, cls, layout), txt)
    if not m:
        return None, "no counter run recorded for this workload / class / layout"
    if m.group(2) != kernel_sources_hash():
        return None, f"counter run was taken on kernel sources {m.group(2)}, these are {kernel_sources_hash()}: not reported"
    return float(m.group(1)), f"profiles/hbm_counters.txt, kernel sources {m.group(2)}"


def _threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(shape, weights):
    """The oracle as it stands, on the host cores: one full-compute step and one speculative attempt of one
    guided sample (2 of the 16 rows); the step rate scales the full step to the 16-row batch."""
    from oracle import dit as odit, sampler as osamp, speca_core as core
    import speca_inputs as si
    om = odit.DiTOracle(shape, weights)
    x = si.make_latents(1, shape.in_channels, shape.latent_hw, 0)
    xr = np.repeat(x, 2, axis=0)
    labels = [1, shape.num_classes]
    cache = core.make_cache("ring", om.n_slots, 2, "taylor", "bf16")
    t0 = time.time()
    osamp.full_step(om, cache, xr, 980.0, labels, 0)
    dt = time.time() - t0
    t1 = time.time()
    osamp.speculative_attempt(om, cache, osamp.SpecaConfig(order=2, interval=5, cache_store="bf16", cache_layout="ring"), xr, 960.0, labels, 1,
                              np.float32(np.inf))
    ds = time.time() - t1
    return {"value": 1.0 / (8.0 * dt), "unit": "steps/s", "cores": _threads(), "kind": "oracle",
            "sample": f"one guided sample (2 of 16 rows, float64 NumPy): full-compute step with cache refresh {dt:.2f} s, accepted speculative "
                      f"attempt (forecast of 56 slots, fold, verify block, Eq. 4, finish) {ds:.2f} s; value = full step scaled x8 to the 16-row batch",
            "full_step_s": dt, "speculative_attempt_s": ds, "speculative_over_full": ds / dt}


def _cls(prof, name, peak, key, scale):
    q = prof[name]
    if not q["launches"]:
        return None
    a = q[key] / (q["ms"] * 1e-3) / scale
    return {"launches": q["launches"], "ms": q["ms"], "achieved": a, "frac": a / peak, "avg_launch_us": 1e3 * q["ms"] / q["launches"]}


def _classes(prof):
    return {"gemm_mfma_TFLOPs": _cls(prof, "gemm", PEAK_BF16_TFLOPS, "flops", 1e12),
            "attention_mfma_TFLOPs": _cls(prof, "attention", PEAK_BF16_TFLOPS, "flops", 1e12),
            "forecast_hbm_GBps": _cls(prof, "forecast", PEAK_HBM_GBPS, "bytes", 1e9),
            "verify_hbm_GBps": _cls(prof, "verify", PEAK_HBM_GBPS, "bytes", 1e9),
            "other_ms": prof["other"]["ms"]}


# ---- configuration 2: the HBM-bound kernels in isolation ------------------------------------------------


def forecast_verify(args, steps, warmup, with_cpu):
    """Cache of 28 slots x 8 rows x 256 tokens x 1152 hidden in bf16, order 2, built from 3 reference steps (0, 4, 8)
    of a seeded quadratic-in-step trajectory plus noise; a step = materialised forecast of every slot at k = 1 +
    Eq. 4 verification of the last slot against a seeded perturbed target.  Also the verification stress shape:
    all 28 slots x 8 rows as 224 rows of one reduction (2 x 132 MB), which shows what the reduction kernels stream
    at when the launch is not latency-bound."""
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

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        err, acc = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile_begin()
    for _ in range(steps):
        step()
    prof = ctx.profile_end()
    # stress shape of the reduction: every slot's forecast against a second tensor of the same size
    allp = out.reshape(slots * B, T * D)
    allt = (allp.float() * 1.01).to(torch.bfloat16)
    e_all, _ = ctx.verify(allp, allt)
    assert np.all(np.isfinite(e_all)) and float(np.max(np.abs(e_all - 0.01))) < 3e-3, e_all
    ctx.profile_begin()
    for _ in range(10):
        ctx.verify(allp, allt)
    pv = ctx.profile_end()["verify"]
    stress = pv["bytes"] / (pv["ms"] * 1e-3) / 1e9
    p, v = prof["forecast"], prof["verify"]
    ach = p["bytes"] / (p["ms"] * 1e-3) / 1e9
    cpu = None
    if with_cpu:
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
    traffic, note = measured_traffic("forecast", "forecast", args.layout)
    res = {
        "steps_per_s": steps / dt, "ms_per_step": 1e3 * dt / steps,
        "forecast": {"achieved_GBps": ach, "frac": ach / PEAK_HBM_GBPS, "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / p["launches"],
                     "bytes_per_launch": p["bytes"] / p["launches"], "traffic": traffic, "traffic_source": note},
        "verify_real_shape": {"avg_launch_us": 1e3 * v["ms"] / max(v["launches"], 1), "bytes_per_launch": v["bytes"] / max(v["launches"], 1),
                              "note": "2 x 4.7 MB: launch latency, not bandwidth"},
        "verify_stress_shape": {"rows": slots * B, "elems_per_row": T * D, "bytes_per_call": pv["bytes"] / 10, "achieved_GBps": stress,
                                "frac": stress / PEAK_HBM_GBPS, "avg_call_us": 1e3 * pv["ms"] / 10,
                                "note": "224 rows x 294912 bf16 elements, prediction and truth read once: 264 MB per call (one partial-sum launch + one final kernel)"},
        "accepted": [bool(a) for a in acc], "errors": [float(e) for e in err], "cpu": cpu,
    }
    ctx.close()
    del out, truth, allp, allt
    torch.cuda.empty_cache()
    return res


def bench_forecast(args):
    r = forecast_verify(args, args.steps, args.warmup, not args.no_cpu_baseline)
    f = r["forecast"]
    print(json.dumps({
        "metric": "forecast_verify_steps_per_s", "value": r["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 2: forecast + verify in isolation, 28 slots x 8 rows x 256 tokens x 1152 hidden, bf16, order 2",
                   "slots": 28, "rows": 8, "tokens": 256, "hidden": 1152, "order": 2},
        "roofline": {"bound": "hbm", "achieved": f["achieved_GBps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": f["frac"],
                     "traffic": f["traffic"], "traffic_source": f["traffic_source"], "kernel": "forecast", "launches": f["launches"],
                     "avg_launch_us": f["avg_launch_us"], "bytes_per_launch": f["bytes_per_launch"]},
        "cpu_baseline": r["cpu"],
        "extras": {k: r[k] for k in ("accepted", "errors", "verify_real_shape", "verify_stress_shape")},
    }))


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


# ---- configurations 4 / 5 --------------------------------------------------------------------------------


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


def mmdit_run(args, which, K, warmup, full=True):
    """FLUX-shaped (4096 image + 512 text tokens) or HunyuanVideo-shaped (27030 video + 256 text tokens)
    rectified-flow MMDiT, bf16, batch 1, Euler steps, Taylor order 2, interval 5.  Weights are seeded random on the
    device; a CPU oracle at this size is out of reach (the kernels are parity-tested at these sizes on sampled
    outputs, the model path on reduced shapes), so the run is checked through properties: finite latents, identical
    bits on a second run, tau = 0 gives an all-full schedule, tau = inf the fixed pattern.  full = False: only the
    timed and the event-profiled trajectory plus one all-accepted trajectory (the long configuration 5)."""
    import torch
    import speca_inputs as si
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    shape = si.mmdit_flux() if which == "flux" else si.mmdit_hunyuan()
    w = device_mmdit_weights(shape)
    _log(f"{which} weights on the device")
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
        _log(f"{which} trajectory of {steps} steps done in {dt:.1f} s")
        return dt, tr, prof, x

    tau = bd.tau_geometric(args.tau0, args.tau_end / args.tau0, K)
    if warmup > 0:
        run(warmup, bd.tau_geometric(args.tau0, args.tau_end / args.tau0, warmup))
    dt, tr, _, x_timed = run(K, tau)
    _, _, prof, x_prof = run(K, tau, profile=True)
    assert torch.equal(x_timed, x_prof), "the same trajectory gave different bits on a second run"
    dt_acc, tr_acc, _, _ = run(K, np.full(K, np.inf, np.float32))
    assert tr_acc["kind"][0].tolist() == [0 if i % args.interval == 0 else 1 for i in range(K)]
    dt_plain = None
    if full:
        dt_plain, tr_plain, _, _ = run(K, np.zeros(K, np.float32))
        assert tr_plain["n_spec"] == 0
    res = {
        "workload": ("config 4: FLUX-shaped MMDiT 1024x1024" if which == "flux" else "config 5: HunyuanVideo-shaped MMDiT 480p 2s")
                    + ", bf16, batch 1, Euler, Taylor order 2",
        "tokens": shape.tokens, "hidden": shape.hidden, "blocks": [shape.depth_dual, shape.depth_single], "steps": K, "warmup": warmup,
        "steps_per_s": K / dt, "ms_per_step": 1e3 * dt / K, "accept_rate": tr["n_spec"] / float(K), "n_full": tr["n_full"],
        "n_spec": tr["n_spec"], "n_reject": tr["n_reject"],
        "errors": [None if np.isnan(e) else float(e) for e in tr["err"][0, :, 0]],
        "plain_sampling_steps_per_s": None if dt_plain is None else K / dt_plain,
        "all_accepted_steps_per_s": K / dt_acc, "all_accepted_accept_rate": tr_acc["n_spec"] / float(K),
        "checks": "finite latents; identical bits on a second run; tau = inf gives the forced-interval pattern" + ("; tau = 0 never speculates" if full else ""),
        "prof": prof,
    }
    res.update(_classes(prof))
    ctx.close()
    del w, ctx, td, vd
    torch.cuda.empty_cache()
    return res


def bench_mmdit(args, which):
    r = mmdit_run(args, which, args.steps, args.warmup)
    prof = r.pop("prof")
    dom = max(("gemm", "attention", "forecast", "verify", "other"), key=lambda k: prof[k]["ms"])
    p = prof[dom]
    ach = p["flops"] / (p["ms"] * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
            "kernel": dom, "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / max(p["launches"], 1),
            "flops_per_launch": p["flops"] / max(p["launches"], 1)}
    print(json.dumps({
        "metric": "denoising_steps_per_s", "value": r["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": r["workload"], "tokens": r["tokens"], "hidden": r["hidden"], "blocks": r["blocks"], "order": 2, "interval": args.interval,
                   "tau0": args.tau0, "tau_end": args.tau_end, "cache_layout": args.layout, "parallelism": "single GPU"},
        "roofline": roof, "cpu_baseline": None,
        "extras": {k: v for k, v in r.items() if k not in ("workload", "tokens", "hidden", "blocks", "steps", "warmup", "steps_per_s", "ms_per_step")},
    }))


def gemm_subbatch_sweep():
    """The four block GEMMs of configuration 3 at the row counts a step can present (M = 512 k: per-sample rejection
    sends any number of guidance pairs to the full pass; four lanes split 16 rows into groups of 4), TFLOP/s with
    weights rotating through 16 copies so that they come from HBM as inside a step."""
    import torch
    from paper_2509_11628_amd import binding as bd
    out = {}
    g = torch.Generator(device="cuda").manual_seed(0)
    for name, N, K, act in (("qkv", 3456, 1152, 0), ("proj", 1152, 1152, 0), ("fc1_gelu", 4608, 1152, 1), ("fc2", 1152, 4608, 0)):
        ws = [(torch.randn((N, K), generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(16)]
        b = torch.zeros((N,), device="cuda", dtype=torch.bfloat16)
        row = {}
        for M in (512, 1024, 1536, 2048, 2560, 3072, 3584, 4096):
            a = torch.randn((M, K), generator=g, device="cuda").to(torch.bfloat16)
            o = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            for i in range(3):
                bd.linear(a, ws[i], b, act, out=o)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(32):
                bd.linear(a, ws[i % 16], b, act, out=o)
            e1.record()
            torch.cuda.synchronize()
            row[str(M)] = round(2.0 * M * N * K * 32 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        out[name] = row
    return out


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
    ap.add_argument("--no-extras", action="store_true",
                    help="only the configured, event-profiled, plain and all-accepted trajectories of configuration 3 (profiling runs)")
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

    def run(steps, tau=None, profile=False, latents=None):
        ts, ab = si.ddim_tables(steps)
        if tau is None:
            tau = bd.tau_geometric(args.tau0, args.tau_end / args.tau0, steps)
        x = torch.from_numpy(lat if latents is None else latents).cuda()
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
    _log(f"configuration 3: {K / dt:.1f} steps/s as configured, {K / dt_plain:.1f} plain, {K / dt_acc:.1f} all accepted")

    dom = max(("gemm", "attention", "forecast", "verify", "other"), key=lambda k: prof[k]["ms"])
    p = prof[dom]
    if dom in ("gemm", "attention"):
        ach = p["flops"] / (p["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS}
    else:
        ach = p["bytes"] / (p["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBPS}
    roof["traffic"], roof["traffic_source"] = measured_traffic("dit_xl2", dom, args.layout)
    roof["measured_on"] = "same trajectory, row groups run serially on one stream (per-kernel event times need no overlap); value is timed with lanes"
    roof.update({"kernel": dom, "launches": p["launches"], "avg_launch_us": 1e3 * p["ms"] / max(p["launches"], 1),
                 "flops_per_launch": p["flops"] / max(p["launches"], 1), "bytes_per_launch": p["bytes"] / max(p["launches"], 1)})

    extras = {"accept_rate": tr["n_spec"] / float(B * K), "n_full": tr["n_full"], "n_spec": tr["n_spec"], "n_reject": tr["n_reject"],
              "plain_sampling_steps_per_s": K / dt_plain, "all_accepted_steps_per_s": K / dt_acc,
              "all_accepted_accept_rate": tr_acc["n_spec"] / float(B * K)}
    extras.update(_classes(prof))

    # images/s is defined on the 50-step trajectory the configuration names, whatever --steps was
    S50 = 50
    if K == S50 or args.no_extras:
        dt50, dt50_plain = dt * S50 / K, dt_plain * S50 / K
    else:
        run(S50)
        dt50, _, _, _ = run(S50)
        dt50_plain, _, _, _ = run(S50, tau=np.zeros(S50, np.float32))
    extras["images_per_s"] = B / dt50
    extras["images_per_s_note"] = f"{B} images per {S50}-step trajectory as configured ({dt50 * 1e3:.0f} ms); plain sampling {B / dt50_plain:.1f} images/s"

    if args.no_extras:
        # profiling runs: only the four trajectories above (configured, event-profiled, plain, all accepted)
        t_full = dt_plain / K
        a_acc = tr_acc["n_spec"] / float(B * K)
        c_s = (dt_acc / K - (1.0 - a_acc) * t_full) / (a_acc * t_full)
        extras["speedup_model"] = {"gamma_nominal": 1.0 / shape.depth, "accepted_step_cost_ratio_measured": c_s,
                                   "all_accepted": {"alpha": a_acc, "measured_vs_plain": dt_plain / dt_acc}}
    else:
        # Thresholds at which the seeded model accepts part of its attempts (0 < alpha < 1): the geometric schedule with the
        # paper's DiT ablation value tau0 = 0.3, decaying to 0.1, calibrated once on this model (its verification errors
        # run from 0.04 to 0.33); and the same threshold level on latents scaled per sample (0.4 .. 2.0), whose errors
        # differ enough that most steps split the batch into a speculative and a full row list.
        tau_cal = bd.tau_geometric(0.3, 0.1 / 0.3, S50)
        run(S50, tau=tau_cal)
        dt_cal, tr_cal, _, x_cal = run(S50, tau=tau_cal)
        scales = np.array([0.4, 0.5, 0.6, 0.7, 1.4, 1.6, 1.8, 2.0], np.float32)
        lat_sc = lat * scales[:, None, None, None]
        tau_mix = np.full(S50, 0.2, np.float32)
        dt_mix, tr_mix, _, x_mix = run(S50, tau=tau_mix, latents=lat_sc)
        dt_mix_plain, _, _, _ = run(S50, tau=np.zeros(S50, np.float32), latents=lat_sc)
        assert bool(torch.isfinite(x_cal).all()) and bool(torch.isfinite(x_mix).all())
        mixed_steps = sum(1 for s_ in range(S50) if len(set(tr_mix["kind"][:, s_].tolist())) > 1)
        if K != S50:
            dt50_acc, tr50_acc, _, _ = run(S50, tau=np.full(S50, np.inf, np.float32))
        else:
            dt50_acc, tr50_acc = dt_acc, tr_acc

        # Speed-up model of the paper's complexity analysis, S = 1 / (1 - alpha (1 - gamma - overhead)), extended by the
        # attempts that are rejected (the paper's count charges only accepted steps): with c_s = cost of an accepted
        # speculative step and c_r = cost of a rejected attempt, both relative to a full step, and rho = rejected
        # attempts per sample-step,  S = 1 / ((1 - alpha) + alpha c_s + rho c_r).  c_s is measured on the all-accepted run,
        # c_r on the all-rejected run (the configured thresholds), both against plain sampling of the same length.
        def ratios(d_run, trc, d_plain, steps):
            return trc["n_spec"] / float(B * steps), trc["n_reject"] / float(B * steps), d_plain / d_run
        t_full = dt50_plain / S50
        a_acc, _, s_acc = ratios(dt50_acc, tr50_acc, dt50_plain, S50)
        c_s = (dt50_acc / S50 - (1.0 - a_acc) * t_full) / (a_acc * t_full)
        a_cfg, r_cfg, s_cfg = ratios(dt, tr, dt_plain, K)
        c_r = (dt / K - (1.0 - a_cfg) * (dt_plain / K) - a_cfg * c_s * (dt_plain / K)) / max(r_cfg, 1e-9) / (dt_plain / K)
        gamma = 1.0 / shape.depth

        def predict(a, r):
            return {"paper_nominal": 1.0 / (1.0 - a * (1.0 - gamma)), "with_measured_costs": 1.0 / ((1.0 - a) + a * c_s + r * c_r)}
        a_cal, r_cal, s_cal = ratios(dt_cal, tr_cal, dt50_plain, S50)
        a_mix, r_mix, s_mix = ratios(dt_mix, tr_mix, dt_mix_plain, S50)
        extras["speedup_model"] = {
            "gamma_nominal": gamma, "accepted_step_cost_ratio_measured": c_s, "rejected_attempt_cost_ratio_measured": c_r,
            "as_configured": {"alpha": a_cfg, "rejected_attempts_per_step": r_cfg, "predicted": predict(a_cfg, r_cfg), "measured_vs_plain": s_cfg},
            "all_accepted": {"alpha": a_acc, "rejected_attempts_per_step": 0.0, "predicted": predict(a_acc, 0.0), "measured_vs_plain": s_acc},
            "calibrated_thresholds": {"alpha": a_cal, "rejected_attempts_per_step": r_cal, "predicted": predict(a_cal, r_cal), "measured_vs_plain": s_cal},
            "mixed_rows": {"alpha": a_mix, "rejected_attempts_per_step": r_mix, "predicted": predict(a_mix, r_mix), "measured_vs_plain": s_mix,
                           "note": "the prediction assumes whole-batch launches; a step that splits the batch pays a full pass at a smaller, less efficient M"},
        }
        extras["calibrated_thresholds_run"] = {"tau": "geometric 0.3 -> 0.1 over 50 steps", "steps_per_s": S50 / dt_cal, "images_per_s": B / dt_cal,
                                               "accept_rate": a_cal, "n_full": tr_cal["n_full"], "n_spec": tr_cal["n_spec"], "n_reject": tr_cal["n_reject"]}
        extras["mixed_rows_run"] = {"tau": "0.2 constant, latents of sample b scaled by (0.4, 0.5, 0.6, 0.7, 1.4, 1.6, 1.8, 2.0)[b]", "steps_per_s": S50 / dt_mix,
                                    "plain_sampling_steps_per_s": S50 / dt_mix_plain, "accept_rate": a_mix, "n_full": tr_mix["n_full"],
                                    "n_spec": tr_mix["n_spec"], "n_reject": tr_mix["n_reject"], "steps_that_split_the_batch": mixed_steps}
        _log(f"calibrated thresholds: alpha {a_cal:.2f}, {S50 / dt_cal:.1f} steps/s; mixed rows: alpha {a_mix:.2f}, {S50 / dt_mix:.1f} steps/s, {mixed_steps} split steps")

    cpu = None if args.no_cpu_baseline else cpu_baseline(shape, weights)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()

    if not args.no_extras:
        extras["gemm_subbatch_TFLOPs"] = gemm_subbatch_sweep()
        fv = forecast_verify(args, 20, 2, False)
        fv.pop("cpu")
        extras["config2_forecast_verify"] = fv
        _log(f"configuration 2: forecast {fv['forecast']['achieved_GBps']:.0f} GB/s, verify stress shape {fv['verify_stress_shape']['achieved_GBps']:.0f} GB/s")
        for which, key, k4, w4, full in (("flux", "config4_flux", 20, 5, True), ("hunyuan", "config5_hunyuan", 6, 1, False)):
            r = mmdit_run(args, which, k4, w4, full)
            r.pop("prof")
            extras[key] = r

    out = {
        "metric": "denoising_steps_per_s", "value": K / dt, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 3: DiT-XL/2-shaped bf16, batch 8 x CFG 1.5 (16 rows), 256 tokens, DDIM, Taylor order 2",
                   "global_batch": B, "rows": 2 * B, "tokens": shape.tokens, "hidden": shape.hidden, "blocks": shape.depth,
                   "order": order, "interval": args.interval, "tau0": args.tau0, "tau_end": args.tau_end, "lanes": args.lanes,
                   "cache_layout": args.layout, "parallelism": "single GPU"},
        "roofline": roof,
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
