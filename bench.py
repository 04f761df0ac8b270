#!/usr/bin/env python3
"""Benchmark of the hot path on ONE MI355X: a "step" is one full denoiser forward of one guidance
branch on the SD3-shaped 1024x1024 workload (24 joint blocks, hidden 1536, 4096 image + 333 text
tokens, bf16), every kernel of the path included, inputs and weights resident in HBM.

Prints one JSON line: the whole-step rate in TFLOP/s of algorithmic work and ms per step, a live
per-kernel roofline for the dominant kernel (events recorded by the library around every launch),
the fused guidance pass at its bandwidth-bound shape, and the CPU oracle timed on a bounded sample."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "ms per denoiser step + TFLOP/s (MFMA %), SD3-shaped MMDiT branch at 1024²"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "pmc_hbm_traffic_cfg2_kernels.md")


def traffic_bytes():
    """HBM-side bytes per launch of the main kernels, from the counter summary under profiles/ (two rocprofv3 --pmc
    runs, FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for a plain copy of known size): the
    summary ends with lines `traffic_bytes <kernel name of the launch trace> <bytes>`.  Missing file: no figures."""
    out = {}
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes":
                    out[parts[1]] = float(parts[2])
    except OSError:
        pass
    return out


CPU_BASELINE_BLOCKS = 4


def cpu_baseline(cfg, synth):
    """The oracle, untuned, on the host cores: FOUR of the 24 joint blocks at the full token count, chained
    (about 1.5 TFLOP of fp64 work, 10-15 s), reported as TFLOP/s of the same algorithmic flop count."""
    import numpy as np
    from oracle import hyb_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    ws = [synth.mmdit_block_weights(cfg, i) for i in range(CPU_BASELINE_BLOCKS)]
    x_img = synth.normal(101, (1, cfg.n_img, cfg.hidden), 1.0, "f32")
    x_txt = synth.normal(102, (1, cfg.n_txt, cfg.hidden), 1.0, "f32")
    temb = synth.normal(103, (1, cfg.hidden), 1.0, "f32")
    t0 = time.time()
    for w in ws:
        x_img, x_txt = O.mmdit_block(x_img, x_txt, temb, w, cfg.heads)
    dt = time.time() - t0
    D, N = cfg.hidden, cfg.n_img + cfg.n_txt
    flops = CPU_BASELINE_BLOCKS * (24 * D * D * N + 4 * N * N * D + 24 * D * D)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d of 24 joint blocks of the same workload (fp64 numpy), %.1f s" % (CPU_BASELINE_BLOCKS, dt),
            "ms_per_step_extrapolated": dt * 1e3 * cfg.blocks / CPU_BASELINE_BLOCKS}


def guidance_roofline(hb, torch, steps, real_shapes=True):
    """The fused CFG + discrepancy + Euler pass at its bandwidth-bound shape: 256 samples of 262144
    latent elements (bf16 velocities, fp32 latent: 12 bytes per element, 805 MB per launch)."""
    batch, n = 256, 262144
    v_c = torch.randn(batch, n, device="cuda").to(torch.bfloat16)
    v_u = torch.randn(batch, n, device="cuda").to(torch.bfloat16)
    x = torch.randn(batch, n, device="cuda")
    xo = x     # the latent is updated in place, as the sampler does (GuidedSampler.step)
    d1, d2 = torch.empty(batch, device="cuda"), torch.empty(batch, device="cuda")
    ws = torch.empty(hb.hyb_discrepancy_workspace_bytes(batch, n), device="cuda", dtype=torch.uint8)
    for _ in range(10):
        hb.hyb_cfg_disc_euler(v_c, v_u, x, xo, 7.0, 0.5, 0.45, d1, d2, ws)
    torch.cuda.synchronize()
    hb.hyb_trace_enable(True)
    for _ in range(steps):
        hb.hyb_cfg_disc_euler(v_c, v_u, x, xo, 7.0, 0.5, 0.45, d1, d2, ws)
    torch.cuda.synchronize()
    tr = hb.hyb_trace_summary()["guidance_pass"]
    hb.hyb_trace_enable(False)
    us = tr["ms"] / tr["launches"] * 1e3
    gbs = tr["work"] / tr["launches"] / (us * 1e-6) / 1e9
    out = {"kernel": "guidance_pass", "shape": "batch 256 x 262144 elements", "bound": "hbm", "achieved": gbs,
           "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "us_per_launch": us,
           "bytes_per_element": 12, "traffic": traffic_bytes().get("guidance_pass"),
           "algorithmic_bytes": tr["work"] / tr["launches"]}
    if not real_shapes:
        return out
    # real latent shapes (latency-bound): time in microseconds
    real = {}
    for name, ne in (("sd3_1024", 262144), ("sd3_2048", 1048576), ("sdxl_1024", 65536)):
        hb.hyb_trace_enable(True)
        for _ in range(20):
            flat = [a.view(-1)[:ne].view(1, -1) for a in (v_c, v_u, x, xo)]
            hb.hyb_cfg_disc_euler(flat[0], flat[1], flat[2], flat[3], 7.0, 0.5, 0.45, d1[0:1], d2[0:1], ws)
        torch.cuda.synchronize()
        tr = hb.hyb_trace_summary()["guidance_pass"]
        hb.hyb_trace_enable(False)
        real[name] = round(tr["ms"] / tr["launches"] * 1e3, 2)
    out["us_at_real_latent_shapes"] = real
    return out


def timed(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def secondary_workloads(m, hb, model, synth, torch):
    """The other workload shapes on the same kernels (reported, not the headline metric): the guided step
    with both branches batched (configs[2]), the 2048 x 2048 branch (configs[3]) and the SDXL-shaped stages
    (configs[4]).  Weights of the MMDiT are reused; only activation buffers change."""
    out = {}
    # configs[2]: batch 2 + fused guidance pass, per guided step
    cfg3 = synth.CFG3
    m.reconfigure(cfg3)
    gs = model.GuidedSampler(m, cfg3.guidance)
    lat, ctx_c, ctx_u = synth.mmdit_inputs(cfg3)
    x = torch.from_numpy(lat).cuda()
    ctx2 = torch.from_numpy(__import__("numpy").stack([ctx_c, ctx_u])).cuda()
    ms = timed(lambda: gs.step(x, ctx2, 0.5, 0.45, 0), 5, 2, torch)
    fl = cfg3.flops_per_sample() * 2
    out["configs[2] guided step (batch 2 + CFG/discrepancy/Euler)"] = {"ms_per_step": round(ms, 3), "tflops": round(fl / ms / 1e9, 1),
                                                                      "ms_for_28_steps": round(ms * 28, 1)}
    # configs[3]: 2048 x 2048 branch
    cfg4 = synth.CFG4
    m.reconfigure(cfg4, pos_np=synth.normal(4, (cfg4.n_img, cfg4.hidden), 0.02, cfg4.dtype))
    lat4, ctx4, _ = synth.mmdit_inputs(cfg4)
    l4, c4 = torch.from_numpy(lat4[None]).cuda(), torch.from_numpy(ctx4[None]).cuda()
    t4 = torch.full((1,), 0.5, device="cuda")
    ms = timed(lambda: m.forward(l4, c4, t4), 3, 1, torch)
    out["configs[3] 2048x2048 branch forward"] = {"ms_per_step": round(ms, 3), "tflops": round(cfg4.flops_per_sample() / ms / 1e9, 1)}
    # beyond the configs: the 2560 x 2560 shape of the paper's high-resolution study (25600 image tokens)
    cfg6 = synth.CFG6
    del l4, c4
    m.reconfigure(cfg6, pos_np=synth.normal(4, (cfg6.n_img, cfg6.hidden), 0.02, cfg6.dtype))
    lat6, ctx6, _ = synth.mmdit_inputs(cfg6)
    l6, c6 = torch.from_numpy(lat6[None]).cuda(), torch.from_numpy(ctx6[None]).cuda()
    ms = timed(lambda: m.forward(l6, c6, t4), 2, 1, torch)
    out["2560x2560 branch forward"] = {"ms_per_step": round(ms, 3), "tflops": round(cfg6.flops_per_sample() / ms / 1e9, 1)}
    return out


def sdxl_workload(hb, model, synth, torch):
    out = {}
    total_ms, total_fl = 0.0, 0.0
    for cfg in (synth.CFG5A, synth.CFG5B):
        st = model.SDXLStage(cfg, (synth.sdxl_block_weights(cfg, i) for i in range(cfg.blocks)))
        x, ctx = synth.sdxl_inputs(cfg)
        dx, dc = torch.from_numpy(x).cuda(), torch.from_numpy(ctx).cuda()
        ms = timed(lambda: st.forward(dx, dc), 5, 2, torch)
        fl = cfg.flops_per_sample() * cfg.batch
        out[cfg.name] = {"ms": round(ms, 3), "tflops": round(fl / ms / 1e9, 1)}
        total_ms += ms
        total_fl += fl
        del st
    out["stages A+B, batch 2"] = {"ms": round(total_ms, 3), "tflops": round(total_fl / total_ms / 1e9, 1)}
    return out


def _device_info(torch):
    """Static properties as the runtime reports them (the clock is the maximum, not the sustained one)."""
    pr = torch.cuda.get_device_properties(0)
    info = {"compute_units": pr.multi_processor_count, "hbm_gib": round(pr.total_memory / 2**30, 1)}
    for name in ("gcnArchName", "clock_rate", "L2_cache_size"):
        if hasattr(pr, name):
            info[name] = getattr(pr, name)
    return info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--guidance-only", action="store_true",
                    help="run only the fused guidance pass at its bandwidth-bound shape (batch 256 x 262144 elements) and "
                         "print its roofline object: a kernel trace of this command holds that one launch shape")
    ap.add_argument("--primary-only", action="store_true",
                    help="time only the headline workload and the guidance pass (profiling runs: a kernel trace of "
                         "this command then holds one shape per kernel); by default the other workload shapes "
                         "(guided step, 2048x2048 and 2560x2560 branches, U-Net stages) are timed too")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the two guidance branches are batched or run "
              "back to back on it); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_21760_amd import binding as hb, model, synth

    hb.lib()    # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.guidance_only:
        print(json.dumps({"guidance_pass_roofline": guidance_roofline(hb, torch, max(args.steps, 10), real_shapes=False)}))
        return
    cfg = synth.CFG2
    t0 = time.time()
    m = model.MMDiT(cfg, synth.mmdit_globals(cfg), synth.mmdit_blocks(cfg))
    lat, ctx_c, _ = synth.mmdit_inputs(cfg)
    latent = torch.from_numpy(lat[None]).cuda()
    ctx = torch.from_numpy(ctx_c[None]).cuda()
    t = torch.full((1,), 0.5, device="cuda")
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    for _ in range(args.warmup):
        m.forward(latent, ctx, t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m.forward(latent, ctx, t)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    flops = cfg.flops_per_sample() * cfg.batch
    tflops = flops / (ms * 1e-3) / 1e12

    # per-kernel timing of the same steps (events around every launch, recorded by the library)
    hb.hyb_trace_enable(True)
    for _ in range(args.steps):
        m.forward(latent, ctx, t)
    torch.cuda.synchronize()
    trace = hb.hyb_trace_summary()
    hb.hyb_trace_enable(False)
    kernels = {}
    for name, r in trace.items():
        per = r["ms"] / r["launches"]
        rate = r["work"] / r["launches"] / (per * 1e-3)
        kernels[name] = {"launches_per_step": r["launches"] / args.steps, "ms_per_step": round(r["ms"] / args.steps, 4),
                         "us_per_launch": round(per * 1e3, 2),
                         ("tflops" if r["unit"] == "flop" else "gbs"): round(rate / (1e12 if r["unit"] == "flop" else 1e9), 1)}
    flop_kernels = {k: v for k, v in trace.items() if v["unit"] == "flop"}
    dom = max(flop_kernels, key=lambda k: flop_kernels[k]["ms"])
    d = flop_kernels[dom]
    dom_ms = d["ms"]
    # the attention kernel leaves a few query blocks as partial results that a small second kernel merges: its
    # time belongs to the attention launch
    helper = {"attention_mfma": "attention_merge"}.get(dom)
    if helper in trace:
        dom_ms += trace[helper]["ms"]
    ach = d["work"] / d["launches"] / (dom_ms / d["launches"] * 1e-3) / 1e12
    roofline = {"kernel": dom if helper not in trace else dom + " + " + helper, "bound": "mfma", "achieved": ach,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic_bytes().get(dom),
                "us_per_launch": dom_ms / d["launches"] * 1e3, "flops_per_launch": d["work"] / d["launches"]}

    guidance = guidance_roofline(hb, torch, max(args.steps, 10))
    secondary = {}
    if not args.primary_only:
        secondary = secondary_workloads(m, hb, model, synth, torch)
        del m
        torch.cuda.empty_cache()
        secondary["configs[4] SDXL-shaped stages"] = sdxl_workload(hb, model, synth, torch)
    line = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic", "mfma_frac_of_peak": tflops / PEAK_BF16_TFLOPS,
        "config": {"workload": "configs[1]: SD3-shaped MMDiT branch, 1024x1024, 24 blocks, hidden 1536, "
                               "4096+333 tokens, batch 1, one denoiser forward", "algorithmic_tflop_per_step": flops / 1e12},
        "roofline": roofline, "guidance_pass_roofline": guidance, "kernels": kernels, "other_workloads": secondary, "setup_s": round(setup_s, 1),
        "device": torch.cuda.get_device_name(0),
        "device_info": _device_info(torch),
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, synth)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
