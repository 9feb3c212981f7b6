#!/usr/bin/env python3
"""Benchmark of the Sign-Muon optimizer hot path on one MI355X.

A step is one signmuon_step call: for every weight block of the workload and all
M simulated workers, momentum -> Newton-Schulz -> sign pack -> majority vote ->
(local polar) -> update.  Inputs are synthetic, seeded, resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E


def ns_flops(shapes, batch_per_block, steps):
    """Nominal Newton-Schulz work: 4 s^2 l per step and matrix (Gram 2 s^2 l + apply 2 s^2 l)."""
    gram = apply_ = 0.0
    for r, c in shapes:
        s, l = min(r, c), max(r, c)
        gram += 2.0 * s * s * l * batch_per_block * steps
        apply_ += 2.0 * s * s * l * batch_per_block * steps
    return gram, apply_


def make_inputs(name, torch, device):
    import workloads as wl
    cfg = wl.WORKLOADS[name]
    M = cfg["M"]
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.BASE_SEED * 1000 + cfg["stream"])
    w, mom, grad = [], [], []
    for r, c in cfg["shapes"]:
        w.append(torch.randn((r, c), generator=gen, device=device) * 0.02)
        mom.append(torch.zeros((M, r, c), device=device))
        kind = cfg["grad"]
        if kind == "normal":
            g = torch.randn((M, r, c), generator=gen, device=device) * cfg["grad_std"]
        elif kind == "lowrank":
            k = cfg["rank"]
            A = torch.randn((r, k), generator=gen, device=device)
            B = torch.randn((c, k), generator=gen, device=device)
            g = (A @ B.T / math.sqrt(k))[None] + torch.randn((M, r, c), generator=gen, device=device)
        elif kind == "student_t":
            nu = cfg["nu"]
            z = torch.randn((M, r, c), generator=gen, device=device)
            chi = torch.zeros((M, r, c), device=device)
            for _ in range(nu):
                chi += torch.randn((M, r, c), generator=gen, device=device) ** 2
            g = z / torch.sqrt(chi / nu)
            del z, chi
        else:
            raise ValueError(kind)
        grad.append(g.contiguous())
    return cfg, w, mom, grad


def run_workload(name, steps, warmup, torch, P, B, scale=None):
    device = torch.device("cuda:0")
    cfg, w, mom, grad = make_inputs(name, torch, device)
    scale = scale or cfg.get("scale", "fro")
    shapes, M = cfg["shapes"], cfg["M"]
    K, Kp = cfg["ns_steps"], cfg["local_polar_steps"]
    ctx = P.Context()
    v0 = None
    if scale == "spectral":
        gen = torch.Generator(device=device)
        gen.manual_seed(7)
        v0 = [torch.randn((M, c), generator=gen, device=device) for _, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-3, ns_steps=K, sign_fmt=cfg["sign_fmt"],
                      local_polar_steps=Kp, scale=scale, power_iters=2, v0=v0)
    for _ in range(warmup):
        P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    # timed region: K steps as a caller runs them, no event taps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    # the same K steps again with HIP events around every launch of the GEMM classes, on the library's stream:
    # launch durations for the roofline (the events cost host time per launch, which the timed region above
    # does not pay; a few dozen launches per step)
    gemm_classes = (B.SM_K_NS_GRAM, B.SM_K_NS_SMALL, B.SM_K_NS_APPLY)
    ctx.profile_reset()
    ctx.profile_enable(sum(1 << k for k in gemm_classes))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    elapsed_tapped = time.perf_counter() - t0
    gemm = {}
    for k in gemm_classes:
        n, ms = ctx.profile_read(k)
        flop, dense, nbytes = ctx.profile_work(k)
        if n == 0:
            continue
        sec = ms * 1e-3
        t_mfma, t_hbm = flop / (MFMA_BF16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
        # flop: the output tiles the launches really computed (a symmetric product: the tiles on and above
        # the diagonal; sizes clipped to the unpadded matrices).  dense: 2 M N K of the same products.
        gemm[P.kernel_name(k)] = {
            "launches_per_step": n / steps, "avg_launch_ms": ms / n, "ms_per_step": ms / steps,
            "flop_per_launch": flop / n, "dense_flop_per_launch": dense / n, "bytes_per_launch": nbytes / n,
            "tflops": flop / sec / 1e12, "frac_of_mfma_peak": flop / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "dense_equiv_tflops": dense / sec / 1e12, "gbs": nbytes / sec / 1e9,
            "bound": "mfma" if t_mfma >= t_hbm else "hbm",
        }
    # second, untimed pass with taps on every kernel class: per-class breakdown
    ctx.profile_reset()
    ctx.profile_enable((1 << B.SM_K_COUNT) - 1)
    for _ in range(steps):
        P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    per_class = {}
    for k in range(B.SM_K_COUNT):
        n, ms = ctx.profile_read(k)
        per_class[P.kernel_name(k)] = {"launches_per_step": n / steps, "ms_per_step": ms / steps}
    ctx.profile_enable(0)
    ws = ctx.workspace_bytes
    standalone = standalone_sign_vote(ctx, cfg, torch, P, B)
    ctx.close()
    graph = graph_replay(w, mom, grad, cfg, scale, v0, steps, warmup, torch, P)

    d_total = sum(r * c for r, c in shapes)
    nominal = sum(ns_flops(shapes, M, K)) + sum(ns_flops(shapes, 1, Kp))
    ns_ms = sum(g["ms_per_step"] for g in gemm.values())
    executed = sum(g["flop_per_launch"] * g["launches_per_step"] for g in gemm.values())
    one_bit = cfg["sign_fmt"] == "1bit"
    pack_bytes = d_total * M * (2 + (0.125 if one_bit else 1.0))
    if Kp:
        vote_bytes = d_total * ((M / 8 if one_bit else M) + 2)          # writes the +-1 bf16 matrix
    else:
        vote_bytes = d_total * ((M / 8 if one_bit else M) + 8)          # fused W read + write
    mom_bytes = d_total * M * 14.0
    ms_pack = per_class[P.kernel_name(B.SM_K_SIGN_PACK)]["ms_per_step"]
    ms_vote = per_class[P.kernel_name(B.SM_K_VOTE)]["ms_per_step"]
    ms_mom = per_class[P.kernel_name(B.SM_K_MOMENTUM)]["ms_per_step"]
    # Alg. PowerIter with P = 2: 2 P + 1 products with X, i.e. 2 P + 1 passes over the bf16 X of every worker before
    # the vote and over the voted matrices after it (algorithmic bytes; the fused pass reads X P + 1 times)
    ms_pi = per_class[P.kernel_name(B.SM_K_POWER_ITER)]["ms_per_step"]
    pi_bytes = 5.0 * 2.0 * d_total * (M + (1 if Kp else 0)) if scale == "spectral" else 0.0
    res = {
        "workload": name, "M": M, "n_blocks": len(shapes), "entries": d_total, "ns_steps": K,
        "local_polar_steps": Kp, "scale": scale,
        "steps_per_s": steps / elapsed, "ms_per_step": 1e3 * elapsed / steps,
        "ms_per_step_with_gemm_taps": 1e3 * elapsed_tapped / steps,
        # executed: the matrix-product tiles actually computed, over the time of all Newton-Schulz launches (the
        # utilisation figure); nominal: the work of Alg. PolarNS as written (4 s^2 l per step and matrix) over the
        # same time, i.e. the rate a step-by-step implementation would need to be as fast (not a utilisation)
        "ns_tflops_executed": executed / (ns_ms * 1e-3) / 1e12 if ns_ms else None,
        "ns_nominal_tflops": nominal / (ns_ms * 1e-3) / 1e12 if ns_ms else None,
        "ns_ms_per_step": ns_ms, "gemm": gemm,
        # the sign pack is part of the last apply GEMM when its class reports no launches: then only the
        # vote's own bytes and time are counted here
        "sign_vote_gbs": ((pack_bytes if ms_pack else 0.0) + vote_bytes) / ((ms_pack + ms_vote) * 1e-3) / 1e9
        if ms_pack + ms_vote else None,
        "sign_pack_fused_into_apply": ms_pack == 0.0,
        "standalone": standalone, "graph_replay": graph,
        "momentum_gbs": mom_bytes / (ms_mom * 1e-3) / 1e9 if ms_mom else None,
        "power_iter": ({"ms_per_step": ms_pi, "algorithmic_gbs": pi_bytes / (ms_pi * 1e-3) / 1e9,
                        "frac_of_hbm_peak": pi_bytes / (ms_pi * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "bytes": "(2P+1) passes over the bf16 X of all workers and, with a local polar step, "
                                 "over the voted matrices"} if ms_pi else None),
        "per_class": per_class, "workspace_GB": ws / 1e9,
    }
    del w, mom, grad, plan
    torch.cuda.empty_cache()
    return res


def graph_replay(w, mom, grad, cfg, scale, v0, steps, warmup, torch, P):
    """The same step captured once into a HIP graph (on a side stream) and replayed: what a caller who
    records the optimizer step pays per step, without the per-launch host overhead.  Reported next to the
    eager figure, which stays the headline (its launches carry the event taps the roofline is taken from)."""
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        ctx = P.Context(stream=side)
        plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-3, ns_steps=cfg["ns_steps"], sign_fmt=cfg["sign_fmt"],
                          local_polar_steps=cfg["local_polar_steps"], scale=scale, power_iters=2, v0=v0)
        P.signmuon_step(ctx, plan)          # plans the workspace
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            P.signmuon_step(ctx, plan)
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ctx.close()
    del g
    return {"ms_per_step": 1e3 * elapsed / steps, "steps_per_s": steps / elapsed}


def standalone_sign_vote(ctx, cfg, torch, P, B, reps=5):
    """The two entry points on their own over the whole set with all M workers, as the paper transports it:
    every worker's blocks concatenated into one buffer of sum(d) entries (each block's d is a multiple of
    64 in every workload, so this is the per-block packing back to back).  signmuon_sign_pack (bf16 in), then
    signmuon_majority_vote (voted bits out for 1-bit signs, voted int8 for int8 signs).  Bytes by the
    per-entry formulas of the kernels' roofline; time = summed kernel time from the event taps."""
    shapes, M, fmt = cfg["shapes"], cfg["M"], cfg["sign_fmt"]
    one_bit = fmt == "1bit"
    d = sum(r * c for r, c in shapes)
    assert all((r * c) % 64 == 0 for r, c in shapes)
    stride = d // 8 if one_bit else d
    u = torch.empty((M, d), dtype=torch.bfloat16, device="cuda")
    for p in range(M):
        u[p] = torch.randn((d,), device="cuda").to(torch.bfloat16)
    sg = torch.zeros((M, stride), dtype=torch.uint8, device="cuda")
    vt = torch.zeros((stride,), dtype=torch.uint8, device="cuda")
    ctx.profile_reset()
    ctx.profile_enable((1 << B.SM_K_SIGN_PACK) | (1 << B.SM_K_VOTE))
    for _ in range(reps):
        P.signmuon_sign_pack(ctx, u, fmt, sg)
        P.signmuon_majority_vote(ctx, sg, fmt, M, d, stride, voted=vt, vfmt="bits" if one_bit else "int8")
    torch.cuda.synchronize()
    _, ms_pack = ctx.profile_read(B.SM_K_SIGN_PACK)
    _, ms_vote = ctx.profile_read(B.SM_K_VOTE)
    ctx.profile_enable(0)
    pack_b = d * M * (2 + (0.125 if one_bit else 1.0)) * reps
    vote_b = d * ((M / 8 + 0.125) if one_bit else (M + 1.0)) * reps
    res = {"sign_pack_gbs": pack_b / (ms_pack * 1e-3) / 1e9, "vote_gbs": vote_b / (ms_vote * 1e-3) / 1e9,
           "sign_vote_gbs": (pack_b + vote_b) / ((ms_pack + ms_vote) * 1e-3) / 1e9,
           "sign_pack_ms": ms_pack / reps, "vote_ms": ms_vote / reps, "entries_per_worker": d}
    del u, sg, vt
    torch.cuda.empty_cache()
    return res


def cpu_baseline(name, budget_s=15.0):
    """Times the oracle (float32 variant, as it stands) on a bounded sample of the workload."""
    import numpy as np
    import workloads as wl
    from oracle import signmuon_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    cpu_model = "unknown"
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.lower().startswith("model name"):
                cpu_model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    cfg = wl.WORKLOADS[name]
    shapes, M = cfg["shapes"], cfg["M"]
    # Blocks and workers are independent, so the step time is the sum over blocks.  Blocks of the
    # workload are timed in order (whole per-block step: momentum, M x PolarNS, pack, vote, local
    # polar, update) until the time budget is used; the rest is scaled by nominal NS work.
    def block_flop(r, c):
        return 4.0 * min(r, c) ** 2 * max(r, c) * (cfg["ns_steps"] * M + cfg["local_polar_steps"])
    total_flop = sum(block_flop(r, c) for r, c in shapes)
    # visit one block of every distinct shape first, then the remaining blocks
    order, seen = [], set()
    for i, sh in enumerate(shapes):
        if sh not in seen:
            seen.add(sh)
            order.append(i)
    order += [i for i in range(len(shapes)) if i not in order]
    t_spent, flop_done, n_done = 0.0, 0.0, 0
    for i in order:
        r, c = shapes[i]
        G = wl.worker_grads(name, i, r, c)
        W = wl.weights(r, c, block=i)
        mom = np.zeros_like(G)
        t0 = time.perf_counter()
        O.signmuon_step(W, mom, G, beta=0.9, lr=1e-3, ns_steps=cfg["ns_steps"], sign_fmt=cfg["sign_fmt"],
                        local_polar_steps=cfg["local_polar_steps"], dtype=np.float32)
        t_spent += time.perf_counter() - t0
        flop_done += block_flop(r, c)
        n_done += 1
        if t_spent > budget_s and n_done >= len(seen):
            break
    step_s = t_spent * total_flop / flop_done
    return {"value": 1.0 / step_s, "unit": "steps/s", "cores": int(cores), "cpu_model": cpu_model, "kind": "oracle",
            "sample": f"float32 oracle (numpy), full per-block step on {n_done} of {len(shapes)} blocks "
                      f"(every distinct shape, all {M} workers) in {t_spent:.1f} s, scaled to the whole set "
                      f"by nominal Newton-Schulz work"}


def mfma_loop_ceiling():
    """Runs the register-resident MFMA loop (paper_2605_16311_amd/mfma_peak, a program of its own, before this
    process touches the GPU): what the matrix cores sustain with nothing else going on, for constant operands
    and for operands of full range, whose switching power lowers the clock the part holds."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2605_16311_amd", "mfma_peak")
    if not os.path.exists(exe):
        return None
    try:
        out = subprocess.run([exe, "60"], capture_output=True, text=True, timeout=120).stdout
    except Exception:
        return None
    res, mode = {}, None
    for ln in out.splitlines():
        if ln.startswith("operands:"):
            mode = ln.split(":", 1)[1].strip()
        elif "GEMM's shape" in ln and "bf16" in ln and mode:
            try:
                res[mode] = float(ln.split("ms")[1].split("TFLOP/s")[0])
            except (IndexError, ValueError):
                pass
    return {"tflops_bf16_by_operands": res, "what": "v_mfma_f32_32x32x16_bf16 loop, registers only, 8 waves/CU, 4x2 "
            "accumulators per wave as in the GEMM kernel"} if res else None


def library_gemm_yardstick(torch):
    """torch.matmul in bf16 (the vendor's GEMM library) on the shapes of the dominant products, in the same run and
    on the same device: a yardstick for what a tuned GEMM reaches on this part, not part of the path."""
    out = {}
    for name, (b, m, n, k) in {"384 x (768 x 768 x 768)": (384, 768, 768, 768),
                               "16 x (4096 x 4096 x 4096)": (16, 4096, 4096, 4096),
                               "8192 x 8192 x 8192": (1, 8192, 8192, 8192)}.items():
        A = torch.randn((b, m, k), device="cuda").to(torch.bfloat16)
        Bm = torch.randn((b, k, n), device="cuda").to(torch.bfloat16)
        for _ in range(3):
            torch.bmm(A, Bm)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for s, e in ev:
            s.record()
            torch.bmm(A, Bm)
            e.record()
        torch.cuda.synchronize()
        ms = sorted(s.elapsed_time(e) for s, e in ev)[len(ev) // 2]
        out[name] = {"median_ms": ms, "tflops": 2.0 * b * m * n * k / ms / 1e9,
                     "frac_of_mfma_peak": 2.0 * b * m * n * k / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS}
        del A, Bm
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="nanogpt124m")
    ap.add_argument("--also", default="resnet50,nanogpt_paper_k10,resnet50_k1,large,int8vote",
                    help="further workloads (comma separated) reported in the same line under 'also' ('' to skip); "
                         "the two large sets run 3 timed steps, the small ones 5 x --steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true",
                    help="skip the register-resident MFMA loop and the library GEMM yardstick (context figures)")
    ap.add_argument("--scale", default=None, choices=["fro", "spectral"],
                    help="scale of Alg. PolarNS: Frobenius norm or PowerIter with P = 2 (default: the workload's own)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three 1 GiB device copies (torch): a kernel of known traffic for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the M workers are a batch dimension); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import __graft_entry__
    __graft_entry__.ensure_built()                                       # loads what is built; compiles only if nothing is
    mfma_loop = None if args.no_calibration else mfma_loop_ceiling()     # before this process uses the GPU
    import torch
    import paper_2605_16311_amd as P
    from paper_2605_16311_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    main_res = run_workload(args.workload, args.steps, args.warmup, torch, P, B, scale=args.scale)
    big = ("large", "int8vote")             # a quarter and an eighth of a second per step
    also = [run_workload(nm, 3 if nm in big else max(args.steps * 5, 50), 1 if nm in big else args.warmup, torch, P, B)
            for nm in args.also.split(",") if nm and nm != args.workload]
    # roofline of the dominant kernel: the GEMM class with the largest share of the step
    dom_name, dom = max(main_res["gemm"].items(), key=lambda kv: kv[1]["ms_per_step"])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(dom_name)
        except Exception:
            traffic = None
    # bound by the matrix cores: achieved = executed flop (tiles really computed) per launch / launch duration
    if dom["bound"] == "mfma":
        ach, peak, unit = dom["tflops"], MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
    else:
        ach, peak, unit = dom["gbs"], HBM_PEAK_GBS, "GB/s"
    line = {
        "metric": "Sign-Muon steps/sec; NS TFLOPS (% MFMA peak); sign+vote GB/s (% HBM)",
        "value": main_res["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        # the K steps repeated with HIP events around every GEMM launch (source of roofline.avg_launch_ms)
        "ms_per_step_with_gemm_taps": main_res["ms_per_step_with_gemm_taps"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "M": main_res["M"], "blocks": main_res["n_blocks"],
                   "entries": main_res["entries"], "ns_steps": main_res["ns_steps"],
                   "local_polar_steps": main_res["local_polar_steps"], "scale": main_res["scale"],
                   # Y, Gram and apply in bf16; the s x s matrices of the regrouped iteration in IEEE half
                   # precision (same MFMA rate); fp32 accumulation, momentum and weights
                   "ns_arithmetic": "bf16 Y / f16 s x s intermediates / f32 accumulate"},
        "roofline": {"kernel": dom_name, "bound": dom["bound"], "achieved": ach, "peak": peak, "unit": unit,
                     "frac": ach / peak, "traffic": traffic, "avg_launch_ms": dom["avg_launch_ms"],
                     "flop_per_launch": dom["flop_per_launch"], "bytes_per_launch": dom["bytes_per_launch"]},
        # tflops / frac_of_mfma_peak: executed tile flop of all Newton-Schulz launches over their time;
        # nominal_tflops: Alg. PolarNS's 4 s^2 l per step and matrix over the same time (algorithm-equivalent rate of
        # the regrouped iteration, which executes about half of that work: a speed figure, not a utilisation)
        "ns": {"tflops": main_res["ns_tflops_executed"],
               "frac_of_mfma_peak": (main_res["ns_tflops_executed"] / MFMA_BF16_PEAK_TFLOPS
                                     if main_res["ns_tflops_executed"] else None),
               "nominal_tflops": main_res["ns_nominal_tflops"], "ms_per_step": main_res["ns_ms_per_step"],
               "gemm": main_res["gemm"]},
        # standalone: signmuon_sign_pack + signmuon_majority_vote on their own over the whole set (the figure the
        # HBM target is quoted on); in_step: what the step itself ran (the pack rides in the apply when fused)
        "sign_vote": {"gbs": main_res["standalone"]["sign_vote_gbs"],
                      "frac_of_hbm_peak": main_res["standalone"]["sign_vote_gbs"] / HBM_PEAK_GBS,
                      "sign_pack_frac_of_hbm_peak": main_res["standalone"]["sign_pack_gbs"] / HBM_PEAK_GBS,
                      "vote_frac_of_hbm_peak": main_res["standalone"]["vote_gbs"] / HBM_PEAK_GBS,
                      "standalone": main_res["standalone"],
                      "in_step_gbs": main_res["sign_vote_gbs"],
                      "in_step_frac_of_hbm_peak": (main_res["sign_vote_gbs"] / HBM_PEAK_GBS
                                                   if main_res["sign_vote_gbs"] else None),
                      "sign_pack_fused_into_apply": main_res["sign_pack_fused_into_apply"]},
        "momentum_gbs": main_res["momentum_gbs"],
        "momentum_frac_of_hbm_peak": main_res["momentum_gbs"] / HBM_PEAK_GBS if main_res["momentum_gbs"] else None,
        "power_iter": main_res["power_iter"],
        "per_class_ms": {k: round(v["ms_per_step"], 4) for k, v in main_res["per_class"].items()},
        "workspace_GB": main_res["workspace_GB"],
        "graph_replay": main_res["graph_replay"],
    }
    if also:
        line["also"] = []
        for a in also:
            e = {k: a[k] for k in ("workload", "M", "n_blocks", "ns_steps", "local_polar_steps", "scale", "steps_per_s",
                                   "ms_per_step", "graph_replay", "ns_tflops_executed", "ns_nominal_tflops",
                                   "momentum_gbs")}
            e["ns_frac_of_mfma_peak"] = (a["ns_tflops_executed"] / MFMA_BF16_PEAK_TFLOPS
                                         if a["ns_tflops_executed"] else None)
            e["gemm"] = {k: {"avg_launch_ms": v["avg_launch_ms"], "launches_per_step": v["launches_per_step"],
                             "tflops": v["tflops"], "frac_of_mfma_peak": v["frac_of_mfma_peak"]}
                         for k, v in a["gemm"].items()}
            e["sign_vote_gbs"] = a["standalone"]["sign_vote_gbs"]
            e["sign_pack_gbs"] = a["standalone"]["sign_pack_gbs"]
            e["vote_gbs"] = a["standalone"]["vote_gbs"]
            e["in_step_sign_vote_gbs"] = a["sign_vote_gbs"]
            if a["power_iter"]:
                e["power_iter"] = {k: a["power_iter"][k] for k in ("ms_per_step", "algorithmic_gbs", "frac_of_hbm_peak")}
            e["per_class_ms"] = {k: round(v["ms_per_step"], 4) for k, v in a["per_class"].items()}
            line["also"].append(e)
    if not args.no_calibration:
        # context for the fractions of the nominal peak above: neither figure is a target or part of the path
        line["calibration"] = {"mfma_loop": mfma_loop, "library_gemm_bf16": library_gemm_yardstick(torch)}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
