#!/usr/bin/env python3
"""Benchmark of the BiGLA + locality-gate forward on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
bigla_fwd(q, k, v, g_fwd, g_bwd) -> o_global, then locality_gate_fwd(x := v, w, z, o_global).
Default workload: the high-resolution ViG-S-shaped block (B=8, H=6, 64x64 grid, L=4096,
dk=dv=64, bf16) -- the configuration the headline metric is quoted on.

Inputs are resident in HBM before the timed region.  The timed loop rotates through several
independent buffer sets whose total size exceeds the 256 MB Infinity Cache, so that every step
streams its operands from HBM rather than from a warm cache.

Prints ONE JSON line.  `roofline` is that of the dominant entry
point, bigla_fwd: its algorithmic bytes over the summed duration of ALL its launches, which are
timed with HIP events recorded on their own stream inside the library (a second pass of the same
K steps, so that event recording does not perturb `value`; the cost of an event pair itself is
estimated from the excess of their sum over the step's wall time and taken off).  `roofline.traffic` is read from the
table in profiles/hbm_traffic.md that the rocprofv3 counter runs wrote.  `cpu_baseline` times the
CPU oracle on the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA peak
CACHE_BYTES = 256 << 20        # Infinity Cache; buffer sets rotate over more than this

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")
BIGLA_KERNELS = ("segment_state", "segment_out", "segment_out_general", "slab", "recurrent")


def measured_traffic():
    """HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs: the rows
    `| workload | kernel | read MB | written MB | bytes |` of profiles/hbm_traffic.md (written by
    `profile_path.py traffic`), keyed by (workload, kernel).  Missing file or row: no figure."""
    table = {}
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[4].isdigit():
                table[(cells[0], cells[1])] = int(cells[4])
    except OSError:
        pass
    return table


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)  # the first few hundred steps after idling run ~5 % slower
    ap.add_argument("--config", type=int, default=4, help="workload index (paper_2405_18425_amd.workloads.CONFIGS)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget-s", type=float, default=12.0)
    ap.add_argument("--single-set", action="store_true", help="reuse one buffer set (cache-warm timing)")
    ap.add_argument("--dk", type=int, default=0, help="override the key/query head width of the workload (side measurement)")
    ap.add_argument("--backward", action="store_true",
                    help="also time bigla_bwd, the gradient of the token mixer, on the same buffers (side "
                         "measurement in detail.backward; not part of the step or of value)")
    ap.add_argument("--gate-width", type=int, default=0,
                    help="also time the step with the forget-gate producer in front (block input of this width), as "
                         "two launches and with the state pass making the gates (side measurement in detail.gated)")
    ap.add_argument("--layout", choices=("bhld", "blhd"), default="bhld",
                    help="activation layout: head-major (default) or token-major [B,L,H,d] (side measurement)")
    ap.add_argument("--fwd-plan", choices=("auto", "four_wave", "wave_specialised", "slab_sweep"), default="auto",
                    help="kernels of the chunkwise forward (side measurement; auto is what bigla_fwd runs)")
    ap.add_argument("--alias-slabs", action="store_true",
                    help="side measurement of the contraction phase: every slab reads the first slab's q, k, v and "
                         "gates (cache-resident inputs; outputs still written; one buffer set)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU; multi-GPU runs are not part of it "
              "(the path shards over (batch, head) slabs with no exchange).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2405_18425_amd import binding as vb
    from paper_2405_18425_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    vb.lib()  # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    w = wl.CONFIGS[args.config]
    if args.dk:
        w = w.replace(name=f"{w.name}_dk{args.dk}", dk=args.dk)
    esize = 2 if w.dtype == "bf16" else 4

    # ---- inputs: one seeded set on the host, further sets are batch-rotated copies on the device
    stored = wl.generate(w, seed=args.seed)
    base = {n: wl.to_torch(a, w.dtype, dev) for n, a in stored.items()}
    set_bytes = sum(t.numel() * t.element_size() for t in base.values()) + 2 * base["v"].numel() * esize
    n_sets = 1 if (args.single_set or args.alias_slabs) else max(2, -(-2 * CACHE_BYTES // set_bytes))
    sets = []
    for i in range(n_sets):
        s = {n: (t if i == 0 or n == "conv_w" else torch.roll(t, shifts=i, dims=0).contiguous())
             for n, t in base.items()}
        if args.layout == "blhd":
            s = {n: (t if n == "conv_w" else t.permute(0, 2, 1, 3).contiguous()) for n, t in s.items()}
        s["o_global"] = torch.empty_like(s["v"])
        s["out"] = torch.empty_like(s["v"])
        sets.append(s)
    code = vb.VIG_BF16 if w.dtype == "bf16" else vb.VIG_F32
    ws_bytes = vb.bigla_workspace_bytes(w.B, w.H, w.L, w.dk, w.dv, code)
    workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def step(i):
        s = sets[i % n_sets]
        vb.bigla_fwd(s["q"], s["k"], s["v"], s["g_fwd"], s["g_bwd"], out=s["o_global"], workspace=workspace,
                     layout=args.layout, plan=args.fwd_plan)
        vb.locality_gate_fwd(s["v"], s["conv_w"], s["gate_logits"], s["o_global"], w.Hg, w.Wg, out=s["out"],
                             layout=args.layout)

    if args.alias_slabs:
        vb.measure_alias_slabs(True)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.tokens / (ms_per_step * 1e-3)

    # ---- per-kernel durations: same K steps again, events recorded by the library on its stream
    vb.timing_enable(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    kern = {}
    for name in vb.KERNELS:
        ms, n = vb.timing_collect(name)
        if n:
            kern[name] = {"avg_us": ms * 1e3 / n, "launches_per_step": n / args.steps}
    vb.timing_enable(False)
    if args.alias_slabs:
        vb.measure_alias_slabs(False)
    # An event pair brackets its kernel plus the cost of the two records.  The launches of a step run back to
    # back on one stream, so their true durations add up to the step's wall time at most: what the raw event
    # times sum to beyond that is the records' cost, shared equally by the launches and taken off.
    raw_sum = sum(k["avg_us"] * k["launches_per_step"] for k in kern.values())
    n_launches = sum(k["launches_per_step"] for k in kern.values())
    pair_us = max(raw_sum - ms_per_step * 1e3, 0.0) / n_launches
    for k in kern.values():
        k["avg_us"] = max(k["avg_us"] - pair_us, 0.0)

    # ---- roofline of the dominant entry point (algorithmic bytes / flops per head-token)
    ht = w.head_tokens
    bigla_bytes = (4 * w.dk + 2 * w.dv) * esize * ht          # q,k,g_fwd,g_bwd,v read once, out written once
    bigla_flops = (8 * w.dk * w.dv + 2 * 64 * (w.dk + w.dv)) * ht  # chunkwise form at the nominal chunk of 64
    loc_bytes = 4 * esize * ht * w.dv                          # x, z, o_global read; out written
    bigla_launches = [n for n in BIGLA_KERNELS if n in kern]
    bigla_us = sum(kern[n]["avg_us"] * kern[n]["launches_per_step"] for n in bigla_launches)
    traffic = measured_traffic()
    per_launch = {n: traffic.get((w.name, n)) for n in bigla_launches}
    # bigla_fwd is the dominant entry point: its algorithmic bytes (q, k, v, both gates read once, out written
    # once) over the time of ALL its launches; the launches one by one are in `launches`
    achieved_gbs = bigla_bytes / (bigla_us * 1e-6) / 1e9
    roofline = {
        "kernel": "bigla_fwd (" + " + ".join(bigla_launches) + ")", "bound": "hbm", "achieved": round(achieved_gbs, 1),
        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
        "traffic": (sum(per_launch.values()) if all(v is not None for v in per_launch.values()) and not args.alias_slabs
                    and args.fwd_plan == "auto" and args.layout == "bhld" and not args.dk else None),
        "avg_us": round(bigla_us, 2), "algorithmic_bytes": bigla_bytes,
        "launches": {n: {"avg_us": round(kern[n]["avg_us"], 2), "traffic": per_launch[n]} for n in bigla_launches},
    }
    extra = {
        "kernels_us": {n: round(k["avg_us"] * k["launches_per_step"], 2) for n, k in kern.items()},
        "event_pair_us": round(pair_us, 2),
        "bigla_us": round(bigla_us, 2),
        "bigla_tokens_per_s": round(w.tokens / (bigla_us * 1e-6), 1),
        "bigla_tflops": round(bigla_flops / (bigla_us * 1e-6) / 1e12, 2),
        "bigla_frac_bf16_mfma_peak": round(bigla_flops / (bigla_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "bigla_hbm_gbs": round(bigla_bytes / (bigla_us * 1e-6) / 1e9, 1),
        "bigla_frac_hbm_peak": round(bigla_bytes / (bigla_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
    }
    if "locality_gate" in kern:
        lus = kern["locality_gate"]["avg_us"]
        extra["locality_hbm_gbs"] = round(loc_bytes / (lus * 1e-6) / 1e9, 1)
        extra["locality_frac_hbm_peak"] = round(loc_bytes / (lus * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        extra["locality_traffic"] = traffic.get((w.name, "locality_gate"))
    if args.alias_slabs:
        extra["alias_slabs"] = True

    # ---- side measurement: the gradient of the token mixer (d_out := the gate logits, any values do)
    if args.backward:
        bws = torch.empty(int(vb.lib().bigla_bwd_workspace_bytes(w.B, w.H, w.L, w.dk, w.dv, code)), dtype=torch.uint8,
                          device=dev)
        n_bwd = max(20, args.steps // 5)

        def bwd(i):
            s = sets[i % n_sets]
            vb.bigla_bwd(s["q"], s["k"], s["v"], s["g_fwd"], s["g_bwd"], s["gate_logits"], workspace=bws,
                         layout=args.layout)

        for i in range(max(5, n_bwd // 5)):
            bwd(i)
        torch.cuda.synchronize()
        b0 = time.perf_counter()
        for i in range(n_bwd):
            bwd(i)
        torch.cuda.synchronize()
        bwd_us = (time.perf_counter() - b0) * 1e6 / n_bwd
        extra["backward"] = {"us": round(bwd_us, 2), "tokens_per_s": round(w.tokens / (bwd_us * 1e-6), 1),
                             "calls": n_bwd, "vs_forward_mixer": round(bwd_us / bigla_us, 2)}

    # ---- side measurement: the step with the gate producer in front of it (Section 3 gate), both plans
    if args.gate_width:
        gi = wl.generate_gate_inputs(w.B, w.L, args.gate_width, w.H, w.dk, w.dtype, seed=args.seed, bias_mu=w.gate_mu)
        gt = {n: wl.to_torch(a, w.dtype, dev) for n, a in gi.items()}
        gw1, gw2 = gt["w1"].t().contiguous(), gt["w2"].t().contiguous()
        xs = [torch.roll(gt["x"], shifts=i, dims=0).contiguous() for i in range(n_sets)]
        gws = torch.empty(int(vb.lib().gated_bigla_workspace_bytes(w.B, w.H, w.L, w.dk, w.dv, code)), dtype=torch.uint8,
                          device=dev)
        gated = {"D": args.gate_width}
        for plan in ("separate", "in_state_pass"):
            def gstep(i):
                s = sets[i % n_sets]
                vb.gated_bigla_fwd(xs[i % n_sets], gw1, gw2, s["q"], s["k"], s["v"], bias=gt["bias"], layout=args.layout,
                                   plan=plan, out=s["o_global"], g_fwd=s["g_fwd"], g_bwd=s["g_bwd"], workspace=gws)
                vb.locality_gate_fwd(s["v"], s["conv_w"], s["gate_logits"], s["o_global"], w.Hg, w.Wg, out=s["out"],
                                     layout=args.layout)
            try:
                for i in range(args.warmup):
                    gstep(i)
            except vb.VigError:
                gated[plan + "_us"] = None
                continue
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            for i in range(args.steps):
                gstep(i)
            torch.cuda.synchronize()
            gated[plan + "_us"] = round((time.perf_counter() - g0) * 1e6 / args.steps, 2)
        extra["gated"] = gated

    # ---- CPU oracle on the host cores (reported baseline, not the target)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        wd = {n: wl.widen(a, w.dtype) for n, a in stored.items()}
        best, spent, reps = float("inf"), 0.0, 0
        while reps < 3 or (spent < args.cpu_budget_s and reps < 2000):
            c0 = time.perf_counter()
            og = oracle.bigla(wd["q"], wd["k"], wd["v"], wd["g_fwd"], wd["g_bwd"])
            oracle.locality_gate(wd["v"], wd["conv_w"], wd["gate_logits"], og, w.Hg, w.Wg)
            dt = time.perf_counter() - c0
            best, spent, reps = min(best, dt), spent + dt, reps + 1
            if spent > 3 * args.cpu_budget_s:
                break
        cpu = {"value": round(w.tokens / best, 1), "unit": "tokens/s", "cores": oracle.max_threads(),
               "kind": "oracle",
               "sample": f"the whole workload ({w.B * w.H} slabs of L={w.L}), fp64, best of {reps} passes "
                         f"({spent:.1f} s of CPU work)"}

    line = {
        "metric": "BiGLA fwd tokens/sec and % bf16 MFMA peak at L=4096, H=6, d=64 (1 GPU)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "L": w.L, "grid": [w.Hg, w.Wg], "dk": w.dk, "dv": w.dv,
                   "gate_logit_mean": w.gate_mu, "layout": args.layout, "buffer_sets": n_sets, "set_bytes": set_bytes,
                   "fwd_plan": args.fwd_plan},
        "roofline": roofline, "cpu_baseline": cpu, "detail": extra,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
