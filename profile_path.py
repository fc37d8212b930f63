"""Driver and summariser for the rocprofv3 runs behind the figures under profiles/.

Run mode (the program that rocprofv3 profiles): a few passes of the BiGLA + locality-gate path on
one workload, plus one plain device-to-device copy of known size that calibrates FETCH_SIZE /
WRITE_SIZE (bytes = counter * factor, factor = known copy bytes / counter of the copy kernel).

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o p -- python3 <repo>/profile_path.py 4 3

Positional arguments: workload index, passes, D, mode.  D > 0 adds the forget-gate producer in front
of every pass (block input of width D for the same B, L, H, dk), feeding the gates it makes to
bigla_fwd.  mode 1 or 2 runs each pass through bigla_locality_fwd with the two-launch plan (1) or the
fused-epilogue plan (2) instead of the two separate entry points; 3 runs bigla_bwd (the gradient of
the token mixer, with the locality step's input as output gradient) after each forward pass, 4 the
same through bigla_bwd_plan with the exact token-by-token kernels only; 5 and 6 (with D > 0) run the gate producer
and the token mixer through gated_bigla_fwd, the state pass making the gates itself (5) or as two launches (6).
Options: --fwd-plan auto|four_wave|wave_specialised|slab_sweep (kernels of the chunkwise forward);
--alias-slabs (every slab reads the first slab's inputs: cache-resident contraction phase).

Summary modes (no GPU): they read the CSV files rocprofv3 wrote and print markdown.

    python3 profile_path.py kernels <dir>                    per-kernel durations of a --kernel-trace --stats run
    python3 profile_path.py counters <dir>                   per-kernel averages of every counter of a --pmc run
    python3 profile_path.py traffic <workload> <fetch dir> <write dir>
                                                             rows for profiles/hbm_traffic.md: HBM bytes per launch
                                                             from a FETCH_SIZE and a WRITE_SIZE run, scaled by the
                                                             calibration copy found in the same runs
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

COPY_BYTES = 256 << 20  # calibration copy: reads 256 MiB, writes 256 MiB
# kernels of the library as the bench line names them
KERNEL_KEYS = (("bigla_segment_state_kernel", "segment_state"), ("bigla_ws_state_kernel", "segment_state"),
               ("bigla_segment_out_kernel", "segment_out"), ("bigla_ws_out_kernel", "segment_out"),
               ("bigla_slab_kernel", "slab"), ("locality_gate_kernel", "locality_gate"),
               ("gate_producer", "gate_producer"), ("gate_lowrank", "gate_lowrank"))


def run(cfg: int, passes: int, gate_width: int, mode: int, fwd_plan: str, alias: bool) -> None:
    import torch

    from paper_2405_18425_amd import binding as vb
    from paper_2405_18425_amd import workloads as wl

    w = wl.CONFIGS[cfg]
    dev = "cuda:0"
    t = {n: wl.to_torch(a, w.dtype, dev) for n, a in wl.generate(w, seed=0).items()}
    gp = None
    if gate_width > 0:
        g = wl.generate_gate_inputs(w.B, w.L, gate_width, w.H, w.dk, w.dtype, seed=0, bias_mu=w.gate_mu)
        gp = {n: wl.to_torch(a, w.dtype, dev) for n, a in g.items()}
        gp["w1"], gp["w2"] = gp["w1"].t().contiguous(), gp["w2"].t().contiguous()
    src = torch.empty(COPY_BYTES // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)  # the calibration kernel (an elementwise copy of COPY_BYTES)
    if alias:
        vb.measure_alias_slabs(True)
    og = out = None
    for _ in range(passes):
        if gp is not None and mode in (5, 6):
            og, _, _ = vb.gated_bigla_fwd(gp["x"], gp["w1"], gp["w2"], t["q"], t["k"], t["v"], bias=gp["bias"],
                                          plan={5: "in_state_pass", 6: "separate"}[mode], g_fwd=t["g_fwd"],
                                          g_bwd=t["g_bwd"])
            out = vb.locality_gate_fwd(t["v"], t["conv_w"], t["gate_logits"], og, w.Hg, w.Wg)
            continue
        if gp is not None:
            vb.gate_producer_fwd(gp["x"], gp["w1"], gp["w2"], w.H, w.dk, bias=gp["bias"], g_fwd=t["g_fwd"],
                                 g_bwd=t["g_bwd"])
        if mode in (1, 2):
            out = vb.bigla_locality_fwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], t["v"], t["conv_w"],
                                        t["gate_logits"], w.Hg, w.Wg,
                                        plan={1: "two_launches", 2: "fused_epilogue"}[mode])
            continue
        og = vb.bigla_fwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], plan=fwd_plan)
        out = vb.locality_gate_fwd(t["v"], t["conv_w"], t["gate_logits"], og, w.Hg, w.Wg)
        if mode in (3, 4):
            vb.bigla_bwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], t["gate_logits"],
                         plan="auto" if mode == 3 else "recurrent")
    torch.cuda.synchronize()
    if alias:
        vb.measure_alias_slabs(False)
    print("profile_path done", w.name, passes, float(out.float().abs().mean()), flush=True)


def _find(directory: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {directory}")
    return hits[0]


def _short(name: str) -> str:
    name = name.replace("void vig::(anonymous namespace)::", "").replace("vig::(anonymous namespace)::", "")
    cut = name.find("(")
    return name[:cut] if cut > 0 else name


def summarize_kernels(directory: str) -> None:
    rows = list(csv.DictReader(open(_find(directory, "kernel_stats.csv"))))
    print("| kernel | calls | avg us | min us | max us | % of GPU time |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        if float(r["Percentage"]) < 0.5:
            continue
        print(f"| {_short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
              f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.1f} |")


def _counter_dispatches(directory: str):
    """kernel -> counter -> dispatch -> value (summed over the dispatch's rows)"""
    per = collections.defaultdict(lambda: collections.defaultdict(lambda: collections.defaultdict(float)))
    for r in csv.DictReader(open(_find(directory, "counter_collection.csv"))):
        per[r["Kernel_Name"]][r["Counter_Name"]][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return per


def _counter_means(directory: str):
    """kernel -> counter -> mean over dispatches"""
    return {k: {c: sum(d.values()) / len(d) for c, d in cs.items()} for k, cs in _counter_dispatches(directory).items()}


def summarize_counters(directory: str) -> None:
    means = _counter_means(directory)
    counters = sorted({c for cs in means.values() for c in cs})
    print("| kernel | " + " | ".join(counters) + " |")
    print("|---" * (len(counters) + 1) + "|")
    for k, cs in means.items():
        print(f"| {_short(k)} | " + " | ".join(f"{cs.get(c, 0):.0f}" for c in counters) + " |")


def summarize_traffic(workload: str, fetch_dir: str, write_dir: str) -> None:
    fetch, write = _counter_means(fetch_dir), _counter_means(write_dir)

    def calibration(directory, counter):
        # the 256 MiB device-to-device copy is the runtime's copy kernel; its largest dispatch is the one meant
        # (the host-to-device uploads of the inputs go through the same kernel with tiny counts)
        for k, cs in _counter_dispatches(directory).items():
            if "copyBuffer" in k and counter in cs and max(cs[counter].values()) > 1000:
                return COPY_BYTES / max(cs[counter].values())
        raise SystemExit(f"no calibration copy with {counter}")

    f_fac, w_fac = calibration(fetch_dir, "FETCH_SIZE"), calibration(write_dir, "WRITE_SIZE")
    print(f"<!-- calibration: FETCH_SIZE * {f_fac:.1f} bytes, WRITE_SIZE * {w_fac:.1f} bytes (a plain 256 MiB copy in the same runs) -->")
    print("| workload | kernel | read MB | written MB | bytes |")
    print("|---|---|---|---|---|")
    for k in fetch:
        key = next((short for needle, short in KERNEL_KEYS if needle in k), None)
        if key is None or k not in write:
            continue
        rd, wr = fetch[k].get("FETCH_SIZE", 0) * f_fac, write[k].get("WRITE_SIZE", 0) * w_fac
        print(f"| {workload} | {key} | {rd / 1e6:.1f} | {wr / 1e6:.1f} | {int(rd + wr)} |")


def main() -> None:
    if len(sys.argv) > 1 and sys.argv[1] in ("kernels", "counters", "traffic"):
        mode, rest = sys.argv[1], sys.argv[2:]
        if mode == "kernels":
            summarize_kernels(rest[0])
        elif mode == "counters":
            summarize_counters(rest[0])
        else:
            summarize_traffic(rest[0], rest[1], rest[2])
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("cfg", type=int, nargs="?", default=4)
    ap.add_argument("passes", type=int, nargs="?", default=3)
    ap.add_argument("gate_width", type=int, nargs="?", default=0)
    ap.add_argument("mode", type=int, nargs="?", default=0)
    ap.add_argument("--fwd-plan", default="auto")
    ap.add_argument("--alias-slabs", action="store_true")
    a = ap.parse_args()
    run(a.cfg, a.passes, a.gate_width, a.mode, a.fwd_plan, a.alias_slabs)


if __name__ == "__main__":
    main()
