"""Driver for rocprofv3 counter runs: a few passes of the BiGLA + locality-gate path on one
workload, plus one plain device-to-device copy of known size that calibrates FETCH_SIZE /
WRITE_SIZE (bytes = counter * factor, factor = known copy bytes / counter of the copy kernel).

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o p -- python3 <repo>/profile_path.py 4 3

A third argument D > 0 adds the forget-gate producer in front of every pass (block input of width D
for the same B, L, H, dk), feeding the gates it makes to bigla_fwd.  A fourth argument 1 or 2 runs
each pass through bigla_locality_fwd with the two-launch plan (1) or the fused-epilogue plan (2)
instead of the two separate entry points; 3 runs bigla_bwd (the gradient of the token mixer, with
the locality step's input as output gradient) after each forward pass, 4 the same through
bigla_bwd_plan with the exact token-by-token kernels only.
"""
from __future__ import annotations

import torch

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

from paper_2405_18425_amd import binding as vb  # noqa: E402
from paper_2405_18425_amd import workloads as wl  # noqa: E402

COPY_BYTES = 256 << 20  # calibration copy: reads 256 MiB, writes 256 MiB


def main(cfg: int = 4, passes: int = 3, gate_width: int = 0, plan: int = 0) -> None:
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
    og = out = None
    for _ in range(passes):
        if gp is not None:
            vb.gate_producer_fwd(gp["x"], gp["w1"], gp["w2"], w.H, w.dk, bias=gp["bias"], g_fwd=t["g_fwd"],
                                 g_bwd=t["g_bwd"])
        if plan in (1, 2):
            out = vb.bigla_locality_fwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], t["v"], t["conv_w"],
                                        t["gate_logits"], w.Hg, w.Wg,
                                        plan={1: "two_launches", 2: "fused_epilogue"}[plan])
            continue
        og = vb.bigla_fwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"])
        out = vb.locality_gate_fwd(t["v"], t["conv_w"], t["gate_logits"], og, w.Hg, w.Wg)
        if plan in (3, 4):
            vb.bigla_bwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], t["gate_logits"],
                         plan="auto" if plan == 3 else "recurrent")
    torch.cuda.synchronize()
    print("profile_path done", w.name, passes, float(out.float().abs().mean()), flush=True)


if __name__ == "__main__":
    main(*(int(a) for a in sys.argv[1:5]))
