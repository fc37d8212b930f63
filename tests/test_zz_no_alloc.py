"""bigla_fwd_static_scratch, the entry point for callers that cannot allocate: through the C ABI,
against bigla_fwd_layout on the same inputs (bit for bit) and against the oracle, on two calls in
a row of which the second is smaller (the library's one scratch array keeps the first call's
contents), and the size limit."""
import ctypes

import numpy as np
import pytest

from paper_2405_18425_amd import workloads as wl
from parity import TOL, assert_close, run_bigla_oracle

pytestmark = pytest.mark.gpu


def _both_entry_points(w, seed, layout):
    """One problem through bigla_fwd_static_scratch and bigla_fwd_layout, raw ctypes calls."""
    import torch
    from paper_2405_18425_amd import binding as vb

    lib = vb.lib()
    s = wl.generate(w, seed=seed, tensors=("q", "k", "v", "g_fwd", "g_bwd"))
    t = {n: wl.to_torch(s[n], w.dtype, "cuda:0") for n in s}
    if layout == "blhd":
        t = {n: a.transpose(1, 2).contiguous() for n, a in t.items()}
    code = vb.VIG_BF16 if w.dtype == "bf16" else vb.VIG_F32
    lay = vb.LAYOUTS[layout]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptrs = [ctypes.c_void_p(t[n].data_ptr()) for n in ("q", "k", "v", "g_fwd", "g_bwd")]
    out_static = torch.full_like(t["v"], float("nan"))
    out_ws = torch.full_like(t["v"], float("nan"))
    need = vb.bigla_workspace_bytes(w.B, w.H, w.L, w.dk, w.dv, code)
    assert 0 < need <= vb.VIG_STATIC_SCRATCH_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = lib.bigla_fwd_static_scratch(*ptrs, ctypes.c_void_p(out_static.data_ptr()), w.B, w.H, w.L, w.dk, w.dv, code,
                                      lay, stream)
    assert st == vb.VIG_OK, vb.status_str(st)
    assert torch.cuda.memory_allocated() == before  # nothing came from torch's allocator either
    st = lib.bigla_fwd_layout(*ptrs, ctypes.c_void_p(out_ws.data_ptr()), w.B, w.H, w.L, w.dk, w.dv, code, lay,
                              ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(need), stream)
    assert st == vb.VIG_OK, vb.status_str(st)
    torch.cuda.synchronize()
    assert torch.equal(out_static.view(torch.int16 if w.dtype == "bf16" else torch.int32),
                       out_ws.view(torch.int16 if w.dtype == "bf16" else torch.int32)), "entry points disagree"
    if layout == "blhd":
        out_static = out_static.transpose(1, 2).contiguous()
    got = wl.widen(wl.from_torch(out_static, w.dtype), w.dtype)
    assert_close(got, run_bigla_oracle(s, w.dtype), TOL[w.dtype], f"static scratch {w.name}")


def test_static_scratch_two_calls_second_smaller():
    big = wl.Workload("noalloc_big", B=2, H=6, Hg=32, Wg=40, dk=64, dv=64, dtype="bf16", gate_mu=1.0)
    small = wl.Workload("noalloc_small", B=1, H=3, Hg=1, Wg=200, dk=64, dv=64, dtype="bf16", gate_mu=0.0)
    print(f"static scratch: {big}", flush=True)
    _both_entry_points(big, seed=21, layout="bhld")
    print(f"static scratch: {small}", flush=True)
    _both_entry_points(small, seed=22, layout="bhld")
    # once more, token-major and with the exact recurrence's scratch (bf16 storage, 16-wide head)
    rec = wl.Workload("noalloc_rec", B=1, H=2, Hg=1, Wg=77, dk=16, dv=32, dtype="bf16", gate_mu=-1.0)
    print(f"static scratch: {rec}", flush=True)
    _both_entry_points(rec, seed=23, layout="blhd")


def test_static_scratch_limit():
    """A problem whose scratch exceeds the static array is refused before anything is launched
    (dummy pointers: the call must not touch them)."""
    from paper_2405_18425_amd import binding as vb

    lib = vb.lib()
    B, H, L = 64, 16, 8192
    assert vb.bigla_workspace_bytes(B, H, L, 64, 64, vb.VIG_BF16) > vb.VIG_STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p(0x10000)
    st = lib.bigla_fwd_static_scratch(p, p, p, p, p, p, B, H, L, 64, 64, vb.VIG_BF16, vb.VIG_LAYOUT_BHLD, None)
    assert st == vb.VIG_ERR_SCRATCH_LIMIT, vb.status_str(st)
    assert "VIG_STATIC_SCRATCH_BYTES" in vb.status_str(st)
