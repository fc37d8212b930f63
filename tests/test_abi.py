"""The C-ABI library loads, exports what include/vig_bigla.h declares, and validates arguments
on the host before anything is launched (CPU only: every call here returns before a launch)."""
import ctypes
import os
import re

import pytest

from paper_2405_18425_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vig_bigla.h")

PTR = 0x10000  # a non-NULL, 16-byte aligned dummy: validation must reject before dereferencing


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"}


def test_header_and_exports_agree():
    names = declared_functions()
    assert names == set(vb.EXPORTS)
    lib = vb.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    for code in range(-9, 1):
        s = vb.status_str(code)
        assert s and "unknown" not in s
    assert "unknown" in vb.status_str(5)
    assert vb.lib().vig_last_hip_error() == 0


def call_bigla(q=PTR, k=PTR, v=PTR, gf=PTR, gb=PTR, out=PTR, B=1, H=1, L=8, dk=16, dv=16, dtype=vb.VIG_F32,
               ws=None, ws_bytes=0):
    return vb.lib().bigla_fwd(q, k, v, gf, gb, out, B, H, L, dk, dv, dtype, ws, ws_bytes, None)


def test_static_scratch_validation_codes():
    """The entry point that allocates nothing validates on the host like bigla_fwd_layout, and refuses
    what its static array cannot hold (no GPU is touched by any of these calls)."""
    f = vb.lib().bigla_fwd_static_scratch

    def call(q=PTR, out=PTR, B=1, H=1, L=8, dk=16, dv=16, dtype=vb.VIG_BF16, layout=vb.VIG_LAYOUT_BHLD):
        return f(q, PTR, PTR, PTR, PTR, out, B, H, L, dk, dv, dtype, layout, None)

    assert call(B=0) == vb.VIG_ERR_SHAPE
    assert call(dtype=9) == vb.VIG_ERR_DTYPE
    assert call(dk=48) == vb.VIG_ERR_UNSUPPORTED
    assert call(B=1 << 20, H=1 << 20, L=1 << 20) == vb.VIG_ERR_SHAPE
    # the five benchmark configurations fit, a much larger problem does not
    for B, H, L in ((64, 3, 196), (64, 6, 196), (16, 12, 1024), (8, 6, 4096)):
        assert 0 < vb.bigla_workspace_bytes(B, H, L, 64, 64, vb.VIG_BF16) <= vb.VIG_STATIC_SCRATCH_BYTES
    assert vb.bigla_workspace_bytes(64, 16, 8192, 64, 64, vb.VIG_BF16) > vb.VIG_STATIC_SCRATCH_BYTES
    assert call(B=64, H=16, L=8192, dk=64, dv=64) == vb.VIG_ERR_SCRATCH_LIMIT
    header = open(HEADER).read()
    assert f"#define VIG_STATIC_SCRATCH_BYTES ({vb.VIG_STATIC_SCRATCH_BYTES >> 20}u << 20)" in header


def test_bigla_validation_codes():
    for name in ("q", "k", "v", "gf", "gb", "out"):
        assert call_bigla(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "L", "dk", "dv"):
        assert call_bigla(**{name: 0}) == vb.VIG_ERR_SHAPE
        assert call_bigla(**{name: -3}) == vb.VIG_ERR_SHAPE
    assert call_bigla(dtype=7) == vb.VIG_ERR_DTYPE
    assert call_bigla(dk=48) == vb.VIG_ERR_UNSUPPORTED
    assert call_bigla(dv=128) == vb.VIG_ERR_UNSUPPORTED
    assert call_bigla(q=PTR + 8) == vb.VIG_ERR_ALIGN
    assert call_bigla(out=PTR + 2) == vb.VIG_ERR_ALIGN
    assert call_bigla(B=1 << 20, H=1 << 20, L=1 << 20) == vb.VIG_ERR_SHAPE
    # bf16 needs scratch for every shape
    for dk, dv in ((16, 16), (64, 64), (32, 64)):
        need = vb.bigla_workspace_bytes(2, 3, 100, dk, dv, vb.VIG_BF16)
        assert need > 0
        assert call_bigla(B=2, H=3, L=100, dk=dk, dv=dv, dtype=vb.VIG_BF16) == vb.VIG_ERR_WORKSPACE
        assert call_bigla(B=2, H=3, L=100, dk=dk, dv=dv, dtype=vb.VIG_BF16, ws=PTR,
                          ws_bytes=need - 1) == vb.VIG_ERR_WORKSPACE
        assert call_bigla(B=2, H=3, L=100, dk=dk, dv=dv, dtype=vb.VIG_BF16, ws=PTR + 4,
                          ws_bytes=need) == vb.VIG_ERR_ALIGN


def test_offset_range_limits():
    """The kernels address one slab's rows (token-major: one batch element's) with 32-bit byte
    offsets; shapes beyond that are refused on the host."""
    L = vb.lib()
    big = 1 << 40
    # chunkwise path: sequence length below 2^24, and (L + 64) rows of 128 bytes (times H when token-major)
    args = (PTR,) * 6 + (1, 1, 1 << 24, 64, 64, vb.VIG_BF16)
    assert L.bigla_fwd_layout(*args, vb.VIG_LAYOUT_BHLD, PTR, big, None) == vb.VIG_ERR_SHAPE
    args = (PTR,) * 6 + (1, 8, (1 << 22) - 32, 64, 64, vb.VIG_BF16)
    assert L.bigla_fwd_layout(*args, vb.VIG_LAYOUT_BLHD, PTR, big, None) == vb.VIG_ERR_SHAPE
    # the exact recurrence has no such limit on L (it is refused for the workspace here, not the shape)
    args = (PTR,) * 6 + (1, 1, 1 << 24, 16, 16, vb.VIG_BF16)
    assert L.bigla_fwd_layout(*args, vb.VIG_LAYOUT_BHLD, None, 0, None) == vb.VIG_ERR_WORKSPACE
    # locality kernel: one slab (one batch element when token-major) below 4 GiB
    assert L.locality_gate_fwd_layout(PTR, PTR, None, PTR, PTR, PTR, 1, 1, 1 << 13, 1 << 13, 64, vb.VIG_F32,
                                      vb.VIG_LAYOUT_BHLD, None) == vb.VIG_ERR_SHAPE
    assert L.locality_gate_fwd_layout(PTR, PTR, None, PTR, PTR, PTR, 1, 64, 1 << 10, 1 << 10, 64, vb.VIG_BF16,
                                      vb.VIG_LAYOUT_BLHD, None) == vb.VIG_ERR_SHAPE


def test_workspace_query():
    assert vb.bigla_workspace_bytes(1, 1, 64, 16, 16, vb.VIG_F32) == 0
    assert vb.bigla_workspace_bytes(0, 1, 64, 16, 16, vb.VIG_F32) == 0
    assert vb.bigla_workspace_bytes(1, 1, 64, 48, 16, vb.VIG_BF16) == 0
    a = vb.bigla_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16)
    b = vb.bigla_workspace_bytes(16, 6, 4096, 64, 64, vb.VIG_BF16)
    assert 0 < a < b and a % 16 == 0


def call_loc(x=PTR, w=PTR, bias=None, z=PTR, og=PTR, out=PTR, B=1, H=1, Hg=4, Wg=4, dv=16, dtype=vb.VIG_BF16):
    return vb.lib().locality_gate_fwd(x, w, bias, z, og, out, B, H, Hg, Wg, dv, dtype, None)


def test_locality_validation_codes():
    for name in ("x", "w", "z", "og", "out"):
        assert call_loc(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "Hg", "Wg", "dv"):
        assert call_loc(**{name: 0}) == vb.VIG_ERR_SHAPE
    assert call_loc(dtype=-1) == vb.VIG_ERR_DTYPE
    assert call_loc(dv=24) == vb.VIG_ERR_UNSUPPORTED
    assert call_loc(bias=PTR + 6) == vb.VIG_ERR_ALIGN
    assert call_loc(w=PTR + 1) == vb.VIG_ERR_ALIGN


def test_layout_entry_points_validate():
    L = vb.lib()
    args = (PTR,) * 6 + (1, 1, 8, 16, 16, vb.VIG_F32)
    assert L.bigla_fwd_layout(*args, 2, None, 0, None) == vb.VIG_ERR_LAYOUT
    assert L.bigla_fwd_layout(*args, -1, None, 0, None) == vb.VIG_ERR_LAYOUT
    assert L.bigla_fwd_layout(None, *args[1:], vb.VIG_LAYOUT_BLHD, None, 0, None) == vb.VIG_ERR_NULL
    # token-major offsets are 32-bit inside a batch element
    big = (PTR,) * 6 + (1, 64, 1 << 23, 64, 64, vb.VIG_BF16)
    assert L.bigla_fwd_layout(*big, vb.VIG_LAYOUT_BLHD, None, 0, None) == vb.VIG_ERR_SHAPE
    largs = (PTR, PTR, None, PTR, PTR, PTR, 1, 1, 4, 4, 16, vb.VIG_BF16)
    assert L.locality_gate_fwd_layout(*largs, 3, None) == vb.VIG_ERR_LAYOUT
    assert L.locality_gate_fwd_layout(PTR, PTR, None, PTR, PTR, PTR, 1, 1, 4, 4, 24, vb.VIG_BF16,
                                      vb.VIG_LAYOUT_BLHD, None) == vb.VIG_ERR_UNSUPPORTED


def test_gate_producer_validation_codes():
    L = vb.lib()

    def call(x=PTR, w1=PTR, w2=PTR, bias=None, gf=PTR, gb=PTR, B=1, H=1, Ln=8, D=32, dk=16, tau=16.0,
             dtype=vb.VIG_BF16, layout=vb.VIG_LAYOUT_BHLD):
        return L.gate_producer_fwd(x, w1, w2, bias, gf, gb, B, H, Ln, D, dk, tau, dtype, layout, None)

    for name in ("x", "w1", "w2", "gf", "gb"):
        assert call(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "Ln", "D", "dk"):
        assert call(**{name: 0}) == vb.VIG_ERR_SHAPE
    assert call(tau=0.0) == vb.VIG_ERR_SHAPE
    assert call(tau=-1.0) == vb.VIG_ERR_SHAPE
    assert call(dtype=5) == vb.VIG_ERR_DTYPE
    assert call(layout=9) == vb.VIG_ERR_LAYOUT
    assert call(dk=48) == vb.VIG_ERR_UNSUPPORTED
    assert call(D=40) == vb.VIG_ERR_UNSUPPORTED
    assert call(bias=PTR + 4) == vb.VIG_ERR_ALIGN
    assert call(x=PTR + 8) == vb.VIG_ERR_ALIGN


def test_bigla_fwd_plan_validation_codes():
    L = vb.lib()

    def call(plan, dk=64, dtype=vb.VIG_BF16, layout=vb.VIG_LAYOUT_BHLD, q=PTR):
        return L.bigla_fwd_plan(q, PTR, PTR, PTR, PTR, PTR, 1, 1, 128, dk, 64, dtype, layout, plan, None, 0, None)

    assert call(4) == vb.VIG_ERR_UNSUPPORTED
    assert call(-1) == vb.VIG_ERR_UNSUPPORTED
    for plan in vb.FWD_PLANS.values():
        assert call(plan, q=None) == vb.VIG_ERR_NULL
        assert call(plan, layout=7) == vb.VIG_ERR_LAYOUT
        assert call(plan, dtype=5) == vb.VIG_ERR_DTYPE
        assert call(plan) == vb.VIG_ERR_WORKSPACE  # a valid chunkwise problem without its workspace


def test_gated_bigla_validation_codes():
    L = vb.lib()

    def call(x=PTR, w1=PTR, w2=PTR, bias=None, q=PTR, k=PTR, v=PTR, gf=PTR, gb=PTR, out=PTR, B=1, H=1, Lq=128, D=64,
             dk=64, dv=64, tau=16.0, dtype=vb.VIG_BF16, layout=vb.VIG_LAYOUT_BHLD, plan=0, ws=PTR, ws_bytes=1 << 30):
        return L.gated_bigla_fwd(x, w1, w2, bias, q, k, v, gf, gb, out, B, H, Lq, D, dk, dv, tau, dtype, layout, plan,
                                 ws, ws_bytes, None)

    for name in ("x", "w1", "w2", "q", "k", "v", "gf", "gb", "out"):
        assert call(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "Lq", "D", "dk", "dv"):
        assert call(**{name: 0}) == vb.VIG_ERR_SHAPE
    assert call(tau=0.0) == vb.VIG_ERR_SHAPE
    assert call(dtype=3) == vb.VIG_ERR_DTYPE
    assert call(layout=2) == vb.VIG_ERR_LAYOUT
    assert call(plan=3) == vb.VIG_ERR_UNSUPPORTED
    assert call(D=48) == vb.VIG_ERR_UNSUPPORTED
    assert call(dk=48) == vb.VIG_ERR_UNSUPPORTED
    assert call(ws=None, ws_bytes=0) == vb.VIG_ERR_WORKSPACE
    assert call(ws_bytes=64) == vb.VIG_ERR_WORKSPACE
    assert call(ws=PTR + 8) == vb.VIG_ERR_ALIGN
    # the plan whose state pass makes the gates: bf16, dk = dv = 64, at least two chunks
    fused = vb.GATES_PLANS["in_state_pass"]
    assert call(plan=fused, dtype=vb.VIG_F32) == vb.VIG_ERR_UNSUPPORTED
    assert call(plan=fused, dk=16, dv=16) == vb.VIG_ERR_UNSUPPORTED
    assert call(plan=fused, Lq=40) == vb.VIG_ERR_UNSUPPORTED
    assert call(plan=fused, q=PTR + 8) == vb.VIG_ERR_ALIGN
    assert L.gated_bigla_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16) >= \
        L.bigla_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16) + 8 * 4096 * 32
    assert L.gated_bigla_workspace_bytes(8, 6, 4096, 48, 64, vb.VIG_BF16) == 0


def test_bigla_locality_validation_codes():
    L = vb.lib()

    def call(q=PTR, k=PTR, v=PTR, gf=PTR, gb=PTR, x=PTR, w=PTR, bias=None, z=PTR, out=PTR, B=1, H=1, Hg=4, Wg=4,
             dk=64, dv=64, dtype=vb.VIG_BF16, layout=vb.VIG_LAYOUT_BHLD, plan=0, ws=None, ws_bytes=0):
        return L.bigla_locality_fwd(q, k, v, gf, gb, x, w, bias, z, out, B, H, Hg, Wg, dk, dv, dtype, layout, plan, ws,
                                    ws_bytes, None)

    for name in ("q", "k", "v", "gf", "gb", "x", "w", "z", "out"):
        assert call(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "Hg", "Wg", "dk", "dv"):
        assert call(**{name: 0}) == vb.VIG_ERR_SHAPE
    assert call(Hg=1 << 12, Wg=1 << 12) == vb.VIG_ERR_SHAPE
    assert call(dtype=9) == vb.VIG_ERR_DTYPE
    assert call(layout=4) == vb.VIG_ERR_LAYOUT
    assert call(plan=3) == vb.VIG_ERR_UNSUPPORTED
    assert call(plan=-1) == vb.VIG_ERR_UNSUPPORTED
    assert call(dk=48) == vb.VIG_ERR_UNSUPPORTED
    for plan in vb.PLANS.values():
        need = L.bigla_locality_workspace_bytes(2, 3, 100, 64, 64, vb.VIG_BF16, plan)
        assert need > 0
        kw = dict(B=2, H=3, Hg=10, Wg=10, plan=plan)
        assert call(**kw) == vb.VIG_ERR_WORKSPACE
        assert call(ws=PTR, ws_bytes=need - 1, **kw) == vb.VIG_ERR_WORKSPACE
        assert call(ws=PTR + 4, ws_bytes=need, **kw) == vb.VIG_ERR_ALIGN
    # the fused plan exists for the chunkwise bf16 shapes only; the others keep the intermediate
    fused, two = vb.PLANS["fused_epilogue"], vb.PLANS["two_launches"]
    assert call(dtype=vb.VIG_F32, plan=fused) == vb.VIG_ERR_UNSUPPORTED
    assert call(dk=16, dv=16, plan=fused) == vb.VIG_ERR_UNSUPPORTED
    assert L.bigla_locality_workspace_bytes(1, 1, 64, 16, 16, vb.VIG_F32, fused) == 0
    assert L.bigla_locality_workspace_bytes(1, 1, 64, 16, 16, vb.VIG_F32, two) == 64 * 16 * 4
    a = L.bigla_locality_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16, fused)
    b = L.bigla_locality_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16, two)
    assert a == vb.bigla_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16)
    assert b >= a + 8 * 6 * 4096 * 64 * 2
    assert L.bigla_locality_workspace_bytes(8, 6, 4096, 64, 64, vb.VIG_BF16, 0) in (a, b)
    assert call(x=PTR + 8, Hg=8, Wg=8, plan=fused, ws=PTR, ws_bytes=1 << 30) == vb.VIG_ERR_ALIGN
    # sequences under 32 tokens are the exact recurrence's (no chunkwise launch to carry the epilogue)
    assert call(Hg=4, Wg=4, plan=fused, ws=PTR, ws_bytes=1 << 30) == vb.VIG_ERR_UNSUPPORTED
    assert L.bigla_locality_workspace_bytes(1, 1, 16, 64, 64, vb.VIG_BF16, fused) == 0
    assert call(Hg=4, Wg=8, plan=fused, ws=PTR + 4, ws_bytes=1 << 30) == vb.VIG_ERR_ALIGN
    # token-major rows of one batch element are addressed with 32-bit byte offsets
    assert call(B=1, H=64, Hg=1 << 10, Wg=1 << 10, layout=vb.VIG_LAYOUT_BLHD, plan=fused, ws=PTR,
                ws_bytes=1 << 40) == vb.VIG_ERR_SHAPE


def test_bigla_bwd_validation_codes():
    L = vb.lib()

    def call(q=PTR, k=PTR, v=PTR, gf=PTR, gb=PTR, do=PTR, dq=PTR, dk_=PTR, dv_=PTR, dgf=PTR, dgb=PTR, B=1, H=1, Ln=8,
             dk=16, dv=16, dtype=vb.VIG_F32, layout=vb.VIG_LAYOUT_BHLD, ws=PTR, ws_bytes=1 << 40):
        return L.bigla_bwd(q, k, v, gf, gb, do, dq, dk_, dv_, dgf, dgb, B, H, Ln, dk, dv, dtype, layout, ws, ws_bytes, None)

    for name in ("q", "k", "v", "gf", "gb", "do", "dq", "dk_", "dv_", "dgf", "dgb"):
        assert call(**{name: None}) == vb.VIG_ERR_NULL
    for name in ("B", "H", "Ln", "dk", "dv"):
        assert call(**{name: 0}) == vb.VIG_ERR_SHAPE
    assert call(dtype=2) == vb.VIG_ERR_DTYPE
    assert call(layout=-1) == vb.VIG_ERR_LAYOUT
    assert call(dk=24) == vb.VIG_ERR_UNSUPPORTED
    assert call(dq=PTR + 4) == vb.VIG_ERR_ALIGN
    need = L.bigla_bwd_workspace_bytes(2, 3, 100, 32, 32, vb.VIG_BF16)
    assert need == 2 * 3 * 100 * (3 * 32 + 32) * 4
    assert call(B=2, H=3, Ln=100, dk=32, dv=32, dtype=vb.VIG_BF16, ws=None, ws_bytes=0) == vb.VIG_ERR_WORKSPACE
    assert call(B=2, H=3, Ln=100, dk=32, dv=32, dtype=vb.VIG_BF16, ws_bytes=need - 1) == vb.VIG_ERR_WORKSPACE
    assert L.bigla_bwd_workspace_bytes(2, 3, 100, 48, 64, vb.VIG_BF16) == 0
    # bf16 with 64-wide values and 64- or 32-wide keys adds the chunkwise kernels' states (four
    # 64 x 64 bf16 matrices per chunk), chunk log-decays and slab marks, each rounded up to 256 bytes
    exact = 2 * 3 * 100 * (3 * 64 + 64) * 4
    chunks = 2 * 3 * 2
    assert L.bigla_bwd_workspace_bytes(2, 3, 100, 64, 64, vb.VIG_F32) == exact
    assert L.bigla_bwd_workspace_bytes(2, 3, 100, 64, 64, vb.VIG_BF16) == exact + chunks * 4 * 8192 + chunks * 512 + 256
    assert L.bigla_bwd_workspace_bytes(2, 3, 100, 32, 64, vb.VIG_BF16) == (
        2 * 3 * 100 * (3 * 32 + 64) * 4 + chunks * 4 * 8192 + chunks * 512 + 256)
    assert L.bigla_bwd_workspace_bytes(2, 3, 100, 64, 32, vb.VIG_BF16) == 2 * 3 * 100 * (3 * 64 + 32) * 4

    def plan_call(plan, Ln=8, H=1, layout=vb.VIG_LAYOUT_BHLD):
        return L.bigla_bwd_plan(PTR, PTR, PTR, PTR, PTR, PTR, PTR, PTR, PTR, PTR, PTR, 1, H, Ln, 64, 64, vb.VIG_BF16,
                                layout, plan, None, 0, None)

    assert plan_call(2) == vb.VIG_ERR_UNSUPPORTED
    assert plan_call(-1) == vb.VIG_ERR_UNSUPPORTED
    assert plan_call(0) == vb.VIG_ERR_WORKSPACE and plan_call(1) == vb.VIG_ERR_WORKSPACE
    # the chunkwise kernels address a slab with 32-bit byte offsets; the exact ones do not
    assert plan_call(0, Ln=1 << 22, H=16, layout=vb.VIG_LAYOUT_BLHD) == vb.VIG_ERR_SHAPE
    assert plan_call(1, Ln=1 << 22, H=16, layout=vb.VIG_LAYOUT_BLHD) == vb.VIG_ERR_WORKSPACE


def test_binding_rejects_cpu_tensors():
    import torch

    t = torch.zeros(1, 1, 4, 16)
    with pytest.raises(vb.VigError):
        vb.bigla_fwd(t, t, t, t, t)
    with pytest.raises(vb.VigError):
        vb.locality_gate_fwd(t, torch.zeros(16, 3, 3), t, t, 2, 2)
