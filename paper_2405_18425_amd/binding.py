"""Thin ctypes binding over the C-ABI library (include/vig_bigla.h).

Argument marshalling only: shapes, dtypes, device pointers and the current HIP stream are
taken from torch tensors and handed to the library; every step of the path runs in the
library's kernels.  There is no CPU or PyTorch fallback: if the HIP library is missing, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvig_bigla.so")

VIG_OK = 0
VIG_ERR_NULL, VIG_ERR_SHAPE, VIG_ERR_DTYPE, VIG_ERR_UNSUPPORTED = -1, -2, -3, -4
VIG_ERR_ALIGN, VIG_ERR_WORKSPACE, VIG_ERR_HIP, VIG_ERR_LAYOUT = -5, -6, -7, -8
VIG_ERR_SCRATCH_LIMIT = -9
VIG_STATIC_SCRATCH_BYTES = 48 << 20
VIG_F32, VIG_BF16 = 0, 1
VIG_LAYOUT_BHLD, VIG_LAYOUT_BLHD = 0, 1
LAYOUTS = {"bhld": VIG_LAYOUT_BHLD, "blhd": VIG_LAYOUT_BLHD}
PLANS = {"auto": 0, "two_launches": 1, "fused_epilogue": 2}
FWD_PLANS = {"auto": 0, "four_wave": 1, "wave_specialised": 2, "slab_sweep": 3}
GATES_PLANS = {"auto": 0, "separate": 1, "in_state_pass": 2}

# every symbol include/vig_bigla.h declares
EXPORTS = ("bigla_workspace_bytes", "bigla_fwd", "bigla_fwd_layout", "bigla_fwd_plan", "bigla_fwd_static_scratch", "locality_gate_fwd",
           "locality_gate_fwd_layout", "bigla_locality_workspace_bytes", "bigla_locality_fwd", "gate_producer_fwd",
           "gated_bigla_workspace_bytes", "gated_bigla_fwd",
           "bigla_bwd_workspace_bytes", "bigla_bwd", "bigla_bwd_plan",
           "vig_status_str", "vig_last_hip_error", "vig_timing_enable",
           "vig_timing_collect", "vig_measure_alias_slabs")
KERNELS = {"segment_state": 0, "gate_lowrank": 1, "segment_out": 2, "recurrent": 3, "locality_gate": 4,
           "segment_out_general": 5, "gate_producer": 6, "slab": 7, "backward": 8}

_lib = None


class VigError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(message)
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libvig_bigla.so (built in-tree by `__graft_entry__.build()`); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "at the repository root (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.bigla_workspace_bytes.argtypes = [ci] * 6
        L.bigla_workspace_bytes.restype = sz
        L.bigla_fwd.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
        L.bigla_fwd.restype = ci
        L.bigla_fwd_layout.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp]
        L.bigla_fwd_layout.restype = ci
        L.bigla_fwd_plan.argtypes = [vp] * 6 + [ci] * 8 + [vp, sz, vp]
        L.bigla_fwd_plan.restype = ci
        L.bigla_fwd_static_scratch.argtypes = [vp] * 6 + [ci] * 7 + [vp]
        L.bigla_fwd_static_scratch.restype = ci
        L.locality_gate_fwd.argtypes = [vp] * 6 + [ci] * 6 + [vp]
        L.locality_gate_fwd.restype = ci
        L.locality_gate_fwd_layout.argtypes = [vp] * 6 + [ci] * 7 + [vp]
        L.locality_gate_fwd_layout.restype = ci
        L.bigla_locality_workspace_bytes.argtypes = [ci] * 7
        L.bigla_locality_workspace_bytes.restype = sz
        L.bigla_locality_fwd.argtypes = [vp] * 10 + [ci] * 9 + [vp, sz, vp]
        L.bigla_locality_fwd.restype = ci
        L.bigla_bwd_workspace_bytes.argtypes = [ci] * 6
        L.bigla_bwd_workspace_bytes.restype = sz
        L.bigla_bwd.argtypes = [vp] * 11 + [ci] * 7 + [vp, sz, vp]
        L.bigla_bwd.restype = ci
        L.bigla_bwd_plan.argtypes = [vp] * 11 + [ci] * 8 + [vp, sz, vp]
        L.bigla_bwd_plan.restype = ci
        L.gate_producer_fwd.argtypes = [vp] * 6 + [ci] * 5 + [ctypes.c_float, ci, ci, vp]
        L.gate_producer_fwd.restype = ci
        L.gated_bigla_workspace_bytes.argtypes = [ci] * 6
        L.gated_bigla_workspace_bytes.restype = sz
        L.gated_bigla_fwd.argtypes = [vp] * 10 + [ci] * 6 + [ctypes.c_float, ci, ci, ci, vp, sz, vp]
        L.gated_bigla_fwd.restype = ci
        L.vig_status_str.argtypes = [ci]
        L.vig_status_str.restype = ctypes.c_char_p
        L.vig_last_hip_error.argtypes = []
        L.vig_last_hip_error.restype = ci
        L.vig_timing_enable.argtypes = [ci]
        L.vig_timing_enable.restype = ci
        L.vig_measure_alias_slabs.argtypes = [ci]
        L.vig_measure_alias_slabs.restype = ci
        L.vig_timing_collect.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_long)]
        L.vig_timing_collect.restype = ci
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().vig_status_str(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != VIG_OK:
        msg = f"{what}: {status_str(status)}"
        if status == VIG_ERR_HIP:
            msg += f" (hipError_t {lib().vig_last_hip_error()})"
        raise VigError(status, msg)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return VIG_F32
    if t.dtype == torch.bfloat16:
        return VIG_BF16
    raise VigError(VIG_ERR_DTYPE, f"unsupported tensor dtype {t.dtype}")


def _dev(t: torch.Tensor, name: str, shape=None, like: torch.Tensor | None = None) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise VigError(VIG_ERR_NULL, f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise VigError(VIG_ERR_SHAPE, f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise VigError(VIG_ERR_SHAPE, f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if like is not None and (t.dtype != like.dtype or t.device != like.device):
        raise VigError(VIG_ERR_DTYPE, f"{name} must match dtype/device of the other tensors")
    return t


def _stream_ptr(device) -> int:
    return int(torch.cuda.current_stream(device).cuda_stream)


def bigla_workspace_bytes(B: int, H: int, L: int, dk: int, dv: int, dtype: int) -> int:
    return int(lib().bigla_workspace_bytes(B, H, L, dk, dv, dtype))


def _layout_code(layout) -> int:
    if layout not in LAYOUTS:
        raise VigError(VIG_ERR_LAYOUT, f"layout must be one of {sorted(LAYOUTS)}")
    return LAYOUTS[layout]


def bigla_fwd(q, k, v, g_fwd, g_bwd, out=None, workspace=None, layout="bhld", static_scratch=False, plan="auto"):
    """BiGLA forward (Section 4.2.1).  q,k,g_fwd,g_bwd: [B,H,L,dk]; v: [B,H,L,dv] -> out [B,H,L,dv]
    (layout "bhld"), or all of them token-major, [B,L,H,d] (layout "blhd").

    g_* are LOG forget gates (<= 0).  `workspace` is an optional uint8 GPU tensor of at least
    bigla_workspace_bytes(...) bytes; one is allocated with torch when absent.
    static_scratch=True calls bigla_fwd_static_scratch instead: the library's own per-GPU scratch
    array serves as workspace and, given `out`, nothing is allocated.  `plan` other than "auto" goes
    through bigla_fwd_plan ("four_wave", "wave_specialised" or "slab_sweep" kernels of the chunkwise path).
    """
    lay = _layout_code(layout)
    q = _dev(q, "q")
    if q.dim() != 4:
        raise VigError(VIG_ERR_SHAPE, "q must be 4-dimensional")
    if lay == VIG_LAYOUT_BHLD:
        B, H, L, dk = q.shape
    else:
        B, L, H, dk = q.shape
    k = _dev(k, "k", q.shape, q)
    g_fwd = _dev(g_fwd, "g_fwd", q.shape, q)
    g_bwd = _dev(g_bwd, "g_bwd", q.shape, q)
    v = _dev(v, "v", like=q)
    if v.dim() != 4 or tuple(v.shape[:3]) != tuple(q.shape[:3]):
        raise VigError(VIG_ERR_SHAPE, "v must have the leading dimensions of q")
    dv = v.shape[3]
    if out is None:
        out = torch.empty(tuple(v.shape), dtype=q.dtype, device=q.device)
    out = _dev(out, "out", tuple(v.shape), q)
    code = _dtype_code(q)
    if static_scratch:
        with torch.cuda.device(q.device):
            st = lib().bigla_fwd_static_scratch(q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(),
                                                g_bwd.data_ptr(), out.data_ptr(), B, H, L, dk, dv, code, lay,
                                                _stream_ptr(q.device))
        _check(st, "bigla_fwd_static_scratch")
        return out
    need = bigla_workspace_bytes(B, H, L, dk, dv, code)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if plan not in FWD_PLANS:
        raise VigError(VIG_ERR_UNSUPPORTED, f"plan must be one of {sorted(FWD_PLANS)}")
    with torch.cuda.device(q.device):
        if plan != "auto":
            st = lib().bigla_fwd_plan(q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(), g_bwd.data_ptr(),
                                      out.data_ptr(), B, H, L, dk, dv, code, lay, FWD_PLANS[plan], ws_ptr, ws_bytes,
                                      _stream_ptr(q.device))
        elif lay == VIG_LAYOUT_BHLD:
            st = lib().bigla_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(), g_bwd.data_ptr(),
                                 out.data_ptr(), B, H, L, dk, dv, code, ws_ptr, ws_bytes, _stream_ptr(q.device))
        else:
            st = lib().bigla_fwd_layout(q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(),
                                        g_bwd.data_ptr(), out.data_ptr(), B, H, L, dk, dv, code, lay, ws_ptr,
                                        ws_bytes, _stream_ptr(q.device))
    _check(st, "bigla_fwd")
    return out


def locality_gate_fwd(x, w, gate_logits, o_global, Hg: int, Wg: int, bias=None, out=None, layout="bhld"):
    """2D gating locality injection (Section 4.2.2).

    x, gate_logits, o_global: [B,H,Hg*Wg,dv] (layout "bhld") or [B,Hg*Wg,H,dv] (layout "blhd");
    w: [H*dv,3,3]; bias: [H*dv] or None -> out like x.
    """
    lay = _layout_code(layout)
    x = _dev(x, "x")
    if x.dim() != 4:
        raise VigError(VIG_ERR_SHAPE, "x must be 4-dimensional")
    if lay == VIG_LAYOUT_BHLD:
        B, H, L, dv = x.shape
    else:
        B, L, H, dv = x.shape
    if L != Hg * Wg:
        raise VigError(VIG_ERR_SHAPE, "x.shape[2] must equal Hg*Wg")
    w = _dev(w, "w", (H * dv, 3, 3), x)
    gate_logits = _dev(gate_logits, "gate_logits", x.shape, x)
    o_global = _dev(o_global, "o_global", x.shape, x)
    if bias is not None:
        bias = _dev(bias, "bias", (H * dv,), x)
    if out is None:
        out = torch.empty_like(x)
    out = _dev(out, "out", x.shape, x)
    with torch.cuda.device(x.device):
        bias_ptr = bias.data_ptr() if bias is not None else None
        if lay == VIG_LAYOUT_BHLD:
            st = lib().locality_gate_fwd(x.data_ptr(), w.data_ptr(), bias_ptr, gate_logits.data_ptr(),
                                         o_global.data_ptr(), out.data_ptr(), B, H, Hg, Wg, dv, _dtype_code(x),
                                         _stream_ptr(x.device))
        else:
            st = lib().locality_gate_fwd_layout(x.data_ptr(), w.data_ptr(), bias_ptr, gate_logits.data_ptr(),
                                                o_global.data_ptr(), out.data_ptr(), B, H, Hg, Wg, dv,
                                                _dtype_code(x), lay, _stream_ptr(x.device))
    _check(st, "locality_gate_fwd")
    return out


def bigla_locality_fwd(q, k, v, g_fwd, g_bwd, x, w, gate_logits, Hg: int, Wg: int, bias=None, out=None,
                       workspace=None, layout="bhld", plan="auto"):
    """Token mixer and locality blend in one call (Sections 4.2.1 and 4.2.2):
    out = G * DWConv3x3(x) + (1 - G) * BiGLA(q, k, v, g_fwd, g_bwd), G = sigmoid(gate_logits).
    Tensors as for bigla_fwd and locality_gate_fwd, L = Hg*Wg.  plan: "auto", "two_launches" or
    "fused_epilogue" (the blend inside the chunkwise output pass; bf16, dv = 64, dk = 64 or 32).
    """
    lay = _layout_code(layout)
    if plan not in PLANS:
        raise VigError(VIG_ERR_UNSUPPORTED, f"plan must be one of {sorted(PLANS)}")
    q = _dev(q, "q")
    if q.dim() != 4:
        raise VigError(VIG_ERR_SHAPE, "q must be 4-dimensional")
    if lay == VIG_LAYOUT_BHLD:
        B, H, L, dk = q.shape
    else:
        B, L, H, dk = q.shape
    if L != Hg * Wg:
        raise VigError(VIG_ERR_SHAPE, "the sequence length must equal Hg*Wg")
    k = _dev(k, "k", q.shape, q)
    g_fwd = _dev(g_fwd, "g_fwd", q.shape, q)
    g_bwd = _dev(g_bwd, "g_bwd", q.shape, q)
    v = _dev(v, "v", like=q)
    if v.dim() != 4 or tuple(v.shape[:3]) != tuple(q.shape[:3]):
        raise VigError(VIG_ERR_SHAPE, "v must have the leading dimensions of q")
    dv = v.shape[3]
    x = _dev(x, "x", v.shape, q)
    gate_logits = _dev(gate_logits, "gate_logits", v.shape, q)
    w = _dev(w, "w", (H * dv, 3, 3), q)
    if bias is not None:
        bias = _dev(bias, "bias", (H * dv,), q)
    if out is None:
        out = torch.empty(tuple(v.shape), dtype=q.dtype, device=q.device)
    out = _dev(out, "out", tuple(v.shape), q)
    code = _dtype_code(q)
    need = int(lib().bigla_locality_workspace_bytes(B, H, L, dk, dv, code, PLANS[plan]))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(q.device):
        st = lib().bigla_locality_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(), g_bwd.data_ptr(),
                                      x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                      gate_logits.data_ptr(), out.data_ptr(), B, H, Hg, Wg, dk, dv, code, lay,
                                      PLANS[plan], ws_ptr, ws_bytes, _stream_ptr(q.device))
    _check(st, "bigla_locality_fwd")
    return out


BWD_PLANS = {"auto": 0, "recurrent": 1}


def bigla_bwd(q, k, v, g_fwd, g_bwd, d_out, workspace=None, layout="bhld", plan="auto"):
    """Gradient of bigla_fwd (Section 4.2.1): returns (dq, dk, dv, dg_fwd, dg_bwd) for the output
    gradient d_out (shaped like v); tensors as for bigla_fwd.  plan: "auto" (bigla_bwd) or
    "recurrent" (bigla_bwd_plan with VIG_BWD_RECURRENT: the exact token-by-token kernels only)."""
    if plan not in BWD_PLANS:
        raise VigError(VIG_ERR_UNSUPPORTED, f"unknown plan {plan!r}")
    lay = _layout_code(layout)
    q = _dev(q, "q")
    if q.dim() != 4:
        raise VigError(VIG_ERR_SHAPE, "q must be 4-dimensional")
    if lay == VIG_LAYOUT_BHLD:
        B, H, L, dk = q.shape
    else:
        B, L, H, dk = q.shape
    k = _dev(k, "k", q.shape, q)
    g_fwd = _dev(g_fwd, "g_fwd", q.shape, q)
    g_bwd = _dev(g_bwd, "g_bwd", q.shape, q)
    v = _dev(v, "v", like=q)
    if v.dim() != 4 or tuple(v.shape[:3]) != tuple(q.shape[:3]):
        raise VigError(VIG_ERR_SHAPE, "v must have the leading dimensions of q")
    dv = v.shape[3]
    d_out = _dev(d_out, "d_out", v.shape, q)
    dq, dk_, dgf, dgb = (torch.empty_like(q) for _ in range(4))
    dv_ = torch.empty_like(v)
    code = _dtype_code(q)
    need = int(lib().bigla_bwd_workspace_bytes(B, H, L, dk, dv, code))
    if need == 0:
        raise VigError(VIG_ERR_UNSUPPORTED, "unsupported shape for bigla_bwd")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), g_fwd.data_ptr(), g_bwd.data_ptr(), d_out.data_ptr(),
                dq.data_ptr(), dk_.data_ptr(), dv_.data_ptr(), dgf.data_ptr(), dgb.data_ptr(), B, H, L, dk, dv, code, lay)
        tail = (workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(q.device))
        if plan == "auto":
            st = lib().bigla_bwd(*args, *tail)
        else:
            st = lib().bigla_bwd_plan(*args, BWD_PLANS[plan], *tail)
    _check(st, "bigla_bwd")
    return dq, dk_, dv_, dgf, dgb


def gate_producer_fwd(x, w1, w2, H: int, dk: int, bias=None, tau: float = 16.0, layout="bhld", g_fwd=None,
                      g_bwd=None):
    """Direction-wise log forget gates (Section 3 gate; Eq. (BiGLA) lines 1-2).

    x: [B,L,D]; w1: [16,D] and w2: [2*H*dk,16] (linear-layer weight layout); bias: [2*H*dk] or None
    -> (g_fwd, g_bwd), each [B,H,L,dk] (layout "bhld") or [B,L,H,dk] ("blhd").
    """
    lay = _layout_code(layout)
    x = _dev(x, "x")
    if x.dim() != 3:
        raise VigError(VIG_ERR_SHAPE, "x must be [B,L,D]")
    B, L, D = x.shape
    w1 = _dev(w1, "w1", (16, D), x)
    w2 = _dev(w2, "w2", (2 * H * dk, 16), x)
    if bias is not None:
        bias = _dev(bias, "bias", (2 * H * dk,), x)
    shape = (B, H, L, dk) if lay == VIG_LAYOUT_BHLD else (B, L, H, dk)
    if g_fwd is None:
        g_fwd = torch.empty(shape, dtype=x.dtype, device=x.device)
    if g_bwd is None:
        g_bwd = torch.empty(shape, dtype=x.dtype, device=x.device)
    g_fwd = _dev(g_fwd, "g_fwd", shape, x)
    g_bwd = _dev(g_bwd, "g_bwd", shape, x)
    with torch.cuda.device(x.device):
        st = lib().gate_producer_fwd(x.data_ptr(), w1.data_ptr(), w2.data_ptr(),
                                     bias.data_ptr() if bias is not None else None, g_fwd.data_ptr(),
                                     g_bwd.data_ptr(), B, H, L, D, dk, float(tau), _dtype_code(x), lay,
                                     _stream_ptr(x.device))
    _check(st, "gate_producer_fwd")
    return g_fwd, g_bwd


def gated_bigla_fwd(x, w1, w2, q, k, v, bias=None, tau: float = 16.0, layout="bhld", plan="auto", out=None,
                    g_fwd=None, g_bwd=None, workspace=None):
    """gate_producer_fwd then bigla_fwd as one call (Section 3 gate; Eq. (BiGLA)): returns (out, g_fwd, g_bwd).

    plan "in_state_pass": the chunkwise state pass makes the gates itself from x W1; "separate": two launches.
    """
    lay = _layout_code(layout)
    if plan not in GATES_PLANS:
        raise VigError(VIG_ERR_UNSUPPORTED, f"plan must be one of {sorted(GATES_PLANS)}")
    q = _dev(q, "q")
    if q.dim() != 4:
        raise VigError(VIG_ERR_SHAPE, "q must be 4-dimensional")
    if lay == VIG_LAYOUT_BHLD:
        B, H, L, dk = q.shape
    else:
        B, L, H, dk = q.shape
    dv = v.shape[-1]
    x = _dev(x, "x", None, q)
    if x.dim() != 3 or x.shape[0] != B or x.shape[1] != L:
        raise VigError(VIG_ERR_SHAPE, "x must be [B,L,D]")
    D = x.shape[2]
    w1 = _dev(w1, "w1", (16, D), q)
    w2 = _dev(w2, "w2", (2 * H * dk, 16), q)
    if bias is not None:
        bias = _dev(bias, "bias", (2 * H * dk,), q)
    kshape = tuple(q.shape)
    vshape = kshape[:-1] + (dv,)
    k = _dev(k, "k", kshape, q)
    v = _dev(v, "v", vshape, q)
    g_fwd = torch.empty(kshape, dtype=q.dtype, device=q.device) if g_fwd is None else _dev(g_fwd, "g_fwd", kshape, q)
    g_bwd = torch.empty(kshape, dtype=q.dtype, device=q.device) if g_bwd is None else _dev(g_bwd, "g_bwd", kshape, q)
    out = torch.empty(vshape, dtype=q.dtype, device=q.device) if out is None else _dev(out, "out", vshape, q)
    code = _dtype_code(q)
    need = lib().gated_bigla_workspace_bytes(B, H, L, dk, dv, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        st = lib().gated_bigla_fwd(x.data_ptr(), w1.data_ptr(), w2.data_ptr(),
                                   bias.data_ptr() if bias is not None else None, q.data_ptr(), k.data_ptr(),
                                   v.data_ptr(), g_fwd.data_ptr(), g_bwd.data_ptr(), out.data_ptr(), B, H, L, D, dk,
                                   dv, float(tau), code, lay, GATES_PLANS[plan], workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(q.device))
    _check(st, "gated_bigla_fwd")
    return out, g_fwd, g_bwd


def timing_enable(on: bool) -> None:
    """Start (and clear) or stop per-kernel HIP-event timing of this thread's launches."""
    _check(lib().vig_timing_enable(1 if on else 0), "vig_timing_enable")


def timing_collect(kernel: str):
    """(total milliseconds, launches) of one kernel since timing was enabled."""
    ms, n = ctypes.c_double(0.0), ctypes.c_long(0)
    _check(lib().vig_timing_collect(KERNELS[kernel], ctypes.byref(ms), ctypes.byref(n)), "vig_timing_collect")
    return ms.value, n.value


def measure_alias_slabs(on: bool) -> None:
    """Measurement aid: make every slab of the chunkwise forward kernels read slab 0's inputs."""
    _check(lib().vig_measure_alias_slabs(1 if on else 0), "vig_measure_alias_slabs")
