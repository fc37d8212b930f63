"""CPU oracle (float64) for the BiGLA + locality-gate path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product path (`paper_2405_18425_amd`) never does.  The
arithmetic lives in `bigla_oracle.c` (plain C, float64, no blocking); this file
only compiles it with gcc and marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bigla_oracle.c")
_SO = os.path.join(_HERE, "libbigla_oracle.so")
_default = None


def build(force: bool = False, src: str = _SRC, so: str = _SO) -> str:
    """Compile the C oracle with gcc (-O2, no fast-math, OpenMP over (b,h) slabs)."""
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", so, src, "-lm"]
        subprocess.run(cmd, check=True)
    return so


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


class Oracle:
    """ctypes front end of one compiled copy of `bigla_oracle.c`."""

    def __init__(self, so_path: str):
        lib = ctypes.CDLL(so_path)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.bigla_ref_f64.argtypes = [dp] * 6 + [ctypes.c_int] * 6
        lib.bigla_ref_f64.restype = ctypes.c_int
        lib.locality_gate_ref_f64.argtypes = [dp] * 6 + [ctypes.c_int] * 6
        lib.locality_gate_ref_f64.restype = ctypes.c_int
        lib.gate_producer_ref_f64.argtypes = [dp] * 6 + [ctypes.c_int] * 6 + [ctypes.c_double, ctypes.c_int]
        lib.gate_producer_ref_f64.restype = ctypes.c_int
        lib.bigla_bwd_ref_f64.argtypes = [dp] * 11 + [ctypes.c_int] * 6
        lib.bigla_bwd_ref_f64.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        self._lib = lib

    def max_threads(self) -> int:
        return int(self._lib.oracle_max_threads())

    def bigla(self, q, k, v, g_fwd, g_bwd, nthreads: int = 0) -> np.ndarray:
        """out[B,H,L,dv] of the BiGLA recurrences (Section 4.2.1), float64.

        q, k, g_fwd, g_bwd: [B,H,L,dk]; v: [B,H,L,dv]; g_* are log gates (<= 0).
        """
        q = _c64(q)
        if q.ndim != 4:
            raise ValueError("q must be [B,H,L,dk]")
        B, H, L, dk = q.shape
        k = _c64(k, q.shape)
        g_fwd = _c64(g_fwd, q.shape)
        g_bwd = _c64(g_bwd, q.shape)
        v = _c64(v)
        if v.ndim != 4 or v.shape[:3] != (B, H, L):
            raise ValueError("v must be [B,H,L,dv]")
        dv = v.shape[3]
        out = np.empty((B, H, L, dv), dtype=np.float64)
        if out.size == 0:
            return out
        rc = self._lib.bigla_ref_f64(_ptr(q), _ptr(k), _ptr(v), _ptr(g_fwd), _ptr(g_bwd), _ptr(out),
                                     B, H, L, dk, dv, int(nthreads))
        if rc != 0:
            raise RuntimeError(f"bigla_ref_f64 failed ({rc})")
        return out

    def bigla_bwd(self, q, k, v, g_fwd, g_bwd, d_out, nthreads: int = 0):
        """(dq, dk, dv, dg_fwd, dg_bwd): the gradient of `bigla` for the output gradient d_out
        [B,H,L,dv] (chain rule on the recurrences of Section 4.2.1), float64."""
        q = _c64(q)
        if q.ndim != 4:
            raise ValueError("q must be [B,H,L,dk]")
        B, H, L, dk = q.shape
        k = _c64(k, q.shape)
        g_fwd = _c64(g_fwd, q.shape)
        g_bwd = _c64(g_bwd, q.shape)
        v = _c64(v)
        if v.ndim != 4 or v.shape[:3] != (B, H, L):
            raise ValueError("v must be [B,H,L,dv]")
        dv = v.shape[3]
        d_out = _c64(d_out, v.shape)
        dq, dk_, dgf, dgb = (np.zeros(q.shape, dtype=np.float64) for _ in range(4))
        dv_ = np.zeros(v.shape, dtype=np.float64)
        if q.size == 0 or v.size == 0:
            return dq, dk_, dv_, dgf, dgb
        rc = self._lib.bigla_bwd_ref_f64(_ptr(q), _ptr(k), _ptr(v), _ptr(g_fwd), _ptr(g_bwd), _ptr(d_out), _ptr(dq),
                                         _ptr(dk_), _ptr(dv_), _ptr(dgf), _ptr(dgb), B, H, L, dk, dv, int(nthreads))
        if rc != 0:
            raise RuntimeError(f"bigla_bwd_ref_f64 failed ({rc})")
        return dq, dk_, dv_, dgf, dgb

    def locality_gate(self, x, w, gate_logits, o_global, Hg: int, Wg: int, bias=None,
                      nthreads: int = 0) -> np.ndarray:
        """out[B,H,Hg*Wg,dv] of the 2D gating locality injection (Section 4.2.2), float64.

        x, gate_logits, o_global: [B,H,Hg*Wg,dv] (token t = y*Wg + x); w: [H*dv,3,3];
        bias: [H*dv] or None.
        """
        x = _c64(x)
        if x.ndim != 4:
            raise ValueError("x must be [B,H,L,dv]")
        B, H, L, dv = x.shape
        if L != Hg * Wg:
            raise ValueError("L != Hg*Wg")
        w = _c64(w, (H * dv, 3, 3))
        z = _c64(gate_logits, x.shape)
        og = _c64(o_global, x.shape)
        b = None if bias is None else _c64(bias, (H * dv,))
        out = np.empty_like(x)
        if out.size == 0:
            return out
        rc = self._lib.locality_gate_ref_f64(_ptr(x), _ptr(w), _ptr(b) if b is not None else None,
                                             _ptr(z), _ptr(og), _ptr(out), B, H, Hg, Wg, dv, int(nthreads))
        if rc != 0:
            raise RuntimeError(f"locality_gate_ref_f64 failed ({rc})")
        return out

    def gate_producer(self, x, w1, w2, H: int, dk: int, bias=None, tau: float = 16.0, nthreads: int = 0):
        """(g_fwd, g_bwd), each [B,H,L,dk]: log forget gates log(sigmoid((x W1) W2 + b)) / tau
        (Section 3 and Eq. (BiGLA) lines 1-2), float64.

        x: [B,L,D]; w1: [D,rank]; w2: [rank, 2*H*dk] (forward half first, heads in order);
        bias: [2*H*dk] or None.
        """
        x = _c64(x)
        if x.ndim != 3:
            raise ValueError("x must be [B,L,D]")
        B, L, D = x.shape
        w1 = _c64(w1)
        if w1.ndim != 2 or w1.shape[0] != D:
            raise ValueError("w1 must be [D,rank]")
        rank = w1.shape[1]
        w2 = _c64(w2, (rank, 2 * H * dk))
        b = None if bias is None else _c64(bias, (2 * H * dk,))
        gf = np.empty((B, H, L, dk), dtype=np.float64)
        gb = np.empty_like(gf)
        if gf.size == 0:
            return gf, gb
        rc = self._lib.gate_producer_ref_f64(_ptr(x), _ptr(w1), _ptr(w2), _ptr(b) if b is not None else None,
                                             _ptr(gf), _ptr(gb), B, H, L, D, rank, dk, float(tau), int(nthreads))
        if rc != 0:
            raise RuntimeError(f"gate_producer_ref_f64 failed ({rc})")
        return gf, gb


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle(build())
    return _default


def max_threads() -> int:
    return default().max_threads()


def bigla(q, k, v, g_fwd, g_bwd, nthreads: int = 0) -> np.ndarray:
    return default().bigla(q, k, v, g_fwd, g_bwd, nthreads)


def bigla_bwd(q, k, v, g_fwd, g_bwd, d_out, nthreads: int = 0):
    return default().bigla_bwd(q, k, v, g_fwd, g_bwd, d_out, nthreads)


def locality_gate(x, w, gate_logits, o_global, Hg: int, Wg: int, bias=None, nthreads: int = 0) -> np.ndarray:
    return default().locality_gate(x, w, gate_logits, o_global, Hg, Wg, bias, nthreads)


def gate_producer(x, w1, w2, H: int, dk: int, bias=None, tau: float = 16.0, nthreads: int = 0):
    return default().gate_producer(x, w1, w2, H, dk, bias, tau, nthreads)


def bigla_locality(q, k, v, g_fwd, g_bwd, x, w, gate_logits, Hg: int, Wg: int, bias=None,
                   nthreads: int = 0) -> np.ndarray:
    """The block's two steps chained (Section 4.2.2, the gating equation with O_global taken from
    Section 4.2.1): the token mixer's output, unrounded, is the global branch of the blend."""
    o_global = bigla(q, k, v, g_fwd, g_bwd, nthreads)
    return locality_gate(x, w, gate_logits, o_global, Hg, Wg, bias, nthreads)
