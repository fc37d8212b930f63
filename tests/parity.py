"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same stored
inputs and compare element by element."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2405_18425_amd import workloads as wl

# tolerances stated for the path: bf16 inputs with fp32 accumulation, and the fp32 path
TOL = {"bf16": 2e-2, "f32": 1e-4}


def assert_close(got64: np.ndarray, ref64: np.ndarray, tol: float, what: str = "") -> float:
    """|got - ref| <= tol*|ref| + tol*rms(ref over the (b,h) slab), element by element.

    Outputs are signed sums that cross zero, so a purely relative bound is meaningless near the
    zero crossings; the slab rms supplies the absolute floor.  Returns max|err| / max|ref|.
    """
    assert got64.shape == ref64.shape, (got64.shape, ref64.shape)
    assert np.all(np.isfinite(got64)), f"{what}: non-finite output"
    rms = np.sqrt(np.mean(ref64 ** 2, axis=(2, 3), keepdims=True))
    err = np.abs(got64 - ref64)
    bound = tol * np.abs(ref64) + tol * rms
    worst = float(np.max(err - bound))
    if worst > 0:
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: |err|={err[idx]:.4e} > bound {bound[idx]:.4e} at {idx} "
                             f"(ref {ref64[idx]:.4e}, got {got64[idx]:.4e}, slab rms {rms[idx[0], idx[1], 0, 0]:.3e})")
    return float(np.max(err) / max(np.max(np.abs(ref64)), 1e-30))


def run_bigla_gpu(stored: dict, dtype: str, **kw) -> np.ndarray:
    """Stored inputs -> HIP path through the C ABI -> float64 array of the stored output."""
    import torch
    from paper_2405_18425_amd import binding as vb

    dev = "cuda:0"
    t = {n: wl.to_torch(stored[n], dtype, dev) for n in ("q", "k", "v", "g_fwd", "g_bwd")}
    out = vb.bigla_fwd(t["q"], t["k"], t["v"], t["g_fwd"], t["g_bwd"], **kw)
    torch.cuda.synchronize()
    return wl.widen(wl.from_torch(out, dtype), dtype)


def run_bigla_oracle(stored: dict, dtype: str, slabs=None) -> np.ndarray:
    w = {n: wl.widen(stored[n], dtype) for n in ("q", "k", "v", "g_fwd", "g_bwd")}
    if slabs is not None:
        B, H = w["q"].shape[:2]
        sel = {n: np.stack([a[b, h] for (b, h) in slabs])[None] for n, a in w.items()}
        return oracle.bigla(sel["q"], sel["k"], sel["v"], sel["g_fwd"], sel["g_bwd"])[0]
    return oracle.bigla(w["q"], w["k"], w["v"], w["g_fwd"], w["g_bwd"])


def run_locality_gpu(x, w, z, og, Hg, Wg, dtype: str, bias=None) -> np.ndarray:
    import torch
    from paper_2405_18425_amd import binding as vb

    dev = "cuda:0"
    tt = lambda a: wl.to_torch(a, dtype, dev)
    out = vb.locality_gate_fwd(tt(x), tt(w), tt(z), tt(og), Hg, Wg, bias=None if bias is None else tt(bias))
    torch.cuda.synchronize()
    return wl.widen(wl.from_torch(out, dtype), dtype)


def run_locality_oracle(x, w, z, og, Hg, Wg, dtype: str, bias=None) -> np.ndarray:
    wd = lambda a: wl.widen(a, dtype)
    return oracle.locality_gate(wd(x), wd(w), wd(z), wd(og), Hg, Wg, bias=None if bias is None else wd(bias))
