"""Seeded synthetic ViG-shaped inputs for the BiGLA + locality-gate path.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
recurrence, no convolution, no blend) and is the one piece of code that both the
CPU oracle's tests and the HIP path's tests / bench use, so that both sides see
the same rounded bits.

Generator: a counter-based stream (splitmix64 of ``stream_key + index``) feeds a
Box-Muller transform in float64; every tensor has its own stream key derived
from (seed, tensor name).  Values are rounded ONCE to the configuration dtype
(float32, or bfloat16 with round-to-nearest-even) and both sides widen those
bits exactly.

Shapes follow the ViG models (Appendix B architecture table: d = 192/384/768,
heads 3/6/12, patch 16) at the resolutions of the paper's resolution sweep
(224, 512, 1024 pixels -> 14x14, 32x32, 64x64 patch grids).  The forget gate
enters as ``log alpha = logsigmoid(z) / tau`` with ``tau = 16`` (Section 3, gated
linear attention), drawn separately for the two directions (Section 4.2.1).
"""
from __future__ import annotations

import dataclasses
import hashlib

import numpy as np

TAU = 16.0  # temperature of the forget gate (Section 3)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    Hg: int  # patch-grid height
    Wg: int  # patch-grid width
    dk: int
    dv: int
    dtype: str  # "f32" | "bf16"
    gate_mu: float  # mean of the gate logits z ~ N(gate_mu, 1)

    @property
    def L(self) -> int:
        return self.Hg * self.Wg

    @property
    def head_tokens(self) -> int:
        return self.B * self.H * self.L

    @property
    def tokens(self) -> int:
        return self.B * self.L

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (index = configuration number).
CONFIGS = (
    Workload("tiny_8x8_f32", B=1, H=1, Hg=8, Wg=8, dk=16, dv=16, dtype="f32", gate_mu=0.0),
    Workload("vig_t_224", B=64, H=3, Hg=14, Wg=14, dk=64, dv=64, dtype="bf16", gate_mu=0.0),
    Workload("vig_s_224", B=64, H=6, Hg=14, Wg=14, dk=64, dv=64, dtype="bf16", gate_mu=0.0),
    Workload("vig_b_512", B=16, H=12, Hg=32, Wg=32, dk=64, dv=64, dtype="bf16", gate_mu=2.0),
    Workload("vig_s_1024", B=8, H=6, Hg=64, Wg=64, dk=64, dv=64, dtype="bf16", gate_mu=-2.0),
)


# --------------------------------------------------------------------------- #
# counter-based random numbers
# --------------------------------------------------------------------------- #
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser applied elementwise to uint64 counters."""
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = x
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        z = z ^ (z >> np.uint64(31))
    return z


def _stream_key(seed: int, name: str) -> np.uint64:
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    return np.uint64(int.from_bytes(h[:8], "little"))


def uniform01(seed: int, name: str, n: int, lane: int = 0) -> np.ndarray:
    """n uniforms in (0,1), float64, from stream (seed, name), sub-stream `lane`."""
    key = _stream_key(seed, f"{name}/{lane}")
    with np.errstate(over="ignore"):
        ctr = (np.arange(n, dtype=np.uint64) + key) & _M64
    bits = _splitmix64(ctr) >> np.uint64(11)  # 53 random bits
    return (bits.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, name: str, shape, mu: float = 0.0, sigma: float = 1.0) -> np.ndarray:
    """N(mu, sigma^2) samples (float64) via Box-Muller on two uniform sub-streams."""
    n = int(np.prod(shape))
    u1 = uniform01(seed, name, n, 0)
    u2 = uniform01(seed, name, n, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mu + sigma * z).reshape(shape)


# --------------------------------------------------------------------------- #
# dtype rounding (storage only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def store(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float64 array once to the storage dtype.

    Returns float32 for "f32" and uint16 bit patterns for "bf16".
    """
    if dtype == "f32":
        return x64.astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x64.astype(np.float32))
    raise ValueError(dtype)


def widen(stored: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of what `store` produced."""
    if dtype == "f32":
        return stored.astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(stored)
    raise ValueError(dtype)


def to_torch(stored: np.ndarray, dtype: str, device="cpu"):
    """Wrap stored bits as a torch tensor of the matching dtype (no value change)."""
    import torch

    if dtype == "f32":
        t = torch.from_numpy(np.ascontiguousarray(stored))
    else:
        t = torch.from_numpy(np.ascontiguousarray(stored).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def from_torch(t, dtype: str) -> np.ndarray:
    """Inverse of `to_torch`: stored representation (float32 / bf16 bits) on the host."""
    import torch

    t = t.detach().cpu().contiguous()
    if dtype == "f32":
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------- #
# the workload recipe
# --------------------------------------------------------------------------- #
def log_gate(z64: np.ndarray) -> np.ndarray:
    """log(sigmoid(z)^(1/tau)) = logsigmoid(z)/tau, evaluated stably in float64."""
    return -(np.logaddexp(0.0, -z64)) / TAU


def generate(w: Workload, seed: int = 0, tensors=None) -> dict:
    """Draw the stored (dtype-rounded) input tensors of one workload.

    q, k : [B,H,L,dk] ~ N(0,1)/4          v : [B,H,L,dv] ~ N(0,1)/4
    g_fwd, g_bwd : [B,H,L,dk] = logsigmoid(N(gate_mu,1))/16, one draw per direction
    conv_w : [H*dv,3,3] ~ N(0, sigma=0.1)  gate_logits : [B,H,L,dv] ~ N(0,1)
    The locality stage takes x := v and o_global := the BiGLA output.
    """
    B, H, L, dk, dv = w.B, w.H, w.L, w.dk, w.dv
    spec = {
        "q": lambda: normal(seed, "q", (B, H, L, dk)) / 4.0,
        "k": lambda: normal(seed, "k", (B, H, L, dk)) / 4.0,
        "v": lambda: normal(seed, "v", (B, H, L, dv)) / 4.0,
        "g_fwd": lambda: log_gate(normal(seed, "z_fwd", (B, H, L, dk), mu=w.gate_mu)),
        "g_bwd": lambda: log_gate(normal(seed, "z_bwd", (B, H, L, dk), mu=w.gate_mu)),
        "conv_w": lambda: normal(seed, "conv_w", (H * dv, 3, 3), sigma=0.1),
        "gate_logits": lambda: normal(seed, "gate_logits", (B, H, L, dv)),
    }
    names = list(spec) if tensors is None else list(tensors)
    return {n: store(spec[n](), w.dtype) for n in names}


def generate_gate_inputs(B: int, L: int, D: int, H: int, dk: int, dtype: str, seed: int = 0, bias_mu: float = 0.0,
                         rank: int = 16) -> dict:
    """Stored inputs of the forget-gate producer, in the mathematical orientation of Section 3:
    x : [B,L,D] ~ N(0,1) (a normalised block input), w1 : [D,rank] ~ N(0,1)/sqrt(D),
    w2 : [rank, 2*H*dk] ~ N(0,1)/sqrt(rank), bias : [2*H*dk] ~ N(bias_mu, 1).  The pre-activation
    then has unit-order spread around bias_mu, like the gate logits of the BiGLA configurations."""
    spec = {
        "x": normal(seed, "gate_x", (B, L, D)),
        "w1": normal(seed, "gate_w1", (D, rank)) / np.sqrt(D),
        "w2": normal(seed, "gate_w2", (rank, 2 * H * dk)) / np.sqrt(rank),
        "bias": normal(seed, "gate_bias", (2 * H * dk,), mu=bias_mu),
    }
    return {n: store(a, dtype) for n, a in spec.items()}
