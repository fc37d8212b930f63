"""Pins for the CPU oracle: facts that the paper's equations and plain mathematics fix.

Each pin takes the implementation under test as a callable, so the same checks
run on the real oracle (tests/test_oracle_pins.py) and on deliberately broken
copies of it (tests/test_oracle_mutants.py: every planted mistake must trip at
least one pin).  None of these re-types the recurrence: they use the O(L^2)
explicit-product expansion, closed forms, symmetries and library routines.
"""
from __future__ import annotations

import json
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _draw(seed, B=2, H=2, L=9, dk=3, dv=4, gate_scale=1.0):
    r = _rng(seed)
    q = r.standard_normal((B, H, L, dk))
    k = r.standard_normal((B, H, L, dk))
    v = r.standard_normal((B, H, L, dv))
    gf = -gate_scale * r.random((B, H, L, dk))
    gb = -gate_scale * r.random((B, H, L, dk))
    return q, k, v, gf, gb


def _close(a, b, tol=1e-11):
    scale = max(1.0, float(np.max(np.abs(b))))
    err = float(np.max(np.abs(np.asarray(a) - np.asarray(b))))
    assert err <= tol * scale, f"max abs err {err:.3e} (scale {scale:.3e})"


# --------------------------------------------------------------------------- #
# BiGLA
# --------------------------------------------------------------------------- #
def quadratic_form(q, k, v, gf, gb):
    """Explicit-product expansion of Eq. (BiGLA), Section 4.2.1, O(L^2), no cumulative sums.

    Unrolling S_t = G_t . S_{t-1} + k_t^T v_t from a zero state gives
      o_fwd_t = sum_{i<=t} sum_c q_tc k_ic (prod_{j=i+1..t} a_fwd_jc) v_i
      o_bwd_t = sum_{i>=t} sum_c q_tc k_ic (prod_{j=t..i-1} a_bwd_jc) v_i
    """
    B, H, L, dk = q.shape
    dv = v.shape[-1]
    af, ab = np.exp(gf), np.exp(gb)
    out = np.zeros((B, H, L, dv))
    for b in range(B):
        for h in range(H):
            for t in range(L):
                acc = np.zeros(dv)
                for i in range(0, t + 1):
                    w = 0.0
                    for c in range(dk):
                        p = 1.0
                        for j in range(i + 1, t + 1):
                            p *= af[b, h, j, c]
                        w += q[b, h, t, c] * k[b, h, i, c] * p
                    acc += w * v[b, h, i]
                for i in range(t, L):
                    w = 0.0
                    for c in range(dk):
                        p = 1.0
                        for j in range(t, i):
                            p *= ab[b, h, j, c]
                        w += q[b, h, t, c] * k[b, h, i, c] * p
                    acc += w * v[b, h, i]
                out[b, h, t] = 0.5 * acc
    return out


def pin_quadratic_bruteforce(bigla):
    for seed, shape in ((1, dict(B=2, H=2, L=9, dk=3, dv=4)), (2, dict(B=1, H=1, L=17, dk=5, dv=2)),
                        (3, dict(B=1, H=3, L=1, dk=2, dv=3))):
        q, k, v, gf, gb = _draw(seed, **shape)
        _close(bigla(q, k, v, gf, gb), quadratic_form(q, k, v, gf, gb))


def pin_handworked_L2(bigla):
    with open(os.path.join(GOLDEN, "bigla_L2_handworked.json")) as f:
        g = json.load(f)
    sh = (1, 1, 2, 1)
    arr = lambda key: np.array(g[key], dtype=np.float64).reshape(sh)
    out = bigla(arr("q"), arr("k"), arr("v"), np.log(arr("alpha_fwd")), np.log(arr("alpha_bwd")))
    _close(out.reshape(-1), np.array(g["out"]), 1e-13)


def pin_all_gates_one(bigla):
    """log-gates = 0: plain bidirectional linear attention (Section 3, linear attention).

    o_fwd_t + o_bwd_t = q_t (sum_i k_i^T v_i) + (q_t . k_t) v_t, one GEMM."""
    q, k, v, gf, _ = _draw(4, B=2, H=3, L=23, dk=6, dv=5)
    z = np.zeros_like(gf)
    kv = np.einsum("bhlc,bhlj->bhcj", k, v)
    want = 0.5 * (np.einsum("bhlc,bhcj->bhlj", q, kv) + np.sum(q * k, -1, keepdims=True) * v)
    _close(bigla(q, k, v, z, z), want)


def pin_gates_vanish(bigla):
    """alpha -> 0 in both directions: only the token's own k^T v survives, twice, then halved."""
    q, k, v, gf, _ = _draw(5, L=11)
    big = np.full_like(gf, -1.0e3)
    _close(bigla(q, k, v, big, big), np.sum(q * k, -1, keepdims=True) * v)


def pin_constant_gate_toeplitz(bigla):
    """One scalar gate gamma everywhere: out_t = sum_i w_|t-i| (q_t.k_i) v_i, w_0 = 1, w_n = gamma^n / 2."""
    q, k, v, gf, _ = _draw(6, B=1, H=2, L=14, dk=4, dv=3)
    gamma = 0.83
    g = np.full_like(gf, np.log(gamma))
    L = q.shape[2]
    n = np.abs(np.arange(L)[:, None] - np.arange(L)[None, :])
    w = np.where(n == 0, 1.0, 0.5 * gamma ** n)
    want = np.einsum("ti,bhti,bhij->bhtj", w, np.einsum("bhtc,bhic->bhti", q, k), v)
    _close(bigla(q, k, v, g, g), want)


def pin_reversal_symmetry(bigla):
    """Reversing the sequence and swapping the two gate streams reverses the output."""
    q, k, v, gf, gb = _draw(7, L=13)
    rev = lambda a: a[:, :, ::-1].copy()
    _close(bigla(rev(q), rev(k), rev(v), rev(gb), rev(gf)), rev(bigla(q, k, v, gf, gb)))
    # and the two gate streams are NOT interchangeable in place
    a, b = bigla(q, k, v, gf, gb), bigla(q, k, v, gb, gf)
    assert np.max(np.abs(a - b)) > 1e-3


def causal_gla(q, k, v, g):
    """Unidirectional GLA (Section 3) by explicit products: o_t = sum_{i<=t} (q_t*k_i*prod a) v_i."""
    B, H, L, dk = q.shape
    out = np.zeros(v.shape)
    a = np.exp(g)
    for t in range(L):
        for i in range(t + 1):
            decay = np.prod(a[:, :, i + 1:t + 1], axis=2)  # [B,H,dk]
            out[:, :, t] += np.sum(q[:, :, t] * k[:, :, i] * decay, -1, keepdims=True) * v[:, :, i]
    return out


def pin_kill_one_direction(bigla):
    q, k, v, gf, gb = _draw(8, L=12)
    dead = np.full_like(gf, -1.0e3)
    self_term = np.sum(q * k, -1, keepdims=True) * v
    # backward killed: causal GLA with the forward gates + the self term, halved
    _close(bigla(q, k, v, gf, dead), 0.5 * (causal_gla(q, k, v, gf) + self_term))
    # forward killed: anti-causal GLA = causal GLA of the reversed sequence; the backward scan
    # applies token t's own gate, so the reversed gate stream lines up without a shift
    rev = lambda a: a[:, :, ::-1].copy()
    anti = rev(causal_gla(rev(q), rev(k), rev(v), rev(gb)))
    _close(bigla(q, k, v, dead, gb), 0.5 * (anti + self_term))
    # causality: with the backward direction dead, tokens > t cannot change out_t
    t0 = 6
    k2, v2, gf2 = k.copy(), v.copy(), gf.copy()
    k2[:, :, t0 + 1:] += 3.0
    v2[:, :, t0 + 1:] -= 2.0
    gf2[:, :, t0 + 1:] *= 0.5
    a, b = bigla(q, k, v, gf, dead), bigla(q, k2, v2, gf2, dead)
    _close(a[:, :, :t0 + 1], b[:, :, :t0 + 1])
    assert np.max(np.abs(a[:, :, t0 + 1:] - b[:, :, t0 + 1:])) > 1e-3


def pin_unused_boundary_gates(bigla):
    """g_fwd[0] and g_bwd[L-1] multiply a zero state: the output cannot depend on them."""
    q, k, v, gf, gb = _draw(9, L=7)
    gf2, gb2 = gf.copy(), gb.copy()
    gf2[:, :, 0] = -5.0
    gb2[:, :, -1] = -7.0
    _close(bigla(q, k, v, gf2, gb2), bigla(q, k, v, gf, gb), 1e-13)
    gf2[:, :, 1] -= 1.0  # any other gate does matter
    assert np.max(np.abs(bigla(q, k, v, gf2, gb2) - bigla(q, k, v, gf, gb))) > 1e-4


def pin_trilinear(bigla):
    q, k, v, gf, gb = _draw(10, L=10)
    q2, k2, v2, _, _ = _draw(11, L=10)
    base = bigla(q, k, v, gf, gb)
    _close(bigla(q + 2 * q2, k, v, gf, gb), base + 2 * bigla(q2, k, v, gf, gb))
    _close(bigla(q, k - 3 * k2, v, gf, gb), base - 3 * bigla(q, k2, v, gf, gb))
    _close(bigla(q, k, v + v2, gf, gb), base + bigla(q, k, v2, gf, gb))


def pin_heads_independent(bigla):
    """Slabs (b,h) do not interact and each equals a B=H=1 call on its own slice (non-square dk != dv)."""
    q, k, v, gf, gb = _draw(12, B=2, H=3, L=8, dk=5, dv=2)
    full = bigla(q, k, v, gf, gb)
    for b in range(2):
        for h in range(3):
            s = (slice(b, b + 1), slice(h, h + 1))
            _close(full[s], bigla(q[s], k[s], v[s], gf[s], gb[s]), 1e-13)


BIGLA_PINS = (pin_quadratic_bruteforce, pin_handworked_L2, pin_all_gates_one, pin_gates_vanish,
              pin_constant_gate_toeplitz, pin_reversal_symmetry, pin_kill_one_direction,
              pin_unused_boundary_gates, pin_trilinear, pin_heads_independent)


# --------------------------------------------------------------------------- #
# locality gate
# --------------------------------------------------------------------------- #
def _draw_loc(seed, B=2, H=2, Hg=5, Wg=7, dv=3):
    r = _rng(seed)
    L = Hg * Wg
    return (r.standard_normal((B, H, L, dv)), r.standard_normal((H * dv, 3, 3)),
            r.standard_normal((B, H, L, dv)), r.standard_normal((B, H, L, dv)))


def pin_loc_library_conv(loc):
    """Against a library depthwise conv2d (groups = channels, zero padding 1) in float64."""
    import torch
    import torch.nn.functional as F

    B, H, Hg, Wg, dv = 2, 2, 5, 7, 3
    x, w, z, og = _draw_loc(20, B, H, Hg, Wg, dv)
    bias = _rng(21).standard_normal(H * dv)
    for bb in (None, bias):
        xi = torch.from_numpy(x).reshape(B, H, Hg, Wg, dv).permute(0, 1, 4, 2, 3).reshape(B, H * dv, Hg, Wg)
        conv = F.conv2d(xi, torch.from_numpy(w).reshape(H * dv, 1, 3, 3),
                        None if bb is None else torch.from_numpy(bb), padding=1, groups=H * dv)
        local = conv.reshape(B, H, dv, Hg, Wg).permute(0, 1, 3, 4, 2).reshape(B, H, Hg * Wg, dv).numpy()
        gate = 1.0 / (1.0 + np.exp(-z))
        _close(loc(x, w, z, og, Hg, Wg, bias=bb), gate * local + (1 - gate) * og)


def pin_loc_centre_delta_and_gate_limits(loc):
    B, H, Hg, Wg, dv = 1, 2, 4, 6, 3
    x, w, z, og = _draw_loc(22, B, H, Hg, Wg, dv)
    delta = np.zeros_like(w)
    delta[:, 1, 1] = 1.0
    _close(loc(x, delta, np.full_like(z, 50.0), og, Hg, Wg), x)          # G -> 1: O_local = x
    _close(loc(x, w, np.full_like(z, -50.0), og, Hg, Wg), og)            # G -> 0: O_global
    local = loc(x, w, np.full_like(z, 50.0), og, Hg, Wg)
    _close(loc(x, w, np.zeros_like(z), og, Hg, Wg), 0.5 * (local + og))  # G = 1/2: the mean


def pin_loc_single_tap_shifts(loc):
    """A single off-centre tap is a pure shift with zero fill: fixes orientation (no kernel flip)."""
    B, H, Hg, Wg, dv = 1, 1, 4, 5, 2
    x, w, z, og = _draw_loc(23, B, H, Hg, Wg, dv)
    big = np.full_like(z, 50.0)
    xg = x.reshape(B, H, Hg, Wg, dv)
    for ky in range(3):
        for kx in range(3):
            tap = np.zeros_like(w)
            tap[:, ky, kx] = 1.0
            want = np.zeros_like(xg)
            dy, dx = ky - 1, kx - 1  # out[y,x] = in[y+dy, x+dx]
            for y in range(Hg):
                for xx in range(Wg):
                    if 0 <= y + dy < Hg and 0 <= xx + dx < Wg:
                        want[:, :, y, xx] = xg[:, :, y + dy, xx + dx]
            _close(loc(x, tap, big, og, Hg, Wg), want.reshape(x.shape))


def pin_loc_ones_kernel_counts(loc):
    """All-ones kernel on a constant image counts in-bounds taps: 9 interior, 6 edge, 4 corner."""
    B, H, Hg, Wg, dv = 1, 1, 4, 5, 2
    x = np.full((B, H, Hg * Wg, dv), 2.5)
    out = loc(x, np.ones((H * dv, 3, 3)), np.full_like(x, 50.0), np.zeros_like(x), Hg, Wg)
    out = out.reshape(Hg, Wg, dv)
    _close(out[1, 2], 9 * 2.5)
    _close(out[0, 2], 6 * 2.5)
    _close(out[2, 0], 6 * 2.5)
    _close(out[0, 0], 4 * 2.5)
    _close(out[Hg - 1, Wg - 1], 4 * 2.5)


def pin_loc_channel_mapping(loc):
    """Filter c = h*dv + j acts on head h, feature j only; bias is added inside O_local."""
    B, H, Hg, Wg, dv = 1, 3, 3, 3, 2
    x, w, z, og = _draw_loc(24, B, H, Hg, Wg, dv)
    big = np.full_like(z, 50.0)
    w2 = np.zeros_like(w)
    w2[:, 1, 1] = np.arange(1, H * dv + 1)
    want = x * np.arange(1, H * dv + 1).reshape(1, H, 1, dv)
    _close(loc(x, w2, big, og, Hg, Wg), want)
    bias = np.arange(H * dv) * 0.5
    _close(loc(x, w2, big, og, Hg, Wg, bias=bias), want + bias.reshape(1, H, 1, dv))


LOC_PINS = (pin_loc_library_conv, pin_loc_centre_delta_and_gate_limits, pin_loc_single_tap_shifts,
            pin_loc_ones_kernel_counts, pin_loc_channel_mapping)


# --------------------------------------------------------------------------- #
# Gate producer (Section 3 gate; Eq. (BiGLA) lines 1-2).  gp(x, w1, w2, H, dk, bias, tau) ->
# (g_fwd, g_bwd), each [B,H,L,dk], log gates.
# --------------------------------------------------------------------------- #
def _gp_draw(seed, B=2, L=7, D=10, rank=4, H=3, dk=5):
    r = _rng(seed)
    return (r.standard_normal((B, L, D)), r.standard_normal((D, rank)) / 2, r.standard_normal((rank, 2 * H * dk)),
            r.standard_normal(2 * H * dk), H, dk)


def _gp_split(z, H, dk):
    """[B,L,2*H*dk] -> two [B,H,L,dk]: forward half first, heads in order inside each half."""
    B, L, _ = z.shape
    f = z[..., :H * dk].reshape(B, L, H, dk).transpose(0, 2, 1, 3)
    b = z[..., H * dk:].reshape(B, L, H, dk).transpose(0, 2, 1, 3)
    return f, b


def pin_gp_library_matmul(gp):
    """alpha = sigmoid((x W1) W2 + b)^(1/tau) with library matmuls and the formula as printed
    (valid where exp does not overflow); checked as alpha, i.e. through exp of the log gate."""
    x, w1, w2, b, H, dk = _gp_draw(1)
    for tau in (16.0, 1.0, 3.5):
        gf, gb = gp(x, w1, w2, H, dk, b, tau)
        alpha = (1.0 / (1.0 + np.exp(-((x @ w1) @ w2 + b)))) ** (1.0 / tau)
        af, ab = _gp_split(alpha, H, dk)
        _close(np.exp(gf), af)
        _close(np.exp(gb), ab)
        assert np.all(gf <= 0) and np.all(gb <= 0)


def pin_gp_zero_projection_gives_bias_gate(gp):
    """W2 = 0 (or x = 0): every token gets log(sigmoid(b))/tau; no bias at all: log(1/2)/tau."""
    x, w1, w2, b, H, dk = _gp_draw(2)
    gf, gb = gp(x, w1, np.zeros_like(w2), H, dk, b, 16.0)
    ref = np.log(1.0 / (1.0 + np.exp(-b))) / 16.0
    _close(gf, np.broadcast_to(ref[:H * dk].reshape(1, H, 1, dk), gf.shape))
    _close(gb, np.broadcast_to(ref[H * dk:].reshape(1, H, 1, dk), gb.shape))
    gf, gb = gp(np.zeros_like(x), w1, w2, H, dk, None, 16.0)
    _close(gf, np.full(gf.shape, np.log(0.5) / 16.0))
    _close(gb, np.full(gb.shape, np.log(0.5) / 16.0))


def pin_gp_split_and_head_mapping(gp):
    """One non-zero column of W2 (bias 0) moves exactly one (direction, head, channel) away from
    log(1/2)/tau: column c < H*dk is forward head c // dk channel c % dk, the rest backward."""
    x, w1, w2, b, H, dk = _gp_draw(3)
    base = np.log(0.5) / 16.0
    for c in (0, dk - 1, dk, H * dk - 1, H * dk, H * dk + dk + 2, 2 * H * dk - 1):
        w = np.zeros_like(w2)
        w[:, c] = w2[:, c]
        gf, gb = gp(x, w1, w, H, dk, None, 16.0)
        moved_f = np.abs(gf - base) > 1e-9
        moved_b = np.abs(gb - base) > 1e-9
        d, h, j = c // (H * dk), (c % (H * dk)) // dk, c % dk
        want = np.zeros(gf.shape, dtype=bool)
        want[:, h, :, j] = True
        if d == 0:
            assert np.array_equal(moved_f, want) and not moved_b.any()
        else:
            assert np.array_equal(moved_b, want) and not moved_f.any()


def pin_gp_low_rank_null_space(gp):
    """Whatever lies in the null space of W1^T cannot change the gates (the gate sees x only
    through the rank-wide product x W1), and the pre-activation is linear in x."""
    x, w1, w2, b, H, dk = _gp_draw(4, D=10, rank=3)
    qmat, _ = np.linalg.qr(w1, mode="complete")
    null = qmat[:, 3:]                                    # D x (D - rank), orthogonal to span(W1)
    r = _rng(40)
    x2 = x + r.standard_normal(x.shape[:2] + (null.shape[1],)) @ null.T
    a = gp(x, w1, w2, H, dk, b, 16.0)
    c = gp(x2, w1, w2, H, dk, b, 16.0)
    _close(c[0], a[0], 1e-10)
    _close(c[1], a[1], 1e-10)
    # logit(alpha^tau) is affine in x: second difference vanishes
    def logit(g):  # log(p / (1 - p)) with p = exp(16 g), 1 - p taken as -expm1 to keep its digits
        return 16.0 * g - np.log(-np.expm1(16.0 * g))
    y = r.standard_normal(x.shape)
    l0, l1, l2 = (logit(gp(x + s * y, w1, w2, H, dk, b, 16.0)[0]) for s in (0.0, 1.0, 2.0))
    _close(l2 - 2 * l1 + l0, np.zeros_like(l0), 1e-8)


def pin_gp_saturation(gp):
    """Far into either tail the log gate is z/tau (z << 0) or -exp(-z)/tau (z >> 0): no overflow,
    no -inf, and the tau-th power of alpha is still the sigmoid."""
    B, L, D, rank, H, dk = 1, 4, 2, 1, 1, 2
    x = np.array([[[1.0, 0.0], [-1.0, 0.0], [50.0, 0.0], [-50.0, 0.0]]])
    w1 = np.array([[1.0], [0.0]])
    w2 = np.array([[20.0, -20.0, 20.0, -20.0]])           # z = +-20 x[.,0]
    gf, gb = gp(x, w1, w2, H, dk, None, 16.0)
    z = 20.0 * x[0, :, 0]
    for t in range(L):
        for j, sgn in enumerate((1.0, -1.0)):
            zz = sgn * z[t]
            want = zz / 16.0 if zz < -30 else (-np.exp(-zz) / 16.0 if zz > 30 else np.log(1 / (1 + np.exp(-zz))) / 16.0)
            assert np.isfinite(gf[0, 0, t, j])
            assert abs(gf[0, 0, t, j] - want) <= 1e-12 * max(1.0, abs(want)), (t, j, gf[0, 0, t, j], want)
            assert gb[0, 0, t, j] == gf[0, 0, t, j]


GP_PINS = (pin_gp_library_matmul, pin_gp_zero_projection_gives_bias_gate, pin_gp_split_and_head_mapping,
           pin_gp_low_rank_null_space, pin_gp_saturation)


# --------------------------------------------------------------------------- #
# BiGLA backward (gradient of the token mixer): pins take bwd(q, k, v, gf, gb, d_out)
# -> (dq, dk, dv, dgf, dgb)
# --------------------------------------------------------------------------- #
def pin_bwd_finite_differences(bwd):
    """Central differences of the O(L^2) explicit-product form (no recurrence, no oracle code)
    in every element of all five inputs, loss = sum(out * d_out)."""
    q, k, v, gf, gb = _draw(21, B=1, H=2, L=5, dk=2, dv=3, gate_scale=1.5)
    d_out = _rng(22).standard_normal(v.shape)
    got = bwd(q, k, v, gf, gb, d_out)
    args = [q, k, v, gf, gb]
    h = 1e-6
    for idx in range(5):
        fd = np.zeros_like(args[idx])
        for i in np.ndindex(*args[idx].shape):
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            plus[idx][i] += h
            minus[idx][i] -= h
            fd[i] = (np.sum(quadratic_form(*plus) * d_out) - np.sum(quadratic_form(*minus) * d_out)) / (2 * h)
        _close(got[idx], fd, 1e-7)


def pin_bwd_gates_closed(bwd):
    """Gates -> 0: out_t = (q_t . k_t) v_t, whose gradients are immediate; the gates get none."""
    q, k, v, _, _ = _draw(23, L=6)
    closed = np.full(q.shape, -800.0)
    d_out = _rng(24).standard_normal(v.shape)
    dq, dk, dv, dgf, dgb = bwd(q, k, v, closed, closed, d_out)
    dov = np.sum(d_out * v, axis=-1, keepdims=True)
    _close(dq, dov * k)
    _close(dk, dov * q)
    _close(dv, np.sum(q * k, axis=-1, keepdims=True) * d_out)
    assert np.all(dgf == 0.0) and np.all(dgb == 0.0)


def pin_bwd_gates_open(bwd):
    """All log-gates 0: out = W V with W = (tril(QK^T) + triu(QK^T)) / 2, plain matrix calculus."""
    q, k, v, _, _ = _draw(25, L=7)
    zero = np.zeros(q.shape)
    d_out = _rng(26).standard_normal(v.shape)
    dq, dk, dv, _, _ = bwd(q, k, v, zero, zero, d_out)
    L = q.shape[2]
    mask = 0.5 * (np.tril(np.ones((L, L))) + np.triu(np.ones((L, L))))
    P = np.einsum("bhtc,bhic->bhti", q, k)
    dP = np.einsum("bhtj,bhij->bhti", d_out, v) * mask
    _close(dv, np.einsum("bhti,bhtj->bhij", P * mask, d_out))
    _close(dq, np.einsum("bhti,bhic->bhtc", dP, k))
    _close(dk, np.einsum("bhti,bhtc->bhic", dP, q))


def pin_bwd_reversal_symmetry(bwd):
    """Reversing the sequence and swapping the gate streams reverses every gradient and swaps the
    two gate gradients."""
    q, k, v, gf, gb = _draw(27, L=8)
    d_out = _rng(28).standard_normal(v.shape)
    a = bwd(q, k, v, gf, gb, d_out)
    rev = lambda x: np.ascontiguousarray(x[:, :, ::-1])
    b = bwd(rev(q), rev(k), rev(v), rev(gb), rev(gf), rev(d_out))
    for x, y in zip(a, (b[0], b[1], b[2], b[4], b[3])):
        _close(rev(y), x)


def pin_bwd_inert_gates_linearity_slabs(bwd):
    """g_fwd[0] and g_bwd[L-1] multiply zero states: no gradient.  The map d_out -> gradients is
    linear, and a slab whose d_out is zero receives none while the others are unchanged."""
    q, k, v, gf, gb = _draw(29, L=6)
    r = _rng(30)
    d1, d2 = r.standard_normal((2,) + v.shape)
    g1, g2, g12 = bwd(q, k, v, gf, gb, d1), bwd(q, k, v, gf, gb, d2), bwd(q, k, v, gf, gb, 2.0 * d1 - 3.0 * d2)
    assert np.all(g1[3][:, :, 0] == 0.0) and np.all(g1[4][:, :, -1] == 0.0)
    assert np.any(g1[3][:, :, 1] != 0.0) and np.any(g1[4][:, :, 0] != 0.0)
    for a, b, c in zip(g1, g2, g12):
        _close(c, 2.0 * a - 3.0 * b)
    d3 = d1.copy()
    d3[0, 1] = 0.0
    g3 = bwd(q, k, v, gf, gb, d3)
    for a, b in zip(g1, g3):
        assert np.all(b[0, 1] == 0.0)
        assert np.array_equal(b[1], a[1]) and np.array_equal(b[0, 0], a[0, 0])


def pin_bwd_library_autodiff(bwd):
    """Reverse-mode differentiation by a library (PyTorch autograd, CPU, fp64) of a vectorised
    explicit-product form: weights exp(difference of cumulative log-gates) under a mask, no
    recurrence and no code of the oracle.  The form itself is first held to the brute-force
    expansion; its gradient then pins all five gradients at a size finite differences do not
    reach, to rounding."""
    import torch

    q, k, v, gf, gb = _draw(29, B=1, H=2, L=9, dk=3, dv=4, gate_scale=1.2)
    d_out = _rng(30).standard_normal(v.shape)
    t = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v, gf, gb)]
    tq, tk, tv, tgf, tgb = t
    L = q.shape[2]
    cf = torch.cumsum(tgf, dim=2)                         # sum_{j<=t} gf_j
    cb = torch.cumsum(tgb, dim=2) - tgb                   # sum_{j<t}  gb_j
    idx = torch.arange(L)
    lower = (idx[None, :] <= idx[:, None]).to(torch.float64)   # [t, i]: i <= t
    upper = (idx[None, :] >= idx[:, None]).to(torch.float64)   # [t, i]: i >= t
    # decay from i to t, forward: prod_{j=i+1..t} a_fwd_j; backward: prod_{j=t..i-1} a_bwd_j
    df = torch.exp((cf[:, :, :, None, :] - cf[:, :, None, :, :]) * lower[None, None, :, :, None])
    db = torch.exp((cb[:, :, None, :, :] - cb[:, :, :, None, :]) * upper[None, None, :, :, None])
    wf = torch.einsum("bhtc,bhic,bhtic->bhti", tq, tk, df) * lower
    wb = torch.einsum("bhtc,bhic,bhtic->bhti", tq, tk, db) * upper
    out = 0.5 * torch.einsum("bhti,bhij->bhtj", wf + wb, tv)
    _close(out.detach().numpy(), quadratic_form(q, k, v, gf, gb), 1e-12)
    (out * torch.tensor(d_out)).sum().backward()
    got = bwd(q, k, v, gf, gb, d_out)
    for g, ref in zip(got, t):
        _close(g, ref.grad.numpy(), 1e-11)


BWD_PINS = (pin_bwd_finite_differences, pin_bwd_gates_closed, pin_bwd_gates_open, pin_bwd_reversal_symmetry,
            pin_bwd_inert_gates_linearity_slabs, pin_bwd_library_autodiff)
