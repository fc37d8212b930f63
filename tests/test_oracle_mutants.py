"""Every planted mistake in a copy of the oracle must trip at least one pin (CPU only).

The mutants are textual edits of oracle/bigla_oracle.c compiled into a temp dir; they show
that the pins in oracle_pins.py would catch a dropped term, a wrong sign or index, a
transposed operand, a swapped stream, a flipped kernel, and so on.
"""
import os
import subprocess

import pytest

import oracle
from oracle_pins import BIGLA_PINS, BWD_PINS, GP_PINS, LOC_PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "bigla_oracle.c")

# (name, old text, new text, occurrence index or None = all, which pin set)
MUTANTS = [
    ("no_half", "0.5 * (o_fwd[(size_t)t * dv + j] + acc)", "(o_fwd[(size_t)t * dv + j] + acc)", None, "bigla"),
    ("fwd_gate_is_bwd", "exp(g_fwd[(size_t)t * dk + c])", "exp(g_bwd[(size_t)t * dk + c])", None, "bigla"),
    ("bwd_gate_is_fwd", "exp(g_bwd[(size_t)t * dk + c])", "exp(g_fwd[(size_t)t * dk + c])", None, "bigla"),
    ("bwd_gate_of_next_token", "exp(g_bwd[(size_t)t * dk + c])",
     "exp(g_bwd[(size_t)(t + 1 < L ? t + 1 : t) * dk + c])", None, "bigla"),
    ("fwd_gate_of_prev_token", "exp(g_fwd[(size_t)t * dk + c])",
     "exp(g_fwd[(size_t)(t > 0 ? t - 1 : t) * dk + c])", None, "bigla"),
    ("gate_not_exponentiated", "exp(g_fwd[(size_t)t * dk + c])", "(1.0 + g_fwd[(size_t)t * dk + c])", None, "bigla"),
    ("readout_before_update_fwd", None, None, None, "bigla"),  # built specially below
    ("bwd_state_not_reset", "    memset(S, 0, sizeof(double) * (size_t)dk * dv);\n    for (int t = L - 1",
     "    for (int t = L - 1", None, "bigla"),
    ("bwd_scans_forward", "for (int t = L - 1; t >= 0; --t)", "for (int t = 0; t < L; ++t)", None, "bigla"),
    ("gate_on_value_dim", "S[(size_t)c * dv + j] = alpha * S[(size_t)c * dv + j] + kc * v[(size_t)t * dv + j];",
     "S[(size_t)c * dv + j] = exp(g_fwd[(size_t)t * dk + (j % dk)]) * S[(size_t)c * dv + j] + kc * v[(size_t)t * dv + j];",
     0, "bigla"),
    ("q_k_swapped_in_readout", "acc += q[(size_t)t * dk + c] * S[(size_t)c * dv + j];",
     "acc += k[(size_t)t * dk + c] * S[(size_t)c * dv + j];", 0, "bigla"),
    ("value_slab_misindexed", "const size_t ok = (size_t)s * L * dk, ov = (size_t)s * L * dv;",
     "const size_t ok = (size_t)s * L * dk, ov = (size_t)(slabs - 1 - s) * L * dv;", None, "bigla"),
    ("self_term_dropped_bwd", None, None, None, "bigla"),  # built specially below
    ("conv_flipped", "w[(size_t)c * 9 + (dy + 1) * 3 + (dx + 1)]", "w[(size_t)c * 9 + (1 - dy) * 3 + (1 - dx)]", None, "loc"),
    ("conv_transposed", "w[(size_t)c * 9 + (dy + 1) * 3 + (dx + 1)]", "w[(size_t)c * 9 + (dx + 1) * 3 + (dy + 1)]", None, "loc"),
    ("conv_wraps_rows", "if (yy < 0 || yy >= Hg || xx < 0 || xx >= Wg) continue;",
     "if (yy < 0 || yy >= Hg) continue; if ((size_t)yy * Wg + xx >= (size_t)Hg * Wg || yy * Wg + xx < 0) continue;", None, "loc"),
    ("gate_swapped", "gate * local + (1.0 - gate) * o_global[o]", "(1.0 - gate) * local + gate * o_global[o]", None, "loc"),
    ("gate_sign", "exp(-z[o])", "exp(z[o])", None, "loc"),
    ("channel_ignores_head", "const int c = h * dv + j;", "const int c = j;", None, "loc"),
    ("bias_outside_gate", "double local = bias ? bias[c] : 0.0;", "double local = 0.0;", None, "loc"),
    ("gp_halves_swapped", "double *g = dir == 0 ? g_fwd : g_bwd;", "double *g = dir == 0 ? g_bwd : g_fwd;", None, "gp"),
    ("gp_heads_interleaved", "const int dir = c / half, h = (c % half) / dk, j = c % dk;",
     "const int dir = c / half, h = (c % half) % H, j = (c % half) / H;", None, "gp"),
    ("gp_w1_transposed", "acc += xt[i] * w1[(size_t)i * rank + r];", "acc += xt[i] * w1[(size_t)r * D + i];", None, "gp"),
    ("gp_w2_transposed", "z += low[r] * w2[(size_t)r * width + c];", "z += low[r] * w2[(size_t)c * rank + r];", None, "gp"),
    ("gp_no_temperature", "log_sigmoid(z) / tau;", "log_sigmoid(z);", None, "gp"),
    ("gp_temperature_inside", "log_sigmoid(z) / tau;", "log_sigmoid(z / tau);", None, "gp"),
    ("gp_bias_dropped", "double z = bias ? bias[c] : 0.0;", "double z = 0.0;", None, "gp"),
    ("gp_sigmoid_sign", "return (z < 0.0 ? z : 0.0) - log1p(exp(-fabs(z)));", "return (z > 0.0 ? -z : 0.0) - log1p(exp(-fabs(z)));", None, "gp"),
    ("gp_naive_log_sigmoid", "return (z < 0.0 ? z : 0.0) - log1p(exp(-fabs(z)));", "return log(1.0 / (1.0 + exp(-z)));", None, "gp"),
    ("gp_token_batch_swapped", "const long b = n / L, t = n % L;", "const long b = n % B, t = n / B;", None, "gp"),
    ("bwd_no_half", "const double dot = 0.5 * d_out[(size_t)t * dv + j];", "const double dot = d_out[(size_t)t * dv + j];",
     None, "bwd"),
    ("bwd_adjoint_decays_by_own_gate", "const double decay = n == L - 1 ? 0.0 : exp(g[(size_t)(t + step) * dk + c]);",
     "const double decay = n == L - 1 ? 0.0 : exp(g[(size_t)t * dk + c]);", None, "bwd"),
    ("bwd_dalpha_from_current_state", "dalpha[(size_t)t * dk + c] += a[c] * states[(size_t)(t - step) * dk + c];",
     "dalpha[(size_t)t * dk + c] += a[c] * states[(size_t)t * dk + c];", None, "bwd"),
    ("bwd_dg_without_alpha", "dg[i] = exp(g[i]) * dalpha[i];", "dg[i] = dalpha[i];", None, "bwd"),
    ("bwd_directions_swapped", "dg_fwd + ok, L, dk, dv, +1, states, a, dalpha);",
     "dg_fwd + ok, L, dk, dv, -1, states, a, dalpha);", None, "bwd"),
    ("bwd_gate_streams_swapped", "bigla_bwd_direction(q + ok, k + ok, v + ov, g_bwd + ok,",
     "bigla_bwd_direction(q + ok, k + ok, v + ov, g_fwd + ok,", None, "bwd"),
    ("bwd_dq_from_adjoint", "dq[(size_t)t * dk + c] += states[(size_t)t * dk + c] * dot;",
     "dq[(size_t)t * dk + c] += a[c] * dot;", None, "bwd"),
    ("bwd_dv_from_q", "kv += k[(size_t)t * dk + c] * a[c];", "kv += q[(size_t)t * dk + c] * a[c];", None, "bwd"),
    ("bwd_dk_without_v", "dk_[(size_t)t * dk + c] += a[c] * v[(size_t)t * dv + j];", "dk_[(size_t)t * dk + c] += a[c];",
     None, "bwd"),
]


def _mutate(src: str, name: str, old, new, occ) -> str:
    if name == "readout_before_update_fwd":
        # forward readout uses S_{t-1} instead of S_t: move the readout loop before the update
        a = src.index("    for (int t = 0; t < L; ++t) {\n        for (int c = 0; c < dk; ++c) {")
        b = src.index("    /* backward direction")
        body = src[a:b]
        upd_start = body.index("        for (int c = 0; c < dk; ++c) {")
        upd_end = body.index("        for (int j = 0; j < dv; ++j) {")
        rd_end = body.rindex("    }\n")
        new_body = body[:upd_start] + body[upd_end:rd_end] + body[upd_start:upd_end] + body[rd_end:]
        return src[:a] + new_body + src[b:]
    if name == "self_term_dropped_bwd":
        # backward readout taken before adding k_t^T v_t (decay applied, own token missing)
        marker = "    for (int t = L - 1; t >= 0; --t) {"
        a = src.index(marker)
        old_upd = "S[(size_t)c * dv + j] = alpha * S[(size_t)c * dv + j] + kc * v[(size_t)t * dv + j];"
        i = src.index(old_upd, a)
        src = src[:i] + "S[(size_t)c * dv + j] = alpha * S[(size_t)c * dv + j];" + src[i + len(old_upd):]
        tail = "            out[(size_t)t * dv + j] = 0.5 * (o_fwd[(size_t)t * dv + j] + acc);\n        }\n"
        i = src.index(tail, a) + len(tail)
        add = ("        for (int c = 0; c < dk; ++c) for (int j = 0; j < dv; ++j)\n"
               "            S[(size_t)c * dv + j] += k[(size_t)t * dk + c] * v[(size_t)t * dv + j];\n")
        return src[:i] + add + src[i:]
    assert old in src, f"mutant {name}: pattern not found"
    if occ is None:
        return src.replace(old, new)
    parts = src.split(old)
    assert len(parts) > occ + 1
    return old.join(parts[:occ + 1]) + new + old.join(parts[occ + 1:])


@pytest.mark.parametrize("name,old,new,occ,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new, occ, which):
    src = open(SRC).read()
    mutated = _mutate(src, name, old, new, occ)
    assert mutated != src
    c_path = tmp_path / f"{name}.c"
    so_path = tmp_path / f"lib{name}.so"
    c_path.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-w", "-o", str(so_path),
                    str(c_path), "-lm"], check=True)
    mutant = oracle.Oracle(str(so_path))
    pins = {"bigla": BIGLA_PINS, "loc": LOC_PINS, "gp": GP_PINS, "bwd": BWD_PINS}[which]
    fn = {"bigla": mutant.bigla, "loc": mutant.locality_gate, "gp": mutant.gate_producer, "bwd": mutant.bigla_bwd}[which]
    tripped = []
    for pin in pins:
        try:
            pin(fn)
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, f"mutant {name} passed every pin"
