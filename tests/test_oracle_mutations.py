"""Do the pins notice a broken oracle?  Each case plants ONE plausible mistake in a copy of
oracle/sasq_oracle.c (on the CPU, never on the GPU), builds it, and runs the pin tests against the
mutant in a subprocess: the pins must fail.  The unmodified copy must pass the same selection."""
from __future__ import annotations

import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sasq_oracle.c")

# (name, text in the source, replacement)
MUTATIONS = [
    ("round_half_away", "e.r = (flags & FLAG_NO_ROUND) ? e.p : rint(e.p);",
     "e.r = (flags & FLAG_NO_ROUND) ? e.p : round(e.p);"),
    ("ste_mask_on_v", "double u = (flags & FLAG_STE_ON_V) ? e.p : e.r;", "double u = e.p;"),
    ("clamp_symmetric", "e.q = e.r < (double)Qn ? (double)Qn", "e.q = e.r < (double)(Qn + 1) ? (double)(Qn + 1)"),
    ("ds_drop_mv_term", "if (e.m) t = isinf(e.p) ? 0.0 : g * (e.q - e.p);", "if (e.m) t = g * e.q;"),
    ("ds_wrong_sign", "if (e.m) t = isinf(e.p) ? 0.0 : g * (e.q - e.p);", "if (e.m) t = isinf(e.p) ? 0.0 : g * (e.p - e.q);"),
    ("ds_clipped_term_zero", "else     t = g * e.q;", "else     t = 0.0;"),
    ("dx_not_masked", "if (dx) dx[idx] = e.m ? dy[idx] : (uint16_t)0;\n            double t;", "if (dx) dx[idx] = dy[idx];\n            double t;"),
    ("true_division_instead_of_reciprocal", "e.p = x * (double)inv_s;", "e.p = x / (1.0 / (double)inv_s) * (1.0 + 1e-7);"),
    ("nibble_order_swapped", "(k & 1) ? (byte >> 4) : (byte & 15u)", "(k & 1) ? (byte & 15u) : (byte >> 4)"),
    ("nibble_unsigned", "static int nibble_to_int(unsigned v) { return (v & 8u) ? (int)v - 16 : (int)v; }",
     "static int nibble_to_int(unsigned v) { return (int)v; }"),
    ("gemm_transposed_weight", "acc += (int32_t)xq[m * K + k] * (int32_t)w8[n * K + k];",
     "acc += (int32_t)xq[m * K + k] * (int32_t)w8[(k % N) * K + (n % K)];"),
    ("epilogue_scale_order", "volatile float c = s * s_w[n];\n                volatile float af = (float)acc;\n                volatile float yf = af * c;",
     "volatile float c = (float)acc * s;\n                volatile float af = s_w[n];\n                volatile float yf = af * c;"),
    ("bias_dropped", "if (bias) { volatile float yb = yf + bias[n]; yf = yb; }", ""),
    ("weight_scale_uses_Qp_plus_1", "volatile float sw = amax / (float)Qp;", "volatile float sw = amax / (float)(Qp + 1);"),
    ("absmax_divides_by_128", "volatile float den = (float)((1 << (bits - 1)) - 1);", "volatile float den = (float)(1 << (bits - 1));"),
    ("f16_subnormal_decode", "if (e == 0)        v = ldexp((double)f, -24);", "if (e == 0)        v = 0.0;"),
    ("bf16_round_truncates", "static uint16_t f32_to_bf16(float f) { return round_to_small_float((double)f, 7, 8, 127); }",
     "static uint16_t f32_to_bf16(float f) { union { float f; uint32_t u; } c; c.f = f; return (uint16_t)(c.u >> 16); }"),
    ("per_channel_uses_first_scale", "        const float sk = s[k];", "        const float sk = s[0];"),
    ("per_channel_ds_row_indexed", "        if (ds64) ds64[k] = acc;", "        if (ds64) ds64[(k + 1) % cols] = acc;"),
    ("grouped_unfused", "f = fmaf((float)acc, s_g[i], f);", "f = f + (float)acc * s_g[i];"),
    ("grouped_scale_index", "reciprocal_f32(s_g[k / group])", "reciprocal_f32(s_g[k % G])"),
    ("grouped_descending", "for (int64_t i = 0; i < G; ++i) {", "for (int64_t i = G - 1; i >= 0; --i) {"),
    ("grouped_group_bounds", "for (int64_t k = i * group; k < (i + 1) * group; ++k)", "for (int64_t k = i * group; k < K; ++k)"),
    ("grouped_weight_factor_first_channel", "volatile float yf = f * s_w[n];", "volatile float yf = f * s_w[0];"),
    ("dynamic_uses_first_row_factor", "volatile float c = srow[m] * s_w[n];", "volatile float c = srow[0] * s_w[n];"),
    ("dynamic_factor_divides_by_128", "volatile float den = (float)Qp;\n        volatile float sm = num / den;",
     "volatile float den = (float)(Qp + 1);\n        volatile float sm = num / den;"),
    ("dynamic_zero_row_unhandled", "if (amax == 0.0) sm = 1.0f;", ""),
    ("bwd_linear_transposed_weight", "load16(w16, n * K + k, dt);", "load16(w16, (k % N) * K + (n % K), dt);"),
    ("bwd_linear_weight_factor_dropped", "volatile float prod = wf32 * s_w[n];", "volatile float prod = wf32;"),
    ("bwd_linear_weight_factor_first_channel", "volatile float prod = wf32 * s_w[n];", "volatile float prod = wf32 * s_w[0];"),
    ("bwd_linear_dy_row_stride", "load16(dy, m * N + n, dt) *", "load16(dy, (m * K + n) % (M * N), dt) *"),
    ("sgd_plus", "volatile float out = s - step;", "volatile float out = s + step;"),
]

PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_pins_pc.py", "tests/test_oracle_pins_grouped.py",
             "tests/test_oracle_pins_dynamic.py", "tests/test_oracle_pins_bwd_linear.py"]
SELECT = ("hand_table or closed_forms or autograd or static_linear or int4 or weight_quantizer or scale_sgd "
          "or encode or decode or per_channel or ds_terms or reciprocal or epilogue or grouped or dynamic or bwd_linear")


def run_pins(src_path: str) -> int:
    env = dict(os.environ, SASQ_ORACLE_MUTANT_SRC=src_path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES, "-k", SELECT],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    return r.returncode


def test_unmodified_copy_passes(tmp_path):
    p = tmp_path / "oracle_copy.c"
    p.write_text(open(SRC).read())
    assert run_pins(str(p)) == 0


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_mutation(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation target for {name} not found in the oracle source"
    p = tmp_path / f"mutant_{name}.c"
    p.write_text(src.replace(old, new, 1))
    assert run_pins(str(p)) != 0, f"no pin noticed the planted mistake: {name}"
