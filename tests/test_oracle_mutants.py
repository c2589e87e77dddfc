"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the
oracle's C source (text substitution, CPU only), builds it, and requires that at
least one pin of tests/test_oracle_pins.py fails on it.
"""
import inspect
import os

import pytest

from oracle import relserve_oracle as ro
from tests import test_oracle_pins as pins

MUTANTS = [
    ("eps_outside_root", "1.0 / sqrt((double)ss / (double)H + (double)eps)", "1.0 / (sqrt((double)ss / (double)H) + (double)eps)"),
    ("norm_weight_dropped", "xr[i] * inv * oracle_bf16_to_f32(w[i])", "xr[i] * inv"),
    ("rope_sign", "vec[i]        = a * c - b * s;", "vec[i]        = a * c + b * s;"),
    ("rope_exponent", "-2.0 * (double)i / (double)d", "-1.0 * (double)i / (double)d"),
    ("rope_k_position", "row + q_dim + (size_t)g * d, d, tok_pos[t]", "row + q_dim + (size_t)g * d, d, 0"),
    ("position_ignores_past", "tok_pos[b->q_start[r] + j] = past + j;", "tok_pos[b->q_start[r] + j] = j;"),
    ("causal_excludes_self", "int32_t n_keys = pos + 1;", "int32_t n_keys = pos > 0 ? pos : 1;"),
    ("scale_1_over_d", "(float)(1.0 / sqrt((double)d));", "(float)(1.0 / (double)d);"),
    ("gqa_interleaved", "int32_t kvh = a / group;", "int32_t kvh = a % n_kv;"),
    ("slot_page_offset", "+ pos % c->page_size;", "+ (pos + 1) % c->page_size;"),
    ("residual_attn_dropped", "x1[(size_t)i * H + j] += xf[(size_t)sel[i] * H + j];", "x1[(size_t)i * H + j] += 0.0f * xf[(size_t)sel[i] * H + j];"),
    ("silu_sign", "g / (1.0f + expf(-g)) * u", "g / (1.0f + expf(g)) * u"),
    ("gate_up_swapped", "float g = gu[(size_t)i * 2 * I + j], u = gu[(size_t)i * 2 * I + I + j];",
     "float u = gu[(size_t)i * 2 * I + j], g = gu[(size_t)i * 2 * I + I + j];"),
    ("residual_mlp_dropped", "float y = x1[i] + mlp[i];", "float y = mlp[i];"),
    ("bf16_truncation", "u += 0x7fffu + lsb;", "(void)lsb;"),
    ("kv_not_rounded_through_cache", "vb[(size_t)t * kv_dim + i] = oracle_f32_to_bf16(row[q_dim + kv_dim + i]);",
     "vb[(size_t)t * kv_dim + i] = oracle_f32_to_bf16(row[q_dim + i]);"),
    ("logits_from_first_token", "x[(size_t)(b->q_start[r + 1] - 1) * H + i]", "x[(size_t)(b->q_start[r]) * H + i]"),
    ("final_norm_dropped", "oracle_linear(m->w_lm_head, m->vocab, H, normed, b->num_reqs, logits);",
     "oracle_linear(m->w_lm_head, m->vocab, H, last, b->num_reqs, logits);"),
    ("layers_share_one_cache", "x, k_pages[l], v_pages[l], num_pages,", "x, k_pages[0], v_pages[0], num_pages,"),
    ("stream_not_rounded_between_layers", "NULL, 0, y, x, NULL, NULL);", "NULL, 0, y, NULL, NULL, NULL); for (size_t i = 0; i < (size_t)T * H; ++i) x[i] = (uint16_t)(oracle_f32_to_bf16(y[i]) & 0xfff0u);"),
    ("greedy_last_of_equals", "if (!have || row[v] > row[best]) { best = v; have = 1; }", "if (!have || row[v] >= row[best]) { best = v; have = 1; }"),
    ("greedy_smallest", "if (!have || row[v] > row[best]) { best = v; have = 1; }", "if (!have || row[v] < row[best]) { best = v; have = 1; }"),
    ("e4m3_truncates", "float n = nearbyintf(ldexpf(a, -q));", "float n = floorf(ldexpf(a, -q));"),
    ("e4m3_no_saturation", "if (a >= 448.0f) return (uint8_t)(sign | 0x7e);", "if (a >= 1e30f) return (uint8_t)(sign | 0x7e);"),
    ("e4m3_bias", "else        mag = ldexpf((float)(8 + m), e - 7 - 3);", "else        mag = ldexpf((float)(8 + m), e - 8 - 3);"),
    ("quantised_scale_dropped_on_read", "return oracle_e4m3_to_f32(((const uint8_t*)pages)[idx]) * scale;", "return oracle_e4m3_to_f32(((const uint8_t*)pages)[idx]);"),
    ("quantised_v_with_k_scale", "v_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[row + i] * v_inv);", "v_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[row + i] * k_inv);"),
    ("quantised_k_before_rotation_slot", "k_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[i] * k_inv);", "k_pages[(size_t)slot * row + i] = oracle_f32_to_e4m3(src[i] * k_scale);"),
    ("quantised_inputs_not_rounded", "for (size_t i = 0; i < (size_t)T * H; ++i) h[i] = oracle_bf16_to_f32(oracle_f32_to_bf16(h[i]));", ";"),
    ("w8a8_row_scale_dropped", "const float scale = a_scale * s_w[n];", "const float scale = a_scale;"),
    ("w8a8_input_scale_dropped", "const float scale = a_scale * s_w[n];", "const float scale = s_w[n];"),
    ("w8a8_scale_of_the_next_row", "const float scale = a_scale * s_w[n];", "const float scale = a_scale * s_w[(n + 1) % N];"),
    ("w8a8_quantiser_multiplies_by_the_scale", "codes[i] = oracle_f32_to_e4m3(in[i] * inv);", "codes[i] = oracle_f32_to_e4m3(in[i] * scale);"),
    ("w8a8_weights_transposed", "wv[k] = lut[Wc[(size_t)n * K + k]];", "wv[k] = lut[Wc[(size_t)k * N + n]];"),
    ("w8a8_attention_output_not_rounded", "for (size_t i = 0; i < (size_t)n_out * q_dim; ++i) attn[i] = oracle_bf16_to_f32(oracle_f32_to_bf16(attn[i]));", ";"),
    ("w8a8_down_input_with_the_gate_up_scale", "q8 ? q8->a_down : 0.0f, H, I, act", "q8 ? q8->a_gate_up : 0.0f, H, I, act"),
    ("w8a8_o_input_with_the_qkv_scale", "q8 ? q8->a_o : 0.0f, H, q_dim, attn", "q8 ? q8->a_qkv : 0.0f, H, q_dim, attn"),
    ("w8a8_gate_up_rows_with_the_qkv_row_scales", "q8 ? q8->s_gate_up : NULL", "q8 ? q8->s_qkv : NULL"),
    ("w8a8_cache_inputs_rounded_as_in_the_16_bit_variant", "if (fp8 && !q8)", "if (fp8 || q8)"),
    ("w8a8_stack_reuses_the_first_layer", "oracle_layer_step_w8a8(c, b, &q8[l], x,", "oracle_layer_step_w8a8(c, b, &q8[0], x,"),
    ("softmax_unnormalised", "out[(size_t)a * d + i] = (float)(o[i] / denom);", "out[(size_t)a * d + i] = (float)(o[i]);"),
]


def _pin_functions():
    out = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        params = list(inspect.signature(fn).parameters)
        extra = [p for p in params if p not in ("oracle", "oracle64")]
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if extra and not marks:
            continue
        cases = [{}]
        for m in marks:
            key, vals = m.args
            cases = [dict(c, **{key: v}) for c in cases for v in vals]
        out.append((name, fn, params, cases))
    return out


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(ro._SRC).read()
    assert src.count(old) == 1, f"mutation anchor for {name} not unique in the oracle source"
    msrc = tmp_path / "mutant.c"
    msrc.write_text(src.replace(old, new))
    lib = str(tmp_path / f"mutant_{name}.so")
    ro.build(force=True, src=str(msrc), out={"f32": lib})
    mutant = ro.Oracle(lib)
    caught = []
    for tname, fn, params, cases in _pin_functions():
        for case in cases:
            kw = dict(case)
            if "oracle" in params:
                kw["oracle"] = mutant
            if "oracle64" in params:
                kw["oracle64"] = mutant
            try:
                fn(**kw)
            except (AssertionError, ValueError, FloatingPointError):
                caught.append(tname)
                break
        if caught:
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"
