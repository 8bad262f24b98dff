"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source (a dropped
term, a wrong sign or index, a swapped operand, a wrong head mapping), compiles the copy on the CPU and runs
the pin tests against it: at least one pin must fail.  The real oracle is never touched; nothing here uses
the GPU.
"""
import os
import subprocess

import pytest

import oracle
import test_oracle_fp8 as fp8
import test_oracle_pins as pins

_SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "ppd_oracle.c")

# (name, text in the source, replacement, which occurrence)
MUTANTS = [
    ("row_does_not_see_itself", "(int64_t)L[i] + j + 1;", "(int64_t)L[i] + j;", 0),
    ("no_causal_mask_among_new_tokens", "(int64_t)L[i] + j + 1;", "(int64_t)L[i] + n[i];", 0),
    ("one_key_too_many", "(int64_t)L[i] + j + 1;", "(int64_t)L[i] + j + 2;", 0),
    ("wrong_kv_head_of_a_query_head", "int g = h / G;", "int g = h % Hkv;", 0),
    ("scale_dropped", "s[t] = (double)scale * dot;", "s[t] = dot;", 0),
    ("exponent_sign", "exp(s[t] - m)", "exp(m - s[t])", 0),
    ("normalisation_dropped", "(float)(acc / l)", "(float)(acc)", 0),
    ("query_read_backwards", "bf16_to_double(qv[d])", "bf16_to_double(qv[D - 1 - d])", 0),
    ("key_page_off_by_one_token", "page_tables[(int64_t)i * max_pages + t / P]",
     "page_tables[(int64_t)i * max_pages + (t + 1) / P]", 0),
    ("value_page_off_by_one_token", "page_tables[(int64_t)i * max_pages + t / P]",
     "page_tables[(int64_t)i * max_pages + (t + 1) / P]", 1),
    ("value_token_offset", "v_index(page, g, (int)(t % P), d, Hkv, D, P)",
     "v_index(page, g, (int)((t + 1) % P), d, Hkv, D, P)", 0),
    ("key_layout_d_reversed_inside_granule", "(int64_t)tok * 8 + d % 8;", "(int64_t)tok * 8 + (7 - d % 8);", 0),
    ("value_layout_d_reversed", "(int64_t)d * 8 +", "(int64_t)(D - 1 - d) * 8 +", 0),
    ("value_layout_token_major", "(int64_t)(tok / 8) * (D * 8) + (int64_t)d * 8 +\n           tok % 8;",
     "(int64_t)tok * D + d;", 0),
    ("k_and_v_halves_swapped", "return page * S + (int64_t)h * P * D + (int64_t)(d / 8)",
     "return page * S + (int64_t)Hkv * P * D + (int64_t)h * P * D + (int64_t)(d / 8)", 0),
    ("slot_offset_wraps_at_half_page", "int tok = (int)(slot % P);", "int tok = (int)(slot % (P / 2));", 0),
    ("skipped_token_written_to_slot_zero", "if (slot < 0) continue;", "if (slot < 0) slot = 0;", 0),
    ("source_heads_transposed", "int64_t src = (t * Hkv + h) * D + d;", "int64_t src = ((int64_t)h * T + t) * D + d;", 0),
    ("layers_land_in_one_pool", "pools + (int64_t)l * layer_stride,", "pools,", 0),
    ("layers_read_the_first_source", "k + (int64_t)l * T * Hkv * D, v + (int64_t)l * T * Hkv * D,", "k, v,", 0),
    ("delay_adds_the_fast_time", "/ beta_target - t_fast;", "/ beta_target + t_fast;", 0),
    ("delay_goes_negative", "return d > 0.0 ? d : 0.0;", "return d;", 0),
    # the FP8 page functions
    ("e4m3_bias_eight", "ldexp(1.0 + (double)m / 8.0, e - 7)", "ldexp(1.0 + (double)m / 8.0, e - 8)", 0),
    ("e4m3_subnormals_as_normals", "mag = ldexp((double)m / 8.0, -6);", "mag = ldexp(1.0 + (double)m / 8.0, -7);", 0),
    ("e4m3_four_mantissa_bits", "int sgn = code >> 7, e = (code >> 3) & 15, m = code & 7;",
     "int sgn = code >> 7, e = (code >> 4) & 7, m = (code & 15) / 2;", 0),
    ("e4m3_sign_dropped", "return sgn ? -mag : mag;", "return mag;", 0),
    ("e4m3_ties_to_the_odd_code", "(c & 1) == 0", "(c & 1) == 1", 0),
    ("e4m3_ties_away_from_zero", "(err == best_err && (c & 1) == 0)", "(err == best_err)", 0),
    ("e4m3_saturates_at_240", "c <= 0x7E; ++c", "c <= 0x77; ++c", 0),
    ("quantise_multiplies_by_the_scale", "volatile float inv = 1.0f / scale;", "volatile float inv = scale;", 0),
    ("values_quantised_with_the_key_scale", "quantise(v[src], v_scale)", "quantise(v[src], k_scale)", 0),
    ("fp8_append_token_offset", "int tok = (int)(slot % P);", "int tok = (int)((slot + 1) % P);", 1),
    ("fp8_layers_land_in_one_pool", "pools + (int64_t)l * layer_stride,", "pools,", 1),
    ("attention_ignores_the_value_scale", "fp8, v_scale);", "fp8, 1.0);", 0),
    ("attention_scales_keys_with_the_value_scale", "fp8, k_scale);", "fp8, v_scale);", 0),
    ("fp8_pool_read_as_16_bit", "if (fp8) return", "if (fp8 > 1) return", 0),
]

# the pins, cheapest and most general first
BATTERY = [
    pins.test_bruteforce_cfg1_all_seeds,
    lambda: pins.test_bruteforce_shapes(8, 1, 128),
    lambda: pins.test_bruteforce_shapes(6, 3, 64),
    pins.test_closed_forms,
    pins.test_append_touches_exactly_its_slots,
    pins.test_stale_pool_contents_never_leak,
    pins.test_append_prefill_equals_tail_of_recompute,
    pins.test_n1_append_prefill_is_decode_and_chunking,
    pins.test_gqa_equals_replicated_mha,
    pins.test_library_sdpa_contiguous_single_sequence,
    pins.test_kv_land_is_one_append_per_layer,
    pins.test_transfer_delay_model_against_the_papers_numbers,
    fp8.test_e4m3_landmarks,
    fp8.test_codes_round_trip_and_are_ordered,
    fp8.test_rounding_ties_and_saturation,
    fp8.test_codes_against_a_library_float8_conversion,
    fp8.test_fp8_append_stores_the_library_codes_in_the_16_bit_layout,
    fp8.test_fp8_attention_is_16_bit_attention_on_the_decoded_pool,
    fp8.test_fp8_scales_act_as_score_scale_and_output_factor,
    fp8.test_fp8_land_is_one_append_per_layer,
]


def _replace_nth(text, old, new, which):
    at = -1
    for _ in range(which + 1):
        at = text.find(old, at + 1)
        assert at >= 0, "the oracle's source no longer contains %r (occurrence %d)" % (old, which)
    return text[:at] + new + text[at + len(old):]


def _first_failing_pin():
    for k, pin in enumerate(BATTERY):
        try:
            pin()
        except (AssertionError, ValueError, FloatingPointError):
            return k
    return None


def test_the_unmodified_oracle_passes_the_battery():
    assert _first_failing_pin() is None


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(name, old, new, which, tmp_path, monkeypatch):
    src = _replace_nth(open(_SRC).read(), old, new, which)
    c_file = tmp_path / (name + ".c")
    so_file = tmp_path / (name + ".so")
    c_file.write_text(src)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-w", "-o", str(so_file), str(c_file), "-lm"])
    oracle.build()
    monkeypatch.setattr(oracle, "_lib", oracle._bind(str(so_file)))
    caught = _first_failing_pin()
    assert caught is not None, "no pin notices the planted mistake '%s'" % name
