"""The pins must have teeth: plant one plausible mistake at a time in a copy of
the oracle's C source (on the CPU, never in the HIP path), rebuild it, and
check that at least one pin test fails for every mutant."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_adam as t_adam
import test_oracle_cast as t_cast
import test_oracle_fp16_scaler as t_f16
import test_oracle_hybrid_accum as t_hyb
import test_oracle_layout as t_layout
import test_oracle_reduce as t_reduce

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

MUTANTS = [
    ("floor_instead_of_ceil", "int64_t S = (N + W - 1) / W;", "int64_t S = N / W;"),
    ("offsets_inclusive", "off[i] = acc;\n        acc += n;", "acc += n;\n        off[i] = acc;"),
    ("pad_value_one", "flat[k] = 0.0f;", "flat[k] = 1.0f;"),
    ("chunk_ignores_rank", "shard[k] = flat[(int64_t)w * S + k];", "shard[k] = flat[k];"),
    ("cast_truncates", "(u + 0x7FFFu + lsb) >> 16", "u >> 16"),
    ("cast_half_up", "(u + 0x7FFFu + lsb) >> 16", "(u + 0x8000u) >> 16"),
    ("cast_half_down", "(u + 0x7FFFu + lsb) >> 16", "(u + 0x7FFFu) >> 16"),
    ("cast_nan_not_special", "(u & 0x007FFFFFu) != 0u)", "(u & 0x007FFFFFu) != 0u && 0)"),
    ("gather_reversed", "orc_cast_bf16(shards[w], S, flat_lp + (int64_t)w * S);",
     "orc_cast_bf16(shards[w], S, flat_lp + (int64_t)(W - 1 - w) * S);"),
    ("gather_f16_reversed", "orc_cast_f16(shards[w], S, flat_lp + (int64_t)w * S);",
     "orc_cast_f16(shards[w], S, flat_lp + (int64_t)(W - 1 - w) * S);"),
    ("gather_f16_ignores_rank", "orc_cast_f16(shards[w], S, flat_lp + (int64_t)w * S);",
     "orc_cast_f16(shards[0], S, flat_lp + (int64_t)w * S);"),
    ("gather_f16_casts_to_bf16", "orc_cast_f16(shards[w], S, flat_lp + (int64_t)w * S);",
     "orc_cast_bf16(shards[w], S, flat_lp + (int64_t)w * S);"),
    ("reduce_acc_from_zero", "float acc = slices[0][k] / pre;", "float acc = 0.0f + slices[0][k] / pre;"),
    ("reduce_reverse_order",
     "float acc = slices[0][k] / pre;\n        for (int32_t w = 1; w < W; ++w) acc = acc + slices[w][k] / pre;",
     "float acc = slices[W - 1][k] / pre;\n        for (int32_t w = W - 2; w >= 0; --w) acc = acc + slices[w][k] / pre;"),
    ("reduce_reciprocal_post", "out[k] = acc / post;", "out[k] = acc * (1.0f / post);"),
    ("reduce_no_post", "out[k] = acc / post;", "out[k] = acc;"),
    ("reduce_pre_after_sum",
     "float acc = slices[0][k] / pre;\n        for (int32_t w = 1; w < W; ++w) acc = acc + slices[w][k] / pre;\n        out[k] = acc / post;",
     "float acc = slices[0][k];\n        for (int32_t w = 1; w < W; ++w) acc = acc + slices[w][k];\n        out[k] = acc / pre / post;"),
    ("scatter_wrong_slice", "sl[w] = gradbufs[w] + (int64_t)r * S;", "sl[w] = gradbufs[w] + (int64_t)(r ? r - 1 : 0) * S;"),
    ("bf16_upcast_shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
    ("gather_lp_ignores_rank", "flat_lp[(int64_t)w * S + k] = lp_shards[w][k];", "flat_lp[(int64_t)w * S + k] = lp_shards[0][k];"),
    ("hybrid_drops_groups", "outer = (i == 0) ? inner : outer + inner;", "outer = inner;"),
    ("hybrid_rank_major_layout", "inner = inner + slices[(int64_t)i * F + l][k] / pre;",
     "inner = inner + slices[(int64_t)l * G + i][k] / pre;"),
    ("hybrid_flat_order", "outer = (i == 0) ? inner : outer + inner;\n        }\n        out[k] = outer / post;",
     "outer = inner;\n        }\n        { float a_ = slices[0][k] / pre; for (int32_t w = 1; w < G * F; ++w) a_ = a_ + slices[w][k] / pre; outer = a_; }\n        out[k] = outer / post;"),
    ("hybrid_post_per_group", "outer = (i == 0) ? inner : outer + inner;", "outer = (i == 0) ? inner / post : outer + inner / post;"),
    ("accumulate_overwrites", "acc[k] = acc[k] + add[k];", "acc[k] = add[k];"),
    ("accumulate_bf16_shift", "acc[k] = acc[k] + bf16_to_f32(add[k]);", "acc[k] = acc[k] + (float)add[k];"),
    ("f16_half_up", "if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;   /* a carry", "if (rem >= 0x1000u) h += 1;   /* a carry"),
    ("f16_truncates", "if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;   /* a carry", "/* a carry"),
    ("f16_subnormal_shift", "int32_t shift = -1 - e;", "int32_t shift = -2 - e;"),
    ("f16_flushes_subnormals", "uint32_t m = man | 0x00800000u;", "return (uint16_t)sign; uint32_t m = man | 0x00800000u;"),
    ("f16_overflow_saturates", "if (e > 15) return (uint16_t)(sign | 0x7C00u);", "if (e > 15) return (uint16_t)(sign | 0x7BFFu);"),
    ("f16_upcast_bias", "u = sign | ((exp + 112u) << 23) | (man << 13);", "u = sign | ((exp + 111u) << 23) | (man << 13);"),
    ("f16_upcast_subnormal", "u = sign | ((uint32_t)(112 - e) << 23) | ((man & 0x03FFu) << 13);", "u = sign | ((uint32_t)(113 - e) << 23) | ((man & 0x03FFu) << 13);"),
    ("unscale_no_check", "if (isinf(g[k]) || isnan(g[k])) found = 1.0f;", ""),
    ("unscale_misses_nan", "if (isinf(g[k]) || isnan(g[k])) found = 1.0f;", "if (isinf(g[k])) found = 1.0f;"),
    ("unscale_divides_by_inv", "g[k] = g[k] * inv_scale;", "g[k] = g[k] / inv_scale;"),
    ("combine_takes_first_rank", "if (flags[w] > m) m = flags[w];", "if (w == 0) m = flags[w];"),
    ("scaler_backoff_growth_swapped", "*scale = *scale * backoff;", "*scale = *scale * growth;"),
    ("scaler_tracker_not_reset", "*scale = *scale * backoff;\n        *growth_tracker = 0;", "*scale = *scale * backoff;"),
    ("scaler_grows_every_step", "if (t == growth_interval) {", "if (t >= 1) {"),
    ("adam_eps_inside_sqrt", "sqrtf(vk) / sqrt_bc2 + eps;", "sqrtf(vk + eps) / sqrt_bc2;"),
    ("adam_no_bias_correction2", "float sqrt_bc2 = sqrtf(bc2);", "float sqrt_bc2 = 1.0f;"),
    ("adam_no_bias_correction1", "float step_size = lr / bc1;", "float step_size = lr;"),
    ("adam_v_not_squared", "one_m_b2 * gk * gk;", "one_m_b2 * gk;"),
    ("adam_betas_swapped", "float mk = beta1 * m[k] + one_m_b1 * gk;", "float mk = beta2 * m[k] + one_m_b2 * gk;"),
    ("adam_ascent", "p[k] = p[k] - step_size", "p[k] = p[k] + step_size"),
    ("adam_state_not_stored", "        m[k] = mk;\n", ""),
]


def _pins():
    pins = [
        lambda: t_layout.test_fig3_worked_example(GOLDEN),
        t_layout.test_layout_special_cases,
        t_layout.test_config_sizes_table,
        t_layout.test_flatten_is_row_major_and_order_sensitive,
        lambda: t_layout.test_padding_closed_form_and_bound(3),
        lambda: t_layout.test_flatten_matches_concatenate_and_views_invert(3),
        lambda: t_layout.test_unshard_bf16_is_cast_of_parameters(3),
        lambda: t_layout.test_gather_of_cast_shards_equals_unshard(3),
        t_cast.test_hand_vectors,
        t_cast.test_nan_stays_quiet_nan_with_sign,
        t_cast.test_nearest_neighbour_in_exact_arithmetic,
        lambda: t_reduce.test_brute_force_sum_then_slice_tiny(4, 2.0, 2.0),
        lambda: t_reduce.test_brute_force_sum_then_slice_tiny(12, 4.0, 3.0),
        lambda: t_reduce.test_brute_force_sum_then_slice_tiny(3, 3.0, 1.0),
        t_reduce.test_pre_divide_happens_before_the_sum,
        t_reduce.test_minus_zero_survives,
        t_reduce.test_order_witness_sequential_rank_order,
        t_reduce.test_integer_gradients_give_exact_mean,
        t_reduce.test_pre_and_post_are_true_divisions,
        t_reduce.test_bf16_inputs_upcast_exactly,
        lambda: t_hyb.test_two_level_order_matches_exact_model(3, 4, 4.0, 3.0),
        lambda: t_hyb.test_two_level_order_matches_exact_model(2, 3, 1.0, 6.0),
        t_hyb.test_eq1_decomposition_is_exact_on_integers,
        t_hyb.test_two_level_order_differs_from_flat_order_in_binary32,
        t_hyb.test_hybrid_bf16_upcast_exact,
        t_hyb.test_accumulate_is_float32_addition,
        t_hyb.test_accumulation_with_and_without_communication_agree_on_integers,
        t_f16.test_f16_hand_vectors,
        t_f16.test_f16_nearest_neighbour_exact,
        lambda: t_f16.test_unshard_f16_is_cast_of_the_concatenated_shards(3),
        t_f16.test_f16_upcast_all_patterns_against_numpy,
        t_f16.test_f16_reduce_is_upcast_then_fp32_reduce,
        t_f16.test_unscale_check_against_torch,
        t_f16.test_sharded_flag_equals_flag_of_the_whole_gradient,
        t_f16.test_scaler_update_against_torch,
        t_adam.test_closed_form_first_step_from_zero_state,
        lambda: t_adam.test_single_step_matches_torch_adam_float64(5),
        t_adam.test_checkpoint_resume,
        t_adam.test_ten_steps_track_torch_adam,
    ]
    return pins


def _load(path):
    lib = ctypes.CDLL(path)
    lib.orc_num_threads.restype = ctypes.c_int
    oracle._configure(lib)
    return lib


def _killed() -> bool:
    for pin in _pins():
        try:
            pin()
        except (AssertionError, ValueError):
            return True
    return False


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new, tmp_path, monkeypatch):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "fsdp_oracle.c")).read()
    assert src.count(old) >= 1, f"mutation site for {name} not found"
    mutated = src.replace(old, new)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", *[f for f in oracle.CFLAGS if not f.startswith("-W")], str(c), "-o", str(so), "-lm"])
    oracle.lib()                                    # make sure the real one is loaded first
    monkeypatch.setattr(oracle, "_lib", _load(str(so)))
    assert _killed(), f"no pin noticed the planted mistake '{name}'"


def test_unmutated_oracle_passes_every_pin():
    for pin in _pins():
        pin()
