"""The pins of the oracle catch planted mistakes.

Each case below plants one plausible mistake in a copy of oracle/gws_oracle.c (a wrong
constant, a dropped term, a wrong sign or index, a transposed operand), compiles the copy
on the CPU and runs the pin that is meant to catch it against the mutated library: the pin
must fail.  Nothing here touches a GPU or the product library."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_arith as arith
import test_oracle_basis as basis
import test_oracle_bitwidth as bw
import test_oracle_mx as mx
import test_oracle_rng as rng
import test_oracle_sample as smp

SRC = os.path.join(os.path.dirname(oracle.__file__), "gws_oracle.c")

# (name, text in the source, replacement, pins expected to fail)
MUTANTS = [
    ("philox multipliers swapped", "(uint64_t)0xD2511F53u * c0", "(uint64_t)0xCD9E8D57u * c0",
     [rng.test_philox_known_answer_vectors]),
    ("philox key increment", "k0 += 0x9E3779B9u;", "k0 += 0x9E3779B1u;", [rng.test_philox_known_answer_vectors]),
    ("philox output order", "out[0] = c0; out[1] = c1;", "out[0] = c1; out[1] = c0;",
     [rng.test_philox_known_answer_vectors]),
    ("philox one round short", "gwso_philox4x32(ctr, key, 10, x);", "gwso_philox4x32(ctr, key, 9, x);",
     [rng.test_noise_uses_counter_col_group_row_step_and_seed_key]),
    ("|R|=2 without the (b or b) factor", "int mag2 = all8 && A;", "int mag2 = all8;",
     [rng.test_bits_to_r_exhaustive_matches_eq10]),
    ("(b or b) reduced to one bit", "int D = (n3 & 0x3u) != 0;", "int D = (n3 & 0x1u) != 0;",
     [rng.test_bits_to_r_exhaustive_matches_eq10]),
    ("|R|=1 not excluded where |R|=2", "int mag1 = C && D && E && !mag2;", "int mag1 = C && D && E;",
     [rng.test_bits_to_r_exhaustive_matches_eq10]),
    ("sign bit shared with a magnitude bit", "int S = (n3 >> 3) & 1;", "int S = (n3 >> 2) & 1;",
     [rng.test_bits_to_r_exhaustive_matches_eq10]),
    ("code not sign-magnitude", "return (code & 8) ? -mag : mag;", "return (code & 8) ? mag - 4 : mag;",
     [rng.test_code_to_r_is_sign_magnitude]),
    ("counter ignores the step", "(uint32_t)step, (uint32_t)(step >> 32)};\n  uint32_t key[2] = {(uint32_t)seed",
     "0u, (uint32_t)(step >> 32)};\n  uint32_t key[2] = {(uint32_t)seed",
     [rng.test_noise_uses_counter_col_group_row_step_and_seed_key]),
    ("element uses the wrong nibble", "return (k >> 1) + 4 * (k & 1);", "return k;",
     [rng.test_noise_uses_counter_col_group_row_step_and_seed_key]),
    ("exp2 coefficient", "0x3E75FDF0u", "0x3E75FDF8u", [arith.test_exp2_within_one_ulp_of_fp64]),
    ("exp2 not scaled by 2^n", "return ldexpf(p, (int)n);", "return ldexpf(p, (int)n + 1);",
     [arith.test_exp2_exact_on_integers]),
    ("bf16 add: ties away from zero", "(rem == half && (sticky || (keep & 1)))", "(rem == half)",
     [arith.test_bf16_add_hand_ties]),
    ("bf16 add: truncation", "int up = (rem > half) ||", "int up = 0 && (rem > half) ||",
     [arith.test_bf16_add_close_exponents_vs_torch]),
    ("cast: one mantissa bit short (E4M3)", "*emax = 8; *emin = -6; *m = 3;", "*emax = 8; *emin = -6; *m = 2;",
     [arith.test_cast_e4m3_vs_torch_float8]),
    ("cast: subnormal threshold (E3M2)", "*emax = 4; *emin = -2; *m = 2;", "*emax = 4; *emin = -1; *m = 2;",
     [arith.test_cast_exhaustive_vs_brute_force]),
    ("cast: no saturation", "if (q > maxv) q = maxv;", "", [arith.test_cast_hand_cases]),
    ("cast: scale exponent off by one", "int xe = Ea + 1 - emax;", "int xe = Ea - emax;",
     [arith.test_cast_exhaustive_vs_brute_force]),
    ("cast: sign of zero dropped", "return (uint16_t)((v16 & 0x8000u) | (r & 0x7FFFu));", "return (uint16_t)(r & 0x7FFFu);",
     [arith.test_cast_exhaustive_vs_brute_force]),
    ("forward: 2^(-b_t) instead of 2^(1-b_t)", "float t = 1.0f - bt[bi * nbc + bj];", "float t = 0.0f - bt[bi * nbc + bj];",
     [smp.test_forward_hand_worked_block]),
    ("forward: b_t indexed transposed", "float t = 1.0f - bt[bi * nbc + bj];", "float t = 1.0f - bt[(bj * nbr + bi) % (nbr * nbc)];",
     [lambda: smp.test_forward_vs_library_composition(oracle.FMT_BF16, (96, 160))]),
    ("forward: noise sign dropped", "((code & 8) ? 0x8000u : 0u));", "0u);", [smp.test_forward_hand_worked_block]),
    ("forward: |R|=2 uses s instead of 2s", "(mag == 1 ? s16 : s2_16)", "(mag == 1 ? s16 : s16)",
     [smp.test_forward_hand_worked_block]),
    ("forward: scale not rounded to BF16", "uint16_t s16 = gwso_bf16_rne(s32);", "uint16_t s16 = (uint16_t)(f32_bits(s32) >> 16);",
     [smp.test_pqn_step_is_the_bf16_rounding_of_the_scale]),
    ("forward: block max misses the last row", "for (int64_t i = i0; i < i1; ++i)\n        for (int64_t j = j0; j < j1; ++j) {\n          uint16_t mag",
     "for (int64_t i = i0; i < i1 - 1; ++i)\n        for (int64_t j = j0; j < j1; ++j) {\n          uint16_t mag",
     [smp.test_block_absmax_sees_every_position_and_only_its_own_block]),
    ("forward: block max taken over signed bit patterns", "uint16_t mag = w[i * ld + j] & 0x7FFFu;", "uint16_t mag = w[i * ld + j];",
     [smp.test_block_absmax_sees_every_position_and_only_its_own_block]),
    ("forward: edge block reads past the tensor", "int64_t j1 = j0 + GWSO_BL < cols ? j0 + GWSO_BL : cols;\n      /* max",
     "int64_t j1 = j0 + GWSO_BL < ld ? j0 + GWSO_BL : ld;\n      /* max", [smp.test_edge_blocks_and_row_padding]),
    ("forward: cast skipped", "(a16 == 0) ? sum : gwso_cast(sum, Ea, fmt)", "sum",
     [smp.test_forward_hand_worked_block]),
    ("backward: sign of ln2", "dbt[bi * nbc + bj] = -ln2 * s * acc;", "dbt[bi * nbc + bj] = ln2 * s * acc;",
     [smp.test_backward_matches_finite_difference_of_eq3]),
    ("backward: scale factor dropped", "dbt[bi * nbc + bj] = -ln2 * s * acc;", "dbt[bi * nbc + bj] = -ln2 * acc;",
     [smp.test_backward_matches_finite_difference_of_eq3]),
    ("backward: dW not a copy", "if (dw) dw[i * ld + j] = g[i * ld + j];", "if (dw) dw[i * ld + j] = g[i * ld + j] ^ 0x8000u;",
     [smp.test_backward_dw_is_g_and_dbt_matches_definition]),
    ("backward: different noise than forward", "group_words(row0 + i, (col0 + j) >> 3, seed, step, x);\n          double r =",
     "group_words(row0 + i, (col0 + j) >> 3, seed, step + 1, x);\n          double r =",
     [smp.test_backward_matches_finite_difference_of_eq3]),
    ("linear: weight layout flag inverted", "w_is_nk ? q[n * ldq + k] : q[k * ldq + n]", "w_is_nk ? q[k * ldq + n] : q[n * ldq + k]",
     [smp.test_linear_vs_numpy_fp64_matmul]),
    ("linear: rounding of Y truncates", "if (rem > half || (rem == half && (keep & 1))) keep += 1;\n  int ef", "int ef",
     [smp.test_linear_bf16_output_rounds_once_to_nearest_even]),
    ("linear: ties of Y rounded away from zero", "if (rem > half || (rem == half && (keep & 1))) keep += 1;\n  int ef",
     "if (rem >= half) keep += 1;\n  int ef", [smp.test_linear_bf16_output_rounds_once_to_nearest_even]),
    ("linear: subnormal Y flushed to zero", "if (E < -126) drop += (-126 - E);", "if (E < -126) return (uint16_t)(sign << 15);",
     [smp.test_linear_bf16_output_rounds_once_to_nearest_even]),
    ("uniform basis: grid shifted by half a step", "2 * (int)(byte & 0xFFu) - 255", "2 * (int)(byte & 0xFFu) - 256",
     [basis.test_uniform_values_enumerated]),
    ("uniform basis: element takes the wrong byte", "(x[k >> 2] >> (8 * (k & 3)))", "(x[k & 3] >> (8 * (k >> 2)))",
     [basis.test_uniform_element_owns_byte_k_mod_4_of_word_k_div_4]),
    ("uniform basis: R * s truncated instead of rounded", "return gwso_bf16_rne(bf16_to_f32(a) * bf16_to_f32(b));",
     "return (uint16_t)(f32_bits(bf16_to_f32(a) * bf16_to_f32(b)) >> 16);", [basis.test_bf16_mul_matches_torch]),
    ("Box-Muller: sine and cosine branches swapped", "z[0] = r * cq;\n  z[1] = r * sq;", "z[0] = r * sq;\n  z[1] = r * cq;",
     [basis.test_box_muller_matches_the_fp64_formula]),
    ("Box-Muller: radius from -ln instead of -2 ln", "float L = -2.0f * bm_log(u1);", "float L = -1.0f * bm_log(u1);",
     [basis.test_box_muller_matches_the_fp64_formula]),
    ("Box-Muller: second quadrant mirrored", "case 1: cq = -sn; sq = c; break;", "case 1: cq = sn; sq = c; break;",
     [basis.test_box_muller_matches_the_fp64_formula]),
    ("Box-Muller: logarithm coefficient", "0x3EAAABC8u", "0x3EABABC8u", [basis.test_box_muller_matches_the_fp64_formula]),
    ("Box-Muller: round(z) instead of round(z / 2)", "float rr = rintf(0.5f * z[k & 1]);", "float rr = rintf(z[k & 1]);",
     [basis.test_box_muller_cells_match_the_rounded_normal]),
    ("Box-Muller: pair takes the wrong word", "gwso_box_muller(x[k >> 1], z);", "gwso_box_muller(x[k >> 2], z);",
     [basis.test_box_muller_pair_d_takes_word_d_cos_then_sin]),
    ("basis forward: step doubled", "pqn = gwso_bf16_mul(r16, s16);", "pqn = gwso_bf16_mul(r16, s2_16);",
     [lambda: basis.test_forward_with_a_basis_vs_library_composition(oracle.BASIS_UNIFORM, (70, 45))]),
    ("basis backward: falls back to the bit basis", "if (basis != GWSO_BASIS_BITS) r = gwso_basis_r", "if (0) r = gwso_basis_r",
     [lambda: basis.test_backward_with_a_basis_matches_the_definition(oracle.BASIS_BOX_MULLER)]),
    ("Eq. 11: offset is b_init instead of b_target", "bt[k] = b_target + prod;", "bt[k] = b_init + prod;",
     [bw.test_eq11_end_points_and_midpoint]),
    ("Eq. 11: slope sign", "float delta = b_init - b_target;\n  for (int64_t k = 0; k < n; ++k) {\n    float prod = bi[k] * delta;\n    bt[k]",
     "float delta = b_target - b_init;\n  for (int64_t k = 0; k < n; ++k) {\n    float prod = bi[k] * delta;\n    bt[k]",
     [bw.test_eq11_end_points_and_midpoint]),
    ("Eq. 12: chain-rule factor dropped", "dbi[k] = (double)delta * (dbt[k]", "dbi[k] = (dbt[k]",
     [bw.test_eq12_gradient_matches_finite_differences]),
    ("Eq. 12: loss term not divided by the layer's block count", "lambda / (double)m * sgn", "lambda * sgn",
     [bw.test_eq12_gradient_matches_finite_differences]),
    ("Eq. 12: divided by the blocks handed in instead of the layer's", "lambda / (double)m * sgn", "lambda / (double)n * sgn",
     [bw.test_eq12_gradient_matches_finite_differences]),
    ("Eq. 12: sign of the loss term", "double sgn = bt > b_target ? 1.0", "double sgn = bt > b_target ? -1.0",
     [bw.test_eq12_special_cases]),
    ("Eq. 12: subgradient at zero not zero", "(bt < b_target ? -1.0 : 0.0)", "-1.0",
     [bw.test_eq12_special_cases]),
    ("MX: shared exponent biased by 128", "xscale[bi * nbc + bj] = (uint8_t)(Ea + 1 - emax + 127);",
     "xscale[bi * nbc + bj] = (uint8_t)(Ea + 1 - emax + 128);", [mx.test_hand_block_scales]),
    ("MX: shared exponent without the headroom binade", "xscale[bi * nbc + bj] = (uint8_t)(Ea + 1 - emax + 127);",
     "xscale[bi * nbc + bj] = (uint8_t)(Ea - emax + 127);", [mx.test_hand_block_scales]),
    ("MX: all-zero block does not get X = 1", "floor_log2_bf16(a16) : emax - 1;", "floor_log2_bf16(a16) : 0;",
     [mx.test_hand_block_scales]),
    ("MX: FP6 fields packed from the top bit of each byte", "(uint8_t)(1u << (bit % 8))", "(uint8_t)(0x80u >> (bit % 8))",
     [lambda: mx.test_mx_output_decodes_to_the_bf16_container_output(oracle.FMT_FP6_E3M2, (40, 50))]),
    ("MX: FP6 field written top bit first", "int64_t bit = 6 * j + b;", "int64_t bit = 6 * j + (5 - b);",
     [lambda: mx.test_mx_output_decodes_to_the_bf16_container_output(oracle.FMT_FP6_E3M2, (40, 50))]),
    ("MX: exponent bias off by one", "int bias = 1 - emin;", "int bias = -emin;",
     [mx.test_e3m2_code_values_match_the_specification_figures, mx.test_e4m3_code_values_match_torch_float8]),
    ("MX: subnormal codes scaled like normals", "ldexp((double)mant, emin - m)", "ldexp((double)mant, emin - m - 1)",
     [mx.test_e3m2_code_values_match_the_specification_figures]),
    ("MX: sign bit one position low", "? nmag : 0);", "? (nmag >> 1) : 0);",
     [lambda: mx.test_encode_inverts_the_code_values_at_any_block_scale(oracle.FMT_FP8_E4M3)]),
]


def _build_mutant(tmp_path, idx, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target not found: {old!r}"
    path_c = tmp_path / f"m{idx}.c"
    path_so = tmp_path / f"m{idx}.so"
    path_c.write_text(text.replace(old, new, 1))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-w",
                    "-o", str(path_so), str(path_c), "-lm"], check=True)
    return oracle.configure(ctypes.CDLL(str(path_so)))


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(idx, tmp_path, monkeypatch):
    name, old, new, pins = MUTANTS[idx]
    oracle.lib()                                     # make sure the genuine library is loaded first
    monkeypatch.setattr(oracle, "_lib", _build_mutant(tmp_path, idx, old, new))
    failed = 0
    for pin in pins:
        try:
            pin()
        except Exception:  # an assertion, or an error the mistake provokes inside the pin
            failed += 1
    assert failed >= 1, f"mutant '{name}' survived {[getattr(p, '__name__', 'pin') for p in pins]}"


def test_the_genuine_oracle_passes_the_same_pins():
    for _, _, _, pins in MUTANTS:
        for pin in pins:
            pin()
