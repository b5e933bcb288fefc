"""The pins must notice plausible mistakes: each case plants ONE wrong token in a copy of the
oracle source (on the CPU, never in the GPU code), rebuilds it, and expects the pin suite to
fail against that copy."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "qa_oracle.cpp")

MUTATIONS = [
    ("threshold_divides_by_n_plus_1", "* S1) / (double)n);", "* S1) / (double)(n + 1));"),
    ("scale_keeps_equal_magnitudes", "if (a > Delta) { S2 += (double)a; ++cnt; }",
     "if (a >= Delta) { S2 += (double)a; ++cnt; }"),
    ("negative_side_compares_wrong_sign", "if (v < -Delta) return -1;", "if (v < Delta) return -1;"),
    ("minus_one_packed_as_10", "code[i] == 1 ? 1u : (code[i] == -1 ? 3u : 0u)",
     "code[i] == 1 ? 1u : (code[i] == -1 ? 2u : 0u)"),
    ("pack_shift_wraps_at_8", "words[i / 16] |= f << (2 * (i % 16));", "words[i / 16] |= f << (2 * (i % 8));"),
    ("reserved_pattern_decodes_minus_one", "return f == 1u ? 1 : (f == 3u ? -1 : 0);",
     "return f == 1u ? 1 : (f >= 2u ? -1 : 0);"),
    ("average_forgets_division", "return (float)(acc / (double)M);", "return (float)(acc);"),
    ("average_uses_wrong_bucket", "const int64_t k = i / bucket_b;", "const int64_t k = i / 16;"),
    ("delta_inside_the_root", "return delta + std::sqrt(*G);", "return std::sqrt(delta + *G);"),
    ("H_without_current_gradient", "  *G = *G + g2;\n  return delta + std::sqrt(*G);",
     "  const float Gold = *G;\n  *G = *G + g2;\n  return delta + std::sqrt(Gold);"),
    ("qcmd_tau_without_eta", "const float tau = (lambda * eta) / H;", "const float tau = lambda / H;"),
    ("qcmd_ascends", "const float u = x - step;", "const float u = x + step;"),
    ("qrda_wrong_sign", "return -std::copysign(mag, z);", "return std::copysign(mag, z);"),
    ("qrda_threshold_without_t", "const float tl = (float)t * lambda;", "const float tl = lambda;"),
    ("qrda_equality_kept", "if (!(r > 0.0f)) return 0.0f;", "if (!(r >= 0.0f)) return 0.0f;"),
    ("qrda_z_subtracts", "    z[i] = z[i] + q[i];\n    x[i] = qrda_component",
     "    z[i] = z[i] - q[i];\n    x[i] = qrda_component"),
    ("logistic_gradient_sign", "*coef_out = (float)((-(double)y * sig) / (double)B);",
     "*coef_out = (float)(((double)y * sig) / (double)B);"),
    ("logistic_sigmoid_branches_swapped", "m >= 0 ? e / (1.0 + e) : 1.0 / (1.0 + e)",
     "m >= 0 ? 1.0 / (1.0 + e) : e / (1.0 + e)"),
    ("requantize_ignores_buckets", "requant == 1 ? bucket : 0, thr_coef, q.data());",
     "0, thr_coef, q.data());"),
    ("exact_threshold_objective", "double obj = run * run / (double)k;", "double obj = run / (double)k;"),
    ("exact_thresholds_drop_the_smallest_kept", "if ((double)a < kept_min && a > Delta) Delta = a;",
     "if ((double)a <= kept_min && a > Delta) Delta = a;"),
    ("exact_thresholds_take_any_smaller_magnitude", "if ((double)a < kept_min && a > Delta) Delta = a;",
     "if ((double)a < kept_min && Delta == 0.0f) Delta = a;"),
    ("tensor_codes_start_at_the_wrong_word", "codes + (int64_t)m * code_stride + begin[s] / 16, 0, sc, th, 0, 0);",
     "codes + (int64_t)m * code_stride + begin[s] / 32, 0, sc, th, 0, 0);"),
    ("tensor_step_uses_first_tensors_scale", "orc_step_qcmd(codes + b / 16, code_stride, scales + s,",
     "orc_step_qcmd(codes + b / 16, code_stride, scales,"),
    ("tensor_step_skips_second_quantization", "x + b, G + b, zs, t, eta, lambda, delta, requant ? 2 : 0);",
     "x + b, G + b, zs, t, eta, lambda, delta, 0);"),
    ("select_codes_takes_unmarked_components", "if ((ind[i / 32] >> (i % 32)) & 1u)\n        code.push_back(",
     "if (!((ind[i / 32] >> (i % 32)) & 1u))\n        code.push_back("),
    ("csr_gradient_uses_row_position", "acc[indices[k]] += (double)coef[b] * (double)vals[k];",
     "acc[indices[k]] += (double)coef[b] * (double)vals[indptr[r]];"),
    ("indicator_needs_both", "if (x[i] != 0.0f || xh != 0.0f) ind_out", "if (x[i] != 0.0f && xh != 0.0f) ind_out"),
    # (dropping g^2 from H^ is not a detectable mistake: whether x^ is zero does not depend on H^
    #  in exact arithmetic -- |x H - eta g| > lambda eta, resp. |z + g| > t lambda)
    ("indicator_qrda_ignores_local_gradient", "const float zh = z[i] + g[i];", "const float zh = z[i];"),
    ("selection_takes_unmarked", "if ((ind[i / 32] >> (i % 32)) & 1u) sel.push_back(g[i]);",
     "if (!((ind[i / 32] >> (i % 32)) & 1u)) sel.push_back(g[i]);"),
    ("philox_key_not_bumped", "if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }",
     "if (round > 1) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }"),
    ("philox_nine_rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
    ("stochastic_keep_probability_inverted", "const bool keep = orc_uniform(seed, step, m, i) < p;",
     "const bool keep = orc_uniform(seed, step, m, i) >= p;"),
    ("stochastic_scale_is_mean_not_max", "      if (a > s) s = a;                        // NaN never wins",
     "      s += a / (float)(hi - lo);"),
    ("stochastic_same_draw_for_all_workers", "const uint32_t ctr[4] = {(uint32_t)j, (uint32_t)(j >> 32), m, step};",
     "const uint32_t ctr[4] = {(uint32_t)j, (uint32_t)(j >> 32), 0, step};"),
    ("decode_advances_on_every_coordinate", "        ++j;\n      }\n  }\n  pack_codes(code.data(), d, dense_words);",
     "      }\n      ++j;\n  }\n  pack_codes(code.data(), d, dense_words);"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not unique/found"
    with tempfile.TemporaryDirectory() as tmp:
        cpp = os.path.join(tmp, "mut.cpp")
        so = os.path.join(tmp, "libmut.so")
        open(cpp, "w").write(src.replace(old, new))
        subprocess.run(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-fPIC", "-shared", cpp, "-o", so],
                       check=True)
        env = dict(os.environ, QA_ORACLE_LIB=so)
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                            os.path.join(ROOT, "tests", "test_oracle_selection_pins.py"),
                            os.path.join(ROOT, "tests", "test_oracle_stochastic_pins.py"),
                            os.path.join(ROOT, "tests", "test_oracle_segments_pins.py")],
                           env=env, cwd=ROOT, capture_output=True, text=True)
        assert r.returncode != 0, f"pins did not notice: {name}"
