"""Plant one plausible mistake at a time in a copy of the oracle's source (on the CPU, never in
the HIP path) and require that the pins notice: a dropped term, a wrong sign, a swapped
operand, a wrong index, a missing normalisation."""
import os
import tempfile

import pytest

import oracle
import oracle_pins

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "ddl_oracle.c")).read()

# (name, text in the oracle, replacement)
MUTANTS = [
    ("delta_sign", "w[m] * (Theta - learner_value(", "w[m] * (-Theta + learner_value("),
    ("delta_drops_theta", "w[m] * (Theta - learner_value(", "w[m] * (0.0 - learner_value("),
    ("delta_unweighted", "Delta += w[m] * (Theta", "Delta += (Theta"),
    ("absent_multiplied_not_skipped",
     "if (w[m] == 0.0)\n                continue;\n            Delta += w[m] * (Theta",
     "Delta += w[m] * (Theta"),
    ("rda_absent_multiplied_not_skipped",
     "if (w[m] == 0.0 || norm[m] == 0.0)\n                    continue;", ""),
    ("momentum_dropped", "double v_new = mu * (double)v[i] + Delta;", "double v_new = Delta;"),
    ("momentum_dampened", "double v_new = mu * (double)v[i] + Delta;",
     "double v_new = mu * (double)v[i] + (1.0 - mu) * Delta;"),
    ("heavy_ball_not_nesterov", "Theta - lr * (Delta + mu * v_new)", "Theta - lr * v_new"),
    ("nesterov_uses_old_v", "Theta - lr * (Delta + mu * v_new)",
     "Theta - lr * (Delta + mu * (double)v[i])"),
    ("step_sign", "Theta - lr * (Delta + mu * v_new)", "Theta + lr * (Delta + mu * v_new)"),
    ("lr_on_buffer", "double v_new = mu * (double)v[i] + Delta;",
     "double v_new = mu * (double)v[i] + lr * Delta;"),
    ("weights_not_normalised", "(double)token_counts[m] / S : 0.0", "(double)token_counts[m] : 0.0"),
    ("weights_ignore_mask_in_sum", "if (quorum_mask[m])\n            S +=", "S +="),
    ("weights_ignore_mask", "quorum_mask[m] ? (double)token_counts[m] / S : 0.0",
     "(double)token_counts[m] / S"),
    ("weights_uniform", "quorum_mask[m] ? (double)token_counts[m] / S : 0.0",
     "quorum_mask[m] ? 1.0 / M : 0.0"),
    ("bf16_shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
    ("learner_index", "return widen_bf16(((const uint16_t*)base)[i]);",
     "return widen_bf16(((const uint16_t*)base)[i ? i - 1 : 0]);"),
    ("quality_tokens_only", "raw[m] = c_tok * (c_tok / (double)step_counts[m]);", "raw[m] = c_tok;"),
    ("quality_inverted", "raw[m] = c_tok * (c_tok / (double)step_counts[m]);",
     "raw[m] = c_tok * ((double)step_counts[m] / c_tok);"),
    ("bf16_round_truncates", "if (dlo < dhi) return (uint16_t)(lo_bits >> 16);\n    if (dhi < dlo) return (uint16_t)(hi_bits >> 16);\n    return (uint16_t)((((lo_bits >> 16) & 1u) == 0 ? lo_bits : hi_bits) >> 16);\n}",
     "return (uint16_t)(lo_bits >> 16);\n}"),
    ("bf16_round_ties_away", "    double dhi = fabs((double)hi - (double)x);\n    if (dlo < dhi) return (uint16_t)(lo_bits >> 16);\n    if (dhi < dlo) return (uint16_t)(hi_bits >> 16);\n    return (uint16_t)((((lo_bits >> 16) & 1u) == 0 ? lo_bits : hi_bits) >> 16);",
     "    double dhi = fabs((double)hi - (double)x);\n    if (dlo < dhi) return (uint16_t)(lo_bits >> 16);\n    return (uint16_t)(hi_bits >> 16);"),
    ("rda_norm_not_sqrt", "norm[m] = sqrt(ss);", "norm[m] = ss;"),
    ("rda_mean_norm_unweighted", "mean_norm += w[m] * norm[m];", "mean_norm += norm[m] / M;"),
    ("rda_direction_not_normalised", "u += w[m] * (d / norm[m]);", "u += w[m] * d;"),
    ("rda_direction_unweighted", "u += w[m] * (d / norm[m]);", "u += (d / norm[m]);"),
    ("rda_mean_direction_not_projected", "mean_norm * (v_out[i] / dir_norm)", "mean_norm * v_out[i]"),
    ("rda_sign", "double d = (double)theta[i] - learner_value(learner_params[m], learner_dtype, i);\n                u +=",
     "double d = learner_value(learner_params[m], learner_dtype, i) - (double)theta[i];\n                u +="),
    ("rda_groups_merged", "size_t hi = n - lo < group_len ? n : lo + group_len;", "size_t hi = n; group_len = n;"),
    ("rda_momentum_dropped",
     "double v_new = (double)mu * (double)v[i] + Delta;\n            theta_out[i] = Theta -",
     "double v_new = Delta;\n            theta_out[i] = Theta -"),
    ("q4_momentum_dropped",
     "double v_new = (double)mu * (double)v[i] + Delta;\n        theta_out[i] = (double)theta[i] -",
     "double v_new = Delta;\n        theta_out[i] = (double)theta[i] -"),
    ("q4_nibble_order", "(i & 1) ? (codes[i >> 1] >> 4) : (codes[i >> 1] & 0x0fu)",
     "(i & 1) ? (codes[i >> 1] & 0x0fu) : (codes[i >> 1] >> 4)"),
    ("q4_no_sign_extension", "return nib >= 8 ? (int)nib - 16 : (int)nib;", "return (int)nib;"),
    ("q4_scale_index", "(double)scales[m][i / block_len]", "(double)scales[m][i / block_len ? 0 : 0]"),
    ("q4_scale_dropped", "double d = (double)scales[m][i / block_len] * (double)q4_code(codes[m], i);",
     "double d = (double)q4_code(codes[m], i);"),
    ("q4_unweighted", "Delta += w[m] * d;", "Delta += d;"),
    ("q4_encode_truncates", "float r = nearbyintf(d / s);", "float r = truncf(d / s);"),
    ("q4_encode_scale_over_8", "float s = a / 7.0f;", "float s = a / 8.0f;"),
    ("q4_encode_sign", "float d = theta[i] - (float)learner_value(learner, learner_dtype, i);\n            float r =",
     "float d = (float)learner_value(learner, learner_dtype, i) - theta[i];\n            float r ="),
    ("q4_encode_pack_order", "(i & 1) ? nib << 4 : nib", "(i & 1) ? nib : nib << 4"),
    ("q4_rda_norm_not_sqrt", "len[m] = sqrt(acc);", "len[m] = acc;"),
    ("q4_rda_mean_norm_unweighted", "R += w[m] * len[m];", "R += len[m] / M;"),
    ("q4_rda_direction_not_normalised",
     "u += w[m] * (q4_value(codes[m], scales[m], i, block_len) / len[m]);",
     "u += w[m] * q4_value(codes[m], scales[m], i, block_len);"),
    ("q4_rda_direction_unweighted",
     "u += w[m] * (q4_value(codes[m], scales[m], i, block_len) / len[m]);",
     "u += (q4_value(codes[m], scales[m], i, block_len) / len[m]);"),
    ("q4_rda_not_projected", "R * (v_out[i] / U)", "R * v_out[i]"),
    ("q4_rda_groups_merged", "size_t g1 = n - g0 < group_len ? n : g0 + group_len;",
     "size_t g1 = n; group_len = n;"),
    ("q4_rda_scale_index", "(double)sc[i / block_len]", "(double)sc[0]"),
    ("q4_rda_momentum_dropped", "double vn = (double)mu * (double)v[i] + Delta;",
     "double vn = Delta;"),
    ("q4_rda_zero_learner_divides",
     "if (w[m] == 0.0 || len[m] == 0.0)\n                    continue;\n                u += w[m] * (q4_value",
     "if (w[m] == 0.0)\n                    continue;\n                u += w[m] * (q4_value"),
    ("chunk_overlap", "size_t lo = per * (size_t)t;", "size_t lo = per * (size_t)t + (t ? 1 : 0);"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new):
    assert SRC.count(old) == 1, f"mutation site for {name} not found exactly once"
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "mutant.c")
        out = os.path.join(d, "mutant.so")
        open(src, "w").write(SRC.replace(old, new))
        oracle.build(force=True, src=src, out=out, extra=["-w"])
        api = oracle_pins.OracleApi(oracle.load(out))
        caught = []
        for pin in oracle_pins.ALL_PINS:
            try:
                pin(api)
            except (AssertionError, oracle.OracleError):
                caught.append(pin.__name__)
        assert caught, f"no pin notices mutant {name}"
