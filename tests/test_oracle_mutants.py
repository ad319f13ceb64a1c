"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the
oracle's source (a dropped term, a wrong sign or index, a swapped operand, a
wrong order of operations), compiles it on the CPU, and requires that at least
one pin of tests/test_oracle_pins.py fails against it.  The unmodified source
must pass the same pins (checked first)."""
import inspect
import os

import pytest

import test_oracle_pins as pins
from oracle import co2_oracle

SRC = os.path.join(os.path.dirname(co2_oracle.__file__), "co2_oracle.cpp")

# (name, text to find in co2_oracle.cpp, replacement); every `find` occurs at least once
# and all its occurrences are replaced.
MUTANTS = [
    ("momentum_sign", "const float mt = bm + pen;", "const float mt = bm - pen;"),
    ("momentum_drops_beta", "const float bm = beta * m[j];", "const float bm = m[j];"),
    ("penalty_multiplies_instead_of_divides", "const float inv = static_cast<float>(1.0 / Lam);",
     "const float inv = static_cast<float>(Lam);"),
    ("penalty_ignored", "const float pen = dbar * inv;", "const float pen = dbar;"),
    ("lambda_misses_plus_one", "std::sqrt(M2) / T + 1.0;\n    }\n    const float inv",
     "std::sqrt(M2) / T;\n    }\n    const float inv"),
    ("lambda_ratio_inverted", "static_cast<double>(alpha)) * std::sqrt(M2) / T + 1.0;",
     "static_cast<double>(alpha)) * T / std::sqrt(M2) + 1.0;"),
    ("lambda_drops_alpha", "Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * std::sqrt(M2)",
     "Lam = (static_cast<double>(c)) * std::sqrt(M2)"),
    ("lambda_uses_squared_norm", "static_cast<double>(alpha)) * std::sqrt(M2) / T + 1.0;",
     "static_cast<double>(alpha)) * M2 / T + 1.0;"),
    ("numerator_not_clipped", "double cm = static_cast<double>(clip_coord<float>(m[j], phi));\n      M2 += cm * cm;",
     "double cm = static_cast<double>(m[j]);\n      M2 += cm * cm;"),
    ("denominator_drops_tau", "T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);",
     "T = static_cast<double>(first_step_norm[s]);"),
    ("denominator_from_wrong_worker", "double dv = static_cast<double>(d[0][j]);",
     "double dv = static_cast<double>(d[K - 1][j]);"),
    ("mean_skips_last_worker", "for (int32_t k = 1; k < K; ++k) sum = sum + d[k][j];",
     "for (int32_t k = 1; k < K - 1; ++k) sum = sum + d[k][j];"),
    ("mean_not_divided", "const float dbar = sum * rK;", "const float dbar = sum;"),
    ("iterate_sign", "const float xn = aj - stepv;", "const float xn = aj + stepv;"),
    ("iterate_drops_alpha", "const float stepv = alpha * cm;", "const float stepv = cm;"),
    ("iterate_not_clipped", "const float cm = clip_coord<float>(mt, phi);", "const float cm = mt;"),
    ("iterate_from_params_not_anchor", "const float xn = aj - stepv;", "const float xn = (x ? x[j] : aj) - stepv;"),
    ("clip_lower_bound_wrong", "return (lo > -phi) ? lo : -phi;", "return (lo > -phi) ? lo : phi;"),
    ("clip_upper_bound_missing", "T lo = (chi < phi) ? chi : phi;", "T lo = chi;"),
    ("pseudo_gradient_sign", "if (x) dout[j] = aj - x[j];\n      // Mean", "if (x) dout[j] = x[j] - aj;\n      // Mean"),
    ("anchor_not_written", "      a_out[j] = xn;\n    }\n  }\n  return 0;\n}\n\n// The same update with every quantity in fp64.",
     "    }\n  }\n  return 0;\n}\n\n// The same update with every quantity in fp64."),
    ("momentum_not_stored", "      m[j] = mt;\n      if (x) x[j] = xn;\n      a_out[j] = xn;\n    }\n  }\n  return 0;\n}\n\n// The same update with every quantity in fp64.",
     "      if (x) x[j] = xn;\n      a_out[j] = xn;\n    }\n  }\n  return 0;\n}\n\n// The same update with every quantity in fp64."),
    ("first_round_updates_momentum", "      a_out[j] = aj;\n    }\n    for (int32_t s = 0; s < S; ++s) {\n      if (lambda_out) lambda_out[s] = 1.0f;",
     "      a_out[j] = aj; m[j] = beta * m[j] + 1.0f;\n    }\n    for (int32_t s = 0; s < S; ++s) {\n      if (lambda_out) lambda_out[s] = 1.0f;"),
    ("segment_off_by_one", "for (int64_t j = lo; j < hi; ++j) {\n      double cm = static_cast<double>(clip_coord<float>(m[j], phi));",
     "for (int64_t j = lo + 1; j < hi; ++j) {\n      double cm = static_cast<double>(clip_coord<float>(m[j], phi));"),
    ("f64_momentum_sign", "const double mt = beta * m[j] + dbar / Lam;", "const double mt = beta * m[j] - dbar / Lam;"),
    ("f64_lambda_misses_plus_one", "if (c != 0.0 && T != 0.0) Lam = c * alpha * std::sqrt(M2) / T + 1.0;",
     "if (c != 0.0 && T != 0.0) Lam = c * alpha * std::sqrt(M2) / T;"),
    ("f64_mean_divides_by_wrong_count", "const double dbar = sum / static_cast<double>(K);",
     "const double dbar = sum / static_cast<double>(K + 1);"),
    ("sqnorms_no_square", "double dv = static_cast<double>(v);\n      acc += dv * dv;", "double dv = static_cast<double>(v);\n      acc += dv;"),
    ("bf16_truncates_instead_of_rounding", "u += 0x7fffu + lsb;", "u += 0u;"),
    ("bf16_ties_round_away", "u += 0x7fffu + lsb;", "u += 0x8000u;"),
    ("bf16_widening_shift_wrong", "cv.u = static_cast<uint32_t>(b) << 16;", "cv.u = static_cast<uint32_t>(b) << 15;"),
    ("bf16_step_skips_rounding_of_dout", "if (x) dout[j] = co2_oracle_f32_to_bf16(aj - x[j]);\n      float sum",
     "if (x) dout[j] = static_cast<uint16_t>(0);\n      float sum"),
    ("f16_truncates_instead_of_rounding", "r += 0x0fffu + lsb;", "r += 0u;"),
    ("f16_ties_round_away", "r += 0x0fffu + lsb;", "r += 0x1000u;"),
    ("f16_exponent_rebias_wrong", "uint32_t r = mag - 0x38000000u;", "uint32_t r = mag - 0x38800000u;"),
    ("f16_no_overflow_to_infinity", "if (mag >= 0x47800000u) return static_cast<uint16_t>(sign | 0x7c00u);",
     "if (mag >= 0x47800000u) return static_cast<uint16_t>(sign | 0x7bffu);"),
    ("f16_subnormals_flushed", "if (mag <= 0x33000000u) return sign;", "if (mag < 0x38800000u) return sign;"),
    ("f16_subnormal_tie_rounds_up", "if (rem > half || (rem == half && (h & 1u))) ++h;", "if (rem >= half) ++h;"),
    ("f16_widening_subnormal_scale", "* 5.9604644775390625e-08f;", "* 1.1920928955078125e-07f;"),
    ("f16_widening_exponent", "cv.u = sign | ((e + 112u) << 23) | (frac << 13);", "cv.u = sign | ((e + 127u) << 23) | (frac << 13);"),
    ("f16_step_reads_bf16_layout", "float sum = co2_oracle_f16_to_f32(d[0][j]);", "float sum = co2_oracle_bf16_to_f32(d[0][j]);"),
    ("f16_step_skips_rounding_of_dout", "if (x) dout[j] = co2_oracle_f32_to_f16(aj - x[j]);\n      float sum",
     "if (x) dout[j] = static_cast<uint16_t>(0);\n      float sum"),
    ("adamw_second_moment_not_squared", "const float v = beta2 * exp_avg_sq[j] + (omb2 * g) * g;",
     "const float v = beta2 * exp_avg_sq[j] + (omb2 * g);"),
    ("adamw_no_bias_correction_1", "const float step_size = static_cast<float>(static_cast<double>(lr) / bc1);",
     "const float step_size = lr;"),
    ("adamw_no_bias_correction_2", "const float denom = std::sqrt(v) / sqrt_bc2 + eps;", "const float denom = std::sqrt(v) + eps;"),
    ("adamw_coupled_decay_missing", "const float pd = p0 * decay;", "const float pd = p0;"),
    ("adamw_update_sign", "const float p1 = pd - upd;", "const float p1 = pd + upd;"),
    ("adamw_eps_inside_root", "const float denom = std::sqrt(v) / sqrt_bc2 + eps;", "const float denom = std::sqrt(v + eps) / sqrt_bc2;"),
    ("adamw_bf16_shift_wrong", "static_cast<uint32_t>(grad_bf16[j]) << 16;", "static_cast<uint32_t>(grad_bf16[j]) << 15;"),
    ("adamw_dout_sign", "if (dout) dout[j] = anchor[j] - p1;", "if (dout) dout[j] = p1 - anchor[j];"),
    ("adamw_step_norm_from_new_value", "const double df = static_cast<double>(p1 - p0);", "const double df = static_cast<double>(p1);"),
    # ---- the variant switches (current-round mean, anchor pull, norm rescale)
    ("variant_own_delta_left_out_of_current_mean", "float sum = nonstale ? dout[j] : d[0][j];",
     "float sum = nonstale ? 0.0f : d[0][j];"),
    ("variant_current_mean_reads_stale_own_delta", "float sum = nonstale ? dout[j] : d[0][j];",
     "float sum = d[0][j];"),
    ("variant_round_zero_skipped_in_current_order", "if (step == 0 && !nonstale) {", "if (step == 0) {"),
    ("variant_numerator_not_capped_by_threshold",
     "if (norm_clip && moved > static_cast<double>(phi)) moved = static_cast<double>(phi);", ""),
    # (clamping the coordinates before that norm would be no mistake: min(||Clip(m)||, phi) == min(||m||, phi))
    ("variant_scale_inverted", "scale = static_cast<float>(static_cast<double>(phi) / nrm);",
     "scale = static_cast<float>(nrm / static_cast<double>(phi));"),
    ("variant_scale_not_applied", "const float cm = norm_clip ? mt * scale : clip_coord<float>(mt, phi);",
     "const float cm = norm_clip ? mt : clip_coord<float>(mt, phi);"),
    ("variant_norm_of_new_momentum_not_squared", "Q += static_cast<double>(mt) * static_cast<double>(mt);",
     "Q += static_cast<double>(mt);"),
    ("variant_norm_taken_of_old_momentum", "Q += static_cast<double>(mt) * static_cast<double>(mt);",
     "Q += static_cast<double>(bm) * static_cast<double>(bm);"),
    ("variant_rescale_also_clamps", "const float cm = norm_clip ? mt * scale : clip_coord<float>(mt, phi);",
     "const float cm = norm_clip ? clip_coord<float>(mt * scale, phi * 0.5f) : clip_coord<float>(mt, phi);"),
    ("variant_pull_sign", "const float gap = x[j] - xn;", "const float gap = xn - x[j];"),
    ("variant_pull_from_anchor", "x[j] = x[j] - pull;", "x[j] = xn - pull;"),
    ("variant_pull_ignores_rho", "const float pull = pull_rho * gap;", "const float pull = gap;"),
    ("variant_pull_moves_anchor_too", "          x[j] = x[j] - pull;\n        }\n      }\n      a_out[j] = xn;",
     "          x[j] = x[j] - pull;\n        }\n      }\n      a_out[j] = x ? x[j] : xn;"),
    ("adamw_f64_first_moment", "const double m1 = beta1 * exp_avg[j] + (1.0 - beta1) * g;", "const double m1 = beta1 * exp_avg[j] + g;"),
]


def _pin_functions():
    out = []
    for name, fn in sorted(vars(pins).items()):
        if name.startswith("test_") and inspect.isfunction(fn):
            out.append((name, fn))
    return out


def _expand(fn):
    """All concrete calls of one pin (its parametrize marks expanded by hand)."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    calls = [dict()]
    for mk in marks:
        argname, values = mk.args[0], mk.args[1]
        calls = [dict(c, **{argname: v}) for c in calls for v in values]
    return calls


def run_all_pins():
    """Run every pin against whatever library co2_oracle currently points to;
    returns the names of the pins that failed."""
    failed = []
    for name, fn in _pin_functions():
        for kw in _expand(fn):
            try:
                fn(oracle=co2_oracle, **kw)
            except AssertionError:
                failed.append(name)
                break
            except Exception as e:      # a crash of a pin is also a detection, but say which
                failed.append(f"{name} ({type(e).__name__})")
                break
    return failed


def test_unmodified_oracle_passes_every_pin():
    co2_oracle.build()
    assert run_all_pins() == []


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, find, repl):
    src = open(SRC).read()
    assert find in src, f"mutant {name}: pattern no longer in the oracle source"
    mutated = tmp_path / f"oracle_{name}.cpp"
    mutated.write_text(src.replace(find, repl))
    lib = co2_oracle.compile_source(str(mutated), str(tmp_path / f"liboracle_{name}.so"))
    with co2_oracle.use_library(lib):
        failed = run_all_pins()
    assert failed, f"no pin notices the planted mistake '{name}'"
