"""The pins must bite: plant plausible mistakes in copies of the oracle's C source (on the CPU, in
a temporary directory) and check that every mutant is rejected by at least one of the pin tests.
The real oracle is never modified."""
import importlib.util
import os
import shutil
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")

# (name, text to find, replacement) -- each is one mistake a re-implementer could plausibly make
MUTANTS = [
    ("residual_sign", "err[a + j] = p[j] - q[j];", "err[a + j] = p[j] + q[j];"),
    ("error_buffer_accumulates", "err[a + j] = p[j] - q[j];", "err[a + j] = err[a + j] + (p[j] - q[j]);"),
    ("error_feedback_dropped", "p[j] = grad[a + j] + err[a + j];     /* g + e */", "p[j] = grad[a + j];"),
    ("tie_goes_down", "if (a >= mid[c]) { mu = c; break; }", "if (a > mid[c]) { mu = c; break; }"),
    ("geometric_midpoint", "mid[c] = 0.5f * (lv[c - 1] + lv[c]);", "mid[c] = 0.70710678f * lv[c];"),
    ("level_off_by_one", "return mu == 0 ? 0.0f : ldexpf(1.0f, mu - 1 - k_g);", "return mu == 0 ? 0.0f : ldexpf(1.0f, mu - 2 - k_g);"),
    ("scale_without_abs", "float a = fabsf(p[j]);\n        if (isnan(a)) saw_nan = 1;", "float a = p[j];\n        if (isnan(a)) saw_nan = 1;"),
    ("negative_zero_code", "int32_t neg = (p[j] < 0.0f) && (mu > 0);", "int32_t neg = (p[j] < 0.0f);"),
    ("beta_theta_swapped", "float vj = (beta2 * v[j]) + (omb2 * g2);", "float vj = (beta1 * v[j]) + (omb1 * g2);"),
    ("second_moment_not_squared", "(omb2 * g2);", "(omb2 * gj);"),
    ("eps_outside_root", "float den = sqrtf(vj + eps);               /* sqrt(v_t + eps) */", "float den = sqrtf(vj) + eps;"),
    ("mean_dropped", "acc[j] = acc[j] / (float)N;", "acc[j] = acc[j];"),
    ("ascent", "x[j] = x[j] - u[j];\n    oq_weight_quantize(cfg, P, index_base, step, x, werr, wcodes, NULL, tie_x);\n    free(acc); free(q); free(u);\n    return status;\n}\n\n/* The same step",
     "x[j] = x[j] + u[j];\n    oq_weight_quantize(cfg, P, index_base, step, x, werr, wcodes, NULL, tie_x);\n    free(acc); free(q); free(u);\n    return status;\n}\n\n/* The same step"),
    ("qx_spacing", "const float per_unit = ldexpf(1.0f, k_x + 1);", "const float per_unit = ldexpf(1.0f, k_x);"),
    ("qx_half_to_even", "jf = roundf(u);", "jf = rintf(u);"),
    ("qx_no_saturation", "if (jf > jmax) jf = jmax;", "if (jf > 4.0f * jmax) jf = jmax;"),
    ("weight_feedback_ignored", "y[j] = (cfg->weight_ef && werr) ? x[j] + werr[j] : x[j];", "y[j] = x[j];"),
    ("pack_bit_order", "wv |= (uint32_t)1 << b;", "wv |= (uint32_t)1 << (31 - b);"),
    ("pack_plane_order", "words[gidx * bits + k] = wv;", "words[gidx * bits + (bits - 1 - k)] = wv;"),
    ("philox_nine_rounds", "for (int round = 0; round < 10; ++round)", "for (int round = 0; round < 9; ++round)"),
    ("philox_constant", "0xCD9E8D57u", "0xCD9E8D56u"),
    ("uniform_low_bits", "(float)(out[j & 3] >> 8) * 0x1p-24f", "(float)(out[j & 3] & 0xffffffu) * 0x1p-24f"),
    ("stochastic_biased", "mu = below + (U < frac ? 1 : 0);", "mu = below + (0.5f < frac ? 1 : 0);"),
    ("variant_w_quantizes_gradient", "status |= worker_message(cfg, seg_off, L, index_base, i, step, u, errs[i],",
     "status |= worker_message(cfg, seg_off, L, index_base, i, step, grads[i], errs[i],"),
    ("variant_w_adds_update", "for (int64_t j = 0; j < P; ++j) x[j] = x[j] - acc[j];", "for (int64_t j = 0; j < P; ++j) x[j] = x[j] + acc[j];"),
    ("window_ignores_given_scale", "oq_qg_window(cfg, p, n, j0, step, worker, s, code, q, tie);\n    for (int64_t j = 0; j < n; ++j) err[j] = p[j] - q[j];",
     "oq_qg_layer(cfg, p, n, j0, step, worker, &s, code, q, tie);\n    for (int64_t j = 0; j < n; ++j) err[j] = p[j] - q[j];"),
    ("decode_ignores_sign", "return neg ? -q : q;\n}\n\n/* element-wise part", "return q;\n}\n\n/* element-wise part"),
    ("bias_correction_missing", "lr1 = lr / bc1;", "lr1 = lr;"),
]


def _load_mutant(tmp, name, find, repl):
    src = open(os.path.join(ORACLE_DIR, "qadam_oracle.c")).read()
    assert src.count(find) >= 1, "mutation site of %s not found in the oracle source" % name
    mdir = os.path.join(tmp, name)
    os.makedirs(mdir)
    open(os.path.join(mdir, "qadam_oracle.c"), "w").write(src.replace(find, repl, 1))
    shutil.copy(os.path.join(ORACLE_DIR, "qadam_oracle.h"), mdir)
    shutil.copy(os.path.join(ORACLE_DIR, "qadam_oracle.py"), mdir)
    spec = importlib.util.spec_from_file_location("qadam_oracle_mutant_" + name, os.path.join(mdir, "qadam_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules[spec.name] = mod          # dataclasses look the module up by name
    spec.loader.exec_module(mod)
    mod.build(force=True)                 # compiles the mutated copy next to the copied wrapper
    return mod


def _battery():
    import test_oracle_philox as tp
    import test_oracle_quantizers as tq
    import test_oracle_steps as ts
    calls = [
        (tq.test_qg_handworked, {}), (tq.test_qx_handworked, {}),
        (tq.test_qg_exact_residual_and_ranges, dict(k_g=2)), (tq.test_qg_exact_residual_and_ranges, dict(k_g=0)),
        (tq.test_pack_unpack_layout, {}), (tq.test_qx_saturation, {}),
        (tq.test_weight_error_feedback_modes, {}), (tq.test_assumption3_bounded_weight_error, dict(k_x=3)),
        (tq.test_qg_bruteforce_argmin, dict(k_g=2)), (tq.test_qx_bruteforce_argmin, dict(k_x=3)),
        (tq.test_assumption2_contraction, dict(k_g=2)), (tq.test_zero_and_nonfinite_layers, {}),
        (tq.test_tie_flags, {}), (tq.test_bit_budget_matches_tables, {}),
        (tp.test_philox_known_answers, {}), (tp.test_uniform_stream_keying, {}),
        (tp.test_stochastic_rounding_is_unbiased_and_adjacent, {}),
        (ts.test_constant_gradient_closed_form, {}), (ts.test_identity_quantizers_reduce_to_generic_adam, {}),
        (ts.test_bias_corrected_flavour_matches_library_adam, {}),
        (ts.test_error_feedback_telescoping_variant_s, dict(k_g=2)), (ts.test_variant_w_telescoping, {}),
        (ts.test_variant_s_server_mean_and_order, {}), (ts.test_fused_step_equals_three_calls, {}),
        (ts.test_window_equals_layer, {}), (ts.test_step_window_equals_step, {}),
        (ts.test_error_buffer_obeys_the_geometric_bound, dict(k_g=2)),
        (ts.test_whole_step_against_the_definitions_in_fp64, dict(variant="s")),
        (ts.test_whole_step_against_the_definitions_in_fp64, dict(variant="w")),
    ]
    return calls


def _first_failure(mod):
    for fn, kw in _battery():
        try:
            fn(mod, **kw)
        except AssertionError:
            return fn.__name__
        except Exception as exc:                     # a crash of the mutant also counts as caught
            return "%s (%s)" % (fn.__name__, type(exc).__name__)
    return None


def test_unmutated_oracle_passes_the_battery(oracle):
    assert _first_failure(oracle) is None


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, find, repl):
    mod = _load_mutant(str(tmp_path), name, find, repl)
    caught = _first_failure(mod)
    assert caught is not None, "mutant %r survived every pin" % name
