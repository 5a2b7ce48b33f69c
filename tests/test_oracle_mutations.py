"""Mutation check of the oracle's pins: one mistake at a time is planted in a COPY of oracle/deeppoly_oracle.c, the
copy is compiled, and the pin named beside the mistake is run against it in a process of its own (the environment
variable DEEPPOLY_ORACLE_SRC makes the oracle's wrapper load the copy).  Every planted mistake must make its pin
fail; the untouched copy must pass all of them.  CPU only; nothing here touches the GPU library.

Each entry: (name, text to find in the C file, replacement, pytest node that has to fail)."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "deeppoly_oracle.c")

PINS = "tests/test_oracle_pins.py::"
DEPTH = "tests/test_oracle_depth.py::"
EARLY = "tests/test_oracle_early_term.py::"
FLOAT = "tests/test_oracle_float_inference.py::"
POOL = "tests/test_oracle_avgpool.py::"

MUTATIONS = [
    # ---- the transformers and the back-substitution (Section 2) -----------------------------------------------
    ("relu_wrong_line_for_the_sign",
     "if (a >= 0.0) use_upper_line = (sense > 0);", "if (a >= 0.0) use_upper_line = (sense < 0);",
     PINS + "test_hand_computed_unstable_relu_example"),
    ("relu_intercept_dropped",
     "acc_scaled(&e->clo, &e->chi, a, b, d);", "(void)d;",
     PINS + "test_hand_computed_unstable_relu_example"),
    ("relu_lower_line_choice_flipped",
     "else lam = (u > -l) ? 1 : 0;", "else lam = (u > -l) ? 0 : 1;",
     PINS + "test_hand_computed_unstable_relu_example"),
    ("relu_slope_from_the_wrong_end",
     "double g = u / sub_up(u, l);", "double g = -l / sub_up(u, l);",
     PINS + "test_second_implementation_agrees"),
    ("dead_relu_passes_its_coefficient",
     "} else if (u <= 0.0) {                /* y = 0 exactly */",
     "} else if (u <= 0.0) { dlo[j] = add_dn(dlo[j], a); dhi[j] = add_up(dhi[j], b);",
     PINS + "test_all_dead_network"),
    ("dense_bias_dropped",
     "acc_scaled(&e->clo, &e->chi, a, b, d->bias[i]);", ";",
     PINS + "test_eps_zero_collapses_to_forward_pass"),
    ("dense_weight_transposed",
     "const double *w = d->wt + (size_t)i * n_in;\n        for (int j = 0; j < n_in; ++j) acc_scaled(&dlo[j], &dhi[j], a, b, w[j]);",
     "for (int j = 0; j < n_in; ++j) acc_scaled(&dlo[j], &dhi[j], a, b, d->wt[((size_t)j * d->n + i) % ((size_t)d->n * n_in)]);",
     PINS + "test_eps_zero_collapses_to_forward_pass"),
    ("conv_taps_swapped",
     "double w = c->wt[(((size_t)d * p->C + ci) * c->kh + f) * c->kw + g];\n                            int j = (ci * p->H + iy) * p->W + ix;\n                            acc_scaled(",
     "double w = c->wt[(((size_t)d * p->C + ci) * c->kh + g) * c->kw + f];\n                            int j = (ci * p->H + iy) * p->W + ix;\n                            acc_scaled(",
     PINS + "test_conv_equals_its_toeplitz_dense_layer"),
    ("conv_padding_ignored",
     "int iy = y * c->sh - c->ph + f;\n                        if (iy < 0 || iy >= p->H) continue;\n                        for (int g = 0; g < c->kw; ++g) {\n                            int ix = x * c->sw - c->pw + g;\n                            if (ix < 0 || ix >= p->W) continue;\n                            double w",
     "int iy = y * c->sh + f;\n                        if (iy < 0 || iy >= p->H) continue;\n                        for (int g = 0; g < c->kw; ++g) {\n                            int ix = x * c->sw + g;\n                            if (ix < 0 || ix >= p->W) continue;\n                            double w",
     PINS + "test_conv_equals_its_toeplitz_dense_layer"),
    ("conv_stride_ignored",
     "int iy = y * c->sh - c->ph + f;\n                        if (iy < 0 || iy >= p->H) continue;\n                        for (int g = 0; g < c->kw; ++g) {\n                            int ix = x * c->sw - c->pw + g;\n                            if (ix < 0 || ix >= p->W) continue;\n                            double w",
     "int iy = y - c->ph + f;\n                        if (iy < 0 || iy >= p->H) continue;\n                        for (int g = 0; g < c->kw; ++g) {\n                            int ix = x - c->pw + g;\n                            if (ix < 0 || ix >= p->W) continue;\n                            double w",
     PINS + "test_conv_equals_its_toeplitz_dense_layer"),
    ("residual_branch_dropped",
     "e->lo[s->b][j] = add_dn(e->lo[s->b][j], a); e->hi[s->b][j] = add_up(e->hi[s->b][j], b);", ";",
     PINS + "test_residual_block_equals_dense_net_carrying_the_skip"),
    ("candidate_uses_the_wrong_interval_end",
     "double m = dmax(dmax(mul_up(a, L), mul_up(a, U)), dmax(mul_up(b, L), mul_up(b, U)));\n            acc = add_up(acc, m);",
     "double m = dmin(dmin(mul_up(a, L), mul_up(a, U)), dmin(mul_up(b, L), mul_up(b, U)));\n            acc = add_up(acc, m);",
     PINS + "test_first_affine_layer_closed_form"),
    ("best_candidate_is_the_worst",
     "best = (sense > 0) ? dmin(best, v) : dmax(best, v);\n        }\n        if (k == 0) return best;",
     "best = (sense > 0) ? dmax(best == INFINITY ? v : best, v) : dmin(best == -INFINITY ? v : best, v);\n        }\n        if (k == 0) return best;",
     PINS + "test_all_candidates_never_looser_than_input_only"),
    # ---- floating point (Section 4.1) ------------------------------------------------------------------------------
    ("interval_times_negative_scalar_ends_swapped",
     "else          { *lo = add_dn(*lo, mul_dn(ahi, w)); *hi = add_up(*hi, mul_up(alo, w)); }",
     "else          { *lo = add_dn(*lo, mul_dn(alo, w)); *hi = add_up(*hi, mul_up(ahi, w)); }",
     DEPTH + "test_scalar_chain_isolates_the_rounding_of_one_product"),
    ("interval_times_negative_scalar_rounded_inward",
     "else          { *lo = add_dn(*lo, mul_dn(ahi, w)); *hi = add_up(*hi, mul_up(alo, w)); }",
     "else          { *lo = add_dn(*lo, mul_up(ahi, w)); *hi = add_up(*hi, mul_dn(alo, w)); }",
     DEPTH + "test_scalar_chain_isolates_the_rounding_of_one_product"),
    ("interval_times_positive_scalar_rounded_inward",
     "if (w >= 0.0) { *lo = add_dn(*lo, mul_dn(alo, w)); *hi = add_up(*hi, mul_up(ahi, w)); }",
     "if (w >= 0.0) { *lo = add_dn(*lo, mul_up(alo, w)); *hi = add_up(*hi, mul_dn(ahi, w)); }",
     DEPTH + "test_interval_coefficient_times_scalar_of_either_sign_is_rounded_outward"),
    ("recentring_forgets_the_width",
     "if (sense > 0) e->chi = add_up(e->chi, slack);\n        else e->clo = add_dn(e->clo, -slack);", "(void)slack;",
     DEPTH + "test_scalar_chain_isolates_the_rounding_of_one_product"),
    ("recentring_pays_the_width_on_the_wrong_side",
     "if (sense > 0) e->chi = add_up(e->chi, slack);\n        else e->clo = add_dn(e->clo, -slack);",
     "if (sense > 0) e->chi = add_up(e->chi, -slack);\n        else e->clo = add_dn(e->clo, slack);",
     DEPTH + "test_scalar_chain_isolates_the_rounding_of_one_product"),
    ("recentring_scales_the_width_wrongly",
     "double slack = mul_up(w, X);", "double slack = mul_up(w, X) * 1e9;",
     DEPTH + "test_deep_networks_recentred_oracle_is_deeppoly_and_the_literal_scheme_is_the_outlier[deep_fc]"),
    # ---- early termination (Sections 3.2, 4.2) --------------------------------------------------------------------
    ("termination_criterion_too_eager",
     "(may_stop && (*lo >= 0.0 || *hi <= 0.0))", "(may_stop && (*lo >= -0.05 || *hi <= 0.05))",
     EARLY + "test_second_implementation_agrees"),
    ("interval_image_ignores_the_sign_of_the_weight",
     "else             { lo = add_dn(lo, mul_dn(w[j], pu[j])); hi = add_up(hi, mul_up(w[j], pl[j])); }",
     "else             { lo = add_dn(lo, mul_dn(w[j], pl[j])); hi = add_up(hi, mul_up(w[j], pu[j])); }",
     EARLY + "test_interval_image_is_the_closed_form"),
    # ---- rounding of the inference (Section 4.1, last paragraph) --------------------------------------------------
    ("inference_error_not_charged_at_a_dense_layer",
     "if (d->has_eta) acc_error(e, a, b, d->eta[i]);", ";",
     FLOAT + "test_float32_evaluations_in_any_order_are_contained"),
    ("inference_error_not_charged_at_a_convolution",
     "if (c->has_eta) acc_error(e, a, b, c->eta[i]);\n                slo[i] = shi[i] = 0.0;\n            }\n    e->active[k] = 0;\n    e->active[c->a] = 1;\n}\n\n/* coefficient interval [alo,ahi] times the pooling weight",
     ";\n                slo[i] = shi[i] = 0.0;\n            }\n    e->active[k] = 0;\n    e->active[c->a] = 1;\n}\n\n/* coefficient interval [alo,ahi] times the pooling weight",
     FLOAT + "test_float32_evaluations_in_any_order_are_contained"),
    ("rounded_sum_not_widened",
     "*lo = add_dn(*lo, -mul_up(fabs(*lo), kU32));\n    *hi = add_up(*hi, mul_up(fabs(*hi), kU32));", ";",
     FLOAT + "test_rounded_sum_hand_example"),
    ("inference_error_leaves_the_bias_out",
     "double s = fabs(l->bias[i]);\n            for (int j = 0; j < p->n; ++j) s = add_up(s, mul_up(fabs(w[j]), dmax(fabs(pl[j]), fabs(pu[j]))));",
     "double s = 0.0;\n            for (int j = 0; j < p->n; ++j) s = add_up(s, mul_up(fabs(w[j]), dmax(fabs(pl[j]), fabs(pu[j]))));",
     FLOAT + "test_bias_term_of_the_error_constant"),
    # ---- average pooling ---------------------------------------------------------------------------------------------------
    ("pool_weight_end_for_the_wrong_sign",
     "*lo = add_dn(*lo, alo >= 0.0 ? mul_dn(alo, w_dn) : mul_dn(alo, w_up));",
     "*lo = add_dn(*lo, alo >= 0.0 ? mul_dn(alo, w_up) : mul_dn(alo, w_dn));",
     POOL + "test_one_ninth_is_enclosed_in_exact_rationals"),
    ("pool_strides_swapped",
     "int iy = y * c->sh - c->ph + f;\n                    if (iy < 0 || iy >= p->H) continue;\n                    for (int g = 0; g < c->kw; ++g) {\n                        int ix = x * c->sw - c->pw + g;",
     "int iy = y * c->sw - c->ph + f;\n                    if (iy < 0 || iy >= p->H) continue;\n                    for (int g = 0; g < c->kw; ++g) {\n                        int ix = x * c->sh - c->pw + g;",
     POOL + "test_rectangular_window_stride_and_padding"),
]


def _run_pin(src, node):
    env = dict(os.environ, DEEPPOLY_ORACLE_SRC=src, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", node], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:] + r.stderr[-500:]


def _plant(tmp, name, find, repl):
    text = open(SRC).read()
    assert text.count(find) == 1, f"{name}: the text to replace must occur exactly once in the oracle (found {text.count(find)})"
    path = os.path.join(tmp, name + ".c")
    with open(path, "w") as f:
        f.write(text.replace(find, repl))
    return path


def test_every_planted_mistake_fails_its_pin(tmp_path):
    tmp = str(tmp_path)
    # (one untouched copy per pin: the jobs run side by side and each builds the library next to its source)
    jobs = []
    for k, node in enumerate(sorted({m[3] for m in MUTATIONS})):
        clean = os.path.join(tmp, f"clean_{k}.c")
        shutil.copy(SRC, clean)
        jobs.append(("clean", clean, node))
    jobs += [(name, _plant(tmp, name, find, repl), node) for name, find, repl, node in MUTATIONS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda j: _run_pin(j[1], j[2]), jobs))
    survivors = []
    for (name, _, node), (rc, out) in zip(jobs, results):
        if name == "clean":
            assert rc == 0, f"the untouched copy fails {node}:\n{out}"
        elif rc == 0:
            survivors.append(f"{name} survives {node}")
        else:
            assert rc == 1, f"{name}: {node} did not run to a verdict (exit {rc}):\n{out}"
    assert not survivors, survivors


@pytest.mark.parametrize("name", [m[0] for m in MUTATIONS])
def test_mutation_texts_are_present_once(name):
    """A mutation whose text has drifted away from the oracle's source would silently test nothing."""
    find = next(m[1] for m in MUTATIONS if m[0] == name)
    assert open(SRC).read().count(find) == 1
