"""Are the oracle's pins sharp?  Each case plants one plausible mistake in a private copy of the oracle's C
source (a flipped sign, a dropped term, a transposed operand, an off-by-one), builds it, and runs the pins of
tests/test_oracle_pins.py against it: at least one of the pins named for that mistake must fail.

Everything here runs on the CPU, in a temporary directory; the real oracle is never touched.
"""
import importlib.util
import os
import shutil

import pytest

from tests import test_oracle_pins as pins

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

# (name, text in cp_oracle.c, replacement, occurrence index or None for the only one, pins expected to notice)
MUTANTS = [
    ("eq8_sign", "double C = (x >= 0) ? z[x] - lse : 0.0;       /* eq. 8 */",
     "double C = (x >= 0) ? lse - z[x] : 0.0;", 0,
     ["test_rank_one_is_independent_cross_entropies", "test_joint_sums_to_one_brute_force"]),
    ("gate_term_dropped", "for (int al = 0; al < r; ++al) a[al] = logw[al];",
     "for (int al = 0; al < r; ++al) a[al] = 0.0 * logw[al];", 0,
     ["test_joint_sums_to_one_brute_force", "test_logspace_equals_probability_space"]),
    ("transposed_head_matrix", "acc += (double)Wsa[(size_t)k * sh->d + j] * (double)h[j];",
     "acc += (double)Wsa[(size_t)j * sh->d + k] * (double)h[j];", None,
     ["test_matches_library_composition", "test_rank_one_is_independent_cross_entropies"]),
    ("logsumexp_off_by_one", "for (int64_t i = 0; i < len; ++i) s += exp(x[i] - mx);",
     "for (int64_t i = 1; i < len; ++i) s += exp(x[i] - mx);", None,
     ["test_joint_sums_to_one_brute_force", "test_gate_weights_normalised"]),
    ("gate_gradient_sign", "dg_all[(size_t)t * r + al] = up * (exp(logw[al]) - gamma);",
     "dg_all[(size_t)t * r + al] = up * (gamma - exp(logw[al]));", 0,
     [("test_gradients_match_central_differences", "G"), ("test_gradients_match_central_differences", "H")]),
    ("onehot_term_dropped", "dz[x] -= up * gamma;", "dz[x] -= 0.0 * up * gamma;", 0,
     ["test_backward_zero_sum_invariants", ("test_gradients_match_central_differences", "U")]),
    ("dh_without_gate_path", "acc += (double)G[(size_t)al * d + j] * dg_all[(size_t)t * r + al];",
     "acc += 0.0 * (double)G[(size_t)al * d + j] * dg_all[(size_t)t * r + al];", 0,
     [("test_gradients_match_central_differences", "H")]),
    ("inverse_cdf_clamp", "return pick < 0 ? len - 1 : pick;", "return pick < 0 ? 0 : pick;", None,
     ["test_draft_boundary_cases"]),
    ("conditional_without_normaliser", "q[al] += z[prefix[k]] - logsumexp(z, V);", "q[al] += z[prefix[k]];", None,
     ["test_chain_of_conditionals_is_the_joint"]),
    ("first_token_without_gate", "t[al] = logw[al] + z[(size_t)al * V + v];", "t[al] = z[(size_t)al * V + v];", None,
     ["test_first_token_logprob"]),
    ("balance_argmin", "if (logw[a] > logw[best]) best = a;", "if (logw[a] < logw[best]) best = a;", None,
     ["test_aux_balance"]),
    ("kl_direction", "kl += exp(lpc[v]) * (lpc[v] - log(m));", "kl += exp(lpc[v]) * (log(m) - lpc[v]);", None,
     ["test_distill_terms_against_library_routines"]),
    ("distill_chain_term_dropped", "dz[x] += D;", "dz[x] += 0.0 * D;", None,
     [("test_distill_gradients_match_central_differences", "U"), ("test_distill_gradients_match_central_differences", "W")]),
    ("full_head_gradient_transposed", "for (int j = 0; j < d; ++j) out[j] += dzv * (double)h[j];",
     "for (int j = 0; j < d; ++j) out[d - 1 - j] += dzv * (double)h[j];", None,
     [("test_full_heads_gradients_match_central_differences", "F"),
      "test_full_heads_reduce_to_the_shared_unembedding_head"]),
    ("bf16_rounding_width", "double q = nearbyint(ldexp(m, 8));", "double q = nearbyint(ldexp(m, 7));", None,
     ["test_bf16_rounding_helper"]),
    ("draft_logq_without_gate", "for (int al = 0; al < r; ++al) a[al] = logw[al];",
     "for (int al = 0; al < r; ++al) a[al] = 0.0 * logw[al];", 2,
     ["test_draft_frequencies_follow_the_joint"]),
    ("sequential_weights_not_updated", "for (int al = 0; al < r; ++al) q[al] += lp[(size_t)al * V + tok];",
     "for (int al = 0; al < r; ++al) q[al] += 0.0 * lp[(size_t)al * V + tok];", None,
     ["test_sequential_scheme_uses_the_pinned_conditionals", "test_sequential_scheme_samples_the_joint"]),
    ("balance_target_share", "- 1.0 / r;", "- 1.0 / (r + 1);", None, ["test_aux_balance"]),
    ("weight_gradient_transposed", "for (int j = 0; j < d; ++j) out[j] += dyk * (double)h[j];",
     "for (int j = 0; j < d; ++j) out[j] += dyk * (double)h[d - 1 - j];", 0,
     [("test_gradients_match_central_differences", "W")]),
    ("unembedding_gradient_without_y", "for (int k = 0; k < d; ++k) out[k] += dzv * y[k];",
     "for (int k = 0; k < d; ++k) out[k] += dzv;", None,
     [("test_gradients_match_central_differences", "U")]),
    ("distill_discount_squared", "for (int k = 0; k < n; ++k, weight *= disc) {",
     "for (int k = 0; k < n; ++k, weight *= disc * disc) {", 0,
     ["test_distill_terms_against_library_routines"]),
    ("distill_terms_swapped", "total += weight * (beta * kl + (1.0 - beta) * ce);",
     "total += weight * ((1.0 - beta) * kl + beta * ce);", None,
     ["test_distill_terms_against_library_routines"]),
    ("distill_prefix_not_applied", "for (int al = 0; al < r; ++al) q[al] += lp[(size_t)al * V + x];",
     "for (int al = 0; al < r; ++al) q[al] += 0.0 * lp[(size_t)al * V + x];", None,
     ["test_distill_without_teacher_term_is_the_joint_likelihood", "test_distill_terms_against_library_routines"]),
    ("distill_backward_discount", "for (int k = 0; k < n; ++k, weight *= disc) {",
     "for (int k = 0; k < n; ++k, weight *= 1.0) {", 1,
     [("test_distill_gradients_match_central_differences", "H"), ("test_distill_gradients_match_central_differences", "W")]),
    # the rounded-y mode and its hooks for rounding ties (several sites at once: old is a list of edits, new is None)
    ("rounding_applied_to_z_not_y",
     [("y[k] = sh->round_y ? round_to_bf16(acc) : acc;", "y[k] = acc;", None),
      ("        z[v] = acc;\n", "        z[v] = sh->round_y ? round_to_bf16(acc) : acc;\n", 0)], None, None,
     ["test_rounded_y_draft_is_the_composition_with_y_rounded", "test_rounding_is_the_identity_on_representable_y",
      "test_rounded_y_first_token_and_sequential_are_the_composition"]),
    ("nudge_added_after_rounding",
     [("        if (nudge) acc += nudge[k];\n", "", None),
      ("y[k] = sh->round_y ? round_to_bf16(acc) : acc;",
       "y[k] = (sh->round_y ? round_to_bf16(acc) : acc) + (nudge ? nudge[k] : 0.0);", None)], None, None,
     ["test_tie_hooks_of_the_draft_routines"]),
    ("y_exact_taken_after_the_nudge",
     [("        if (y_exact) y_exact[k] = acc;\n        if (nudge) acc += nudge[k];\n",
       "        if (nudge) acc += nudge[k];\n        if (y_exact) y_exact[k] = acc;\n", None)], None, None,
     ["test_tie_hooks_of_the_draft_routines"]),
    ("rounded_mode_ignored_by_first_token", "head_y_ex(sh, h, W, 0, al, y_nudge ? y_nudge + ((size_t)b * r + al) * d : NULL, NULL, y);",
     "head_y(&(cpo_shape){sh->T, sh->d, sh->V, sh->n, sh->r, 0}, h, W, 0, al, y);", None,
     ["test_rounded_y_first_token_and_sequential_are_the_composition"]),
    ("nudge_of_the_wrong_row_in_sequential", "y_nudge ? y_nudge + (((size_t)b * n + s) * r + al) * d : NULL, NULL, y);",
     "y_nudge ? y_nudge + (((size_t)b * r + al) * n + s) * d : NULL, NULL, y);", None,
     ["test_tie_hooks_of_the_draft_routines"]),
]


def mutated_oracle(tmp_path, old, new, occurrence):
    """A private module object of the oracle's front end whose C source carries the planted mistake."""
    d = os.path.join(str(tmp_path), "oracle_mutant")
    os.makedirs(d, exist_ok=True)
    src = open(os.path.join(ORACLE_DIR, "cp_oracle.c")).read()
    edits = [(old, new, occurrence)] if isinstance(old, str) else old
    for old, new, occurrence in edits:
        count = src.count(old)
        assert count >= 1, f"mutation site not found: {old!r}"
        if occurrence is None:
            assert count == 1, f"mutation site is not unique ({count}): {old!r}"
            src = src.replace(old, new)
        else:
            parts = src.split(old)
            assert occurrence < len(parts) - 1
            src = old.join(parts[:occurrence + 1]) + new + old.join(parts[occurrence + 1:])
    with open(os.path.join(d, "cp_oracle.c"), "w") as f:
        f.write(src)
    shutil.copy(os.path.join(ORACLE_DIR, "cp_oracle.py"), os.path.join(d, "cp_oracle.py"))
    spec = importlib.util.spec_from_file_location("cp_oracle_mutant", os.path.join(d, "cp_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)            # its _HERE/_SRC point into the temporary directory
    mod.build(force=True)
    return mod


def pin_fails(mod, pin):
    name, arg = (pin, None) if isinstance(pin, str) else pin
    fn = getattr(pins, name)
    try:
        fn(mod) if arg is None else fn(mod, arg)
    except Exception:                        # an assertion, or the oracle refusing outright
        return True
    return False


@pytest.mark.parametrize("name,old,new,occurrence,expected", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, occurrence, expected):
    mod = mutated_oracle(tmp_path, old, new, occurrence)
    caught = [p for p in expected if pin_fails(mod, p)]
    assert caught, f"no pin noticed the planted mistake {name!r}: tried {expected}"


def test_the_unmutated_copy_passes(tmp_path):
    """The harness itself: an unchanged private copy passes the same pins."""
    mod = mutated_oracle(tmp_path, "return pick < 0 ? len - 1 : pick;", "return pick < 0 ? len - 1 : pick;", None)
    for m in MUTANTS:
        for p in m[4]:
            assert not pin_fails(mod, p), p
