"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the C oracle (on
the CPU; nothing here touches the GPU path), rebuilds it, and requires that at least one of
the pins that rest on the paper and on mathematics alone - brute-force ledger, Fig. 7
walk-through, allreduce special case against torch, conservation, Lemma 2 identity, closed
forms, torch's bf16 - fails.  The pin that compares the C code with the oracle package's own
fp64 version is deliberately not in the list: the oracle must not be pinned only to itself.
"""
import os

import pytest

import test_oracle_pins as pins
from oracle import eager_oracle as eo

MUTATIONS = {
    "stale term dropped when a process catches up":
        ("c = R[p][i] + g;", "c = g;"),
    "late gradient not stored in the send buffer":
        ("R[p][i] = g;", ";"),
    "contribution subtracted":
        ("s = s + c;", "s = s - c;"),
    "late process contributes its fresh gradient":
        ("s = s + R[p][i];", "s = s + g;"),
    "average over the contributors instead of P":
        ("const float inv_P = 1.0f / (float)P;",
         "const float inv_P = 1.0f / (float)__builtin_popcountll(mask);"),
    "momentum operands swapped":
        ("vn = fmaf(mu, *v, g);", "vn = fmaf(mu, g, *v);"),
    "step added instead of subtracted":
        ("*w = fmaf(-lr, step, *w);", "*w = fmaf(lr, step, *w);"),
    "mask bits read in reverse rank order":
        ("(int)((mask >> p) & 1u)", "(int)((mask >> (P - 1 - p)) & 1u)"),
    "bf16 widened with the wrong shift":
        ("(uint32_t)h << 16", "(uint32_t)h << 15"),
    "empty send buffers read as if they held a gradient":
        ("(int)((valid >> p) & 1u)", "1"),
    "Nesterov step from the old momentum":
        ("step = fmaf(mu, vn, g);", "step = fmaf(mu, *v, g);"),
    "weight decay applied to the update instead of the parameter":
        ("g = fmaf(wd, *w, u);", "g = fmaf(wd, u, *w);"),
    "stashed gradient overwrites a pending one":
        ("R[i] = has_stale ? R[i] + g : g;", "R[i] = g;"),
    "layer-wise rate inverted":
        ("(double)trust * nw / (nu + (double)wd * nw + (double)eps)",
         "(double)trust * nu / (nw + (double)wd * nu + (double)eps)"),
    "layer-wise rate without the weight-decay term":
        ("(nu + (double)wd * nw + (double)eps)", "(nu + (double)eps)"),
    "layer-wise rate from squared norms":
        ("nu = sqrt(ssu);", "nu = ssu;"),
    "layer-wise rate scales the learning rate instead of the gradient":
        ("update_rule(rate * g, &w[i], &v[i], lr, mu, 0.0f, nesterov);",
         "update_rule(g, &w[i], &v[i], rate * lr, mu, 0.0f, nesterov);"),
    "absent process contributes nothing":
        ("""                if (has_stale)
                    s = s + R[p][i];
                if (!is_absent)""", """                if (has_stale && !is_absent)
                    s = s + R[p][i];
                if (!is_absent)"""),
}


def _pins():
    yield lambda: pins.test_brute_force_every_mask_sequence(2, 3)
    yield lambda: pins.test_brute_force_every_mask_sequence(3, 2)
    yield lambda: pins.test_fig7_walkthrough("catches_up")
    yield lambda: pins.test_fig7_walkthrough("late_again")
    yield pins.test_full_participation_is_allreduce_mean_with_torch_sgd
    yield lambda: pins.test_conservation_every_gradient_applied_exactly_once(4)
    yield pins.test_lemma2_distance_to_clean_iterate
    yield pins.test_momentum_closed_form_and_plain_sgd
    yield lambda: pins.test_update_rule_variants_against_torch_sgd(0.01, True)
    yield pins.test_divides_by_P_not_by_contributors
    yield pins.test_bf16_widening_matches_torch
    yield pins.test_nonfinite_gradients_propagate
    yield lambda: pins.test_brute_force_with_absent_processes_and_stashes(2, 3)
    yield pins.test_layerwise_rate_closed_forms
    yield pins.test_layerwise_rate_properties_and_torch


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_a_planted_mistake_fails_a_pin(name, tmp_path):
    old, new = MUTATIONS[name]
    src = open(eo._SRC).read()
    assert src.count(old) == 1, f"mutation site not unique: {old!r}"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    saved = (eo._SRC, eo._LIB, eo._lib)
    eo._SRC, eo._LIB, eo._lib = str(mutated), str(tmp_path / "libmutant.so"), None
    try:
        caught = None
        for pin in _pins():
            try:
                pin()
            except AssertionError as e:
                caught = e
                break
        assert caught is not None, f"no pin noticed: {name}"
    finally:
        eo._SRC, eo._LIB, eo._lib = saved
    assert os.path.exists(saved[1])


def test_the_unmutated_oracle_passes_the_same_pins():
    for pin in _pins():
        pin()
