"""The pins must catch plausible mistakes: each case plants one mistake in a copy of the
oracle's source (on the CPU), rebuilds it, and requires that at least one pin fails."""
import os

import pytest

import oracle
import tests.test_oracle_backward as bwd
import tests.test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "dchag_oracle.c")

MUTATIONS = {
    "no_softmax_scale": ("s[c] = acc * scale;", "s[c] = acc;"),
    "key_uses_value_weights": ("affine(lv->Wk + wo, lv->bk ? lv->bk + bo : NULL,", "affine(lv->Wv + wo, lv->bk ? lv->bk + bo : NULL,"),
    "patch_pixels_transposed": ("u[r * p + s] =", "u[s * p + r] ="),
    "no_channel_embedding": ("tc[d] += (double)ce[(size_t)c * D + d];", "tc[d] += 0.0;"),
    "every_head_reads_head_zero": ("const int r0 = a * dh;", "const int r0 = 0 * a * dh;"),
    "no_value_bias": ("lv->bv ? lv->bv + bo : NULL", "NULL"),
    "no_output_bias": ("lv->bo ? lv->bo + bo : NULL", "NULL"),
    "no_query_bias": ("lv->bq ? lv->bq + bo : NULL", "NULL"),
    "no_tokenizer_bias": ("be ? be + (size_t)c * D : NULL", "NULL"),
    "patch_grid_column_major": ("const int pi = n / pw, pj = n % pw;", "const int pi = n % (H / p), pj = n / (H / p);"),
    "query_not_projected": ("affine(lv->Wq + wo, lv->bq ? lv->bq + bo : NULL, qv, D, D, Q);",
                            "memcpy(Q, qv, sizeof(double) * (size_t)D);"),
    "softmax_not_normalised": ("s[c] /= den;", "s[c] /= 1.0;"),
    "all_groups_use_group_zero_weights": ("const size_t wo = (size_t)k * D * D, bo = (size_t)k * D;",
                                          "const size_t wo = 0 * (size_t)k, bo = 0;"),
    "value_of_wrong_member": ("acc += s[c] * V[(size_t)c * D + r0 + i];", "acc += s[c] * V[(size_t)(m - 1 - c) * D + r0 + i];"),
    "groups_overlap": ("const int c0 = k * g;", "const int c0 = k * g > 0 ? k * g - 1 : 0;"),
}


# planted in the backward half of the source; caught by the backward pins
BACKWARD_MUTATIONS = {
    "bwd_softmax_jacobian_without_the_mean": ("(dal[c] - dot);", "(dal[c]);"),
    "bwd_no_scale_on_the_query_gradient": ("dQ[r0 + i] += scale * ds * K[(size_t)c * D + r0 + i];",
                                           "dQ[r0 + i] += ds * K[(size_t)c * D + r0 + i];"),
    "bwd_key_gradient_uses_keys": ("dK[(size_t)c * D + r0 + i] = scale * ds * Q[r0 + i];",
                                   "dK[(size_t)c * D + r0 + i] = scale * ds * K[(size_t)c * D + r0 + i];"),
    "bwd_value_gradient_without_alpha": ("dV[(size_t)c * D + r0 + i] = al[(size_t)c * heads + a] * d_o[r0 + i];",
                                         "dV[(size_t)c * D + r0 + i] = d_o[r0 + i];"),
    "bwd_outer_product_transposed": ("gr[j] += yi * x[j];", "gr[j] += y[j % rows] * x[i % cols];"),
    "bwd_input_gradient_misses_the_key_path": (
        "affine_transposed_add(lv->Wk + wo, dK + (size_t)c * D, D, D, dzc);", ""),
    "bwd_output_projection_not_transposed": (
        "affine_transposed_add(lv->Wo + wo, dy, D, D, d_o);", "affine(lv->Wo + wo, NULL, dy, D, D, d_o);"),
    "bwd_patch_pixels_transposed": ("u[r * p + s] = (double)img[(size_t)(pi * p + r) * W + (pj * p + s)];\n      const double *dt",
                                    "u[s * p + r] = (double)img[(size_t)(pi * p + r) * W + (pj * p + s)];\n      const double *dt"),
    "bwd_linear_level_input_gradient_without_weight": ("dz[(size_t)c * D + d] = (double)lv->Wv[wi] * dy[d];",
                                                       "dz[(size_t)c * D + d] = dy[d];"),
    "bwd_level_gradients_of_group_zero_only": ("const double *dy = dzs[l + 1] + ((size_t)i * G + k) * D;",
                                               "const double *dy = dzs[l + 1] + ((size_t)i * G + 0 * k) * D;"),
}


def run_backward_pins():
    checks = [
        ("autograd", lambda: bwd.test_backward_matches_library_autograd(bwd.CASES[1])),
        ("autograd_linear", lambda: bwd.test_backward_matches_library_autograd(bwd.CASES[4])),
        ("fd", lambda: bwd.test_backward_matches_finite_differences_of_the_forward(bwd.CASES[1])),
        ("dbk", bwd.test_key_bias_has_zero_gradient_and_token_biases_share_theirs),
        ("dbv", bwd.test_value_bias_gradient_is_the_output_projection_of_the_output_bias_gradient),
    ]
    failed = []
    for name, fn in checks:
        try:
            fn()
        except AssertionError:
            failed.append(name)
    return failed


def run_pins():
    """A subset of the pins that together covers every step; returns the names of those that failed."""
    checks = [
        ("conv2d", lambda: pins.test_tokenizer_is_a_grouped_conv2d(2, 4, 6)),
        ("conv2d_p4", lambda: pins.test_tokenizer_is_a_grouped_conv2d(4, 8, 12)),
        ("mha", lambda: pins.test_one_group_is_library_multihead_attention(2, 8, 3)),
        ("brute", lambda: pins.test_forward_matches_brute_force_micro(
            dict(C=5, D=6, heads=1, group_sizes=(2, 3), p=1, H=3, W=4), True)),
        ("brute3", lambda: pins.test_forward_matches_brute_force_micro(
            dict(C=6, D=4, heads=4, group_sizes=(2, 2, 2), p=2), True)),
        ("g1", pins.test_group_of_one_is_value_then_output_projection),
        ("mean", lambda: pins.test_identical_keys_give_the_mean_of_values("zero_wk")),
        ("convex", pins.test_softmax_weights_are_a_convex_combination),
        ("short", pins.test_short_last_group_attends_only_over_real_members),
        ("local", pins.test_output_depends_only_on_its_own_patch),
    ]
    failed = []
    for name, fn in checks:
        try:
            fn()
        except AssertionError:
            failed.append(name)
    return failed


def test_unmutated_source_passes_the_subset():
    assert run_pins() == []
    assert run_backward_pins() == []


@pytest.mark.parametrize("name", sorted(BACKWARD_MUTATIONS))
def test_planted_backward_mistake_is_caught(name, tmp_path):
    old, new = BACKWARD_MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for {name} not found exactly once in the oracle source"
    bad_src = tmp_path / "bad_oracle.c"
    bad_src.write_text(text.replace(old, new))
    bad_lib = str(tmp_path / f"libbad_{name}.so")
    oracle.compile_source(str(bad_src), bad_lib)
    oracle.use_library(bad_lib)
    try:
        failed = run_backward_pins()
    finally:
        oracle.use_library(None)
    assert failed, f"no backward pin noticed the planted mistake {name!r}"


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation anchor for {name} not found in the oracle source"
    bad_src = tmp_path / "bad_oracle.c"
    bad_src.write_text(text.replace(old, new))
    bad_lib = str(tmp_path / f"libbad_{name}.so")
    oracle.compile_source(str(bad_src), bad_lib)
    oracle.use_library(bad_lib)
    try:
        failed = run_pins()
    finally:
        oracle.use_library(None)
    assert failed, f"no pin noticed the planted mistake {name!r}"
