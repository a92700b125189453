"""The pins really pin: plant one plausible mistake at a time in a copy of the oracle's C source
(on the CPU; the committed oracle is never touched) and check that the pin suite notices."""

import importlib.util
import os
import shutil
import subprocess
import sys

import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = {
    "relu_dropped": ("a1[i] = active ? a0 : 0.0;", "a1[i] = a0;"),
    "rms_mean_over_wrong_count": ("sumsq / (double)E + L->eps", "sumsq / (double)(E > 1 ? E - 1 : 1) + L->eps"),
    "eps_outside_root": ("sqrt(sumsq / (double)E + L->eps)", "(sqrt(sumsq / (double)E) + L->eps)"),
    "gain_dropped": ("(float)(g * a1[i] / rms)", "(float)(a1[i] / rms)"),
    "bias_dropped": ("L->b_router ? (double)L->b_router[i] : 0.0", "0.0"),
    "non_strict_activation": ("(float)a0 > 0.0f", "(float)a0 >= 0.0f"),
    "router_weight_transposed": ("widen(L->w_router, L->wdtype, (size_t)i * d + j)",
                                 "widen(L->w_router, L->wdtype, (size_t)j * E + i)"),
    "list_tail_not_minus_one": ("active_idx[c * E + s] = -1;", "active_idx[c * E + s] = 0;"),
    "counts_swapped": ("stats[0] += tls_inactive;\n    stats[1] += cls_inactive;",
                       "stats[1] += tls_inactive;\n    stats[0] += cls_inactive;"),
    "union_misses_last_token": ("for (int t = 0; t < k; ++t)\n      for (int i = 0; i < E; ++i) {",
                                "for (int t = 0; t < (k > 1 ? k - 1 : 1); ++t)\n      for (int i = 0; i < E; ++i) {"),
    "swish_on_the_up_branch": ("h[j] = swish(g) * u;", "h[j] = swish(u) * g;"),
    "swish_sign": ("return u / (1.0 + exp(-u));", "return u / (1.0 + exp(u));"),
    "w_down_transposed": ("size_t row = ((size_t)i * d + c) * de;\n    double e = 0.0;\n    for (int j = 0; j < de; ++j) e += h[j] * widen(L->w_down, L->wdtype, row + j);",
                          "double e = 0.0;\n    for (int j = 0; j < de; ++j) e += h[j] * widen(L->w_down, L->wdtype, ((size_t)i * de + j) * d + c);"),
    "w_up_transposed": ("for (int c = 0; c < d; ++c) u += (double)xt[c] * widen(L->w_up, L->wdtype, row + c);",
                        "for (int c = 0; c < d; ++c) u += (double)xt[c] * widen(L->w_up, L->wdtype, ((size_t)i * d + c) * de + j);"),
    "mask_ignored_by_sparse_path": ("if (!((token_mask[tok * W + i / 64] >> (i % 64)) & 1)) continue;", ""),
    "score_dropped": ("y[c] += a * e;", "y[c] += e;"),
    "bf16_shift": ("<< 16;", "<< 15;"),
    "mask_bit_position": ("token_mask[t * W + i / 64] |= (uint64_t)1 << (i % 64);",
                          "token_mask[t * W + i / 64] |= (uint64_t)1 << ((i + 1) % 64);"),
}


def pin_calls(o):
    yield lambda: pins.test_router_hand_worked_golden(o)
    yield lambda: pins.test_router_bf16_weights_widen_exactly(o)
    for E, d in [(5, 16), (65, 8)]:
        yield lambda E=E, d=d: pins.test_router_invariants(o, E, d)
    yield lambda: pins.test_router_single_expert_closed_form(o)
    yield lambda: pins.test_router_matches_matmul_library(o)
    yield lambda: pins.test_router_exact_arithmetic_fixture_any_order(o)
    yield lambda: pins.test_router_sign_patterns_bruteforce(o)
    for E, k in [(16, 4), (65, 3), (128, 8)]:
        yield lambda E=E, k=k: pins.test_union_bruteforce_sets(o, E, k)
    yield lambda: pins.test_union_k1_and_repeated_tokens_and_monotonicity(o)
    yield lambda: pins.test_ffn_hand_worked_golden(o)
    for dt in ("f32", "bf16"):
        yield lambda dt=dt: pins.test_ffn_single_expert_is_a_two_matmul_mlp(o, dt)
    yield lambda: pins.test_ffn_one_hot_weights_closed_form(o)
    yield lambda: pins.test_ffn_multi_expert_is_weighted_sum_of_single_experts(o)
    yield lambda: pins.test_gated_with_gate_equal_up_reduces_to_nongated(o)
    for gated in (False, True):
        yield lambda gated=gated: pins.test_sparse_equals_dense_bitwise_and_skips(o, gated)


def load_mutant(tmp_path, name, old, new):
    src = open(os.path.join(ROOT, "oracle", "blockffn_oracle.c")).read()
    assert src.count(old) == 1, "mutation target must occur exactly once: " + name
    pkg = tmp_path / ("oracle_mut_" + name)
    pkg.mkdir()
    (pkg / "blockffn_oracle.c").write_text(src.replace(old, new))
    shutil.copy(os.path.join(ROOT, "oracle", "__init__.py"), pkg / "__init__.py")
    spec = importlib.util.spec_from_file_location("oracle_mut_" + name, str(pkg / "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.build(force=True)
    return mod


def test_unmutated_copy_passes(tmp_path):
    mod = load_mutant(tmp_path, "identity", "int oracle_max_experts(void) { return 1024; }",
                      "int oracle_max_experts(void) { return 1024; } ")
    for call in pin_calls(mod):
        call()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTATIONS[name]
    mod = load_mutant(tmp_path, name, old, new)
    caught = []
    for i, call in enumerate(pin_calls(mod)):
        try:
            call()
        except (AssertionError, StopIteration) as e:
            caught.append(i)
    assert caught, "no pin noticed the planted mistake '%s'" % name
