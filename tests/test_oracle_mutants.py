"""The pins must bite: plant one plausible mistake at a time in a copy of the
oracle's source (on the CPU, in a temporary directory), rebuild it, and check
that at least one pin in test_oracle_arith / test_oracle_layout fails."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_arith as A
import test_oracle_layout as L

SUM = "    float s = g[0][i];\n    for (int32_t w = 1; w < W; ++w) s = s + g[w][i];\n"

MUTANTS = {
    "reverse worker order": (SUM, "    float s = g[W-1][i];\n    for (int32_t w = W - 2; w >= 0; --w) s = s + g[w][i];\n"),
    "mean instead of sum": ("    float t = wd * p[i];", "    s = s / (float)W;\n    float t = wd * p[i];"),
    "pairwise sum": (SUM, "    float tmp[64];\n    for (int32_t w = 0; w < W; ++w) tmp[w] = g[w][i];\n"
                          "    for (int32_t m = W; m > 1; m = (m + 1) / 2)\n"
                          "      for (int32_t a = 0; a < m / 2; ++a) tmp[a] = tmp[a] + tmp[m - 1 - a];\n"
                          "    float s = tmp[0];\n"),
    "sum seeded with +0": (SUM, "    float s = 0.0f;\n    for (int32_t w = 0; w < W; ++w) s = s + g[w][i];\n"),
    "weight decay dropped": ("float d = s + t;", "float d = s;"),
    "weight decay sign": ("float d = s + t;", "float d = s - t;"),
    "weight decay decoupled": ("float d = s + t;\n", "float d = s;\n    p[i] = p[i] - lr * t;\n"),
    "step sign": ("float pn = p[i] - q;", "float pn = p[i] + q;"),
    "nesterov": ("float q = lr * vn;", "float q = lr * (d + mu * vn);"),
    "dampening": ("float vn = u + d;", "float vn = u + (1.0f - mu) * d;"),
    "stale momentum in step": ("float q = lr * vn;", "float q = lr * v[i];"),
    "lr folded into momentum": ("float vn = u + d;\n    float q = lr * vn;", "float vn = u + lr * d;\n    float q = vn;"),
    "fma in decay": ("float d = s + t;", "float d = __builtin_fmaf(wd, p[i], s);"),
    "fma in momentum": ("float vn = u + d;", "float vn = __builtin_fmaf(mu, v[i], d);"),
    "fma in step": ("float pn = p[i] - q;", "float pn = __builtin_fmaf(-lr, vn, p[i]);"),
    "double accumulation of the sum": (SUM, "    double sd = g[0][i];\n    for (int32_t w = 1; w < W; ++w) sd = sd + g[w][i];\n    float s = (float)sd;\n"),
    "telemetry after decay": ("acc += (double)s * (double)s;", "acc += (double)d * (double)d;"),
    "equal-size split": ("if (len > cap_elems) len = cap_elems;",
                         "{ int64_t k = (n + cap_elems - 1) / cap_elems; int64_t e = (n + k - 1) / k; if (len > e) len = e; }"),
    "arrival first layer first": ("for (int32_t b = begin; b < end; ++b) out_order[k++] = b;\n    end = begin;",
                                  "for (int32_t b = begin; b < end; ++b) out_order[b] = b;\n    end = begin; k = 0;"),
    "arrival offsets descending": ("for (int32_t b = begin; b < end; ++b) out_order[k++] = b;",
                                   "for (int32_t b = end - 1; b >= begin; --b) out_order[k++] = b;"),
    "interleave ties to higher job": ("if (lhs < rhs) best = j;", "if (lhs <= rhs) best = j;"),
    "interleave position k/n": ("(2 * (int64_t)head[j] + 1)", "(2 * (int64_t)head[j])"),
}

PINS = [
    A.test_constant_gradient_geometric_momentum, A.test_pure_weight_decay_is_geometric,
    A.test_zero_gradient_momentum_coasts, A.test_full_recurrence_matrix_power,
    lambda o: A.test_identical_workers_give_W_times_g(o, 4),
    A.test_sum_order_is_sequential_in_worker_index, A.test_sum_starts_from_worker_zero_value,
    A.test_sum_matches_independent_sequential_loop, A.test_no_fused_multiply_add_anywhere,
    A.test_weight_decay_uses_pre_update_parameter, lambda o: A.test_against_torch_sgd(o, 4),
    A.test_within_rounding_bound_of_exact,
    L.test_split_rule_full_blocks_then_remainder, L.test_arrival_is_last_layer_first_offsets_ascending,
    L.test_interleave_hand_cases, L.test_interleave_equals_sort_by_exact_fraction,
]


def _all_pins_pass(orc) -> bool:
    for pin in PINS:
        try:
            pin(orc)
        except (AssertionError, ValueError):
            return False
    return True


def test_unmutated_oracle_passes(orc):
    assert _all_pins_pass(orc)


@pytest.mark.parametrize("name", list(MUTANTS))
def test_pins_catch_mutant(orc, name, monkeypatch):
    old, new = MUTANTS[name]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "ps_oracle.cpp")).read()
    assert old in src, "mutation site not found: the oracle changed, update this table"
    with tempfile.TemporaryDirectory() as td:
        cpp, so = os.path.join(td, "m.cpp"), os.path.join(td, "m.so")
        open(cpp, "w").write(src.replace(old, new))
        subprocess.check_call(["g++", *oracle.CXXFLAGS, "-mfma", "-o", so, cpp])
        good = oracle.lib()
        bad = ctypes.CDLL(so)
        for fn in ("orc_split_layers", "orc_arrival_order", "orc_interleave",
                   "orc_aggregate_block", "orc_sum_block"):
            getattr(bad, fn).restype = getattr(good, fn).restype
            getattr(bad, fn).argtypes = getattr(good, fn).argtypes
        monkeypatch.setattr(oracle, "_lib", bad)
        assert not _all_pins_pass(orc), f"no pin noticed: {name}"
