"""Show that the pins bite: each plausible mistake planted in a COPY of the oracle fails a pin.

The mistakes are planted in the CPU oracle's C source (never in GPU code): the
source is edited as text, compiled to a temporary shared object and run through
the same check functions as the real oracle.
"""
import os

import pytest

import oracle
from test_oracle_pins import ALL_CHECKS
from test_oracle_next_pins import NEXT_CHECKS

MUTANTS = {
    "beta1_beta2_swapped_in_sign": ("float a = beta1 * mi[j];", "float a = beta2 * mi[j];"),
    "beta2_replaced_in_momentum": ("float a2 = beta2 * mi[j];", "float a2 = beta1 * mi[j];"),
    "one_minus_beta_mixed_up": ("float b2 = one_minus_beta2 * gij;", "float b2 = one_minus_beta1 * gij;"),
    "gradient_weight_dropped": ("float b = one_minus_beta1 * gij;", "float b = gij;"),
    "sign_of_zero_is_minus": ("int plus = !(c < 0.0f);", "int plus = (c > 0.0f);"),
    "sign_flipped": ("int plus = !(c < 0.0f);", "int plus = (c < 0.0f);"),
    "fused_multiply_add": ("float c = a + b;", "float c = __builtin_fmaf(beta1, mi[j], b);"),
    "msb_first_bits": ("pi[j / 64] |= (uint64_t)1 << (j % 64);", "pi[j / 64] |= (uint64_t)1 << (63 - j % 64);"),
    "new_momentum_feeds_sign": ("float a = beta1 * mi[j];",
                                "float a = beta1 * (beta2 * mi[j] + one_minus_beta2 * gij);"),
    "tie_votes_plus": ("Delta = (float)((S > 0) - (S < 0));", "Delta = (float)((S >= 0) - (S < 0));"),
    "sum_not_centred": ("int32_t S = 2 * (int32_t)counts[j] - N;", "int32_t S = (int32_t)counts[j];"),
    "average_by_wrong_count": ("Delta = (float)S / (float)N;", "Delta = (float)S / (float)(N + 1);"),
    "update_added": ("x[j] = x[j] - v;", "x[j] = x[j] + v;"),
    "weight_decay_dropped": ("float u = Delta + t;", "float u = Delta;"),
    "weight_decay_outside_lr": ("float v = lr * u;", "float v = lr * Delta + t;"),
    "count_skips_last_worker": ("for (int32_t i = 0; i < N; ++i) {\n            uint64_t word",
                                "for (int32_t i = 0; i + 1 < N || i == 0; ++i) {\n            uint64_t word"),
    "momentum_not_stored": ("mi[j] = a2 + b2;", "(void)(a2 + b2);"),
    # the wider rows
    "plus_plane_includes_ties": ("if (S > 0)\n                planes[j / 64] |= bit;", "if (S >= 0)\n                planes[j / 64] |= bit;"),
    "tie_plane_dropped": ("if (S == 0)\n                planes[plane_stride + j / 64] |= bit;", "if (S == 0 && 0)\n                planes[plane_stride + j / 64] |= bit;"),
    "count_planes_one_short": ("while (((int64_t)1 << bits) <= (int64_t)N)", "while (((int64_t)1 << bits) < (int64_t)N)"),
    "decoded_tie_is_minus": ("Delta = plus ? 1.0f : (tie ? 0.0f : -1.0f);", "Delta = plus ? 1.0f : -1.0f;"),
    "decoded_count_not_centred": ("Delta = (float)(2 * p - N) / (float)N;", "Delta = (float)p / (float)N;"),
    "per_worker_beta_uses_worker_0": ("float a = beta1[i] * mi[j];", "float a = beta1[0] * mi[j];"),
    "per_worker_beta2_swapped": ("float a2 = beta2[i] * mi[j];", "float a2 = beta1[i] * mi[j];"),
    "global_sign_of_last_worker": ("sum = sum + c;", "sum = c;"),
    "global_sign_zero_is_minus": ("float Delta = (mean < 0.0f) ? -1.0f : 1.0f;", "float Delta = (mean > 0.0f) ? 1.0f : -1.0f;"),
    "global_momentum_from_blend": ("*mij = a2 + b2;", "*mij = c;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    with open(oracle.SOURCE) as f:
        src = f.read()
    # the first occurrence is the one meant (later functions repeat some lines of earlier ones)
    assert src.count(old) >= 1, f"mutation site for {name} not found"
    c_path = os.path.join(tmp_path, f"mutant_{name}.c")
    with open(c_path, "w") as f:
        f.write(src.replace(old, new, 1))
    so_path = os.path.join(tmp_path, f"mutant_{name}.so")
    oracle.compile_source(c_path, so_path)
    mutant = oracle.Oracle(so_path)
    caught = []
    for check in ALL_CHECKS + NEXT_CHECKS:
        try:
            check(mutant)
        except AssertionError:
            caught.append(check.__name__)
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"
