"""CPU-only: the float64 oracle of the scan's neighbours (conv1d(4) + SiLU, gated RMSNorm)
against a library convolution, autodiff, closed forms, invariants and finite differences; and
the same checks against copies of the oracle with one planted mistake each (planted in the
oracle, on the CPU), which at least one check must notice."""
import os
import subprocess

import pytest

import oracle
from block_oracle_pins import ALL_CHECKS

SRC = os.path.join(os.path.dirname(oracle.block.__file__), "m2rnn_block_oracle.c")


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda c: c.__name__)
def test_block_oracle_pin(check):
    check(oracle.block)


MUTATIONS = {
    "taps_reversed": ("const int ts = t - (CONV_TAPS - 1) + j;\n    if (ts >= 0) a +=",
                      "const int ts = t - j;\n    if (ts >= 0) a +="),
    "anti_causal": ("const int ts = t - (CONV_TAPS - 1) + j;\n    if (ts >= 0) a +=",
                    "const int ts = t + j;\n    if (ts >= 0 && ts < T) a +="),
    "silu_gradient": ("return sg * (1.0 + u * (1.0 - sg));", "return sg * (1.0 + u * sg);"),
    "conv_dw_uses_output_step": ("dw[(size_t)c * CONV_TAPS + j] += da * x[((size_t)b * T + ts) * C + c];",
                                 "dw[(size_t)c * CONV_TAPS + j] += da * x[((size_t)b * T + t) * C + c];"),
    "conv_bias_dropped": ("double a = bias ? bias[c] : 0.0;", "double a = 0.0;"),
    "norm_mean_not_divided": ("const double s = 1.0 / sqrt(ss / D + eps);\n    if (s_out)",
                              "const double s = 1.0 / sqrt(ss + eps);\n    if (s_out)"),
    "norm_gate_without_silu": ("const double xi = yt[i] * (at[i] * sigmoid(at[i]));\n      out[",
                               "const double xi = yt[i] * at[i];\n      out["),
    "norm_bwd_s_cubed": ("const double dxi = s * p - r * s * s * s * xi / D;",
                         "const double dxi = s * p - r * s * s * xi / D;"),
    "norm_bwd_missing_projection": ("const double dxi = s * p - r * s * s * s * xi / D;",
                                    "const double dxi = s * p;"),
    "norm_dw_without_s": ("dw[i] += dot[i] * xi * s;", "dw[i] += dot[i] * xi;"),
    "norm_dy_da_swapped": ("dy[tok * D + i] = dxi * g;", "dy[tok * D + i] = dxi * yt[i];"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_block_pins_catch_mutation(name, tmp_path):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, "mutation site not found: " + old
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-fPIC", "-shared", "-o", str(lib), str(mutated), "-lm"])
    variant = oracle.block.Variant(str(lib))
    caught = []
    for check in ALL_CHECKS:
        try:
            check(variant)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin noticed the planted mistake '%s'" % name
