"""CPU-only: the pins must notice mistakes.  Each case plants one plausible
error in a copy of the oracle's C source (a dropped term, a transposed
operand, a wrong sign or index), builds it, and requires at least one pin
to fail.  The mistakes are planted in the oracle, on the CPU, never on a GPU.
"""
import os
import subprocess

import pytest

import oracle
from oracle import m2rnn_oracle
from oracle_pins import ALL_CHECKS

SRC = os.path.join(os.path.dirname(m2rnn_oracle.__file__), "m2rnn_oracle.c")

MUTATIONS = {
    "carried_gradient_dropped":
        ("G[i * V + j] = qt[i] * dyt[j] + C[i * V + j];", "G[i * V + j] = qt[i] * dyt[j];"),
    "carry_is_product_not_sum":
        ("C[i * V + c] = ft * G[i * V + c] + acc;", "C[i * V + c] = ft * G[i * V + c] * acc;"),
    "carry_misses_gate_path":
        ("C[i * V + c] = ft * G[i * V + c] + acc;", "C[i * V + c] = acc;"),
    "W_transposed_in_forward":
        ("s += H[i * V + c] * W[c * V + j];", "s += H[i * V + c] * W[j * V + c];"),
    "W_not_transposed_in_backward":
        ("acc += dS[i * V + j] * Wn[c * V + j];", "acc += dS[i * V + j] * Wn[j * V + c];"),
    "gate_sign":
        ("H[e] = ft * H[e] + (1.0 - ft) * z;", "H[e] = ft * H[e] + (1.0 + ft) * z;"),
    "gate_swapped":
        ("H[e] = ft * H[e] + (1.0 - ft) * z;", "H[e] = (1.0 - ft) * H[e] + ft * z;"),
    "dW_transposed":
        ("dWu[c * V + j] += acc;", "dWu[j * V + c] += acc;"),
    "df_uses_new_state":
        ("dft += G[e] * (Hprev[e] - Z[e]);", "dft += G[e] * (Hnext[e] - Z[e]);"),
    "dq_uses_old_state":
        ("acc += Hnext[i * V + j] * dyt[j];", "acc += Hprev[i * V + j] * dyt[j];"),
    "tanh_derivative":
        ("dS[e] = (1.0 - ft) * G[e] * (1.0 - Z[e] * Z[e]);",
         "dS[e] = (1.0 - ft) * G[e] * (1.0 - Z[e]);"),
    "dS_misses_gate_factor":
        ("dS[e] = (1.0 - ft) * G[e] * (1.0 - Z[e] * Z[e]);",
         "dS[e] = G[e] * (1.0 - Z[e] * Z[e]);"),
    "outer_product_dropped":
        ("S[i * V + j] = s + kt[i] * vt[j];", "S[i * V + j] = s;"),
    "dk_dv_swapped_operands":
        ("acc += dS[i * V + j] * vt[j];", "acc += dS[i * V + j] * kt[i];"),
    "head_group_mapping":
        ("const int g = n / heads_per_group;", "const int g = n % Nqk;"),
    "residual_without_v":
        ("acc += w_r[(size_t)n * V + j] * v[IDX_V(b, t, n, j)];", "acc += w_r[(size_t)n * V + j];"),
    "residual_missing_in_dv":
        ("if (w_r) acc += w_r[(size_t)n * V + j] * dyt[j];", ""),
    "dw_r_head_index":
        ("dw_r[(size_t)n * V + j] = s;", "dw_r[(size_t)(N - 1 - n) * V + j] = s;"),
    "clip_one_sided":
        ("C[e] = C[e] > clip ? clip : (C[e] < -clip ? -clip : C[e]);",
         "C[e] = C[e] > clip ? clip : C[e];"),
    "clip_after_readout_term":
        ("G[i * V + j] = qt[i] * dyt[j] + C[i * V + j];",
         "{ G[i * V + j] = qt[i] * dyt[j] + C[i * V + j]; if (clip > 0.0) G[i * V + j] = "
         "G[i * V + j] > clip ? clip : (G[i * V + j] < -clip ? -clip : G[i * V + j]); }"),
    "gate_exponent_sign":
        ("return exp(-alpha[n] * softplus(x + beta[n]));", "return exp(alpha[n] * softplus(x + beta[n]));"),
    "gate_beta_not_added":
        ("return exp(-alpha[n] * softplus(x + beta[n]));", "return exp(-alpha[n] * softplus(x));"),
    "gate_dx_misses_alpha":
        ("const double dx = -g * alpha[n] * psi / (1.0 + exp(-u));",
         "const double dx = -g * psi / (1.0 + exp(-u));"),
    "gate_dalpha_uses_sigmoid":
        ("sa += -g * psi * sp;", "sa += -g * psi / (1.0 + exp(-u));"),
    "readout_before_update":
        ("acc += H[i * V + j] * qt[i];", "acc += S[i * V + j] * qt[i];"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_mutation(name, tmp_path):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, "mutation site not found: " + old
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-o",
                           str(lib), str(mutated), "-lm"])
    fwd, bwd = oracle.m2rnn_oracle.variant(str(lib))
    caught = []
    for check in ALL_CHECKS:
        try:
            check(fwd, bwd)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin noticed the planted mistake '%s'" % name
