"""CPU checks of the seeded input generator (it feeds both the oracle and the GPU library, so
the two must see identical, storage-exact values)."""
import numpy as np

from paper_2603_14360_amd.synth_inputs import (WORKLOADS, Workload, bf16_bits_to_f32, make_inputs,
                                                round_to_bf16, select_heads)


def test_generator_is_deterministic_and_shaped():
    wl = WORKLOADS["C1"]
    a, b = make_inputs(wl), make_inputs(wl)
    for name in ("q", "k", "v", "f", "W", "dy"):
        assert np.array_equal(a[name], b[name]), name
    assert a["q"].shape == (wl.B, wl.T, wl.N, wl.K) and a["v"].shape == (wl.B, wl.T, wl.N, wl.V)
    assert a["W"].shape == (wl.N, wl.V, wl.V) and a["f"].shape == (wl.B, wl.T, wl.N)
    assert a["H0"] is None and a["dHT"] is None
    assert (a["f"] > 0).all() and (a["f"] < 1).all() and a["f"].dtype == np.float32


def test_bf16_rounding_is_nearest_even_and_idempotent():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(10000).astype(np.float32) * np.float32(3.0)
    r, bits = round_to_bf16(x)
    assert np.array_equal(bf16_bits_to_f32(bits), r)
    assert np.array_equal(round_to_bf16(r)[0], r)                 # already representable
    assert (np.abs(r - x) <= np.abs(x) * 2.0 ** -8).all()         # half an ulp of 8 bits
    # ties go to the even mantissa: 1 + 2^-8 is exactly between 1 and 1 + 2^-7
    tie = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert np.array_equal(round_to_bf16(tie)[0], np.array([1.0, 1.0 + 2.0 ** -6], dtype=np.float32))


def test_bf16_workloads_hold_storage_exact_values():
    wl = Workload("t", 2, 9, 3, 16, 16, "bf16", 11, 0.25, 1.0, use_H0=True, use_dHT=True)
    inp = make_inputs(wl)
    for name in ("q", "k", "v", "W", "dy"):
        assert np.array_equal(round_to_bf16(inp[name])[0], inp[name]), name
    assert inp["H0"].dtype == np.float32 and inp["dHT"].shape == (2, 3, 16, 16)


def test_normalised_k_and_shared_heads():
    wl = Workload("t", 2, 5, 4, 16, 16, "f32", 3, 0.25, 0.0, normalise_k=True, Nqk=1)
    inp = make_inputs(wl)
    assert inp["q"].shape == (2, 5, 1, 16)
    assert np.allclose(np.linalg.norm(inp["k"].astype(np.float64), axis=-1), 1.0, atol=1e-6)
    sub = select_heads(inp, [1, 3])
    assert sub["q"].shape == (2, 5, 1, 16) and sub["v"].shape == (2, 5, 2, 16)
    assert np.array_equal(sub["W"], inp["W"][[1, 3]]) and np.array_equal(sub["f"], inp["f"][:, :, [1, 3]])
    per_head = select_heads(make_inputs(Workload("t", 1, 4, 4, 16, 16, "f32", 3, 0.25, 0.0)), [2])
    assert per_head["q"].shape == (1, 4, 1, 16)


def test_shorter_T_is_its_own_draw_not_a_prefix():
    # documented behaviour: reduced shapes are drawn directly (tests that need prefixes slice)
    wl = WORKLOADS["C1"]
    full, short = make_inputs(wl), make_inputs(wl, T=8)
    assert short["q"].shape[1] == 8 and full["q"].shape[1] == wl.T
