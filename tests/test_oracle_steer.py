"""Pins for the steering injection H <- H + alpha_t * v (Sec. 4.2) and the bf16 rounding it uses."""
import numpy as np
import torch

from oracle import round_to_bf16, steer_add


def test_bf16_rounding_matches_library_on_fp32_inputs():
    # torch rounds fp32 -> bf16 to nearest even; on fp32-representable inputs a single
    # rounding and torch's agree bit for bit.
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(2000) * 1e-30).astype(np.float32),
        (rng.standard_normal(2000) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 3.0e-39, -2.5e-40], dtype=np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16)
    vals, bits = round_to_bf16(x.astype(np.float64))
    np.testing.assert_array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(vals, ref.to(torch.float64).numpy())


def test_bf16_ties_go_to_even_and_no_double_rounding():
    # bf16 has 8 significant bits: spacing 2^-7 in [1, 2)
    v, _ = round_to_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8)]))
    np.testing.assert_array_equal(v, [1.0, 1 + 2.0 ** -6, -1.0])
    # just above a tie must round up even though float32 would first round it onto the tie
    x = 1 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(x) == np.float32(1 + 2.0 ** -8)
    assert round_to_bf16(np.array([x]))[0][0] == 1 + 2.0 ** -7


def test_steer_is_axpy_in_fp32_storage():
    rng = np.random.default_rng(2)
    h = rng.standard_normal((5, 64)).astype(np.float32)
    v = rng.standard_normal(64).astype(np.float32)
    got = steer_add(h, v, 1.25, dtype="f32")
    ref = (h.astype(np.float64) + 1.25 * v.astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(got, ref.astype(np.float64))


def test_steer_bf16_per_row_coefficients_and_mask():
    rng = np.random.default_rng(3)
    h = torch.from_numpy(rng.standard_normal((6, 96)).astype(np.float32)).to(torch.bfloat16)
    v = torch.from_numpy(rng.standard_normal(96).astype(np.float32)).to(torch.bfloat16)
    coef = np.array([1.0, 1.02, 1.04, 0.0, 2.0, 0.5], dtype=np.float32)
    mask = np.array([1, 0, 1, 1, 0, 1], dtype=np.uint8)
    h64, v64 = h.to(torch.float64).numpy(), v.to(torch.float64).numpy()
    got = steer_add(h64, v64, coef, mask, dtype="bf16")
    # unmasked rows unchanged, zero coefficient is the identity
    np.testing.assert_array_equal(got[[1, 4]], h64[[1, 4]])
    np.testing.assert_array_equal(got[3], h64[3])
    # masked rows: within half a bf16 ulp of the exact value, and representable in bf16
    exact = h64 + coef.astype(np.float64)[:, None] * v64[None, :]
    rows = [0, 2, 5]
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact[rows]), 1e-30))) - 7)
    assert np.all(np.abs(got[rows] - exact[rows]) <= 0.5 * ulp + 1e-300)
    back = torch.from_numpy(got).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(back, got)
    # library cross-check: float64 -> float32 -> bf16 differs from one rounding only on
    # double-rounding cases, which are at most one bf16 ulp away and rare
    lib = torch.from_numpy(exact).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    diff = np.abs(lib[rows] - got[rows])
    assert np.all(diff <= ulp * 1.0000001) and (diff > 0).mean() < 1e-2


def test_adaptive_strength_is_the_initial_strength_plus_gamma_per_non_execution_thought():
    from oracle import steer_strength
    # Sec. 4.2: alpha_t = alpha_0 + gamma * N_o: alpha_0 with no non-execution thought so far,
    # one gamma more for every one counted, independently per sample
    np.testing.assert_array_equal(steer_strength([0, 0], 1.5, 0.25), [1.5, 1.5])
    np.testing.assert_array_equal(steer_strength([0, 1, 2, 8], 1.0, 0.5), [1.0, 1.5, 2.0, 5.0])
    a = steer_strength(np.arange(10), 0.3, 0.07)
    np.testing.assert_allclose(np.diff(a), 0.07, rtol=1e-12)
