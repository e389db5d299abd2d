"""Pins for the oracle's 8-bit draft format (E4M3 elements + E8M0 block scales; the two-step
direct cast of arXiv 2503.13565, section 3.4.3, with the 8-bit element format that sections 1
and 3.2 name as a drop-in).  Expected values come from the field widths, exact rational
arithmetic, and a library's float8 conversion and decode; none is computed by the oracle.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import synth
from test_oracle_cast import bf16_bits, bits_value


def grid_from_fields():
    g = []
    for code in range(127):
        e, m = code >> 3, code & 7
        g.append(Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7))
    return g


GRID = grid_from_fields()


def library_code(r: np.ndarray) -> np.ndarray:
    """A library's round-to-nearest-even conversion to E4M3 (valid below 464; it has no saturation)."""
    return torch.from_numpy(np.asarray(r, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def cast_block(values):
    q8, s = oracle.e4m3_direct_cast(bf16_bits(values).reshape(1, 32))
    return q8[0], int(s[0, 0])


def test_grid_matches_field_widths_and_library_decode():
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for code in range(127):
        assert oracle.e4m3_magnitude(code) == float(GRID[code]) == lib[code]
    assert float(GRID[126]) == 448.0 and float(GRID[1]) == 2.0 ** -9 and float(GRID[8]) == 2.0 ** -6
    assert np.isnan(lib[127])


def test_every_code_point_round_trips_at_every_scale():
    mags = np.array([float(g) for g in GRID])
    for j in list(range(-117, 120, 7)) + [-117, 119, 0]:
        for lo in range(0, 127, 31):
            codes = list(range(lo, min(lo + 31, 127)))
            signs = [(-1.0) ** c for c in codes]
            vals = np.zeros(32)
            vals[: len(codes)] = mags[codes] * np.array(signs)
            vals[31] = 448.0                            # fixes floor(log2 amax) = 8
            q8, sc = cast_block(vals * 2.0 ** j)
            assert sc == j + 127, (j, sc)
            want = [c | (0x80 if sg < 0 else 0) for c, sg in zip(codes, signs)]
            assert q8[: len(codes)].tolist() == want, (j, lo)
            assert q8[31] == 126
            back = oracle.e4m3_dequant(q8.reshape(1, 32), np.array([[sc]], np.uint8))[0]
            assert np.array_equal(back, vals * 2.0 ** j)


def test_midpoints_go_to_the_even_code_and_neighbours_to_the_nearer():
    for c in range(126):
        mid = (GRID[c] + GRID[c + 1]) / 2
        even = c if c % 2 == 0 else c + 1
        # one BF16 ulp: mid has at most 5 significant bits, BF16 holds 8
        f = float(mid)
        ulp = 2.0 ** (np.floor(np.log2(f)) - 7)
        for E in (-60, 0, 31):
            vals = np.zeros(32)
            vals[0] = 256.0
            vals[1], vals[2], vals[3] = f, f - ulp, -(f + ulp)
            q8, sc = cast_block(vals * 2.0 ** E)
            assert sc == E + 127
            assert (q8[1], q8[2], q8[3]) == (even, c, 0x80 | (c + 1)), (c, E, q8[:4])


def test_elements_match_a_library_conversion_below_the_saturation_point():
    rng = np.random.default_rng(3)
    for E in (-40, -8, 0, 9):
        # magnitudes 2^-27 .. 2^9: from far below the smallest subnormal target to the top binade
        bits = ((rng.integers(100, 136, size=(400, 32)) << 7) | rng.integers(0, 128, size=(400, 32))).astype(np.uint16)
        bits |= (rng.integers(0, 2, size=bits.shape) << 15).astype(np.uint16)
        v = bits_value(bits)
        keep = np.abs(v) < 464.0                                               # the library has no saturation
        v = np.where(keep & np.isfinite(v), v, 0.0)
        v[:, 0] = 300.0                                                        # floor(log2 amax) = 8
        q8, s = oracle.e4m3_direct_cast(bf16_bits((v * 2.0 ** E).astype(np.float32)))
        assert np.all(s == E + 127)
        want = library_code(v)
        assert np.array_equal(q8 & 0x7F, want & 0x7F)
        assert np.array_equal(q8 >> 7, (np.signbit(v)).astype(np.uint8))


def test_beyond_the_largest_magnitude_saturates_never_nan():
    # amax in (448, 512) keeps floor(log2 amax) = 8: such elements cannot be represented and clamp
    for r in (450.0, 464.0, 466.0, 480.0, 510.0):
        vals = np.zeros(32)
        vals[5], vals[6] = r, -r
        q8, sc = cast_block(vals)
        assert sc == 127 and q8[5] == 126 and q8[6] == 0x80 | 126, (r, q8[5], q8[6])


def test_scale_rule_zero_blocks_tiny_blocks_and_non_finite_inputs():
    for amax, want in [(1.0, 127 - 8), (1.9921875, 127 - 8), (2.0, 127 - 7), (255.0, 127 - 1), (256.0, 127),
                       (2.0 ** -100, 127 - 108), (2.0 ** -126, 0), (2.0 ** -120, 0), (2.0 ** 127, 127 + 119)]:
        vals = np.zeros(32)
        vals[17] = -amax
        _, sc = cast_block(vals)
        assert sc == want, (amax, sc, want)
    q8, sc = cast_block(np.zeros(32))
    assert sc == 0 and not q8.any()
    neg_zero = np.zeros(32, np.float32)
    neg_zero[3] = -0.0
    q8, _ = cast_block(neg_zero)
    assert q8[3] == 0x80
    for bad in (np.inf, -np.inf, np.nan):
        w = bf16_bits(np.ones(32)).copy()
        w[9] = (np.array([bad], np.float32).view(np.uint32)[0] >> 16).astype(np.uint16)
        q8, s = oracle.e4m3_direct_cast(w.reshape(1, 32))
        assert s[0, 0] == 0xFF and not q8.any()
        assert np.all(np.isnan(oracle.e4m3_dequant(q8, s)))


def test_error_bound_of_the_cast():
    w = synth.weights_student_t(64, 512, seed=4)
    bits = synth.to_bits(w)
    q8, s = oracle.e4m3_direct_cast(bits)
    back = oracle.e4m3_dequant(q8, s)
    v = bits_value(bits)
    X = 2.0 ** (s.astype(np.float64) - 127).repeat(32, axis=1)
    # half a quantum: 2^-4 relative for normal targets, 2^-10 X below the smallest normal,
    # and up to 64 X for the elements that saturate
    bound = np.maximum(np.abs(v) * 2.0 ** -4, X * 2.0 ** -10)
    bound = np.where(np.abs(v) > 448.0 * X, 64.0 * X, bound)
    assert np.all(np.abs(back - v) <= bound)
    assert np.all(np.abs(back) <= 448.0 * X)


def test_product_matches_library_matmul_on_library_decoded_weights():
    m, n, k = 5, 37, 192
    w = synth.weights_student_t(n, k, seed=5)
    x = synth.activations_outlier_channels(m, k, seed=6)
    q8, s = oracle.e4m3_direct_cast(synth.to_bits(w))
    w_lib = torch.from_numpy(q8).view(torch.float8_e4m3fn).to(torch.float64) * \
        torch.from_numpy(2.0 ** (s.astype(np.float64) - 127)).repeat_interleave(32, dim=1)
    y, a = oracle.e4m3_woq_gemm(synth.to_bits(x), q8, s)
    y_lib = (x.double() @ w_lib.T).numpy()
    a_lib = (x.double().abs() @ w_lib.abs().T).numpy()
    assert y.shape == (m, n)
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)
    assert np.array_equal(oracle.e4m3_dequant(q8, s), w_lib.numpy())


def test_one_hot_rows_pick_single_weights():
    n, k = 7, 64
    w = synth.weights_gaussian_outliers(n, k, seed=8)
    q8, s = oracle.e4m3_direct_cast(synth.to_bits(w))
    wd = oracle.e4m3_dequant(q8, s)
    x = torch.zeros((3, k), dtype=torch.bfloat16)
    x[0, 5], x[1, 63], x[2, 32] = 1.0, -2.0, 0.5
    y = oracle.e4m3_woq_gemm(synth.to_bits(x), q8, s, want_abs=False)
    assert np.array_equal(y[0], wd[:, 5]) and np.array_equal(y[1], -2.0 * wd[:, 63])
    assert np.array_equal(y[2], 0.5 * wd[:, 32])
