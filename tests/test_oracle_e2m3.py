"""Pins for the oracle's 6-bit draft format (E2M3 elements + E8M0 block scales; the two-step direct
cast of arXiv 2503.13565, section 3.4.3, with a 6-bit element format).  Expected values come from
the field widths, a bit string written out here, exact rational arithmetic and a library FP64
matmul on a decode table built here; none is computed by the oracle.
"""
from fractions import Fraction

import numpy as np
import torch

import oracle
from paper_2503_13565_amd import synth
from test_oracle_cast import bf16_bits, bits_value

GRID = [Fraction(m, 8) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 1)
        for e in range(4) for m in range(8)]


def unpack(block24: np.ndarray) -> list:
    """The 32 six-bit codes of one block: a little-endian bit string, code i in bits 6i .. 6i+5."""
    big = int.from_bytes(bytes(block24.tolist()), "little")
    return [(big >> (6 * i)) & 63 for i in range(32)]


def cast_block(values):
    q6, s = oracle.e2m3_direct_cast(bf16_bits(values).reshape(1, 32))
    return unpack(q6[0]), int(s[0, 0])


def test_grid_from_field_widths():
    assert [oracle.e2m3_magnitude(c) for c in range(32)] == [float(g) for g in GRID]
    assert float(GRID[31]) == 7.5 and float(GRID[1]) == 0.125 and float(GRID[8]) == 1.0


def test_packing_is_the_stated_bit_string():
    vals = np.zeros(32)
    vals[0], vals[1], vals[2], vals[31] = 4.0, -0.125, 7.5, -1.0       # codes 24, 32|1, 31, 32|8
    q6, s = oracle.e2m3_direct_cast(bf16_bits(vals).reshape(1, 32))
    want = 24 | (33 << 6) | (31 << 12) | (40 << (6 * 31))
    assert int.from_bytes(bytes(q6[0].tolist()), "little") == want and int(s[0, 0]) == 127
    assert q6.shape == (1, 24)


def test_every_code_point_round_trips_at_every_scale():
    mags = np.array([float(g) for g in GRID])
    for j in list(range(-123, 124, 7)) + [-123, 123, 0]:
        for lo in (0, 16):
            codes = list(range(lo, lo + 16))
            vals = np.zeros(32)
            vals[:16] = mags[codes] * np.array([(-1.0) ** c for c in codes])
            vals[31] = 4.0                              # fixes floor(log2 amax) = 2 (7.5 keeps it too)
            got, sc = cast_block(vals * 2.0 ** j)
            assert sc == j + 127, (j, sc)
            assert got[:16] == [c | (32 if c % 2 else 0) for c in codes] and got[31] == 24
            q6, s = oracle.e2m3_direct_cast(bf16_bits(vals * 2.0 ** j).reshape(1, 32))
            assert np.array_equal(oracle.e2m3_dequant(q6, s)[0], vals * 2.0 ** j)


def test_midpoints_go_to_the_even_code_and_saturation():
    for c in range(31):
        f = float((GRID[c] + GRID[c + 1]) / 2)           # at most 5 significant bits: a BF16 number
        ulp = 2.0 ** (np.floor(np.log2(f)) - 7)
        even = c if c % 2 == 0 else c + 1
        for E in (-50, 0, 40):
            vals = np.zeros(32)
            vals[0] = 4.0
            vals[1], vals[2], vals[3] = f, f - ulp, -(f + ulp)
            got, sc = cast_block(vals * 2.0 ** E)
            assert sc == E + 127
            assert got[1:4] == [even, c, 32 | (c + 1)], (c, E, got[:4])
    for r in (7.5, 7.625, 7.75, 7.875, 7.96875):          # amax below 8 keeps the scale; all clamp to 7.5
        vals = np.zeros(32)
        vals[9], vals[10] = r, -r
        got, sc = cast_block(vals)
        assert sc == 127 and got[9] == 31 and got[10] == 63, (r, got[9], got[10])


def test_scale_rule_zero_blocks_and_non_finite_inputs():
    for amax, want in [(1.0, 125), (3.984375, 126), (4.0, 127), (2.0 ** -100, 25), (2.0 ** -126, 0), (2.0 ** 127, 252)]:
        vals = np.zeros(32)
        vals[17] = -amax
        _, sc = cast_block(vals)
        assert sc == want, (amax, sc, want)
    got, sc = cast_block(np.zeros(32))
    assert sc == 0 and not any(got)
    neg_zero = np.zeros(32, np.float32)
    neg_zero[3] = -0.0
    got, _ = cast_block(neg_zero)
    assert got[3] == 32
    w = bf16_bits(np.ones(32)).copy()
    w[9] = 0x7F80                                       # +Inf
    q6, s = oracle.e2m3_direct_cast(w.reshape(1, 32))
    assert s[0, 0] == 0xFF and not q6.any() and np.all(np.isnan(oracle.e2m3_dequant(q6, s)))


def test_error_bound_and_library_matmul_on_a_decode_table_built_here():
    m, n, k = 5, 37, 192
    w = synth.weights_student_t(n, k, seed=5)
    x = synth.activations_outlier_channels(m, k, seed=6)
    bits = synth.to_bits(w)
    q6, s = oracle.e2m3_direct_cast(bits)
    table = np.array([float(g) for g in GRID] + [-float(g) for g in GRID])
    codes = np.array([[c for b in range(k // 32) for c in unpack(q6[r, 24 * b:24 * b + 24])] for r in range(n)])
    X = 2.0 ** (s.astype(np.float64) - 127).repeat(32, axis=1)
    w_here = table[codes] * X
    assert np.array_equal(oracle.e2m3_dequant(q6, s), w_here)
    v = bits_value(bits)
    bound = np.where(np.abs(v) > 7.5 * X, 0.5 * X, np.maximum(np.abs(v) * 2.0 ** -4, X * 2.0 ** -4))
    assert np.all(np.abs(w_here - v) <= bound)
    y, a = oracle.e2m3_woq_gemm(synth.to_bits(x), q6, s)
    y_lib = (x.double() @ torch.from_numpy(w_here).T).numpy()
    a_lib = (x.double().abs() @ torch.from_numpy(np.abs(w_here)).T).numpy()
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)
