"""Pins for the oracle's generic element formats (arXiv 2503.13565, sections 1, 3.2 and 5: 8-bit and
lower-bit drafts as drop-ins; the two-step direct cast of section 3.4.3 with another element
format): E5M2 (8 bits), E3M2 (6 bits) and the 2-bit ternary T2, each with one E8M0 scale per 32
elements.  Expected values come from the field widths in exact rationals, a library float8
conversion, closed-form intervals, brute force and a library FP64 matmul on a decode table built
here; none is computed by the oracle.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import synth
from test_oracle_cast import bf16_bits, bits_value

E5M2, E3M2, T2 = oracle.FMT_E5M2, oracle.FMT_E3M2, oracle.FMT_T2


def grid(ebits, mbits, bias, top_exp):
    """Finite magnitudes of a sign-magnitude minifloat, code = e << mbits | m, exponent fields 0 .. top_exp."""
    out = []
    for e in range(top_exp + 1):
        for m in range(1 << mbits):
            frac = Fraction(m, 1 << mbits)
            out.append(frac * Fraction(2) ** (1 - bias) if e == 0 else (1 + frac) * Fraction(2) ** (e - bias))
    return out


GRIDS = {E5M2: grid(5, 2, 15, 30), E3M2: grid(3, 2, 3, 7), T2: [Fraction(0), Fraction(1)]}
BITS = {E5M2: 8, E3M2: 6, T2: 2}
EMAX = {E5M2: 15, E3M2: 4, T2: 0}
FORMATS = [E5M2, E3M2, T2]


def unpack(fmt, block: np.ndarray) -> list:
    """The 32 codes of one block: a little-endian bit string, code i in bits bits*i .. bits*i + bits - 1."""
    b = BITS[fmt]
    big = int.from_bytes(bytes(block.tolist()), "little")
    return [(big >> (b * i)) & ((1 << b) - 1) for i in range(32)]


def cast_block(fmt, values):
    q, s = oracle.mx_direct_cast(fmt, bf16_bits(values).reshape(1, 32))
    assert q.shape == (1, BITS[fmt] * 4)
    return unpack(fmt, q[0]), int(s[0, 0])


def nearest_even(fmt, r: Fraction) -> int:
    """Brute force in exact rationals: nearest magnitude, a tie to the even code, saturate at the top."""
    g = GRIDS[fmt]
    best = min(range(len(g)), key=lambda c: (abs(r - g[c]), c % 2))
    return best


@pytest.mark.parametrize("fmt", FORMATS)
def test_grid_from_field_widths(fmt):
    g = GRIDS[fmt]
    assert [oracle.mx_magnitude(fmt, c) for c in range(len(g))] == [float(v) for v in g]
    assert oracle.mx_block_bytes(fmt) == BITS[fmt] * 4
    assert float(g[-1]) == {E5M2: 57344.0, E3M2: 28.0, T2: 1.0}[fmt]
    # the largest power of two of the format is 2^emax
    assert max(v for v in g if v.numerator == 1 or v.denominator == 1 and (v.numerator & (v.numerator - 1)) == 0
               ) == Fraction(2) ** EMAX[fmt]


def test_packing_is_the_stated_bit_string():
    vals = np.zeros(32)
    vals[0], vals[1], vals[2], vals[31] = 1.0, -1.0, 0.5, -0.75        # amax 1: T2 scale byte 127
    got, sc = cast_block(T2, vals)
    # codes: +1 -> 1, -1 -> 3, 0.5 is the tie -> 0, -0.75 -> sign | 1 = 3
    assert sc == 127 and got[:3] == [1, 3, 0] and got[31] == 3 and not any(got[3:31])
    q, _ = oracle.mx_direct_cast(T2, bf16_bits(vals).reshape(1, 32))
    assert int.from_bytes(bytes(q[0].tolist()), "little") == (1 | (3 << 2) | (3 << 62))
    vals = np.zeros(32)
    vals[0], vals[1], vals[31] = 16.0, -28.0, 0.03125                   # E3M2: amax 28 -> scale byte 127
    got, sc = cast_block(E3M2, vals)
    # 16 = 2^(7-3): exponent field 7, mantissa 0; 28 is the top code; 1/32 is the tie between 0 and the
    # smallest subnormal 2^(1-3) / 4 = 1/16 and goes to the even code 0
    assert sc == 127 and got[0] == (7 << 2) and got[1] == 32 | 31 and got[31] == 0
    vals[31] = 0.09375                                                  # the tie between codes 1 and 2
    got, _ = cast_block(E3M2, vals)
    assert got[31] == 2
    q, _ = oracle.mx_direct_cast(E3M2, bf16_bits(vals).reshape(1, 32))
    assert int.from_bytes(bytes(q[0].tolist()), "little") == (28 | (63 << 6) | (2 << 186))


@pytest.mark.parametrize("fmt", FORMATS)
def test_every_code_point_round_trips(fmt):
    g = GRIDS[fmt]
    top = float(g[-1])
    for j in (-60, -7, 0, 9, 50):
        for lo in range(0, len(g), 24):
            codes = list(range(lo, min(lo + 24, len(g))))
            vals = np.zeros(32)
            vals[:len(codes)] = [float(g[c]) * (-1.0) ** c for c in codes]
            vals[31] = top                                  # fixes floor(log2 amax) = emax
            got, sc = cast_block(fmt, vals * 2.0 ** j)
            assert sc == j + 127, (fmt, j, sc)
            sign = 1 << (BITS[fmt] - 1)
            assert got[:len(codes)] == [c | (sign if c % 2 else 0) for c in codes]
            q, s = oracle.mx_direct_cast(fmt, bf16_bits(vals * 2.0 ** j).reshape(1, 32))
            assert np.array_equal(oracle.mx_dequant(fmt, q, s)[0], vals * 2.0 ** j)


@pytest.mark.parametrize("fmt", [E5M2, E3M2])
def test_midpoints_neighbours_and_saturation_against_exact_rationals(fmt):
    g = GRIDS[fmt]
    top = g[-1]
    # every BF16 value between two neighbouring magnitudes that fits 8 significant bits, for a few binades
    rng = np.random.default_rng(5)
    cands = []
    for c in range(len(g) - 1):
        mid = (g[c] + g[c + 1]) / 2
        cands += [mid, g[c], g[c + 1]]
    for r in cands:
        f = float(r)
        if f == 0.0 or r > top:
            continue
        # representable in BF16?
        u = np.float32(f).view(np.uint32)
        if u & 0xFFFF:
            continue
        for E in (-30, 0, 20):
            vals = np.zeros(32)
            vals[0] = float(top)
            vals[1] = f
            vals[2] = -f
            got, sc = cast_block(fmt, vals * 2.0 ** E)
            assert sc == E + 127
            want = nearest_even(fmt, r)
            assert got[1] == want and got[2] == want | (1 << (BITS[fmt] - 1)), (fmt, f, got[1], want)
    # random BF16 values under a fixed block maximum: brute force in rationals
    vals = (rng.standard_normal(31) * float(top) / 3).astype(np.float32)
    vals = (vals.view(np.uint32) & 0xFFFF0000).view(np.float32)
    block = np.concatenate([[float(top)], np.clip(vals, -float(top), float(top))]).astype(np.float32)
    got, sc = cast_block(fmt, block)
    assert sc == 127
    for i in range(32):
        r = Fraction(float(abs(block[i])))
        assert got[i] & ((1 << (BITS[fmt] - 1)) - 1) == nearest_even(fmt, r), (fmt, i, block[i])
    # saturation band: amax in (top, 2^(emax+1)) keeps the scale and clamps to the top code
    for mult in (1.03125, 1.0625, 1.125):
        vals = np.zeros(32)
        vals[4], vals[5] = float(top) * mult, -float(top) * mult
        got, sc = cast_block(fmt, vals)
        assert sc == 127 and got[4] == len(g) - 1 and got[5] == (len(g) - 1) | (1 << (BITS[fmt] - 1))


def test_e5m2_against_a_library_float8_conversion():
    # in-range values under a block maximum of 57344 (scale byte 127: X = 1): the library's
    # round-to-nearest-even conversion gives the same codes
    rng = np.random.default_rng(11)
    for scale in (1.0, 2.0 ** -9, 2.0 ** 3):
        mags = np.abs(rng.standard_normal(31) * 8000.0 * scale).astype(np.float32)
        mags = (mags.view(np.uint32) & 0xFFFF0000).view(np.float32)
        vals = np.concatenate([[57344.0], np.minimum(mags, 57344.0)]).astype(np.float32)
        vals[1::2] *= -1.0
        got, sc = cast_block(E5M2, vals)
        assert sc == 127
        lib = torch.from_numpy(vals).to(torch.float8_e5m2).view(torch.uint8).numpy()
        assert got == [int(v) for v in lib]
        back = torch.from_numpy(lib.copy()).view(torch.float8_e5m2).to(torch.float64).numpy()
        q, s = oracle.mx_direct_cast(E5M2, bf16_bits(vals).reshape(1, 32))
        assert np.array_equal(oracle.mx_dequant(E5M2, q, s)[0], back)


def test_t2_closed_form_intervals():
    # X = 2^floor(log2 amax); |v| / X in [0, 1/2] -> 0 (1/2 is the tie), (1/2, 2) -> 1
    for E in (-20, 0, 13):
        for amax_m in (1.0, 1.5, 1.9921875):
            vals = np.zeros(32)
            vals[0] = amax_m
            probe = [0.5, 0.50390625, 0.49609375, 0.75, 1.0, 0.25, 0.0, 0.001953125]
            vals[1:1 + len(probe)] = probe
            vals[20:20 + len(probe)] = [-p for p in probe]
            got, sc = cast_block(T2, vals * 2.0 ** E)
            assert sc == E + 127 and got[0] == 1
            want = [0, 1, 0, 1, 1, 0, 0, 0]
            assert got[1:1 + len(probe)] == want
            assert got[20:20 + len(probe)] == [w | 2 for w in want]


@pytest.mark.parametrize("fmt", FORMATS)
def test_scale_rule_zero_blocks_and_non_finite_inputs(fmt):
    e = EMAX[fmt]
    for amax, fl in [(1.0, 0), (3.984375, 1), (4.0, 2), (2.0 ** -100, -100), (2.0 ** 127, 127)]:
        vals = np.zeros(32)
        vals[17] = -amax
        _, sc = cast_block(fmt, vals)
        assert sc == max(fl - e, -127) + 127, (fmt, amax, sc)
    got, sc = cast_block(fmt, np.zeros(32))
    assert sc == 0 and not any(got)
    neg_zero = np.zeros(32, np.float32)
    neg_zero[3] = -0.0
    got, _ = cast_block(fmt, neg_zero)
    assert got[3] == 1 << (BITS[fmt] - 1)
    w = bf16_bits(np.ones(32)).copy()
    w[9] = 0x7F80                                       # +Inf
    q, s = oracle.mx_direct_cast(fmt, w.reshape(1, 32))
    assert s[0, 0] == 0xFF and not q.any() and np.all(np.isnan(oracle.mx_dequant(fmt, q, s)))
    # a power of two moves the scale byte and nothing else; a sign flip moves the sign bits only
    v = synth.weights_student_t(1, 32, seed=3)
    vb = bits_value(synth.to_bits(v))[0]
    q0, s0 = oracle.mx_direct_cast(fmt, bf16_bits(vb).reshape(1, 32))
    q1, s1 = oracle.mx_direct_cast(fmt, bf16_bits(vb * 2.0 ** 11).reshape(1, 32))
    assert np.array_equal(q0, q1) and int(s1[0, 0]) == int(s0[0, 0]) + 11
    q2, s2 = oracle.mx_direct_cast(fmt, bf16_bits(-vb).reshape(1, 32))
    sign = 1 << (BITS[fmt] - 1)
    assert np.array_equal(s2, s0) and unpack(fmt, q2[0]) == [c ^ sign for c in unpack(fmt, q0[0])]


@pytest.mark.parametrize("fmt", FORMATS)
def test_product_against_a_library_matmul_on_a_decode_table_built_here(fmt):
    m, n, k = 5, 37, 192
    w = synth.weights_student_t(n, k, seed=5)
    x = synth.activations_outlier_channels(m, k, seed=6)
    q, s = oracle.mx_direct_cast(fmt, synth.to_bits(w))
    g = [float(v) for v in GRIDS[fmt]]
    pad = (1 << (BITS[fmt] - 1)) - len(g)               # E5M2: the Inf/NaN codes, never produced
    table = np.array(g + [np.nan] * pad + [-v for v in g] + [np.nan] * pad)
    bb = BITS[fmt] * 4
    codes = np.array([[c for b in range(k // 32) for c in unpack(fmt, q[r, bb * b:bb * b + bb])] for r in range(n)])
    X = 2.0 ** (s.astype(np.float64) - 127).repeat(32, axis=1)
    w_here = table[codes] * X
    assert not np.isnan(w_here).any()
    assert np.array_equal(oracle.mx_dequant(fmt, q, s), w_here)
    y, a = oracle.mx_woq_gemm(fmt, synth.to_bits(x), q, s)
    y_lib = (x.double() @ torch.from_numpy(w_here).T).numpy()
    a_lib = (x.double().abs() @ torch.from_numpy(np.abs(w_here)).T).numpy()
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)
    # error bound of the cast: half a quantum of the value's binade, one X below the smallest normal
    v = bits_value(synth.to_bits(w))
    assert np.all(np.abs(w_here - v) <= np.maximum(np.abs(v), X) * {E5M2: 0.125, E3M2: 0.125, T2: 0.5}[fmt] + 1e-300)
