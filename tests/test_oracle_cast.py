"""Pins for the CPU oracle's direct cast (arXiv 2503.13565, section 3.4.3).

No reference implementation exists, so the oracle is pinned against what the
section and the arithmetic fix: the E2M1 grid from its field widths, the scale
rule floor(log2 amax) - 2, hand-written decision points of round-to-nearest-even
(tests/golden), an independent interval table in exact rational arithmetic, an
integer form on BF16 bit patterns, and invariants (power-of-two scaling, sign,
permutation, idempotence, error bound).  None of the expected values below is
computed by the oracle.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


# ----------------------------------------------------------------------------------------
# helpers that restate BF16 and the rule independently of the oracle
# ----------------------------------------------------------------------------------------
def bf16_bits(values) -> np.ndarray:
    """float values that are exactly BF16-representable -> their 16-bit patterns."""
    f = np.asarray(values, dtype=np.float32)
    u = f.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not representable in BF16"
    return (u >> 16).astype(np.uint16)


def bits_value(bits) -> np.ndarray:
    return (np.asarray(bits, np.uint32) << 16).view(np.float32).astype(np.float64)


def nibbles_of(q_row: np.ndarray) -> np.ndarray:
    """Unpack bytes: element 2j = low nibble of byte j, element 2j+1 = high nibble."""
    out = np.empty(q_row.size * 2, np.uint8)
    out[0::2] = q_row & 0xF
    out[1::2] = q_row >> 4
    return out


def interval_code(r: Fraction) -> int:
    """Decision intervals of round-to-nearest, ties to the even code, saturating."""
    F = Fraction
    if r <= F(1, 4):
        return 0
    if r < F(3, 4):
        return 1
    if r <= F(5, 4):
        return 2
    if r < F(7, 4):
        return 3
    if r <= F(5, 2):
        return 4
    if r < F(7, 2):
        return 5
    if r <= 5:
        return 6
    return 7


def integer_form(mag_bits: int, scale_byte: int) -> int:
    """Code from the 15 magnitude bits of a BF16 and the block's scale byte, in integers
    only: r*4 = significand * 2^(exp_eff - 5 - scale_byte)... compared against the
    quarter-unit thresholds 1, 3, 5, 7, 10, 14, 20."""
    exp = mag_bits >> 7
    man = mag_bits & 0x7F
    sig = man if exp == 0 else (0x80 | man)
    exp_eff = max(exp, 1)
    sh = exp_eff - 5 - scale_byte          # r * 4 = sig * 2^sh
    num, den = (sig << sh, 1) if sh >= 0 else (sig, 1 << (-sh))
    # compare num/den with thresholds t: num <= t*den etc.
    if num <= 1 * den:
        return 0
    if num < 3 * den:
        return 1
    if num <= 5 * den:
        return 2
    if num < 7 * den:
        return 3
    if num <= 10 * den:
        return 4
    if num < 14 * den:
        return 5
    if num <= 20 * den:
        return 6
    return 7


def cast_block(values_bits):
    """Cast a single 32-element block given as bit patterns; returns (nibbles[32], scale)."""
    w = np.asarray(values_bits, np.uint16).reshape(1, 32)
    q, s = oracle.direct_cast(w)
    return nibbles_of(q[0]), int(s[0, 0])


# ----------------------------------------------------------------------------------------
# the grid
# ----------------------------------------------------------------------------------------
def test_grid_from_field_widths():
    assert [oracle.e2m1_magnitude(c) for c in range(8)] == GRID


def test_every_code_point_round_trips():
    # A block holding all 16 code values times 2^j (padded with zeros) casts to exactly
    # those codes with scale byte j + 127.
    signed = GRID + [-g for g in GRID]
    for j in range(-124, 125):
        vals = np.array(signed + [0.0] * 16, np.float64) * 2.0 ** j
        nib, sc = cast_block(bf16_bits(vals))
        assert sc == j + 127, (j, sc)
        expect = list(range(8)) + [8 + c for c in range(8)] + [0] * 16
        assert nib.tolist() == expect, j
        # and dequantisation gives the values back exactly
        q, s = oracle.direct_cast(bf16_bits(vals).reshape(1, 32))
        assert np.array_equal(oracle.dequant(q, s)[0], vals)


def test_golden_decision_points():
    pts = []
    for line in open(os.path.join(GOLDEN, "e2m1_decision_points.txt")):
        if line.startswith("#") or not line.strip():
            continue
        r, c = line.split()
        pts.append((float(r), int(c)))
    assert len(pts) >= 30
    for E in (-100, -3, 0, 5, 90):
        X = 2.0 ** E
        for r, code in pts:
            for sign in (1.0, -1.0):
                # amax = 4*X fixes the scale at X unless r itself is larger (r < 8 keeps
                # floor(log2 amax) = E + 2 either way)
                vals = np.zeros(32)
                vals[0] = 4.0 * X
                vals[7] = sign * r * X
                nib, sc = cast_block(bf16_bits(vals))
                assert sc == E + 127
                got = int(nib[7])
                want = code | (8 if sign < 0 else 0)
                if r == 0.0 and sign < 0:
                    want = 8                      # reading: -0.0 keeps its sign bit
                assert got == want, (E, r, sign, got, want)


# ----------------------------------------------------------------------------------------
# the scale
# ----------------------------------------------------------------------------------------
def test_scale_over_every_bf16_magnitude():
    # amax ranges over every finite BF16 magnitude; block = amax at a moving position
    mags = np.arange(0, 0x7F80, dtype=np.uint16)           # 0x7F80 = +Inf
    blocks = np.zeros((mags.size, 32), np.uint16)
    pos = np.arange(mags.size) % 32
    blocks[np.arange(mags.size), pos] = mags | ((np.arange(mags.size) & 1).astype(np.uint16) << 15)
    q, s = oracle.direct_cast(blocks)
    # integer form on the bit pattern
    expect_int = np.maximum((mags >> 7).astype(np.int64) - 2, 0)
    assert np.array_equal(s[:, 0].astype(np.int64), expect_int)
    # floor(log2 amax) - 2, through the math library, where no clamp applies
    vals = bits_value(mags)
    for i in range(1, mags.size, 37):
        E = math.floor(math.log2(vals[i])) - 2
        assert s[i, 0] == max(E, -127) + 127, (i, vals[i])
    # an unclamped non-zero block always holds a 6 (code 7) or 4 (code 6) at its amax
    nib = np.stack([nibbles_of(r) for r in q[::101]])
    codes_at_pos = nib[np.arange(nib.shape[0]), pos[::101]] & 7
    unclamped = (mags[::101] >> 7) >= 2
    assert np.all(np.isin(codes_at_pos[unclamped], (6, 7)))


def test_scale_uses_block_max_not_first_or_last():
    rng = np.random.default_rng(1)
    for _ in range(200):
        exps = rng.integers(100, 140, size=32)
        vals = np.ldexp(1.0 + rng.integers(0, 128, size=32) / 128.0, exps - 127)
        vals *= rng.choice([-1.0, 1.0], size=32)
        _, sc = cast_block(bf16_bits(vals))
        assert sc - 127 == math.floor(math.log2(np.abs(vals).max())) - 2


# ----------------------------------------------------------------------------------------
# rounding: exhaustive agreement of the oracle with two independent statements
# ----------------------------------------------------------------------------------------
def _blocks_for_amax_exp(ea: int, test_mags: np.ndarray) -> np.ndarray:
    """Blocks whose amax is the largest magnitude with biased exponent `ea` (so the scale
    byte is max(ea-2,0)) and whose other 31 slots hold the magnitudes under test."""
    amax = (ea << 7) | 0x7F
    n = (test_mags.size + 30) // 31
    pad = np.zeros(n * 31, np.uint16)
    pad[: test_mags.size] = test_mags
    blocks = np.empty((n, 32), np.uint16)
    blocks[:, 0] = amax
    blocks[:, 1:] = pad.reshape(n, 31)
    return blocks


@pytest.mark.parametrize("ea", list(range(0, 255)))
def test_rounding_near_every_scale(ea):
    # every magnitude within 7 binades below the block maximum, for every possible scale
    lo = max(ea - 7, 0) << 7
    hi = ((ea << 7) | 0x7F) + 1
    mags = np.arange(lo, hi, dtype=np.uint16)
    blocks = _blocks_for_amax_exp(ea, mags)
    q, s = oracle.direct_cast(blocks)
    e = max(ea - 2, 0)
    assert np.all(s == e)
    nib = np.stack([nibbles_of(r) for r in q])[:, 1:].reshape(-1)[: mags.size]
    for m, got in zip(mags.tolist(), nib.tolist()):
        r = Fraction(float(bits_value(m))) / (Fraction(2) ** (e - 127))
        assert got == interval_code(r) == integer_form(m, e), (ea, m, got)


@pytest.mark.parametrize("ea", [0, 1, 2, 3, 9, 127, 128, 200, 254])
def test_rounding_all_magnitudes_below_amax(ea):
    # all magnitudes not above the block maximum (most flush to zero far below it)
    hi = ((ea << 7) | 0x7F) + 1
    mags = np.arange(0, hi, dtype=np.uint16)
    blocks = _blocks_for_amax_exp(ea, mags)
    q, s = oracle.direct_cast(blocks)
    e = max(ea - 2, 0)
    nib = np.stack([nibbles_of(r) for r in q])[:, 1:].reshape(-1)[: mags.size]
    expect = np.array([integer_form(m, e) for m in mags.tolist()], np.uint8)
    assert np.array_equal(nib, expect)
    # spot-check the rational statement too
    for m in mags[:: max(1, mags.size // 500)].tolist():
        r = Fraction(float(bits_value(m))) / (Fraction(2) ** (e - 127))
        assert int(nib[m]) == interval_code(r)


def test_brute_force_nearest_on_tiny_blocks():
    # nearest grid point by exhaustive search in exact arithmetic, tie -> even code
    rng = np.random.default_rng(7)
    for _ in range(300):
        E = int(rng.integers(-20, 20))
        bits = rng.integers(0, 0x7F80, size=32).astype(np.uint16)
        # keep values within a few binades of each other so codes are not all zero
        exps = rng.integers(120 + E, 130 + E, size=32)
        bits = ((exps << 7) | (bits & 0x7F)).astype(np.uint16)
        bits |= (rng.integers(0, 2, size=32).astype(np.uint16) << 15)
        nib, sc = cast_block(bits)
        vals = bits_value(bits & 0x7FFF)
        assert sc - 127 == math.floor(math.log2(vals.max())) - 2
        X = Fraction(2) ** (sc - 127)
        for i in range(32):
            r = Fraction(float(vals[i])) / X
            cands = sorted(range(8), key=lambda c: (abs(r - Fraction(GRID[c])), c & 1))
            assert (int(nib[i]) & 7) == cands[0]
            assert (int(nib[i]) >> 3) == int(bits[i] >> 15)


# ----------------------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------------------
def _random_blocks(rng, n, spread=6, center=120):
    exps = rng.integers(center - spread, center + 1, size=(n, 32))
    man = rng.integers(0, 128, size=(n, 32))
    sign = rng.integers(0, 2, size=(n, 32))
    return ((sign << 15) | (exps << 7) | man).astype(np.uint16)


def test_power_of_two_invariance():
    rng = np.random.default_rng(2)
    w = _random_blocks(rng, 400)
    q0, s0 = oracle.direct_cast(w)
    for t in (-60, -7, -1, 1, 13, 90):
        wt = (w.astype(np.int32) + (t << 7)).astype(np.uint16)    # exponent field + t
        qt, st = oracle.direct_cast(wt)
        assert np.array_equal(qt, q0)
        assert np.array_equal(st.astype(np.int32), s0.astype(np.int32) + t)


def test_sign_symmetry_and_permutation():
    rng = np.random.default_rng(3)
    w = _random_blocks(rng, 300)
    q0, s0 = oracle.direct_cast(w)
    qn, sn = oracle.direct_cast(w ^ np.uint16(0x8000))
    assert np.array_equal(sn, s0)
    assert np.array_equal(qn, q0 ^ np.uint8(0x88))
    perm = rng.permutation(32)
    qp, sp = oracle.direct_cast(w[:, perm])
    assert np.array_equal(sp, s0)
    n0 = np.stack([nibbles_of(r) for r in q0])
    npm = np.stack([nibbles_of(r) for r in qp])
    assert np.array_equal(npm, n0[:, perm])


def test_idempotence_and_error_bound():
    import torch
    rng = np.random.default_rng(4)
    w = _random_blocks(rng, 500, spread=9)
    q, s = oracle.direct_cast(w)
    wh = oracle.dequant(q, s)
    # dequantised values are BF16-representable; casting them again changes nothing
    wh_bits = torch.from_numpy(wh.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits_value(wh_bits), wh)
    q2, s2 = oracle.direct_cast(wh_bits)
    assert np.array_equal(q2, q) and np.array_equal(s2, s)
    # |v - w_hat| <= X inside the grid's range, < 2X in the saturated band, <= amax/2 always
    v = bits_value(w)
    X = np.ldexp(1.0, s.astype(np.int32) - 127)
    err = np.abs(v - wh)
    r = np.abs(v) / X
    assert np.all(err[r <= 6] <= X.repeat(32, axis=1)[r <= 6] * 1.0)
    assert np.all(err[r > 6] < 2 * X.repeat(32, axis=1)[r > 6])
    amax = np.abs(v).max(axis=1, keepdims=True)
    assert np.all(err <= amax / 2)
    assert np.all(np.sign(wh) * np.sign(v) >= 0)


def test_zero_subnormal_and_nonfinite_blocks():
    z = np.zeros(32, np.uint16)
    nib, sc = cast_block(z)
    assert sc == 0 and not nib.any()
    z[5] = 0x8000                                   # -0.0 keeps its sign bit
    nib, sc = cast_block(z)
    assert sc == 0 and nib[5] == 8 and nib.sum() == 8
    # BF16 subnormal maximum: scale byte clamps to 0, X = 2^-127; 0x0040 = 2^-127 -> r = 1
    sub = np.zeros(32, np.uint16)
    sub[0] = 0x0040
    sub[1] = 0x0020                                 # 2^-128 -> r = 0.5
    sub[2] = 0x0010                                 # 2^-129 -> r = 0.25 -> tie to 0
    sub[3] = 0x007F                                 # (127/64) 2^-127 -> r = 1.984 -> 2 (code 4)
    nib, sc = cast_block(sub)
    assert sc == 0 and nib[:4].tolist() == [2, 1, 0, 4]
    for bad in (0x7F80, 0xFF80, 0x7FC0):            # +Inf, -Inf, NaN
        b = _random_blocks(np.random.default_rng(5), 1)[0]
        b[11] = bad
        nib, sc = cast_block(b)
        assert sc == 0xFF and not nib.any()
    q = np.zeros((1, 16), np.uint8)
    assert np.all(np.isnan(oracle.dequant(q, np.full((1, 1), 0xFF, np.uint8))))


def test_saturation_band():
    # amax/X lies in [4, 8): everything in (6, 8) saturates to 6, never wraps
    for man in range(0x40, 0x80):                   # 1.5 .. 1.992 times 4 -> r in [6, 8)
        b = np.zeros(32, np.uint16)
        b[3] = (130 << 7) | man                     # value (1+man/128)*8; X = 2, so r = value/2 in [6, 8)
        nib, sc = cast_block(b)
        assert sc == 130 - 2 and nib[3] == 7


def test_layout_and_byte_accounting():
    rng = np.random.default_rng(6)
    w = _random_blocks(rng, 3 * 4).reshape(3, 128)         # N=3, K=128 -> 4 blocks per row
    q, s = oracle.direct_cast(w)
    assert q.shape == (3, 64) and s.shape == (3, 4)
    assert q.nbytes + s.nbytes == 3 * 128 * 0.53125
    assert abs(2 / 0.53125 - 3.76) < 0.01                   # the paper's 3.76x byte reduction
    # blocks are along K: block b of row n only depends on w[n, 32b:32b+32]
    for n in range(3):
        for b in range(4):
            nib, sc = cast_block(w[n, 32 * b: 32 * b + 32])
            assert sc == s[n, b]
            assert np.array_equal(nibbles_of(q[n, 16 * b: 16 * b + 16]), nib)
    # explicit nibble order: element 0 = 1.0 (code 2), element 1 = -6.0 (code 15)
    blk = bf16_bits([1.0, -6.0] + [0.0] * 30)
    q1, s1 = oracle.direct_cast(blk.reshape(1, 32))
    assert q1[0, 0] == 0xF2 and s1[0, 0] == 127
    with pytest.raises(ValueError):
        oracle.direct_cast(np.zeros((2, 48), np.uint16))
