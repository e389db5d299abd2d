"""Pins for the oracle's fused epilogue (bias, gated activation, residual add around the
contraction; arXiv 2503.13565, section 3.4 for the fusion, sections 4.2 and 4.3 for the gated-MLP
targets).  Values that do not come from the oracle: closed forms of the logistic function, a
library FP64 silu on de-interleaved columns, the odd-part identity, additivity with a padded
non-square layout, and a numeric maximum of the slope used in the error scale.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from test_oracle_gemm import f64_to_bf16_bits


def bits(a):
    """BF16 bit patterns of values that are exactly representable."""
    b = f64_to_bf16_bits(np.asarray(a, np.float64))
    back = (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(back, np.asarray(a, np.float64)), "test value is not a BF16 number"
    return b


def test_no_option_is_the_identity():
    rng = np.random.default_rng(0)
    y = rng.standard_normal((3, 10))
    a = np.abs(rng.standard_normal((3, 10))) + 1
    out, a_out = oracle.epilogue(y, a)
    assert np.array_equal(out, y) and np.array_equal(a_out, a)


def test_bias_goes_by_column_and_residual_by_element_with_a_padded_stride():
    m, n = 3, 5                                       # non-square: a transposed index fails
    y = np.arange(m * n, dtype=np.float64).reshape(m, n) * 0.25
    a = np.full((m, n), 2.0)
    bias = np.array([1.0, -2.0, 0.5, 4.0, -8.0])
    res_padded = np.full((m, n + 3), 77.0)            # the padding must never be read
    res = np.array([[0.5, 1.5, -2.5, 3.0, -4.0], [8.0, -16.0, 32.0, -64.0, 128.0], [0.0, 0.125, -0.25, 0.375, 1.0]])
    res_padded[:, :n] = res
    rb = bits(res_padded)[:, :n]
    assert rb.strides[0] == 2 * (n + 3)
    out, a_out = oracle.epilogue(y, a, bias_bits=bits(bias), residual_bits=rb)
    assert np.array_equal(out, y + bias[None, :] + res)
    assert np.array_equal(a_out, a + np.abs(bias)[None, :] + np.abs(res))
    out_b, _ = oracle.epilogue(y, a, bias_bits=bits(bias))
    assert np.array_equal(out_b, y + bias[None, :])
    out_r, _ = oracle.epilogue(y, a, residual_bits=np.ascontiguousarray(rb))
    assert np.array_equal(out_r, y + res)


def test_gate_closed_forms():
    # sigma(ln 3) = 3/4, sigma(-ln 3) = 1/4, sigma(0) = 1/2, sigma(ln 7) = 7/8
    g = np.array([math.log(3.0), -math.log(3.0), 0.0, math.log(7.0), 1.0])
    u = np.array([2.0, -4.0, 123.0, 0.5, 1.0])
    want = np.array([math.log(3.0) * 0.75 * 2.0, -math.log(3.0) * 0.25 * -4.0, 0.0, math.log(7.0) * 0.875 * 0.5,
                     0.7310585786300049])          # the last: 1 / (1 + 1/e), a tabulated constant
    y = np.empty((1, 10))
    y[0, 0::2] = g
    y[0, 1::2] = u
    out, _ = oracle.epilogue(y, np.abs(y), act=oracle.ACT_SWIGLU)
    assert out.shape == (1, 5)
    np.testing.assert_allclose(out[0], want, rtol=1e-15, atol=0)


def test_gate_saturates_and_never_overflows():
    y = np.array([[800.0, 3.0, -800.0, 3.0, 40.0, -2.0, -40.0, 5.0]])
    out, a_out = oracle.epilogue(y, np.abs(y), act=oracle.ACT_SWIGLU)
    assert out[0, 0] == 2400.0                        # silu(v) -> v
    assert out[0, 1] == 0.0 or abs(out[0, 1]) < 1e-300    # silu(v) -> 0-
    assert abs(out[0, 2] - -80.0) < 1e-14 and abs(out[0, 3]) < 1e-14
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(a_out))


def test_gate_against_library_silu_on_deinterleaved_columns():
    rng = np.random.default_rng(5)
    m, f = 4, 33
    y = rng.standard_normal((m, 2 * f)) * 3.0
    bias = np.round(rng.standard_normal(2 * f) * 8) / 8           # BF16-exact
    res = np.round(rng.standard_normal((m, f)) * 16) / 16
    a = np.abs(y) * 1.5
    out, _ = oracle.epilogue(y, a, bias_bits=bits(bias), residual_bits=bits(res), act=oracle.ACT_SWIGLU)
    z = torch.from_numpy(y + bias[None, :])
    want = (torch.nn.functional.silu(z[:, 0::2]) * z[:, 1::2]).numpy() + res
    np.testing.assert_allclose(out, want, rtol=1e-14, atol=1e-15)


def test_odd_part_of_the_gate_is_the_identity():
    # silu(v) - silu(-v) = v: with up = 1, out(v) - out(-v) = v
    v = np.linspace(-30, 30, 241)
    y = np.empty((2, 2 * v.size))
    y[0, 0::2], y[1, 0::2] = v, -v
    y[:, 1::2] = 1.0
    out, _ = oracle.epilogue(y, np.abs(y), act=oracle.ACT_SWIGLU)
    np.testing.assert_allclose(out[0] - out[1], v, rtol=0, atol=1e-14)


def test_error_scale_bounds_a_perturbed_product():
    """a_out is an upper bound: perturb z by e * A (any signs) and the result moves by at most
    e * a_out, also where the slope of the gate is largest."""
    rng = np.random.default_rng(9)
    m, f = 6, 200
    y = rng.standard_normal((m, 2 * f)) * 4.0
    y[0, 0::2] = 2.3993572805154676                   # argmax of silu'
    a = np.abs(y) + np.abs(rng.standard_normal((m, 2 * f))) * 5.0
    res = np.round(rng.standard_normal((m, f)) * 16) / 16
    out, a_out = oracle.epilogue(y, a, residual_bits=bits(res), act=oracle.ACT_SWIGLU)
    e = 1e-3
    for trial in range(8):
        sign = rng.choice([-1.0, 1.0], size=y.shape)
        out_p, _ = oracle.epilogue(y + sign * e * a, a, residual_bits=bits(res), act=oracle.ACT_SWIGLU)
        assert np.all(np.abs(out_p - out) <= e * (a_out - np.abs(res)) * (1 + 1e-12))
    # the slope constant: a numeric maximum of the central difference of a library silu
    v = torch.linspace(2.0, 3.0, 2000001, dtype=torch.float64)
    s = torch.nn.functional.silu(v)
    slope = ((s[2:] - s[:-2]) / (v[2:] - v[:-2])).max().item()
    out1, a1 = oracle.epilogue(np.array([[0.0, 1.0]]), np.array([[1.0, 0.0]]), act=oracle.ACT_SWIGLU)
    assert abs(a1[0, 0] - slope) < 1e-7               # a_out = L * A_g * |z_u| here


def test_rejects_odd_width_for_the_gate_and_short_residual_stride():
    with pytest.raises(RuntimeError):
        oracle.epilogue(np.zeros((1, 3)), np.zeros((1, 3)), act=oracle.ACT_SWIGLU)
    with pytest.raises(ValueError):
        oracle.epilogue(np.zeros((2, 4)), np.zeros((2, 4)), residual_bits=np.zeros((2, 3), np.uint16))
