"""Pins for the oracle's BF16-weight product (the target model's unquantised linear layer;
arXiv 2503.13565, section 3.2 for who runs it, section 3.4.3 for its role as the byte yardstick).
A library FP64 matmul on the exact BF16 values, closed forms that catch a transposed operand or
a stride mistake, and the quantised product on weights the cast represents exactly.
"""
import numpy as np
import torch

import oracle
from paper_2503_13565_amd import synth
from test_oracle_gemm import on_grid_weights, f64_to_bf16_bits


def test_matches_library_fp64_matmul():
    m, n, k = 5, 37, 200                             # ragged, K not a multiple of 32
    x = synth.activations_outlier_channels(m, k, seed=1)
    w = synth.weights_student_t(n, k, seed=2)
    y, a = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    y_lib = torch.matmul(x.double(), w.double().T).numpy()
    a_lib = torch.matmul(x.double().abs(), w.double().abs().T).numpy()
    assert y.shape == (m, n)
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)


def test_one_hot_rows_pick_single_weights_and_columns_are_not_transposed():
    n, k = 7, 40
    w = synth.weights_gaussian_outliers(n, k, seed=3)
    x = torch.zeros((3, k), dtype=torch.bfloat16)
    x[0, 5] = 1.0
    x[1, 39] = -2.0
    x[2, 0] = 0.5
    y = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w), want_abs=False)
    wd = w.double().numpy()
    assert np.array_equal(y[0], wd[:, 5])
    assert np.array_equal(y[1], -2.0 * wd[:, 39])
    assert np.array_equal(y[2], 0.5 * wd[:, 0])


def test_all_ones_gives_row_sums_in_index_order():
    n, k = 4, 64
    w = torch.arange(n * k, dtype=torch.float32).reshape(n, k).remainder(17).sub(8).to(torch.bfloat16)
    x = torch.ones((1, k), dtype=torch.bfloat16)
    y, a = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    assert np.array_equal(y[0], w.double().sum(dim=1).numpy())
    assert np.array_equal(a[0], w.double().abs().sum(dim=1).numpy())


def test_agrees_with_quantised_product_when_the_cast_is_exact():
    rng = np.random.default_rng(4)
    n, k, m = 21, 96, 3
    w, _, _ = on_grid_weights(rng, n, k)
    wb = f64_to_bf16_bits(w)
    q, s = oracle.direct_cast(wb)
    x = synth.to_bits(synth.activations_gaussian(m, k, seed=5))
    y_q, a_q = oracle.woq_gemm(x, q, s)
    y_b, a_b = oracle.bf16_gemm(x, wb)
    assert np.array_equal(y_q, y_b) and np.array_equal(a_q, a_b)


def test_quantisation_error_of_the_product_is_within_the_format_bound():
    # |w - w_hat| <= amax_block / 2 elementwise (section 3.4.3's rounding), hence
    # |y_bf16 - y_mxfp4| <= sum_k |x_k| * amax_block(k) / 2
    n, k, m = 16, 256, 2
    w = synth.weights_student_t(n, k, seed=6)
    xb = synth.activations_gaussian(m, k, seed=7)
    q, s = oracle.direct_cast(synth.to_bits(w))
    y_q = oracle.woq_gemm(synth.to_bits(xb), q, s, want_abs=False)
    y_b = oracle.bf16_gemm(synth.to_bits(xb), synth.to_bits(w), want_abs=False)
    amax = w.double().abs().reshape(n, k // 32, 32).amax(dim=2).repeat_interleave(32, dim=1)
    bound = torch.matmul(xb.double().abs(), (amax / 2).T).numpy()
    assert np.all(np.abs(y_q - y_b) <= bound + 1e-12)
    assert np.abs(y_q - y_b).max() > 0
