"""Pins for the oracle's product along the rows of a stored MXFP4 tensor (arXiv 2503.13565, section
5: a quantised attention cache as the next step; one token per row, blocks along the head dimension,
so the score side is the ordinary product and the value side contracts over the rows).  Expected
values come from one-hot inputs, a library FP64 matmul on the transpose of the pinned ordinary
product, and loops written out here; none is computed by the function under test."""
import numpy as np
import torch

import oracle
from paper_2503_13565_amd import synth
from test_oracle_cast import bf16_bits

E2M1 = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]      # section 3.4.3: the eight magnitudes of the element format


def decode_here(q, s):
    n, k = q.shape[0], q.shape[1] * 2
    out = np.empty((n, k))
    for r in range(n):
        for c in range(k):
            nib = (int(q[r, c // 2]) >> (4 * (c & 1))) & 0xF
            out[r, c] = (-1.0 if nib & 8 else 1.0) * E2M1[nib & 7] * 2.0 ** (int(s[r, c // 32]) - 127)
    return out


def test_one_hot_rows_pick_dequantised_rows_and_sums_add():
    w = synth.weights_student_t(40, 64, seed=2)
    q, s = oracle.direct_cast(synth.to_bits(w))
    table = decode_here(q, s)
    x = np.zeros((3, 40))
    x[0, 7], x[1, 39], x[2, 0], x[2, 5] = 1.0, -2.0, 0.5, 4.0
    y, a = oracle.woq_gemm_t(bf16_bits(x).reshape(3, 40), q, s)
    assert np.array_equal(y[0], table[7]) and np.array_equal(y[1], -2.0 * table[39])
    assert np.array_equal(y[2], 0.5 * table[0] + 4.0 * table[5])
    assert np.array_equal(a[2], 0.5 * np.abs(table[0]) + 4.0 * np.abs(table[5]))


def test_against_a_library_matmul_and_the_transpose_of_the_ordinary_product():
    n, k, m = 333, 128, 5
    w = synth.weights_student_t(n, k, seed=3)
    q, s = oracle.direct_cast(synth.to_bits(w))
    x = synth.activations_outlier_channels(m, n, seed=4)
    y, a = oracle.woq_gemm_t(synth.to_bits(x), q, s)
    eye = torch.eye(k, dtype=torch.bfloat16)
    d_t = oracle.woq_gemm(synth.to_bits(eye), q, s, want_abs=False)     # [k, n]: the dequantised tensor, transposed
    y_lib = x.double().numpy() @ d_t.T
    a_lib = np.abs(x.double().numpy()) @ np.abs(d_t.T)
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)
    assert np.array_equal(d_t.T, decode_here(q, s))


def test_loops_written_out_on_a_tiny_case_with_a_nan_block():
    w = synth.weights_student_t(6, 64, seed=5)
    q, s = oracle.direct_cast(synth.to_bits(w))
    s = s.copy()
    s[4, 1] = 0xFF
    x = synth.activations_outlier_channels(2, 6, seed=6)
    xb = synth.to_bits(x)
    xv = x.double().numpy()
    y, _ = oracle.woq_gemm_t(xb, q, s)
    table = decode_here(q, s)
    table[4, 32:] = np.nan
    for m in range(2):
        for c in range(64):
            want = 0.0
            for r in range(6):
                want += xv[m, r] * table[r, c]
            assert (np.isnan(want) and np.isnan(y[m, c])) or want == y[m, c]
    assert np.isnan(y[:, 32:]).all() and not np.isnan(y[:, :32]).any()
