"""Pins for the CPU oracle's dequantisation, FP64 product and argmax (arXiv 2503.13565,
section 3.4.3, Eq. 2).  The product is pinned by the special case where the weights already
lie on the MXFP4 grid: then dequant(cast(W)) == W exactly and the oracle must agree with a
library FP64 matmul on W itself.  One-hot and all-ones activations give closed forms that
catch a transposed operand, a wrong nibble order or a dropped scale.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import synth

GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def on_grid_weights(rng, n, k, e_lo=110, e_hi=130):
    """Random E2M1 codes times a random power of two per 32-block; every block holds a 4 or
    a 6 so that the cast reproduces its scale.  Returns (values float64 [n,k], codes, bytes)."""
    codes = rng.integers(0, 16, size=(n, k))
    nblk = k // 32
    top = rng.integers(6, 8, size=(n, nblk)) | (rng.integers(0, 2, size=(n, nblk)) << 3)
    pos = rng.integers(0, 32, size=(n, nblk))
    c3 = codes.reshape(n, nblk, 32)
    np.put_along_axis(c3, pos[..., None], top[..., None], axis=2)
    codes = c3.reshape(n, k)
    sb = rng.integers(e_lo, e_hi, size=(n, nblk))
    mag = GRID[codes & 7] * np.where(codes & 8, -1.0, 1.0)
    vals = mag * np.ldexp(1.0, sb - 127).repeat(32, axis=1)
    return vals, codes.astype(np.uint8), sb.astype(np.uint8)


def f64_to_bf16_bits(v):
    t = torch.from_numpy(np.asarray(v, np.float64)).to(torch.float32)
    b = t.to(torch.bfloat16)
    assert torch.equal(b.to(torch.float64), torch.from_numpy(np.asarray(v, np.float64))), "not BF16-exact"
    return synth.to_bits(b)


def test_on_grid_weights_survive_cast_and_match_library_matmul():
    rng = np.random.default_rng(0)
    n, k, m = 37, 96 * 2, 5                      # N != K, several blocks, ragged sizes
    w, codes, sb = on_grid_weights(rng, n, k)
    q, s = oracle.direct_cast(f64_to_bf16_bits(w))
    assert np.array_equal(s, sb)
    assert np.array_equal(q, (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8))
    assert np.array_equal(oracle.dequant(q, s), w)
    x = synth.activations_outlier_channels(m, k, seed=3)
    y, a = oracle.woq_gemm(synth.to_bits(x), q, s)
    y_lib = torch.matmul(x.to(torch.float64), torch.from_numpy(w).T).numpy()
    a_lib = torch.matmul(x.to(torch.float64).abs(), torch.from_numpy(np.abs(w)).T).numpy()
    assert y.shape == (m, n)
    np.testing.assert_allclose(y, y_lib, rtol=0, atol=1e-12 * a_lib.max())
    np.testing.assert_allclose(a, a_lib, rtol=1e-13)
    assert np.all(a >= np.abs(y) - 1e-12 * a)


def test_one_hot_activation_reads_single_weights():
    rng = np.random.default_rng(1)
    n, k = 9, 128
    w, codes, sb = on_grid_weights(rng, n, k)
    q, s = oracle.direct_cast(f64_to_bf16_bits(w))
    for kk in (0, 1, 31, 32, 33, 126, 127):
        x = np.zeros((2, k))
        x[0, kk] = 1.0
        x[1, kk] = -2.0
        y, a = oracle.woq_gemm(f64_to_bf16_bits(x), q, s)
        assert np.array_equal(y[0], w[:, kk])
        assert np.array_equal(y[1], -2.0 * w[:, kk])
        assert np.array_equal(a[1], 2.0 * np.abs(w[:, kk]))


def test_explicit_bytes_dequantise_by_hand():
    # q byte 0x72: element 0 = code 2 (1.0), element 1 = code 7 (6.0); 0xB9: 0.5 with sign, 1.5 with sign
    q = np.zeros((1, 16), np.uint8)
    q[0, 0] = 0x72
    q[0, 1] = 0xB9
    s = np.array([[129]], np.uint8)                              # 2^2
    wh = oracle.dequant(q, s)[0]
    assert wh[:4].tolist() == [4.0, 24.0, -2.0, -6.0] and not wh[4:].any()
    x = np.zeros((1, 32))
    x[0, :4] = [1.0, 0.5, 3.0, -1.0]
    y, a = oracle.woq_gemm(f64_to_bf16_bits(x), q, s)
    assert y[0, 0] == 4.0 + 12.0 - 6.0 + 6.0 and a[0, 0] == 4.0 + 12.0 + 6.0 + 6.0


def test_all_ones_activation_block_constant_weights():
    n, k = 4, 96
    w = np.zeros((n, k))
    for r in range(n):
        for b in range(3):
            w[r, 32 * b: 32 * b + 32] = GRID[6] * 2.0 ** (r - b)     # 4 * 2^(r-b)
    q, s = oracle.direct_cast(f64_to_bf16_bits(w))
    y, _ = oracle.woq_gemm(f64_to_bf16_bits(np.ones((1, k))), q, s)
    want = [32 * 4.0 * sum(2.0 ** (r - b) for b in range(3)) for r in range(n)]
    assert y[0].tolist() == want


def test_late_scaling_identity_eq2():
    # scf * sum(w_i a_i) == sum(scf w_i a_i): exact in FP64 because scf is a power of two
    data = synth.llama_linear(synth.ModelShape("tiny", 256, 64, 256, 48, 1), "down", m=3, seed=5)
    q, s = oracle.direct_cast(synth.to_bits(data["w"]))
    xb = synth.to_bits(data["x"])
    y_early = oracle.woq_gemm(xb, q, s, want_abs=False)
    y_late = oracle.woq_gemm_late_scaled(xb, q, s)
    # per-block partial sums are rounded at a different point, so agreement is to FP64 round-off
    np.testing.assert_allclose(y_late, y_early, rtol=0, atol=1e-13 * np.abs(y_early).max())
    # with a single block per row the two orders are the same sum and must agree exactly
    w1 = synth.weights_student_t(8, 32, seed=9)
    q1, s1 = oracle.direct_cast(synth.to_bits(w1))
    x1 = synth.to_bits(synth.activations_gaussian(2, 32, seed=10))
    assert np.array_equal(oracle.woq_gemm(x1, q1, s1, want_abs=False),
                          oracle.woq_gemm_late_scaled(x1, q1, s1))


def test_threads_do_not_change_results():
    data = synth.llama_linear(synth.ModelShape("tiny", 128, 96, 128, 100, 1), "lm_head", m=4, seed=2)
    wb, xb = synth.to_bits(data["w"]), synth.to_bits(data["x"])
    q1, s1 = oracle.direct_cast(wb, threads=1)
    q4, s4 = oracle.direct_cast(wb, threads=4)
    assert np.array_equal(q1, q4) and np.array_equal(s1, s4)
    y1, a1 = oracle.woq_gemm(xb, q1, s1, threads=1)
    y4, a4 = oracle.woq_gemm(xb, q1, s1, threads=4)
    assert np.array_equal(y1, y4) and np.array_equal(a1, a4)


def test_quantised_product_is_close_to_the_unquantised_one():
    # sanity of the whole chain on config-0-like data: relative error of the MXFP4 product
    # against the BF16-weight product is a few percent of sum |x w|, never more than 1/2
    g = torch.Generator().manual_seed(0)
    w = synth.weights_gaussian_outliers(64, 512, gen=g)
    x = synth.activations_gaussian(2, 512, gen=g)
    q, s = oracle.direct_cast(synth.to_bits(w))
    y, a = oracle.woq_gemm(synth.to_bits(x), q, s)
    y_bf16 = torch.matmul(x.double(), w.double().T).numpy()
    a_bf16 = torch.matmul(x.double().abs(), w.double().abs().T).numpy()
    assert np.all(np.abs(y - y_bf16) <= 0.5 * a_bf16)
    assert np.abs(y - y_bf16).mean() < 0.05 * a_bf16.mean()


def test_argmax_brute_force_ties_and_planted_max():
    rng = np.random.default_rng(11)
    y = rng.standard_normal((6, 50))
    y[1, 17] = 9.0
    y[2, 40] = y[2, 3] = 7.5                      # exact tie -> lowest index
    y[3, :] = -1.0                                # all equal -> index 0
    y[4, 49] = 5.0                                # last column
    idx, val = oracle.argmax(y)
    for m in range(6):
        best = max(range(50), key=lambda n: (y[m, n], -n))
        assert idx[m] == best and val[m] == y[m, best]
    assert idx[1] == 17 and idx[2] == 3 and idx[3] == 0 and idx[4] == 49


def test_tolerance_terms():
    assert oracle.bf16_ulp(1.0) == 2.0 ** -7
    assert oracle.bf16_ulp(1.999) == 2.0 ** -7
    assert oracle.bf16_ulp(-2.0) == 2.0 ** -6
    assert oracle.bf16_ulp(0.75) == 2.0 ** -8
    assert oracle.bf16_ulp(0.0) == 2.0 ** -133
    # BF16 subnormals m * 2^-133, m = 1 .. 127, are 2^-133 apart; the first normal binade too
    assert oracle.bf16_ulp(2.0 ** -133) == 2.0 ** -133 and oracle.bf16_ulp(1.5e-40) == 2.0 ** -133
    assert oracle.bf16_ulp(127 * 2.0 ** -133) == 2.0 ** -133 and oracle.bf16_ulp(2.0 ** -126) == 2.0 ** -133
    assert oracle.bf16_ulp(2.0 ** -125) == 2.0 ** -132
    assert torch.tensor([1.5 * 2.0 ** -133], dtype=torch.float64).to(torch.bfloat16).double().item() == 2.0 ** -132
    t = oracle.tolerance(np.array([1.0]), np.array([10.0]))
    assert t[0] == 1e-2 + 2.0 ** -7


def test_shape_errors():
    with pytest.raises(ValueError):
        oracle.woq_gemm(np.zeros((1, 64), np.uint16), np.zeros((2, 16), np.uint8), np.zeros((2, 1), np.uint8))
    with pytest.raises(ValueError):
        oracle.dequant(np.zeros((2, 16), np.uint8), np.zeros((2, 2), np.uint8))
