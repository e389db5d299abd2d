"""GPU parity of the BF16-weight product (the target model's linear layer; arXiv 2503.13565,
section 3.2) against the CPU oracle, element by element, through the C ABI.

Bar: |y_gpu - y_ref| <= 1e-3 * sum_k |x_k w_k| + 1 BF16 ulp of |y_ref| (FP32 accumulation of exact
BF16 products in another order than the oracle's, then one rounding to BF16); argmax as for the
quantised product.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth
from helpers import DEV, assert_gemm_close, assert_argmax_ok

pytestmark = pytest.mark.gpu


def run_case(w, x, what, argmax=True):
    y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    wg, xg = w.to(DEV), x.to(DEV)
    y = binding.mxfp4_bf16_gemm(xg, wg)
    torch.cuda.synchronize()
    worst = assert_gemm_close(y, y_ref, a_ref, what)
    if argmax:
        idx, val = binding.mxfp4_bf16_gemm_argmax(xg, wg)
        torch.cuda.synchronize()
        assert_argmax_ok(idx, val, y_ref, a_ref, what + " argmax")
    return worst


@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 8, 9, 16, 19])
@pytest.mark.parametrize("n,k", [(1, 8), (3, 72), (17, 512), (33, 520), (250, 4096), (1030, 1024), (64, 11008),
                                 (20, 28672)])
def test_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=700 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=800 + m + k)
    run_case(w, x, "BF16 N=%d K=%d M=%d" % (n, k, m))


@pytest.mark.parametrize("n,k", [(2048, 8), (2049, 520), (2100, 4096), (2060, 2056), (2050, 5000), (2500, 8192),
                                 (2051, 8200)])
def test_decode_frame_shapes(n, k):
    # one activation row and enough weight rows: the decode-step kernel (K up to 8192, ragged and
    # whole steps of 512, odd N), and just beyond its range the general one
    w = synth.weights_student_t(n, k, seed=900 + n + k)
    x = synth.activations_outlier_channels(1, k, seed=950 + k)
    run_case(w, x, "BF16 decode frame N=%d K=%d" % (n, k))


def test_decode_frame_strided_weights_and_ties():
    n, k = 2100, 1024
    wbig = synth.weights_student_t(n, k + 64, seed=41)
    x = synth.activations_gaussian(1, k, seed=42)
    w = wbig[:, :k].contiguous()
    y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    best = int(np.argmax(y_ref[0]))
    for rows in ([7, 2099], [0, 1]):
        wt = wbig.clone()
        for r in rows:
            wt[r] = wbig[best]
        lo = min(rows + [best])
        wg = wt.to(DEV)[:, :k]                              # row stride k + 64
        idx, _ = binding.mxfp4_bf16_gemm_argmax(x.to(DEV), wg)
        y = binding.mxfp4_bf16_gemm(x.to(DEV), wg)
        torch.cuda.synchronize()
        assert int(idx[0]) == lo, (rows, best, int(idx[0]))
        y_t, a_t = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(wt[:, :k].contiguous()))
        assert_gemm_close(y, y_t, a_t, "BF16 decode frame strided")


@pytest.mark.parametrize("m", [3, 4, 5, 8, 9, 16, 17, 33])
@pytest.mark.parametrize("n,k", [(16, 128), (2050, 4096), (4100, 1024), (300, 8192), (530, 11008)])
def test_matrix_core_passes(n, k, m):
    # three and more rows with K % 128 == 0: the matrix-core kernel where a pass's rows fit the LDS
    w = synth.weights_student_t(n, k, seed=1000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=1050 + m + k)
    run_case(w, x, "BF16 matrix cores N=%d K=%d M=%d" % (n, k, m))


@pytest.mark.parametrize("n,k,m", [(2100, 28672, 8), (300, 11008, 8), (4100, 11008, 7), (70, 28672, 3),
                                   (2050, 20480, 16)])
def test_long_k_passes_in_phases(n, k, m):
    # the rows of a pass do not fit the LDS whole: K in phases, one pass over the weights
    w = synth.weights_student_t(n, k, seed=1100 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=1150 + m + k)
    run_case(w, x, "BF16 phased N=%d K=%d M=%d" % (n, k, m))


def test_matrix_core_exact_ties_pick_lowest_index():
    n, k, m = 600, 512, 4
    w = synth.weights_student_t(n, k, seed=51) * 0.1
    top = synth.weights_student_t(1, k, seed=52)
    x = top.clone().repeat(m, 1)
    for rows in ([5, 300, 599], [0, 1], [598, 599], [15, 16, 17]):
        wt = w.clone()
        wt[rows] = top
        idx, val = binding.mxfp4_bf16_gemm_argmax(x.to(DEV), wt.to(DEV))
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == [rows[0]] * m, (rows, idx)


@pytest.mark.parametrize("m", [1, 8])
def test_config0_shape(m):
    w = synth.weights_gaussian_outliers(4096, 4096, seed=0)
    x = synth.activations_gaussian(m, 4096, seed=1)
    run_case(w, x, "BF16 4096x4096 M=%d" % m)


def test_lm_head_shape_argmax_sampled_columns():
    # full size on the GPU; the oracle checks a seeded sample of columns and the picked column
    n, k, m = 32000, 4096, 4
    w = synth.weights_student_t(n, k, seed=11)
    x = synth.activations_outlier_channels(m, k, seed=12)
    wg, xg = w.to(DEV), x.to(DEV)
    y = binding.mxfp4_bf16_gemm(xg, wg)
    idx, val = binding.mxfp4_bf16_gemm_argmax(xg, wg)
    torch.cuda.synchronize()
    cols = np.unique(np.concatenate([np.random.default_rng(5).integers(0, n, 512), idx.cpu().numpy(),
                                     y.float().argmax(dim=1).cpu().numpy()]))
    y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w[cols]))
    assert_gemm_close(y[:, cols], y_ref, a_ref, "BF16 lm_head sampled")
    # the fused pick and the pick from the stored outputs agree up to the tolerance
    tol = oracle.tolerance(y_ref, a_ref)
    pos = {int(c): i for i, c in enumerate(cols)}
    for r in range(m):
        g, h = pos[int(idx[r])], pos[int(y[r].float().argmax())]
        assert y_ref[r, g] >= y_ref[r, h] - (tol[r, g] + tol[r, h])
        assert abs(float(val[r]) - y_ref[r, g]) <= 1e-3 * a_ref[r, g] + abs(y_ref[r, g]) * 2.0 ** -20


def test_strided_operands():
    n, k, m = 100, 512, 3
    wbig = synth.weights_student_t(n, k + 64, seed=21)
    xbig = synth.activations_gaussian(m, k + 32, seed=22)
    w, x = wbig[:, :k], xbig[:, :k]
    y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x.contiguous()), synth.to_bits(w.contiguous()))
    wg, xg = wbig.to(DEV)[:, :k], xbig.to(DEV)[:, :k]
    ybig = torch.zeros((m, n + 8), dtype=torch.bfloat16, device=DEV)
    binding.mxfp4_bf16_gemm(xg, wg, y=ybig[:, :n])
    torch.cuda.synchronize()
    assert_gemm_close(ybig[:, :n], y_ref, a_ref, "BF16 strided")
    assert not ybig[:, n:].float().abs().sum().item()


def test_exact_ties_pick_lowest_index_and_run_to_run_determinism():
    n, k, m = 300, 1024, 2
    w = synth.weights_student_t(n, k, seed=31)
    x = synth.activations_gaussian(m, k, seed=32)
    y_ref, _ = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    best = int(np.argmax(y_ref[0]))
    w[7] = w[best]
    w[250] = w[best]                                      # three identical rows: exact ties
    lo = min(7, best)
    wg, xg = w.to(DEV), x.to(DEV)
    idx, _ = binding.mxfp4_bf16_gemm_argmax(xg, wg)
    y1 = binding.mxfp4_bf16_gemm(xg, wg)
    y2 = binding.mxfp4_bf16_gemm(xg, wg)
    torch.cuda.synchronize()
    assert int(idx[0]) == lo
    assert torch.equal(y1, y2)


def test_errors_are_reported():
    x = torch.zeros((1, 64), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((4, 64), dtype=torch.bfloat16, device=DEV)
    lib = binding.load()
    st = 0
    assert lib.mxfp4_bf16_gemm(x.data_ptr(), 1, 64, None, 4, 64, 64, w.data_ptr(), 4, st) == 1
    assert lib.mxfp4_bf16_gemm(x.data_ptr(), 1, 64, w.data_ptr(), 4, 60, 64, w.data_ptr(), 4, st) == 2
    assert lib.mxfp4_bf16_gemm(x.data_ptr(), 1, 64, w.data_ptr() + 2, 4, 64, 64, w.data_ptr(), 4, st) == 3
    assert lib.mxfp4_bf16_gemm_argmax(x.data_ptr(), 1, 64, w.data_ptr(), 4, 64, 64, w.data_ptr(), None, None, 0, st) == 4
