"""GPU parity of the 6-bit draft format (E2M3 elements packed as a 192-bit string per block + E8M0
scales: mxfp4_e2m3_direct_cast, _dequant, _woq_gemm, _woq_gemm_argmax) with the CPU oracle
(arXiv 2503.13565, section 3.4.3 for the cast rule and the product; sections 1 and 5 for other bit
widths as drop-ins).  The cast is bit-exact, the product within 1e-3 of the sum of absolute
products plus one BF16 ulp."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_gemm_close  # noqa: E402


def codes_of(block24):
    big = int.from_bytes(bytes(np.asarray(block24).tolist()), "little")
    return [(big >> (6 * i)) & 63 for i in range(32)]


def cast_both_ways(w: torch.Tensor, what=""):
    q_ref, s_ref = oracle.e2m3_direct_cast(synth.to_bits(w))
    wg = w.to(DEV)
    q, s = binding.mxfp4_e2m3_direct_cast(wg)
    q2, s2 = binding.mxfp4_e2m3_direct_cast(wg, integer_rule=True)
    torch.cuda.synchronize()
    for name, (qq, ss) in (("integer rule", (q2, s2)), ("convert", (q, s))):
        sg, qg = ss.cpu().numpy(), qq.cpu().numpy()
        bad = np.argwhere(sg != s_ref)
        assert bad.size == 0, "%s %s: %d scale bytes differ, first at %r: gpu %d ref %d" % (
            what, name, len(bad), tuple(bad[0]), sg[tuple(bad[0])], s_ref[tuple(bad[0])])
        bad = np.argwhere(qg != q_ref)
        if bad.size:
            r, c = bad[0]
            b = c // 24
            raise AssertionError("%s %s: %d bytes differ; first in row %d block %d\n gpu codes %r\n ref codes %r\n input bits %r" % (
                what, name, len(bad), r, b, codes_of(qg[r, 24 * b:24 * b + 24]), codes_of(q_ref[r, 24 * b:24 * b + 24]),
                [hex(v) for v in synth.to_bits(w)[r, 32 * b:32 * b + 32]]))
    return q, s, q_ref, s_ref


def test_cast_every_bf16_magnitude_under_several_block_scales():
    for amax_exp in (1, 2, 60, 127, 129, 200, 254):
        amax_bits = (amax_exp << 7) | 0x7F                       # 1.9921875 * 2^(amax_exp - 127): r just below 8
        mags = np.arange(0, amax_bits + 1, dtype=np.int64)
        lo = max(0, ((amax_exp - 12) << 7))                     # 2^-12 of the maximum and below all round to zero
        mags = np.concatenate([mags[mags >= lo], np.array([0, 1, 0x7F, 0x80], np.int64)])
        mags = np.concatenate([mags, np.zeros((-len(mags)) % 31, np.int64)])
        blocks = mags.reshape(-1, 31)
        signs = (np.arange(blocks.size).reshape(blocks.shape) % 3 == 0).astype(np.int64) << 15
        rows = np.concatenate([np.full((blocks.shape[0], 1), amax_bits, np.int64), blocks | signs], axis=1)
        w = synth.from_bits(rows.astype(np.uint16).reshape(1, -1))
        cast_both_ways(w, "amax exponent %d" % amax_exp)


def test_cast_special_blocks_shapes_and_dequant():
    w = synth.weights_student_t(8, 256, seed=1)
    w[0, :32] = 0.0
    w[1, 5] = float("inf")
    w[2, 40] = float("nan")
    w[3, 64:96] = -0.0
    w[4, :32] = 1e-38
    w[5, :32] = 3e38
    cast_both_ways(w, "special blocks")
    for n, k in [(1, 32), (5, 96), (33, 4096), (130, 11008)]:
        w = synth.weights_student_t(n, k, seed=n + k)
        q, s, q_ref, s_ref = cast_both_ways(w, "N=%d K=%d" % (n, k))
        back = binding.mxfp4_e2m3_dequant(q, s)
        torch.cuda.synchronize()
        assert np.array_equal(back.to(torch.float64).cpu().numpy(), oracle.e2m3_dequant(q_ref, s_ref))


@pytest.mark.parametrize("n,k", [(2048, 128), (2100, 256), (2049, 2176), (2500, 4096), (2300, 8192),
                                 (2100, 11008), (2049, 14336), (2050, 28672)])
@pytest.mark.parametrize("m", [1, 2, 3])
def test_product_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=100 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=200 + m + k)
    q, s, q_ref, s_ref = cast_both_ways(w)
    y_ref, a_ref = oracle.e2m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_e2m3_woq_gemm(xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e2m3 N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_e2m3_woq_gemm_argmax(xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "e2m3 argmax N=%d K=%d M=%d" % (n, k, m))


@pytest.mark.parametrize("n,k", [(1, 128), (7, 256), (100, 4096), (1000, 2176), (2047, 11008), (300, 18944)])
@pytest.mark.parametrize("m", [1, 2, 3, 9])
def test_product_small_n(n, k, m):
    # fewer weight rows than the decode kernel takes: the tiles, at any row count
    w = synth.weights_student_t(n, k, seed=700 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=800 + m + k)
    q, s, q_ref, s_ref = cast_both_ways(w)
    y_ref, a_ref = oracle.e2m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_e2m3_woq_gemm(xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e2m3 small N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_e2m3_woq_gemm_argmax(xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "e2m3 small N argmax N=%d K=%d M=%d" % (n, k, m))


@pytest.mark.parametrize("n,k", [(2048, 128), (2500, 4096), (2049, 2176), (2100, 11008)])
@pytest.mark.parametrize("m", [4, 5, 8, 9, 16, 17])
def test_product_verification_rows(n, k, m):
    # three and more rows: the matrix-core tiles where a pass's rows fit the LDS, else passes
    w = synth.weights_student_t(n, k, seed=500 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=600 + m + k)
    q, s, q_ref, s_ref = cast_both_ways(w)
    y_ref, a_ref = oracle.e2m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_e2m3_woq_gemm(xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e2m3 tiles N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_e2m3_woq_gemm_argmax(xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "e2m3 tiles argmax N=%d K=%d M=%d" % (n, k, m))


def test_product_llama_shape_refusals_and_nan_block():
    data = synth.llama_linear(synth.LLAMA_7B, "o", m=1, seed=4)
    q, s, q_ref, s_ref = cast_both_ways(data["w"], "o")
    y_ref, a_ref = oracle.e2m3_woq_gemm(synth.to_bits(data["x"]), q_ref, s_ref)
    y = binding.mxfp4_e2m3_woq_gemm(data["x"].to(DEV), q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e2m3 o")
    s2 = s.clone()
    s2[17, 3] = 0xFF
    y2 = binding.mxfp4_e2m3_woq_gemm(data["x"].to(DEV), q, s2).float().cpu().numpy()
    keep = np.arange(4096) != 17
    assert np.isnan(y2[0, 17]) and np.array_equal(y2[:, keep], y.float().cpu().numpy()[:, keep])
    for n, k in [(100, 20480), (4096, 96)]:                      # few rows and K beyond the tiles' LDS; K % 128
        x = torch.zeros((1, k), dtype=torch.bfloat16, device=DEV)
        q0 = torch.zeros((n, k // 32 * 24), dtype=torch.uint8, device=DEV)
        s0 = torch.zeros((n, k // 32), dtype=torch.uint8, device=DEV)
        with pytest.raises(binding.Mxfp4Error) as e:
            binding.mxfp4_e2m3_woq_gemm(x, q0, s0)
        assert e.value.code == 2
