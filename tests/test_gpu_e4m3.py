"""GPU parity of the 8-bit draft format (E4M3 elements + E8M0 block scales: mxfp4_e4m3_direct_cast,
_dequant, _woq_gemm, _woq_gemm_argmax) with the CPU oracle (arXiv 2503.13565, section 3.4.3 for the
cast rule and the product; sections 1 and 3.2 for 8-bit drafts as drop-ins).  The cast is
bit-exact, the product within 1e-3 of the sum of absolute products plus one BF16 ulp."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_gemm_close  # noqa: E402


def cast_both_ways(w: torch.Tensor, what=""):
    q_ref, s_ref = oracle.e4m3_direct_cast(synth.to_bits(w))
    wg = w.to(DEV)
    q, s = binding.mxfp4_e4m3_direct_cast(wg)
    q2, s2 = binding.mxfp4_e4m3_direct_cast(wg, integer_rule=True)
    torch.cuda.synchronize()
    for name, (qq, ss) in (("convert", (q, s)), ("integer rule", (q2, s2))):
        sg, qg = ss.cpu().numpy(), qq.cpu().numpy()
        bad = np.argwhere(sg != s_ref)
        assert bad.size == 0, "%s %s: %d scale bytes differ, first at %r: gpu %d ref %d" % (
            what, name, len(bad), tuple(bad[0]), sg[tuple(bad[0])], s_ref[tuple(bad[0])])
        bad = np.argwhere(qg != q_ref)
        assert bad.size == 0, "%s %s: %d elements differ, first at %r: gpu %#x ref %#x (input bits %#x)" % (
            what, name, len(bad), tuple(bad[0]), qg[tuple(bad[0])], q_ref[tuple(bad[0])],
            synth.to_bits(w)[tuple(bad[0])])
    return q, s, q_ref, s_ref


def test_cast_every_bf16_magnitude_under_several_block_scales():
    """Blocks of one maximum that fixes the scale and 31 probes: every finite BF16 magnitude up to
    that maximum, both signs, for block maxima across the exponent range (including maxima just
    below 512 X, whose neighbours saturate, and blocks whose scale clamps at byte 0)."""
    for amax_exp in (3, 8, 60, 127, 135, 200, 254):
        amax_bits = (amax_exp << 7) | 0x7F                       # 1.9921875 * 2^(amax_exp - 127)
        mags = np.arange(0, amax_bits + 1, dtype=np.int64)
        lo = max(0, ((amax_exp - 22) << 7))                     # 2^-22 of the maximum and below all round to zero
        mags = np.concatenate([mags[mags >= lo], np.array([0, 1, 0x7F, 0x80], np.int64)])
        pad = (-len(mags)) % 31
        mags = np.concatenate([mags, np.zeros(pad, np.int64)])
        blocks = mags.reshape(-1, 31)
        signs = (np.arange(blocks.size).reshape(blocks.shape) % 3 == 0).astype(np.int64) << 15
        rows = np.concatenate([np.full((blocks.shape[0], 1), amax_bits, np.int64), blocks | signs], axis=1)
        w = synth.from_bits(rows.astype(np.uint16).reshape(1, -1))
        cast_both_ways(w, "amax exponent %d" % amax_exp)


def test_cast_special_blocks():
    w = synth.weights_student_t(8, 256, seed=1)
    w[0, :32] = 0.0
    w[1, 5] = float("inf")
    w[2, 40] = float("nan")
    w[3, 64:96] = -0.0
    w[4, :32] = 1e-38                                            # scale clamps at byte 0
    w[5, :32] = 3e38
    w[6, 3] = -float("inf")
    cast_both_ways(w, "special blocks")


@pytest.mark.parametrize("n,k", [(1, 32), (5, 96), (33, 4096), (130, 11008)])
def test_cast_shapes_and_dequant(n, k):
    w = synth.weights_student_t(n, k, seed=n + k)
    q, s, q_ref, s_ref = cast_both_ways(w, "N=%d K=%d" % (n, k))
    back = binding.mxfp4_e4m3_dequant(q, s)
    torch.cuda.synchronize()
    want = oracle.e4m3_dequant(q_ref, s_ref)                     # four significant bits: exact in BF16
    assert np.array_equal(back.to(torch.float64).cpu().numpy(), want)


@pytest.mark.parametrize("n,k", [(1, 32), (2, 96), (35, 160), (250, 4096), (1000, 1024), (300, 16384),
                                 (8200, 2048), (130, 11008)])
@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 9])
def test_product_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=100 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=200 + m + k)
    q, s, q_ref, s_ref = cast_both_ways(w)
    y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_e4m3_woq_gemm(xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e4m3 N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_e4m3_woq_gemm_argmax(xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "e4m3 argmax N=%d K=%d M=%d" % (n, k, m))


@pytest.mark.parametrize("n,k", [(2048, 128), (2100, 256), (2049, 2176), (2500, 4096), (2300, 8192),
                                 (2100, 11008), (2049, 14336), (2050, 28672), (2051, 32768)])
@pytest.mark.parametrize("m", [1, 2])
def test_product_decode_frame_shapes(n, k, m):
    # enough rows, K % 128 == 0, one or two activation rows: the decode-step kernel (two half blocks
    # per lane); every step count, ragged and whole K, odd N
    w = synth.weights_student_t(n, k, seed=300 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=400 + m + k)
    q, s, q_ref, s_ref = cast_both_ways(w)
    y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_e4m3_woq_gemm(xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "e4m3 decode frame N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_e4m3_woq_gemm_argmax(xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "e4m3 decode frame argmax N=%d K=%d M=%d" % (n, k, m))


def test_decode_frame_ties_nan_scale_and_non_finite_rows():
    n, k = 2100, 6144                                    # three steps: ragged, activations in registers
    w = synth.weights_student_t(n, k, seed=21) * 0.1
    top = synth.weights_student_t(1, k, seed=22)
    x = top.clone()
    for rows in ([5, 300, 2099], [0, 1], [2098, 2099]):
        wt = w.clone()
        wt[rows] = top
        q, s, q_ref, s_ref = cast_both_ways(wt)
        y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
        idx, val = binding.mxfp4_e4m3_woq_gemm_argmax(x.to(DEV), q, s)
        assert idx.cpu().numpy().tolist() == [rows[0]], (rows, idx)
        assert_argmax_ok(idx, val, y_ref, a_ref)
    q, s, q_ref, s_ref = cast_both_ways(w)
    s2 = s.clone()
    s2[17, 3] = 0xFF                                     # one NaN block in row 17 ...
    s2[18, k // 32 - 1] = 0xFF                           # ... and one at the very end of row 18
    y = binding.mxfp4_e4m3_woq_gemm(x.to(DEV), q, s2).float().cpu().numpy()
    y0 = binding.mxfp4_e4m3_woq_gemm(x.to(DEV), q, s).float().cpu().numpy()
    assert np.all(np.isnan(y[:, [17, 18]]))
    keep = ~np.isin(np.arange(n), [17, 18])
    assert np.array_equal(y[:, keep], y0[:, keep])


def test_product_llama_shapes_and_padded_strides():
    sh = synth.LLAMA_7B
    for name, m in (("o", 1), ("down", 5)):
        data = synth.llama_linear(sh, name, m=m, seed=4)
        q, s, q_ref, s_ref = cast_both_ways(data["w"], name)
        y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(data["x"]), q_ref, s_ref)
        k, n = data["x"].shape[1], data["w"].shape[0]
        xbuf = torch.zeros((m, k + 8), dtype=torch.bfloat16, device=DEV)
        xbuf[:, :k] = data["x"].to(DEV)
        ybuf = torch.full((m, n + 6), 3.0, dtype=torch.bfloat16, device=DEV)
        binding.mxfp4_e4m3_woq_gemm(xbuf[:, :k], q, s, y=ybuf[:, :n])
        torch.cuda.synchronize()
        assert_gemm_close(ybuf[:, :n], y_ref, a_ref, "e4m3 %s M=%d" % (name, m))
        assert torch.all(ybuf[:, n:] == 3.0)


def test_exact_ties_pick_lowest_index_and_nan_scale_stays_in_its_row():
    w = synth.weights_student_t(600, 512, seed=11) * 0.1
    top = synth.weights_student_t(1, 512, seed=12)
    x = top.clone().repeat(3, 1)
    for rows in ([5, 300, 599], [0, 1], [598, 599]):
        wt = w.clone()
        wt[rows] = top
        q, s, q_ref, s_ref = cast_both_ways(wt)
        y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
        idx, val = binding.mxfp4_e4m3_woq_gemm_argmax(x.to(DEV), q, s)
        assert idx.cpu().numpy().tolist() == [rows[0]] * 3, (rows, idx)
        assert_argmax_ok(idx, val, y_ref, a_ref)
    q, s, q_ref, s_ref = cast_both_ways(w)
    s2 = s.clone()
    s2[17, 3] = 0xFF                                              # one NaN block in row 17
    y = binding.mxfp4_e4m3_woq_gemm(x.to(DEV), q, s2).float().cpu().numpy()
    y0 = binding.mxfp4_e4m3_woq_gemm(x.to(DEV), q, s).float().cpu().numpy()
    assert np.all(np.isnan(y[:, 17]))
    keep = np.arange(600) != 17
    assert np.array_equal(y[:, keep], y0[:, keep])
