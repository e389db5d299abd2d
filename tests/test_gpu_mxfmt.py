"""GPU parity of the block formats chosen by id (E5M2, E3M2 and the 2-bit ternary T2, each with E8M0
scales per 32 elements: mxfp4_fmt_direct_cast, _dequant, _woq_gemm, _woq_gemm_argmax) with the CPU
oracle (arXiv 2503.13565, section 3.4.3 for the cast rule and the product; sections 1, 3.2 and 5 for
8-bit and lower-bit drafts as drop-ins).  The cast is bit-exact, the product within 1e-3 of the sum
of absolute products plus one BF16 ulp."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_gemm_close  # noqa: E402

FORMATS = [binding.FMT_E5M2, binding.FMT_E3M2, binding.FMT_T2]
BITS = {binding.FMT_E5M2: 8, binding.FMT_E3M2: 6, binding.FMT_T2: 2}
EMAX = {binding.FMT_E5M2: 15, binding.FMT_E3M2: 4, binding.FMT_T2: 0}
SPAN = {binding.FMT_E5M2: 36, binding.FMT_E3M2: 12, binding.FMT_T2: 4}     # binades below amax that matter


def codes_of(fmt, block):
    b = BITS[fmt]
    big = int.from_bytes(bytes(np.asarray(block).tolist()), "little")
    return [(big >> (b * i)) & ((1 << b) - 1) for i in range(32)]


def cast_both_ways(fmt, w: torch.Tensor, what=""):
    assert oracle.FMT_E5M2 == binding.FMT_E5M2 and oracle.FMT_E3M2 == binding.FMT_E3M2 and oracle.FMT_T2 == binding.FMT_T2
    q_ref, s_ref = oracle.mx_direct_cast(fmt, synth.to_bits(w))
    wg = w.to(DEV)
    q, s = binding.mxfp4_fmt_direct_cast(fmt, wg)
    q2, s2 = binding.mxfp4_fmt_direct_cast(fmt, wg, integer_rule=True)
    torch.cuda.synchronize()
    bb = BITS[fmt] * 4
    assert binding.mxfp4_fmt_block_bytes(fmt) == bb == oracle.mx_block_bytes(fmt)
    for name, (qq, ss) in (("ALU rule", (q2, s2)), ("convert", (q, s))):
        sg, qg = ss.cpu().numpy(), qq.cpu().numpy()
        bad = np.argwhere(sg != s_ref)
        assert bad.size == 0, "fmt %d %s %s: %d scale bytes differ, first at %r: gpu %d ref %d" % (
            fmt, what, name, len(bad), tuple(bad[0]), sg[tuple(bad[0])], s_ref[tuple(bad[0])])
        bad = np.argwhere(qg != q_ref)
        if bad.size:
            r, c = bad[0]
            b = c // bb
            raise AssertionError("fmt %d %s %s: %d bytes differ; first in row %d block %d\n gpu codes %r\n ref codes %r\n input bits %r" % (
                fmt, what, name, len(bad), r, b, codes_of(fmt, qg[r, bb * b:bb * b + bb]),
                codes_of(fmt, q_ref[r, bb * b:bb * b + bb]), [hex(v) for v in synth.to_bits(w)[r, 32 * b:32 * b + 32]]))
    return q, s, q_ref, s_ref


@pytest.mark.parametrize("fmt", FORMATS)
def test_cast_every_bf16_magnitude_under_several_block_scales(fmt):
    for amax_exp in (1, 2, 20, 60, 127, 129, 200, 254):
        for amax_man in (0x7F, 0x00, 0x60, 0x61):
            amax_bits = (amax_exp << 7) | amax_man
            lo = max(0, ((amax_exp - SPAN[fmt]) << 7))              # further below everything rounds to zero
            mags = np.arange(lo, amax_bits + 1, dtype=np.int64)
            mags = np.concatenate([mags, np.array([0, 1, 0x7F, 0x80], np.int64)])
            mags = mags[mags <= amax_bits]
            mags = np.concatenate([mags, np.zeros((-len(mags)) % 31, np.int64)])
            blocks = mags.reshape(-1, 31)
            signs = (np.arange(blocks.size).reshape(blocks.shape) % 3 == 0).astype(np.int64) << 15
            rows = np.concatenate([np.full((blocks.shape[0], 1), amax_bits, np.int64), blocks | signs], axis=1)
            w = synth.from_bits(rows.astype(np.uint16).reshape(1, -1))
            cast_both_ways(fmt, w, "amax exponent %d mantissa %#x" % (amax_exp, amax_man))


@pytest.mark.parametrize("fmt", FORMATS)
def test_cast_special_blocks_shapes_and_dequant(fmt):
    w = synth.weights_student_t(8, 256, seed=1)
    w[0, :32] = 0.0
    w[1, 5] = float("inf")
    w[2, 40] = float("nan")
    w[3, 64:96] = -0.0
    w[4, :32] = 1e-38
    w[5, :32] = 3e38
    cast_both_ways(fmt, w, "special blocks")
    for n, k in [(1, 32), (5, 96), (33, 4096), (130, 11008)]:
        w = synth.weights_student_t(n, k, seed=n + k)
        q, s, q_ref, s_ref = cast_both_ways(fmt, w, "N=%d K=%d" % (n, k))
        back = binding.mxfp4_fmt_dequant(fmt, q, s)
        torch.cuda.synchronize()
        assert np.array_equal(back.to(torch.float64).cpu().numpy(), oracle.mx_dequant(fmt, q_ref, s_ref))
    # the ternary dequantisation is exact at the ends of the scale range too
    w = synth.from_bits(np.array([[0x0001] + [0] * 31 + [0x7F00] + [0x8001] * 31], np.uint16))
    q, s, q_ref, s_ref = cast_both_ways(binding.FMT_T2, w, "scale ends")
    back = binding.mxfp4_fmt_dequant(binding.FMT_T2, q, s).to(torch.float64).cpu().numpy()
    assert np.array_equal(back, oracle.mx_dequant(binding.FMT_T2, q_ref, s_ref))


_CAST = {}


def product_case(fmt, n, k, m, seed, what):
    x = synth.activations_outlier_channels(m, k, seed=seed + 100 + m + k)
    key = (fmt, n, k, seed)
    if key not in _CAST:                                            # one cast (both sides) per weight tensor
        _CAST.clear()
        _CAST[key] = cast_both_ways(fmt, synth.weights_student_t(n, k, seed=seed + n + k))
    q, s, q_ref, s_ref = _CAST[key]
    y_ref, a_ref = oracle.mx_woq_gemm(fmt, synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    y = binding.mxfp4_fmt_woq_gemm(fmt, xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "fmt %d %s N=%d K=%d M=%d" % (fmt, what, n, k, m))
    idx, val = binding.mxfp4_fmt_woq_gemm_argmax(fmt, xg, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "fmt %d %s argmax N=%d K=%d M=%d" % (fmt, what, n, k, m))


@pytest.mark.parametrize("m", [1, 2, 3, 4])
@pytest.mark.parametrize("n,k", [(4500, 2048), (4100, 2176), (8200, 4096), (4099, 8192), (4100, 11008), (1030, 28672)])
@pytest.mark.parametrize("fmt", FORMATS)
def test_product_wide_rows(fmt, n, k, m):
    # 64 and more blocks per row, or a count that is no power of two: one weight row per wave slot,
    # several steps along K with a ragged last one; row counts that are no multiple of the slots
    product_case(fmt, n, k, m, 100, "wide")


@pytest.mark.parametrize("m", [1, 2, 5, 9])
@pytest.mark.parametrize("n,k", [(1, 32), (7, 64), (70000, 128), (33333, 256), (5000, 512), (4097, 1024), (100, 96), (300, 4096)])
@pytest.mark.parametrize("fmt", FORMATS)
def test_product_short_rows_and_small_n(fmt, n, k, m):
    # K/32 a power of two below 64: 64 / (K/32) rows per wave slot (attention-head sized rows);
    # few weight rows: one slot per step; more than four activation rows: several passes
    product_case(fmt, n, k, m, 300, "short")


@pytest.mark.parametrize("fmt", FORMATS)
def test_product_llama_shapes_ties_nan_block_and_refusals(fmt):
    data = synth.llama_linear(synth.LLAMA_7B, "o", m=1, seed=4)
    q, s, q_ref, s_ref = cast_both_ways(fmt, data["w"], "o")
    y_ref, a_ref = oracle.mx_woq_gemm(fmt, synth.to_bits(data["x"]), q_ref, s_ref)
    xg = data["x"].to(DEV)
    y = binding.mxfp4_fmt_woq_gemm(fmt, xg, q, s)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "o")
    s2 = s.clone()
    s2[17, 3] = 0xFF
    y2 = binding.mxfp4_fmt_woq_gemm(fmt, xg, q, s2).float().cpu().numpy()
    keep = np.arange(4096) != 17
    assert np.isnan(y2[0, 17]) and np.array_equal(y2[:, keep], y.float().cpu().numpy()[:, keep])
    # identical weight rows: the lowest index wins
    q3, s3 = q.clone(), s.clone()
    top = int(np.argmax(y_ref[0]))
    for r in (5, 900, 4095):
        q3[r], s3[r] = q[top], s[top]
    idx, _ = binding.mxfp4_fmt_woq_gemm_argmax(fmt, xg, q3, s3)
    torch.cuda.synchronize()
    assert int(idx[0]) == min(5, top)
    bb = BITS[fmt] * 4
    x = torch.zeros((1, 128), dtype=torch.bfloat16, device=DEV)
    q0 = torch.zeros((4, 4 * bb), dtype=torch.uint8, device=DEV)
    s0 = torch.zeros((4, 4), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_fmt_woq_gemm(7, x, q0, s0)
    assert e.value.code == 2
    xk = torch.zeros((1, 1 << 17), dtype=torch.bfloat16, device=DEV)                 # a row beyond the LDS
    qk = torch.zeros((4, (1 << 12) * bb), dtype=torch.uint8, device=DEV)
    sk = torch.zeros((4, 1 << 12), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_fmt_woq_gemm(fmt, xk, qk, sk)
    assert e.value.code == 2
    assert binding.mxfp4_fmt_block_bytes(0) == 0 and binding.mxfp4_fmt_block_bytes(4) == 0
