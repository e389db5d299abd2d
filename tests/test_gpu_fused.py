"""GPU parity of the fused epilogue (mxfp4_woq_gemm_fused: bias, gate of the gated MLP on
interleaved gate/up rows, residual add) with the CPU oracle, on every kernel family that has the
fused form (arXiv 2503.13565, section 3.4 for the fusion; sections 4.2 and 4.3 for the targets
whose linear layers carry these operators)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_cast_bit_exact, assert_gemm_close  # noqa: E402

AUTO, CVT, REG = binding.PATH_AUTO, binding.PATH_VALU_CVT, binding.PATH_VALU_REG
MFMA, MFMA_GENERAL = binding.PATH_MFMA, binding.PATH_MFMA_GENERAL
NONE, SWIGLU = binding.ACT_NONE, binding.ACT_SWIGLU

OPTIONS = [  # (bias, act, residual)
    (True, NONE, False), (False, NONE, True), (True, NONE, True), (False, SWIGLU, False), (True, SWIGLU, True),
]


def bf16_randn(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


def fused_case(n, k, m, paths, options=OPTIONS, seed=0, what=""):
    w = synth.weights_student_t(n, k, seed=9000 + seed + n + k)
    x = synth.activations_outlier_channels(m, k, seed=9500 + seed + m + k)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    xg = x.to(DEV)
    spread = float(np.abs(y_ref).mean()) + 1e-3      # bias and residual of the product's own size
    ws_bytes = binding.mxfp4_woq_gemm_workspace_bytes(m, n, k)
    for has_bias, act, has_res in options:
        if act == SWIGLU and n % 2:
            continue
        c = n // 2 if act == SWIGLU else n
        bias = bf16_randn((n,), seed + 1, spread) if has_bias else None
        res = bf16_randn((m, c), seed + 2, spread) if has_res else None
        out_ref, a_out = oracle.epilogue(y_ref, a_ref, None if bias is None else synth.to_bits(bias),
                                         None if res is None else synth.to_bits(res), act)
        bg = None if bias is None else bias.to(DEV)
        rg = None if res is None else res.to(DEV)
        for p in paths:
            tag = "%s N=%d K=%d M=%d bias=%d act=%d res=%d path=%d" % (what, n, k, m, has_bias, act, has_res, p)
            y = binding.mxfp4_woq_gemm_fused(xg, q, s, bias=bg, act=act, residual=rg, path=p)
            torch.cuda.synchronize()
            assert_gemm_close(y, out_ref, a_out, tag)
            if ws_bytes and p in (AUTO, MFMA, MFMA_GENERAL):
                ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=DEV)
                y2 = binding.mxfp4_woq_gemm_fused(xg, q, s, bias=bg, act=act, residual=rg, path=p, workspace=ws)
                torch.cuda.synchronize()
                assert_gemm_close(y2, out_ref, a_out, tag + " with workspace")


@pytest.mark.parametrize("n,k", [(2048, 128), (2050, 4096), (2112, 6144), (2050, 12288), (4096, 2048)])
@pytest.mark.parametrize("m", [1, 2, 3])
def test_fused_register_gemv(n, k, m):
    fused_case(n, k, m, [REG, AUTO], what="register GEMV")


@pytest.mark.parametrize("n,k", [(2, 32), (34, 96), (250, 4096), (1000, 160), (300, 16384)])
@pytest.mark.parametrize("m", [1, 2, 5])
def test_fused_general_gemv(n, k, m):
    fused_case(n, k, m, [CVT], what="general GEMV")


@pytest.mark.parametrize("n,k", [(16, 128), (18, 256), (250, 11008), (1000, 4096), (48, 8192), (2050, 2048)])
@pytest.mark.parametrize("m", [3, 4, 8, 16, 17])
def test_fused_mfma_tiles(n, k, m):
    fused_case(n, k, m, [MFMA, MFMA_GENERAL], what="MFMA")


@pytest.mark.parametrize("n,k,m", [(18, 256, 3), (250, 11008, 4), (1000, 4096, 8), (2050, 2048, 17)])
def test_fused_on_tile_major_weights(n, k, m):
    w = synth.weights_student_t(n, k, seed=n + 1)
    x = synth.activations_outlier_channels(m, k, seed=k + 1)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    tw = binding.mxfp4_tile_repack(q, s)
    bias = bf16_randn((n,), 1, 2.0)
    for act in (NONE, SWIGLU):
        c = n // 2 if act == SWIGLU else n
        res = bf16_randn((m, c), 2, 2.0)
        out_ref, a_out = oracle.epilogue(y_ref, a_ref, synth.to_bits(bias), synth.to_bits(res), act)
        y = binding.mxfp4_woq_gemm_tiled_fused(x.to(DEV), tw, bias=bias.to(DEV), act=act, residual=res.to(DEV))
        torch.cuda.synchronize()
        assert_gemm_close(y, out_ref, a_out, "tile-major fused N=%d K=%d M=%d act=%d" % (n, k, m, act))


def test_fused_split_in_space_many_tiles():
    # 16 rows of K = 11008 do not fit the LDS and 12288 weight rows are too many tiles per workgroup
    # for the in-kernel running sums: with a workspace the finish kernel applies the epilogue
    fused_case(12288, 11008, 16, [AUTO], options=[(True, SWIGLU, True), (True, NONE, True)], what="split in space")


def test_fused_llama_layer_shapes_auto():
    # o projection + residual, gate+up with the gate, down projection + residual, one and five rows
    sh = synth.LLAMA_7B
    for m in (1, 5):
        fused_case(sh.hidden, sh.hidden, m, [AUTO], options=[(False, NONE, True)], seed=m, what="o")
        fused_case(2 * sh.mlp, sh.hidden, m, [AUTO], options=[(False, SWIGLU, False)], seed=m, what="gate_up")
        fused_case(sh.hidden, sh.mlp, m, [AUTO], options=[(False, NONE, True)], seed=m, what="down")


def test_fused_residual_in_place_and_padded_strides():
    n, k, m = 2050, 4096, 5
    w = synth.weights_student_t(n, k, seed=77)
    x = synth.activations_outlier_channels(m, k, seed=78)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    res = bf16_randn((m, n), 5, 3.0)
    out_ref, a_out = oracle.epilogue(y_ref, a_ref, None, synth.to_bits(res), NONE)
    xg = x.to(DEV)
    for rows in (slice(0, 5), slice(0, 1), slice(0, 2)):
        mm = rows.stop
        for p in ([AUTO, CVT] if mm <= 2 else [AUTO, MFMA_GENERAL]):
            buf = torch.full((m, n + 14), 7.0, dtype=torch.bfloat16, device=DEV)      # padded row stride
            stream = buf[:, :n]
            stream.copy_(res.to(DEV))
            binding.mxfp4_woq_gemm_fused(xg[rows], q, s, residual=stream[rows], y=stream[rows], path=p)
            torch.cuda.synchronize()
            assert_gemm_close(stream[rows], out_ref[rows], a_out[rows], "in place M=%d path %d" % (mm, p))
            assert torch.all(buf[:, n:] == 7.0), "the padding of the rows was written"
            assert torch.equal(stream[mm:].cpu(), res[mm:]), "rows beyond M were written"


def test_fused_without_options_equals_the_plain_product_bit_for_bit():
    for n, k, m in [(2050, 4096, 1), (2050, 4096, 2), (1000, 4096, 4), (250, 11008, 16), (300, 160, 1)]:
        w = synth.weights_student_t(n, k, seed=n + m)
        x = synth.activations_outlier_channels(m, k, seed=k + m)
        q, s, _, _ = assert_cast_bit_exact(w)
        xg = x.to(DEV)
        y0 = binding.mxfp4_woq_gemm(xg, q, s)
        y1 = binding.mxfp4_woq_gemm_fused(xg, q, s)
        zero_is_signless = (y0.float() == 0) & (y1.float() == 0)
        assert torch.all((y0.view(torch.int16) == y1.view(torch.int16)) | zero_is_signless), (n, k, m)


def test_fused_argument_errors():
    q = torch.zeros((35, 64), dtype=torch.uint8, device=DEV)
    s = torch.zeros((35, 4), dtype=torch.uint8, device=DEV)
    x = torch.zeros((1, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_fused(x, q, s, act=SWIGLU, y=torch.empty((1, 17), dtype=torch.bfloat16, device=DEV))
    assert e.value.code == 2                            # odd N with the gate
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_fused(x, q, s, act=7)
    assert e.value.code == 6
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_fused(x, q, s, path=binding.PATH_VALU_LUT)
    assert e.value.code == 6
