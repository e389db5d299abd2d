"""GPU parity of mxfp4_woq_gemm / mxfp4_woq_gemm_argmax with the CPU oracle
(arXiv 2503.13565, section 3.4.3, Eq. 2; section 4.4 for the 1..k+1 row range)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import (ALL_VALU, DEV, assert_argmax_ok, assert_cast_bit_exact,  # noqa: E402
                     assert_gemm_close, run_gemm_case)

AUTO = binding.PATH_AUTO


def test_config0_all_paths():
    data = synth.config0()
    worst = run_gemm_case(data["w"], data["x"], ALL_VALU + [AUTO], "config0")
    print("worst err/tol per path:", worst)


@pytest.mark.parametrize("linear", ["qkv", "o", "gate_up", "down", "lm_head"])
def test_llama7b_decode_linears_m1(linear):
    data = synth.llama_linear(synth.LLAMA_7B, linear, m=1, seed=0)
    run_gemm_case(data["w"], data["x"], [AUTO, binding.PATH_VALU_LUT], "7B " + linear,
                  argmax=(linear == "lm_head"))


@pytest.mark.parametrize("m", [2, 4, 8, 16, 32])
def test_verification_sweep_config0_shape(m):
    g = torch.Generator().manual_seed(0)
    w = synth.weights_gaussian_outliers(4096, 4096, gen=g)
    x = synth.activations_gaussian(m, 4096, gen=g)
    run_gemm_case(w, x, [AUTO], "cfg2 4096x4096 M=%d" % m)


@pytest.mark.parametrize("m", [2, 4, 8, 16, 32])
def test_verification_sweep_lm_head_argmax(m):
    data = synth.llama_linear(synth.LLAMA_7B, "lm_head", m=m, seed=0)
    run_gemm_case(data["w"], data["x"], [AUTO], "cfg2 lm_head M=%d" % m, argmax=True)


@pytest.mark.parametrize("n,k", [(1, 32), (3, 64), (5, 2048), (17, 2080), (64, 11008), (33, 28672),
                                 (1000, 4096), (7, 65536)])
@pytest.mark.parametrize("m", [1, 2, 3, 5])
def test_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=1000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=2000 + m + k)
    paths = ALL_VALU if k <= 32768 else [binding.PATH_VALU_CVT]
    run_gemm_case(w, x, paths, "N=%d K=%d M=%d" % (n, k, m), argmax=True)


REG = binding.PATH_VALU_REG


@pytest.mark.parametrize("n,k", [(2048, 128), (2100, 256), (2049, 2176), (2500, 4096), (2111, 6144),
                                 (2300, 8192), (2222, 10240), (2100, 11008), (2050, 12288), (2049, 14336),
                                 (2060, 16384), (2111, 20480), (2050, 28672), (2048, 32768),
                                 (10241, 4096), (12001, 3968), (11000, 1024), (10240, 2176), (10500, 6144)])
@pytest.mark.parametrize("m", [1, 2, 3])
def test_register_gemv_edge_shapes(n, k, m):
    """The decode-step kernel: full, ragged and padded step counts, rows that do not fill the last
    round of a workgroup, one and two activation rows per pass, the fused argmax; few and many rows
    per compute unit (12 waves, or two workgroups of 8, up to K = 4096)."""
    w = synth.weights_student_t(n, k, seed=5000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=6000 + m + k)
    run_gemm_case(w, x, [REG, binding.PATH_VALU_CVT], "REG N=%d K=%d M=%d" % (n, k, m), argmax=True)


def test_register_gemv_refuses_what_it_cannot_run():
    for n, k in [(100, 4096), (4096, 96), (4096, 32768 + 128)]:
        x = torch.zeros((1, k), dtype=torch.bfloat16, device=DEV)
        q = torch.zeros((n, k // 2), dtype=torch.uint8, device=DEV)
        s = torch.zeros((n, k // 32), dtype=torch.uint8, device=DEV)
        with pytest.raises(binding.Mxfp4Error) as e:
            binding.mxfp4_woq_gemm(x, q, s, path=REG)
        assert e.value.code == 6
        y = binding.mxfp4_woq_gemm(x, q, s)                # AUTO takes the general kernel
        assert not y.float().abs().sum().item()


def test_register_gemv_long_k_ignores_non_finite_activations_of_other_rows():
    # from K = 14336 on the activations stay in LDS in padded rows; what pads them is zero, so a
    # NaN in the next activation row cannot reach this row's outputs
    n, k = 2048, 20480
    w = synth.weights_student_t(n, k, seed=31)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    x = synth.activations_gaussian(2, k, seed=32)
    x[1, :64] = float("nan")
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x[:1]), q_ref, s_ref)
    y = binding.mxfp4_woq_gemm(x.to(DEV), q, s, path=REG)
    assert_gemm_close(y[:1], y_ref, a_ref, "row 0 beside a NaN row")
    assert torch.isnan(y[1].float()).all()


def test_register_gemv_nan_scale_stays_in_its_row():
    # ragged K: the lanes past the end of a row see the next row's scale bytes; a NaN block there
    # (scale 0xFF) must not leak into this row
    n, k = 2048, 2176
    w = synth.weights_student_t(n, k, seed=17)
    w[11, 5] = float("nan")
    q, s = binding.mxfp4_direct_cast(w.to(DEV))
    x = synth.activations_gaussian(1, k, seed=18).to(DEV)
    y = binding.mxfp4_woq_gemm(x, q, s, path=REG).float().cpu()
    assert torch.isnan(y[0, 11]) and torch.isfinite(y[0, :11]).all() and torch.isfinite(y[0, 12:]).all()


def test_register_gemv_exact_ties_pick_lowest_index():
    w = synth.weights_student_t(2600, 512, seed=21) * 0.1
    top = synth.weights_student_t(1, 512, seed=22)
    x = top.clone()
    for rows in ([5, 300, 2599], [0, 1], [2598, 2599], [255, 256, 257, 1300]):
        wt = w.clone()
        wt[rows] = top
        q, s, q_ref, s_ref = assert_cast_bit_exact(wt)
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
        assert oracle.argmax(y_ref)[0][0] == rows[0]
        idx, val = binding.mxfp4_woq_gemm_argmax(x.to(DEV), q, s, path=REG)
        assert int(idx[0]) == rows[0], (rows, int(idx[0]))
        assert_argmax_ok(idx, val, y_ref, a_ref)


MFMA = binding.PATH_MFMA
MFMA_GENERAL = binding.PATH_MFMA_GENERAL


@pytest.mark.parametrize("n,k", [(1, 128), (16, 128), (17, 256), (33, 2048), (250, 11008), (1000, 4096),
                                 (48, 8192), (31, 12288)])
@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 8, 9, 16, 17, 33])
def test_mfma_tiles_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=3000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=4000 + m + k)
    run_gemm_case(w, x, [MFMA, MFMA_GENERAL], "MFMA N=%d K=%d M=%d" % (n, k, m), argmax=True)


def test_mfma_needs_k_multiple_of_128():
    x = torch.zeros((4, 96), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((8, 48), dtype=torch.uint8, device=DEV)
    s = torch.zeros((8, 3), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm(x, q, s, path=MFMA)
    assert e.value.code == 6
    y = binding.mxfp4_woq_gemm(x, q, s)                    # AUTO falls back to the vector path
    assert not y.float().abs().sum().item()


@pytest.mark.parametrize("n,k,m", [(130, 11008, 8), (130, 11008, 16), (75, 11008, 20), (40, 28672, 3),
                                   (40, 28672, 16), (100, 8192, 32), (20, 65536, 5), (4200, 11008, 9),
                                   (4200, 11008, 7), (9000, 5120 * 3, 6)])
def test_mfma_split_k(n, k, m):
    """K cut into phases: inside the kernel when there is no workspace (up to eight rows: accumulators in
    registers, the activation rows of two phases in LDS; wider passes: running sums in LDS), across
    workgroups through the workspace when there is (or the first form again where a workgroup has one
    tile); rows in passes of unequal width; several tiles per workgroup.  The fused argmax always has its workspace and so takes the second form."""
    assert binding.mxfp4_woq_gemm_workspace_bytes(m, n, k) > 0
    w = synth.weights_gaussian_outliers(n, k, seed=31 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=32 + m)
    worst = run_gemm_case(w, x, [MFMA], "split-K N=%d K=%d M=%d" % (n, k, m), argmax=True)
    assert any(isinstance(key, tuple) for key in worst)


def test_mfma_large_k_runs_with_and_without_workspace():
    n, k, m = 8, 65536, 4
    x = torch.zeros((m, k), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((n, k // 2), dtype=torch.uint8, device=DEV)
    s = torch.zeros((n, k // 32), dtype=torch.uint8, device=DEV)
    y = binding.mxfp4_woq_gemm(x, q, s, path=MFMA)                # split in time, no scratch needed
    assert not y.float().abs().sum().item()
    ws = torch.empty((binding.mxfp4_woq_gemm_workspace_bytes(m, n, k),), dtype=torch.uint8, device=DEV)
    y = binding.mxfp4_woq_gemm(x, q, s, path=MFMA, workspace=ws)  # split across workgroups
    assert not y.float().abs().sum().item()
    small = torch.empty((16,), dtype=torch.uint8, device=DEV)     # too small: ignored
    y = binding.mxfp4_woq_gemm(x, q, s, path=MFMA, workspace=small)
    assert not y.float().abs().sum().item()


def test_mfma_config0_and_llama_shapes():
    data = synth.config0()
    run_gemm_case(data["w"], data["x"], [MFMA, MFMA_GENERAL], "config0 MFMA")
    for linear in ("down", "o"):
        d = synth.llama_linear(synth.LLAMA_7B, linear, m=8, seed=0)
        run_gemm_case(d["w"], d["x"], [MFMA, MFMA_GENERAL], "7B %s M=8 MFMA" % linear)


@pytest.mark.parametrize("m", [17, 33])
def test_many_rows(m):
    w = synth.weights_student_t(260, 1024, seed=5)
    x = synth.activations_outlier_channels(m, 1024, seed=6)
    run_gemm_case(w, x, [AUTO], "M=%d" % m, argmax=True)


def test_strided_activations_and_output():
    w = synth.weights_student_t(100, 512, seed=7)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    xb = synth.activations_outlier_channels(3, 1024, seed=8).to(DEV)
    x = xb[:, 256:768]                                      # ldx = 1024, offset 512 bytes
    ybuf = torch.zeros((3, 160), dtype=torch.bfloat16, device=DEV)
    y = ybuf[:, :100]                                       # ldy = 160
    binding.mxfp4_woq_gemm(x, q, s, y=y)
    torch.cuda.synchronize()
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x.contiguous()), q_ref, s_ref)
    assert_gemm_close(y, y_ref, a_ref, "strided")
    assert not ybuf[:, 100:].any()                          # nothing written past N


def test_on_grid_weights_and_one_hot_rows():
    # weights on the MXFP4 grid: products are exact small sums, so the GPU result must equal
    # the BF16 rounding of the exact value whenever that value needs few bits
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 16, size=(48, 128)).astype(np.uint8)
    codes[:, ::32] = 6
    sb = rng.integers(120, 130, size=(48, 4)).astype(np.uint8)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    wh = oracle.dequant(q, sb)
    x = np.zeros((4, 128))
    x[0, 0] = 1.0
    x[1, 33] = -2.0
    x[2, 127] = 0.5
    x[3, 64] = 1.0
    x[3, 65] = 1.0
    xt = torch.from_numpy(x).to(torch.bfloat16)
    qd, sd = torch.from_numpy(q).to(DEV), torch.from_numpy(sb).to(DEV)
    for p in ALL_VALU + [binding.PATH_MFMA, binding.PATH_MFMA_GENERAL]:
        y = binding.mxfp4_woq_gemm(xt.to(DEV), qd, sd, path=p).double().cpu().numpy()
        assert np.array_equal(y[0], wh[:, 0]), p
        assert np.array_equal(y[1], -2.0 * wh[:, 33]), p
        assert np.array_equal(y[2], 0.5 * wh[:, 127]), p
        assert np.array_equal(y[3], wh[:, 64] + wh[:, 65]), p


def test_argmax_exact_ties_pick_lowest_index():
    # identical weight rows give bit-identical accumulators: only the lowest index is correct
    w = synth.weights_student_t(600, 512, seed=11) * 0.1
    top = synth.weights_student_t(1, 512, seed=12)
    x = top.clone()                                          # x aligned with `top` -> that row wins by far
    for rows in ([5, 300, 599], [0, 1], [598, 599], [255, 256, 257]):
        wt = w.clone()
        wt[rows] = top
        q, s, q_ref, s_ref = assert_cast_bit_exact(wt)
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
        assert oracle.argmax(y_ref)[0][0] == rows[0]
        for p in ALL_VALU + [binding.PATH_MFMA, binding.PATH_MFMA_GENERAL]:
            idx, val = binding.mxfp4_woq_gemm_argmax(x.to(DEV), q, s, path=p)
            assert int(idx[0]) == rows[0], (rows, p, int(idx[0]))
            assert_argmax_ok(idx, val, y_ref, a_ref)


def test_argmax_near_tie_accepts_either_within_tolerance():
    # two rows whose exact products differ by far less than the tolerance: either index is right
    rng = np.random.default_rng(13)
    k = 2048
    codes = rng.integers(0, 16, size=(64, k)).astype(np.uint8)
    sb = np.full((64, k // 32), 120, np.uint8)
    x = synth.activations_gaussian(1, k, seed=14)
    xs = np.sign(x.float().numpy()[0])
    winner = np.where(xs >= 0, 7, 15).astype(np.uint8)         # +-6 aligned with the sign of x: the largest product
    codes[10] = winner
    codes[40] = winner
    x[0, 77] = 2.0 ** -12                                        # a tiny activation ...
    codes[40, 77] = 6                                            # ... times a weight one code lower in row 40
    codes[10, 77] = 7
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q, sb)
    assert oracle.argmax(y_ref)[0][0] == 10 and y_ref[0, 10] - y_ref[0, 40] < 1e-6 * a_ref[0, 10]
    for p in ALL_VALU + [binding.PATH_MFMA, binding.PATH_MFMA_GENERAL]:
        idx, val = binding.mxfp4_woq_gemm_argmax(x.to(DEV), torch.from_numpy(q).to(DEV),
                                                 torch.from_numpy(sb).to(DEV), path=p)
        got = assert_argmax_ok(idx, val, y_ref, a_ref)
        assert got[0] in (10, 40)


def test_deterministic_run_to_run():
    data = synth.llama_linear(synth.LLAMA_7B, "o", m=2, seed=1)
    q, s = binding.mxfp4_direct_cast(data["w"].to(DEV))
    x = data["x"].to(DEV)
    y1 = binding.mxfp4_woq_gemm(x, q, s).clone()
    i1, v1 = binding.mxfp4_woq_gemm_argmax(x, q, s)
    i1, v1 = i1.clone(), v1.clone()
    for _ in range(3):
        y2 = binding.mxfp4_woq_gemm(x, q, s)
        i2, v2 = binding.mxfp4_woq_gemm_argmax(x, q, s)
        assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
        assert torch.equal(i1, i2) and torch.equal(v1, v2)


def test_nan_block_propagates():
    w = synth.weights_student_t(8, 64, seed=15)
    w[3, 40] = float("inf")
    q, s = binding.mxfp4_direct_cast(w.to(DEV))
    x = synth.activations_gaussian(1, 64, seed=16).to(DEV)
    y = binding.mxfp4_woq_gemm(x, q, s).float().cpu()
    assert torch.isnan(y[0, 3]) and torch.isfinite(y[0, [0, 1, 2, 4, 5, 6, 7]]).all()


def test_errors_are_reported_not_fatal():
    x = torch.zeros((1, 64), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((4, 32), dtype=torch.uint8, device=DEV)
    s = torch.zeros((4, 2), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm(x, q, s, path=99)
    assert e.value.code == 6
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_argmax(x, q, s, workspace=torch.zeros(8, dtype=torch.uint8, device=DEV))
    assert e.value.code == 4
