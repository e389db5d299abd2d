"""GPU parity of mxfp4_direct_cast / mxfp4_dequant with the CPU oracle: bit-exact nibbles and
scale bytes (arXiv 2503.13565, section 3.4.3)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_cast_bit_exact  # noqa: E402


def bits_tensor(bits: np.ndarray) -> torch.Tensor:
    return synth.from_bits(bits)


def test_config0_weights_bit_exact():
    data = synth.config0()
    assert_cast_bit_exact(data["w"], "config0 W[4096,4096]")


@pytest.mark.parametrize("ea", [0, 1, 2, 3, 9, 127, 128, 200, 254])
def test_every_magnitude_below_amax(ea):
    # block = [largest magnitude with exponent ea, 31 magnitudes under test]; all magnitudes <= amax
    hi = ((ea << 7) | 0x7F) + 1
    mags = np.arange(0, hi, dtype=np.uint16)
    n = (mags.size + 30) // 31
    pad = np.zeros(n * 31, np.uint16)
    pad[: mags.size] = mags
    pad[1::2] |= 0x8000                                   # alternate signs
    blocks = np.empty((n, 32), np.uint16)
    blocks[:, 0] = (ea << 7) | 0x7F
    blocks[:, 1:] = pad.reshape(n, 31)
    assert_cast_bit_exact(bits_tensor(blocks), "ea=%d" % ea)


def test_every_scale_near_its_maximum():
    rows = []
    for ea in range(0, 255):
        lo = max(ea - 7, 0) << 7
        hi = ((ea << 7) | 0x7F) + 1
        mags = np.arange(lo, hi, dtype=np.uint16)
        n = (mags.size + 30) // 31
        pad = np.zeros(n * 31, np.uint16)
        pad[: mags.size] = mags
        blocks = np.empty((n, 32), np.uint16)
        blocks[:, 0] = (ea << 7) | 0x7F
        blocks[:, 1:] = pad.reshape(n, 31)
        rows.append(blocks)
    blocks = np.concatenate(rows)
    rng = np.random.default_rng(0)
    perm = rng.permuted(np.tile(np.arange(32), (blocks.shape[0], 1)), axis=1)
    blocks = np.take_along_axis(blocks, perm, axis=1)       # amax at a random position
    blocks ^= (rng.integers(0, 2, size=blocks.shape).astype(np.uint16) << 15)
    assert_cast_bit_exact(bits_tensor(blocks), "near-max sweep")


def test_special_blocks():
    b = np.zeros((8, 64), np.uint16)
    b[1, 5] = 0x8000                                        # -0.0
    b[2, 0:4] = [0x0040, 0x0020, 0x0010, 0x007F]            # BF16 subnormals
    b[3, 40] = 0x7F80                                       # +Inf in the second block only
    b[3, 0:8] = 0x3F80
    b[4, 3] = 0x7FC1                                        # NaN
    b[5, :] = 0x7F7F                                        # largest finite everywhere
    b[6, :] = 0xFF7F
    b[7, 0:32] = 0x0080                                     # smallest normal
    q, s, _, s_ref = assert_cast_bit_exact(bits_tensor(b), "special")
    assert s_ref[3].tolist() == [125, 255] and s_ref[4, 0] == 255 and s_ref[0].tolist() == [0, 0]


@pytest.mark.parametrize("n,k", [(1, 32), (3, 64), (5, 96), (17, 11008), (2, 28672), (129, 4096), (0, 64)])
def test_ragged_shapes(n, k):
    w = synth.weights_student_t(max(n, 1), k, seed=n * 7 + k)[:n]
    if n == 0:
        q, s = binding.mxfp4_direct_cast(w.to(DEV))
        assert q.shape == (0, k // 2) and s.shape == (0, k // 32)
        return
    assert_cast_bit_exact(w, "N=%d K=%d" % (n, k))


def test_row_stride():
    base = synth.weights_student_t(9, 256, seed=3).to(DEV)
    view = base[:, 64:192]                                  # ldw = 256 > K = 128, offset 128 bytes
    q, s = binding.mxfp4_direct_cast(view)
    torch.cuda.synchronize()
    q_ref, s_ref = oracle.direct_cast(synth.to_bits(view.contiguous()))
    assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("linear", ["qkv", "o", "gate_up", "down", "lm_head"])
def test_llama7b_linears_bit_exact(linear):
    data = synth.llama_linear(synth.LLAMA_7B, linear, m=1, seed=0)
    assert_cast_bit_exact(data["w"], "7B " + linear)


@pytest.mark.parametrize("hw", [False, True])
def test_dequant_matches_oracle_for_every_byte_and_scale(hw):
    # all 256 byte values in every position, scale bytes 16..250 (BF16-normal results)
    scales = np.arange(16, 251, dtype=np.uint8)
    n = scales.size
    q = np.empty((n, 16 * 16), np.uint8)                    # 16 blocks per row
    for i in range(16):
        q[:, i * 16:(i + 1) * 16] = (np.arange(16)[None, :] + 16 * i).astype(np.uint8)
    rng = np.random.default_rng(1)
    q = rng.permuted(q, axis=1)
    s = scales[(np.arange(n)[:, None] + 7 * np.arange(16)[None, :]) % n].astype(np.uint8)
    want = oracle.dequant(q, s)
    got = binding.mxfp4_dequant(torch.from_numpy(q).to(DEV), torch.from_numpy(s).to(DEV), hw_convert=hw)
    torch.cuda.synchronize()
    got = got.to(torch.float64).cpu().numpy()
    assert np.array_equal(got, want), np.argwhere(got != want)[:5]
    assert np.array_equal(np.signbit(got), np.signbit(want))


def test_cast_then_dequant_round_trip_on_grid():
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 16, size=(64, 256)).astype(np.uint8)
    codes[:, ::32] = 7                                      # a 6 in every block pins the scale
    sb = rng.integers(20, 240, size=(64, 8)).astype(np.uint8)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    w = oracle.dequant(q, sb)
    wt = torch.from_numpy(w).to(torch.bfloat16)
    assert torch.equal(wt.double(), torch.from_numpy(w))
    qg, sg = binding.mxfp4_direct_cast(wt.to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(qg.cpu().numpy(), q) and np.array_equal(sg.cpu().numpy(), sb)
    back = binding.mxfp4_dequant(qg, sg)
    assert torch.equal(back.cpu(), wt)
