"""GPU parity of the tile-major weight copy and the products that read it (mxfp4_tile_repack,
mxfp4_woq_gemm_tiled, _argmax, _verify) with the CPU oracle on the canonical tensors
(arXiv 2503.13565, section 3.4.3, Eq. 2; section 4.4 for the verification batches; section 3.1
for the accept rule)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_cast_bit_exact, assert_gemm_close  # noqa: E402


def tile_major_by_definition(q: np.ndarray, s: np.ndarray):
    """The layout the header states, written as index arithmetic on the canonical arrays."""
    n, kb = q.shape
    k = kb * 2
    steps, nblk = k // 128, k // 32
    items = (steps + 3) // 4
    tiles = (n + 15) // 16
    qp = np.zeros((tiles * 16, kb), np.uint8)
    qp[:n] = q
    # [tile][row i][step][g][16]  ->  [tile][step][g][i][16]  (lane = i + 16 g)
    qt = qp.reshape(tiles, 16, steps, 4, 16).transpose(0, 2, 3, 1, 4).reshape(-1)
    sp = np.full((tiles * 16, items * 16), 0x7F, np.uint8)
    sp[:n, :nblk] = s
    st = sp.reshape(tiles, 16, items, 16).transpose(0, 2, 1, 3).reshape(-1)
    return qt, st


@pytest.mark.parametrize("n,k", [(16, 128), (33, 256), (100, 11008), (250, 4096), (4101, 1024)])
def test_tile_repack_is_the_stated_permutation(n, k):
    rng = np.random.default_rng(n + k)
    q = rng.integers(0, 256, size=(n, k // 2)).astype(np.uint8)
    s = rng.integers(0, 255, size=(n, k // 32)).astype(np.uint8)
    w = binding.mxfp4_tile_repack(torch.from_numpy(q).to(DEV), torch.from_numpy(s).to(DEV))
    torch.cuda.synchronize()
    qt, st = tile_major_by_definition(q, s)
    assert w.q.numel() == qt.size and w.s.numel() == st.size
    assert np.array_equal(w.q.cpu().numpy(), qt)
    assert np.array_equal(w.s.cpu().numpy(), st)


@pytest.mark.parametrize("n,k", [(16, 128), (17, 256), (250, 11008), (1000, 4096), (48, 8192), (2050, 2048),
                                 (31, 12288), (4100, 11008), (530, 28672), (8300, 11008)])
@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 8, 16, 17, 33])
def test_tiled_product_edge_shapes(n, k, m):
    w = synth.weights_student_t(n, k, seed=7000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=8000 + m + k)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    tw = binding.mxfp4_tile_repack(q, s)
    xg = x.to(DEV)
    # the widest pass (4, 8 or 16 rows) keeps its rows, padded to whole items of 512 columns, in the LDS
    width = 16 if m > 8 else (8 if m > 4 else 4)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    ws_bytes = binding.mxfp4_woq_gemm_workspace_bytes(m, n, k)
    # one and two rows run the decode kernel of this layout: the rows and 1 KiB of partial sums per row
    # and tile of a workgroup in the LDS
    tiles = (n + 15) // 16
    slots = -(-tiles // min(tiles, 256))
    decode = m <= 2 and m * k * 2 + slots * (1088 * m + 4) + 512 <= 160 * 1024
    if not decode and (k + 511) // 512 * 1024 * width + 8192 > 160 * 1024:
        assert ws_bytes > 0
        ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=DEV)
        if m > 8:
            # no workspace: refused; with one, K is split over grid rows
            with pytest.raises(binding.Mxfp4Error) as e:
                binding.mxfp4_woq_gemm_tiled(xg, tw)
            assert e.value.code == 6
        else:
            # up to eight rows walk K in phases inside the workgroup, no workspace needed; with one, the
            # same kernel where a workgroup has few tiles, else K split over grid rows
            y0 = binding.mxfp4_woq_gemm_tiled(xg, tw)
            torch.cuda.synchronize()
            assert_gemm_close(y0, y_ref, a_ref, "tiled, K in phases, N=%d K=%d M=%d" % (n, k, m))
        y = binding.mxfp4_woq_gemm_tiled(xg, tw, workspace=ws)
    else:
        y = binding.mxfp4_woq_gemm_tiled(xg, tw)
        if ws_bytes == 0:                               # a workspace changes nothing when K is not split
            y2 = binding.mxfp4_woq_gemm_tiled(xg, tw, workspace=torch.empty((64,), dtype=torch.uint8, device=DEV))
            assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "tiled N=%d K=%d M=%d" % (n, k, m))
    idx, val = binding.mxfp4_woq_gemm_tiled_argmax(xg, tw)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "tiled argmax N=%d K=%d M=%d" % (n, k, m))


def test_tiled_llama_lm_head_verify():
    data = synth.llama_linear(synth.LLAMA_7B, "lm_head", m=5, seed=3)
    q, s, q_ref, s_ref = assert_cast_bit_exact(data["w"])
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(data["x"]), q_ref, s_ref)
    picks, _ = oracle.argmax(y_ref)
    tw = binding.mxfp4_tile_repack(q, s)
    xg = data["x"].to(DEV)
    # a draft that agrees with the verifier's picks for two positions, then differs
    draft = np.array([picks[0], picks[1], (picks[2] + 1) % 32000, picks[3]], np.int32)
    accept, idx, val = binding.mxfp4_woq_gemm_tiled_verify(xg, tw, torch.from_numpy(draft).to(DEV))
    torch.cuda.synchronize()
    got = assert_argmax_ok(idx, val, y_ref, a_ref, "tiled verify")
    g_ref, next_ref = oracle.greedy_accept(got.astype(np.int32), draft)
    assert accept.cpu().numpy().tolist() == [g_ref, next_ref]
    # and the same answer as the canonical tensors give
    accept2, idx2, _ = binding.mxfp4_woq_gemm_verify(xg, q, s, torch.from_numpy(draft).to(DEV))
    assert torch.equal(idx, idx2) and torch.equal(accept, accept2)


def test_tiled_exact_ties_pick_lowest_index():
    w = synth.weights_student_t(600, 512, seed=11) * 0.1
    top = synth.weights_student_t(1, 512, seed=12)
    x = top.clone().repeat(4, 1)
    for rows in ([5, 300, 599], [0, 1], [598, 599], [15, 16, 17]):
        wt = w.clone()
        wt[rows] = top
        q, s, q_ref, s_ref = assert_cast_bit_exact(wt)
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
        idx, val = binding.mxfp4_woq_gemm_tiled_argmax(x.to(DEV), binding.mxfp4_tile_repack(q, s))
        assert idx.cpu().numpy().tolist() == [rows[0]] * 4, (rows, idx)
        assert_argmax_ok(idx, val, y_ref, a_ref)


def test_tiled_refuses_what_does_not_fit_and_bad_k():
    q = torch.zeros((64, 11008 // 2), dtype=torch.uint8, device=DEV)
    s = torch.zeros((64, 11008 // 32), dtype=torch.uint8, device=DEV)
    tw = binding.mxfp4_tile_repack(q, s)
    x = torch.zeros((16, 11008), dtype=torch.bfloat16, device=DEV)     # 16 x 11008 BF16 = 352 KB
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_tiled(x, tw)
    assert e.value.code == 6
    for rows in (4, 8):                                                 # whole in the LDS; K in phases
        y = binding.mxfp4_woq_gemm_tiled(x[:rows], tw)
        assert not y.float().abs().sum().item()
    q96 = torch.zeros((16, 48), dtype=torch.uint8, device=DEV)
    s96 = torch.zeros((16, 3), dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_tile_repack(q96, s96)
    assert e.value.code == 2


@pytest.mark.parametrize("n,k", [(1, 128), (15, 128), (16, 256), (4096, 4096), (4097, 4096), (12288, 4096),
                                 (22016, 4096), (4096, 11008), (32000, 4096), (2050, 3072), (777, 8192),
                                 (5000, 2176), (300, 28672), (9000, 6144), (128256, 2048), (66000, 1024)])
@pytest.mark.parametrize("m", [1, 2])
def test_tiled_decode_rows(n, k, m):
    """One and two rows on the tile-major copy: every count of steps per wave (K = 128 .. 28672: in
    registers up to four, from LDS beyond), waves beyond K, ragged N, one to 32 tiles per workgroup;
    the same pick as from the row-major tensors."""
    w = synth.weights_student_t(n, k, seed=9000 + n + k)
    x = synth.activations_outlier_channels(m, k, seed=9100 + m + k)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    tw = binding.mxfp4_tile_repack(q, s)
    xg = x.to(DEV)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    y = binding.mxfp4_woq_gemm_tiled(xg, tw)
    torch.cuda.synchronize()
    assert_gemm_close(y, y_ref, a_ref, "tiled decode N=%d K=%d M=%d" % (n, k, m))
    again = binding.mxfp4_woq_gemm_tiled(xg, tw)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), again.view(torch.int16))          # the same bits on every call
    idx, val = binding.mxfp4_woq_gemm_tiled_argmax(xg, tw)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "tiled decode argmax N=%d K=%d M=%d" % (n, k, m))
    s2 = s.clone()
    s2[n // 2, 0] = 0xFF                                                       # a NaN block stays in its row
    y2 = binding.mxfp4_woq_gemm_tiled(xg, binding.mxfp4_tile_repack(q, s2)).float().cpu().numpy()
    keep = np.arange(n) != n // 2
    assert np.isnan(y2[:, n // 2]).all() and np.array_equal(y2[:, keep], y.float().cpu().numpy()[:, keep])
