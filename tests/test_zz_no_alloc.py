"""The entry point that allocates nothing (mxfp4_woq_gemm_argmax_noalloc): same picks and winning
accumulators as mxfp4_woq_gemm_argmax, bit for bit, on two calls in a row, the second smaller (the
library's own scratch keeps the first call's contents); sizes beyond the buffer are refused."""
import pytest
import torch

from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _case(m, n, k, seed):
    w = synth.weights_student_t(n, k, seed=seed).to(DEV)
    q, s = binding.mxfp4_direct_cast(w)
    x = synth.activations_outlier_channels(m, k, seed=seed + 1).to(DEV)
    idx = torch.full((m,), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros((m,), dtype=torch.float32, device=DEV)
    return x, q, s, (idx, val)


def test_noalloc_pick_equals_workspace_form_twice_in_a_row():
    # first a verification batch on the LM-head shape (tile kernel, many partial winners), then a
    # single token on a smaller matrix (decode kernel, fewer partial winners)
    for m, n, k, seed in ((8, 32000, 4096, 31000), (1, 5000, 2048, 31010), (3, 4096, 11008, 31020)):
        x, q, s, out = _case(m, n, k, seed)
        binding.mxfp4_woq_gemm_argmax_noalloc(x, q, s, out)
        ref_idx, ref_val = binding.mxfp4_woq_gemm_argmax(x, q, s)
        torch.cuda.synchronize()
        assert torch.equal(out[0], ref_idx), (m, n, k, out[0].tolist(), ref_idx.tolist())
        assert torch.equal(out[1].view(torch.int32), ref_val.view(torch.int32)), (m, n, k)


def test_noalloc_refuses_what_does_not_fit():
    cap = int(binding.load().mxfp4_woq_gemm_argmax_noalloc_max_bytes())
    assert cap == 4 << 20
    # 16 rows on a long K: the split-K partial products alone exceed the buffer
    m, n, k = 16, 16384, 28672
    assert binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k) > cap
    q = torch.zeros((n, k // 2), dtype=torch.uint8, device=DEV)
    s = torch.full((n, k // 32), 127, dtype=torch.uint8, device=DEV)
    x = torch.zeros((m, k), dtype=torch.bfloat16, device=DEV)
    out = (torch.full((m,), -7, dtype=torch.int32, device=DEV), torch.zeros((m,), dtype=torch.float32, device=DEV))
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.mxfp4_woq_gemm_argmax_noalloc(x, q, s, out)
    assert e.value.code == 4
    torch.cuda.synchronize()
    assert torch.all(out[0] == -7)
