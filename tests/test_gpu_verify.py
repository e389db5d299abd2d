"""GPU parity of the fused draft verification (arXiv 2503.13565, section 3.1): product, greedy pick
and accept rule in one call, for the MXFP4 and the BF16 weights, against the CPU oracle.

The picks are held to the argmax bar (an index is correct iff its oracle value is within the
tolerance of the oracle maximum); the accept pair is integer work and must equal the oracle's rule
applied to the picks the GPU reported, bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth
from helpers import DEV, assert_argmax_ok, oracle_cast_t

pytestmark = pytest.mark.gpu


def drafts_for(picks, kind, vocab):
    """Draft tokens for M - 1 positions: all equal to the picks, or with the first mismatch planted."""
    d = np.array(picks[:-1], dtype=np.int32)
    if kind == "all":
        return d
    pos = {"first": 0, "mid": len(d) // 2, "last": len(d) - 1}[kind]
    if len(d):
        d[pos] = (d[pos] + 1) % vocab
        if pos + 1 < len(d):
            d[pos + 1:] = picks[pos + 1:-1]               # later matches must not count
    return d


def check(accept, idx, val, draft, y_ref, a_ref, what):
    assert_argmax_ok(idx, val, y_ref, a_ref, what)
    got = tuple(int(v) for v in accept.cpu().numpy())
    want = oracle.greedy_accept(idx.cpu().numpy(), draft)
    assert got == want, "%s: accept %r, oracle rule on the reported picks %r" % (what, got, want)
    return got


@pytest.mark.parametrize("kind", ["all", "first", "mid", "last"])
@pytest.mark.parametrize("m", [1, 2, 5, 8, 9, 17, 33])
def test_mxfp4_verify(m, kind):
    n, k = 1000, 1024
    w = synth.weights_student_t(n, k, seed=900 + m)
    x = synth.activations_outlier_channels(m, k, seed=901 + m)
    q_ref, s_ref = oracle_cast_t(w)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    picks, _ = oracle.argmax(y_ref)
    draft = drafts_for(picks, kind, n)
    q, s = binding.mxfp4_direct_cast(w.to(DEV))
    dg = torch.from_numpy(draft).to(DEV) if m > 1 else None
    accept, idx, val = binding.mxfp4_woq_gemm_verify(x.to(DEV), q, s, dg)
    torch.cuda.synchronize()
    g, nxt = check(accept, idx, val, draft, y_ref, a_ref, "MXFP4 verify M=%d %s" % (m, kind))
    if np.array_equal(idx.cpu().numpy(), picks):          # no near-tie flipped a pick: the planted outcome
        want_g = {"all": m - 1, "first": 0, "mid": (m - 1) // 2, "last": max(m - 2, 0)}[kind]
        assert g == want_g and nxt == picks[g]


@pytest.mark.parametrize("kind", ["all", "first", "mid"])
@pytest.mark.parametrize("m", [1, 3, 8, 12])
def test_bf16_verify(m, kind):
    n, k = 777, 512
    w = synth.weights_gaussian_outliers(n, k, seed=910 + m)
    x = synth.activations_gaussian(m, k, seed=911 + m)
    y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
    picks, _ = oracle.argmax(y_ref)
    draft = drafts_for(picks, kind, n)
    dg = torch.from_numpy(draft).to(DEV) if m > 1 else None
    accept, idx, val = binding.mxfp4_bf16_gemm_verify(x.to(DEV), w.to(DEV), dg)
    torch.cuda.synchronize()
    check(accept, idx, val, draft, y_ref, a_ref, "BF16 verify M=%d %s" % (m, kind))


def test_verify_lm_head_shape_and_agreement_with_argmax_call():
    n, k, m = 32000, 4096, 5
    d = synth.llama_linear(synth.LLAMA_7B, "lm_head", m=m, seed=3)
    q, s = binding.mxfp4_direct_cast(d["w"].to(DEV))
    xg = d["x"].to(DEV)
    idx0, val0 = binding.mxfp4_woq_gemm_argmax(xg, q, s)
    draft = idx0[:-1].clone()
    draft[2] = (draft[2] + 7) % n
    accept, idx, val = binding.mxfp4_woq_gemm_verify(xg, q, s, draft)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx0) and torch.equal(val, val0)      # same kernels, same picks
    assert accept.tolist() == [2, int(idx0[2])]


def test_verify_errors():
    lib = binding.load()
    x = torch.zeros((2, 128), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((8, 64), dtype=torch.uint8, device=DEV)
    s = torch.zeros((8, 4), dtype=torch.uint8, device=DEV)
    out = torch.zeros((8,), dtype=torch.int32, device=DEV)
    ws = torch.zeros((binding.mxfp4_woq_gemm_argmax_workspace_bytes(2, 8, 128),), dtype=torch.uint8, device=DEV)
    args = (x.data_ptr(), 2, 128, q.data_ptr(), s.data_ptr(), 8, 128)
    assert lib.mxfp4_woq_gemm_verify(*args, None, out.data_ptr(), out.data_ptr(), None, ws.data_ptr(), ws.numel(), 0) == 1
    assert lib.mxfp4_woq_gemm_verify(*args, out.data_ptr(), None, out.data_ptr(), None, ws.data_ptr(), ws.numel(), 0) == 1
    assert lib.mxfp4_woq_gemm_verify(*args, out.data_ptr(), out.data_ptr(), out.data_ptr(), None, None, 0, 0) == 4
