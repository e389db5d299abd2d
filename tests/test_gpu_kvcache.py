"""GPU parity of attention over a cache held in MXFP4 (arXiv 2503.13565, section 5 names the
quantised cache as the next step and gives no procedure; the reading tested here: one token per
row, blocks of section 3.4.3 along the head dimension, a token cast on its own when appended; the
score side is mxfp4_woq_gemm with N = tokens, the value side is mxfp4_woq_gemm_t).  Casts are
bit-exact, products within 1e-3 of the sum of absolute products plus one BF16 ulp."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_gemm_close  # noqa: E402


def cache(tokens, d, seed):
    """Keys or values of one head: Student-t rows scaled like projected hidden states."""
    w = synth.weights_student_t(tokens, d, seed=seed) * 40.0
    return w.to(torch.bfloat16)


@pytest.mark.parametrize("d", [64, 128, 256])
def test_tokens_appended_one_at_a_time_give_the_bits_of_one_cast(d):
    tokens = 70
    k_all = cache(tokens, d, seed=d).to(DEV)
    q_ref, s_ref = oracle.direct_cast(synth.to_bits(k_all.cpu()))
    q = torch.zeros((tokens, d // 2), dtype=torch.uint8, device=DEV)
    s = torch.zeros((tokens, d // 32), dtype=torch.uint8, device=DEV)
    for t in range(tokens):
        binding.mxfp4_direct_cast(k_all[t:t + 1], q=q[t:t + 1], s=s[t:t + 1])
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("d", [64, 96, 128, 256, 2048])
@pytest.mark.parametrize("tokens", [1, 5, 31, 32, 33, 1000, 4096, 20001])
@pytest.mark.parametrize("m", [1, 3, 4, 8, 9])
def test_scores_and_values_over_the_quantised_cache(d, tokens, m):
    if d == 2048 and tokens > 4096:
        pytest.skip("covered by the smaller head dimensions")
    keys, values = cache(tokens, d, seed=tokens + d), cache(tokens, d, seed=tokens + d + 1)
    qk, sk = binding.mxfp4_direct_cast(keys.to(DEV))
    qv, sv = binding.mxfp4_direct_cast(values.to(DEV))
    qk_ref, sk_ref = oracle.direct_cast(synth.to_bits(keys))
    qv_ref, sv_ref = oracle.direct_cast(synth.to_bits(values))
    assert np.array_equal(qk.cpu().numpy(), qk_ref) and np.array_equal(sv.cpu().numpy(), sv_ref)
    assert np.array_equal(qv.cpu().numpy(), qv_ref) and np.array_equal(sk.cpu().numpy(), sk_ref)
    query = (synth.activations_outlier_channels(m, d, seed=7 * m + d).float() * d ** -0.5).to(torch.bfloat16)
    scores = binding.mxfp4_woq_gemm(query.to(DEV), qk, sk)
    torch.cuda.synchronize()
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(query), qk_ref, sk_ref)
    assert_gemm_close(scores, y_ref, a_ref, "scores d=%d T=%d M=%d" % (d, tokens, m))
    # attention weights from the oracle's scores, rounded to BF16 once: the same input on both sides
    p = torch.softmax(torch.from_numpy(y_ref), dim=1).to(torch.bfloat16)
    out = binding.mxfp4_woq_gemm_t(p.to(DEV), qv, sv)
    torch.cuda.synchronize()
    o_ref, oa_ref = oracle.woq_gemm_t(synth.to_bits(p), qv_ref, sv_ref)
    assert_gemm_close(out, o_ref, oa_ref, "values d=%d T=%d M=%d" % (d, tokens, m))
    # signed inputs of full size too (the softmax is mostly tiny)
    x = synth.activations_outlier_channels(m, tokens, seed=3 * m + tokens)
    out = binding.mxfp4_woq_gemm_t(x.to(DEV), qv, sv)
    torch.cuda.synchronize()
    o_ref, oa_ref = oracle.woq_gemm_t(synth.to_bits(x), qv_ref, sv_ref)
    assert_gemm_close(out, o_ref, oa_ref, "values, signed d=%d T=%d M=%d" % (d, tokens, m))


def test_same_bits_on_every_call_nan_block_padded_rows_and_refusals():
    tokens, d, m = 3000, 128, 4
    values = cache(tokens, d, seed=1)
    qv, sv = binding.mxfp4_direct_cast(values.to(DEV))
    xp = torch.zeros((m, 3008), dtype=torch.bfloat16)
    xp[:, :tokens] = synth.activations_outlier_channels(m, tokens, seed=2)
    xg = xp.to(DEV)[:, :tokens]                                   # row stride 3008
    yp = torch.full((m, 160), 7.0, dtype=torch.bfloat16, device=DEV)
    y = binding.mxfp4_woq_gemm_t(xg, qv, sv, y=yp[:, :d])
    torch.cuda.synchronize()
    o_ref, oa_ref = oracle.woq_gemm_t(synth.to_bits(xp[:, :tokens].contiguous()), qv.cpu().numpy(), sv.cpu().numpy())
    assert_gemm_close(y, o_ref, oa_ref, "padded")
    assert torch.all(yp[:, d:] == 7.0)
    for _ in range(3):
        again = binding.mxfp4_woq_gemm_t(xg, qv, sv)
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), y.contiguous().view(torch.int16))
    s2 = sv.clone()
    s2[1234, 2] = 0xFF
    y2 = binding.mxfp4_woq_gemm_t(xg, qv, s2).float().cpu().numpy()
    assert np.isnan(y2[:, 64:96]).all() and not np.isnan(y2[:, :64]).any() and not np.isnan(y2[:, 96:]).any()
    with pytest.raises(binding.Mxfp4Error) as e:                   # K beyond a head dimension
        binding.mxfp4_woq_gemm_t(torch.zeros((1, 8), dtype=torch.bfloat16, device=DEV),
                                 torch.zeros((8, 2048), dtype=torch.uint8, device=DEV),
                                 torch.zeros((8, 128), dtype=torch.uint8, device=DEV))
    assert e.value.code == 2
    assert binding.mxfp4_woq_gemm_t_workspace_bytes(1, 8, 4096) == 0
    with pytest.raises(binding.Mxfp4Error) as e:                   # workspace too small
        binding.mxfp4_woq_gemm_t(xg, qv, sv, workspace=torch.empty((64,), dtype=torch.uint8, device=DEV))
    assert e.value.code == 4
    with pytest.raises(binding.Mxfp4Error) as e:                   # more rows than the call takes
        binding.mxfp4_woq_gemm_t(torch.zeros((65, tokens), dtype=torch.bfloat16, device=DEV), qv, sv,
                                 workspace=torch.empty((1 << 20,), dtype=torch.uint8, device=DEV))
    assert e.value.code == 2
