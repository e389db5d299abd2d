"""GPU checks of mxfp4_woq_gemm_chain: a chain of dependent one-token products in one persistent
launch (arXiv 2503.13565, section 3.2: the decode step streams the model's weights; sections 3.1
and 3.4: a forward pass is a fixed chain of contractions with fused operators around them).

Three bars.  (1) The chained launch gives the bits of the same descriptors issued one launch at a
time (mxfp4_woq_gemm_grouped), outputs of every link and the pick.  (2) A real chain -- output
projection with residual, gate+up with the gate, down projection with the residual stream updated
in place, LM head with the pick -- stays within the tolerance of the oracle run as a chain, the
tolerance carried from link to link: a link's input differs from the oracle's (its own exact
output rounded to BF16) by at most the previous link's bar plus one rounding, and that difference
reaches the next output through sum_k |w_k| delta_k.  (3) A wait that cannot be met is given up:
every wave ends, the status word says so, nothing hangs.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_cast_bit_exact  # noqa: E402

NONE, SWIGLU = binding.ACT_NONE, binding.ACT_SWIGLU


def make_linear(n, k, seed, scale=0.02):
    w = synth.weights_student_t(n, k, seed=seed, scale=scale)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    return q, s, q_ref, s_ref


def bf16_randn(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """FP64 -> BF16 bit patterns, round to nearest even (the oracle side of a link's output)."""
    return synth.to_bits(torch.from_numpy(np.asarray(a, np.float64)).to(torch.float32).to(torch.bfloat16))


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return synth.from_bits(bits).to(torch.float64).numpy()


def clone_items(items, remap):
    """The same descriptors on fresh output buffers: `remap` maps data_ptr of a chained tensor to
    its twin, so that a tensor written by one link and read by a later one stays the same tensor."""
    out = []
    for it in items:
        c = dict(it)
        for key in ("x", "residual", "y"):
            t = it.get(key)
            if t is not None and t.data_ptr() in remap:
                twin = remap[t.data_ptr()]
                c[key] = twin if twin.shape == t.shape else twin[:, :t.shape[1]]    # a leading slice
        if "out" in c:
            c["out"] = (torch.empty_like(c["out"][0]), torch.empty_like(c["out"][1]))
        out.append(c)
    return out


def run_both(items, chained_tensors, mode=binding.CHAIN_PERSISTENT):
    """Run `items` chained and as single launches on twin buffers; compare every output's bits."""
    remap = {t.data_ptr(): t.clone() for t in chained_tensors}
    twin = clone_items(items, remap)
    chain = binding.GemmGroup(items, chained=True, mode=mode)
    chain.run()
    single = binding.GemmGroup(twin)
    single.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0
    for i, (a, b) in enumerate(zip(chain.ys, single.ys)):
        if isinstance(a, tuple):
            assert torch.equal(a[0], b[0]), "pick of link %d: %r against %r" % (i, a[0].tolist(), b[0].tolist())
            assert torch.equal(a[1].view(torch.int32), b[1].view(torch.int32)), "winning value of link %d" % i
        else:
            same = torch.equal(a.view(torch.int16), b.view(torch.int16))
            if not same:
                bad = (a.view(torch.int16) != b.view(torch.int16)).nonzero()
                raise AssertionError("link %d: %d outputs differ from the single launch, first at %r: %r against %r"
                                     % (i, len(bad), bad[0].tolist(), a.flatten()[bad[0][-1]].item(),
                                        b.flatten()[bad[0][-1]].item()))
    return chain, single


def decoder_chain(h, f, vocab, seed, with_bias=False):
    """o -> gate+up (gated) -> down (+ residual stream in place) -> LM head pick, really chained."""
    lo = make_linear(h, h, seed)
    lg = make_linear(2 * f, h, seed + 1)
    ld = make_linear(h, f, seed + 2)
    lh = make_linear(vocab, h, seed + 3)
    x0 = synth.activations_outlier_channels(1, h, seed=seed + 4)
    r0 = bf16_randn((1, h), seed + 5, 0.5)
    bias = bf16_randn((h,), seed + 6, 0.25) if with_bias else None
    xg, rg = x0.to(DEV), r0.to(DEV)
    y_o = torch.zeros((1, h), dtype=torch.bfloat16, device=DEV)
    y_g = torch.zeros((1, f), dtype=torch.bfloat16, device=DEV)
    items = [
        dict(x=xg, q=lo[0], s=lo[1], residual=rg, y=y_o),
        dict(x=y_o, q=lg[0], s=lg[1], act=SWIGLU, y=y_g),
        dict(x=y_g, q=ld[0], s=ld[1], residual=y_o, y=y_o, **({"bias": bias.to(DEV)} if with_bias else {})),
        dict(x=y_o, q=lh[0], s=lh[1], argmax=True),
    ]
    return items, [y_o, y_g], (lo, lg, ld, lh), (x0, r0, bias)


def oracle_chain(lins, inputs, f):
    """The same chain in the oracle (FP64 products, BF16 rounding between links), with the bar of
    every link: its own tolerance plus what the previous links' bars can move its inputs by."""
    lo, lg, ld, lh = lins
    x0, r0, bias = inputs
    # link 0: exact inputs
    y, a = oracle.woq_gemm(synth.to_bits(x0), lo[2], lo[3])
    out0, a0 = oracle.epilogue(y, a, None, synth.to_bits(r0), NONE)
    tol0 = oracle.tolerance(out0, a0)
    x1_bits = to_bf16_bits(out0)
    d1 = tol0 + oracle.bf16_ulp(out0)                           # |x1_gpu - x1_ref| at most
    # link 1: gate+up; the input's uncertainty enters the error scale of the epilogue
    y, a = oracle.woq_gemm(x1_bits, lg[2], lg[3])
    a_eff = a + (np.abs(oracle.dequant(lg[2], lg[3])) @ d1[0])[None, :] / 1e-3
    out1, a1 = oracle.epilogue(y, a_eff, None, None, SWIGLU)
    tol1 = oracle.tolerance(out1, a1)
    x2_bits = to_bf16_bits(out1)
    d2 = tol1 + oracle.bf16_ulp(out1)
    # link 2: down projection + (bias) + residual = link 0's output, itself uncertain by d1
    y, a = oracle.woq_gemm(x2_bits, ld[2], ld[3])
    a_eff = a + (np.abs(oracle.dequant(ld[2], ld[3])) @ d2[0])[None, :] / 1e-3
    out2, a2 = oracle.epilogue(y, a_eff, synth.to_bits(bias) if bias is not None else None, x1_bits, NONE)
    tol2 = oracle.tolerance(out2, a2) + d1
    x3_bits = to_bf16_bits(out2)
    d3 = tol2 + oracle.bf16_ulp(out2)
    # link 3: LM head logits (FP32 accumulators, no rounding)
    y3, a3 = oracle.woq_gemm(x3_bits, lh[2], lh[3])
    tol3 = 1e-3 * a3 + (np.abs(oracle.dequant(lh[2], lh[3])) @ d3[0])[None, :]
    return (out0, tol0), (out1, tol1), (out2, tol2), (y3, tol3)


@pytest.mark.parametrize("mode", [binding.CHAIN_PERSISTENT, binding.CHAIN_AUTO, binding.CHAIN_SEPARATE])
@pytest.mark.parametrize("h,f,vocab,bias", [(1024, 1408, 4096, False), (2048, 2816, 8192, True)])
def test_real_chain_equals_single_launches_and_the_oracle_chain(h, f, vocab, bias, mode):
    items, chained, lins, inputs = decoder_chain(h, f, vocab, 21000 + h, with_bias=bias)
    chain, single = run_both(items, chained, mode)
    y_o, y_g = chained
    (out0, tol0), (out1, tol1), (out2, tol2), (y3, tol3) = oracle_chain(lins, inputs, f)
    # y_o holds link 2's output (link 0's was updated in place); the twin run keeps no copy either
    err1 = np.abs(y_g.double().cpu().numpy() - out1)
    assert np.all(err1 <= tol1), "gated link: worst err/tol %g" % float((err1 / tol1).max())
    err2 = np.abs(y_o.double().cpu().numpy() - out2)
    assert np.all(err2 <= tol2), "down link: worst err/tol %g" % float((err2 / tol2).max())
    idx, val = chain.ys[3]
    g = int(idx[0])
    ref_idx, ref_val = oracle.argmax(y3)
    assert 0 <= g < vocab
    assert y3[0, g] >= ref_val[0] - (tol3[0, g] + tol3[0, ref_idx[0]]), "pick %d (%r), oracle %d (%r)" % (
        g, y3[0, g], ref_idx[0], ref_val[0])
    assert abs(float(val[0]) - y3[0, g]) <= tol3[0, g] + abs(y3[0, g]) * 2.0 ** -20


def test_first_link_against_the_oracle_alone():
    # one link, exact inputs: the plain bar of the single call
    h = 1536
    lo = make_linear(h, h, 21500)
    x0 = synth.activations_outlier_channels(1, h, seed=21501)
    r0 = bf16_randn((1, h), 21502, 0.5)
    chain = binding.GemmGroup([dict(x=x0.to(DEV), q=lo[0], s=lo[1], residual=r0.to(DEV))], chained=True)
    chain.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0
    y, a = oracle.woq_gemm(synth.to_bits(x0), lo[2], lo[3])
    out, a_out = oracle.epilogue(y, a, None, synth.to_bits(r0), NONE)
    err = np.abs(chain.ys[0].double().cpu().numpy() - out)
    tol = oracle.tolerance(out, a_out)
    assert np.all(err <= tol), float((err / tol).max())


@pytest.mark.parametrize("n,k", [(256, 128), (300, 384), (4096, 11008), (4099, 4096), (77, 2048), (12288, 4096)])
def test_ragged_shapes_one_link(n, k):
    # fewer rows than workgroups, rows that do not divide, a ragged last step, the smallest K
    lin = make_linear(n, k, 22000 + n)
    x = synth.activations_outlier_channels(1, k, seed=22001 + n)
    items = [dict(x=x.to(DEV), q=lin[0], s=lin[1]), dict(x=x.to(DEV), q=lin[0], s=lin[1], argmax=True)]
    run_both(items, [])


def test_llama7b_decode_step_equals_single_launches():
    # the benchmark's chain at full size: qkv -> o (reads the first 4096 outputs of qkv) -> gate+up
    # (gated) -> down (+ residual in place) -> LM head pick
    h, f, vocab = 4096, 11008, 32000
    seeds = iter(range(23000, 23100))
    lq = make_linear(3 * h, h, next(seeds))
    lo = make_linear(h, h, next(seeds))
    lg = make_linear(2 * f, h, next(seeds))
    ld = make_linear(h, f, next(seeds))
    lh = make_linear(vocab, h, next(seeds))
    x0 = synth.activations_outlier_channels(1, h, seed=next(seeds)).to(DEV)
    y_q = torch.zeros((1, 3 * h), dtype=torch.bfloat16, device=DEV)
    y_o = torch.zeros((1, h), dtype=torch.bfloat16, device=DEV)
    y_g = torch.zeros((1, f), dtype=torch.bfloat16, device=DEV)
    items = [
        dict(x=x0, q=lq[0], s=lq[1], y=y_q),
        dict(x=y_q[:, :h], q=lo[0], s=lo[1], residual=x0, y=y_o),
        dict(x=y_o, q=lg[0], s=lg[1], act=SWIGLU, y=y_g),
        dict(x=y_g, q=ld[0], s=ld[1], residual=y_o, y=y_o),
        dict(x=y_o, q=lh[0], s=lh[1], argmax=True),
    ]
    run_both(items, [y_q, y_o, y_g], binding.CHAIN_AUTO)
    chain, _ = run_both(items, [y_q, y_o, y_g])
    # replays of the same chain (new epochs every time) give the same bits
    first = [y.clone() if not isinstance(y, tuple) else (y[0].clone(), y[1].clone()) for y in chain.ys]
    for _ in range(3):
        chain.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0
    # (y_o is updated in place by link 3 from link 1's fresh output, so replays reproduce it)
    for a, b in zip(first, chain.ys):
        if isinstance(a, tuple):
            assert torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))
        else:
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_long_chain_takes_several_launches():
    # 100 small links, each reading the one before: more than one launch's worth of links
    h = 512
    lins = [make_linear(h, h, 24000 + i, scale=0.03) for i in range(4)]
    x0 = synth.activations_gaussian(1, h, seed=24100).to(DEV)
    bufs = [torch.zeros((1, h), dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    items, src = [], x0
    for i in range(100):
        dst = bufs[i & 1]
        lin = lins[i % 4]
        items.append(dict(x=src, q=lin[0], s=lin[1], y=dst))
        src = dst
    run_both(items, bufs)


def test_give_up_is_reported_and_nothing_hangs():
    h = 1024
    lin = make_linear(h, h, 25000)
    x = synth.activations_gaussian(1, h, seed=25001).to(DEV)
    y0 = torch.zeros((1, h), dtype=torch.bfloat16, device=DEV)
    y1 = torch.zeros((1, h), dtype=torch.bfloat16, device=DEV)
    items = [dict(x=x, q=lin[0], s=lin[1], y=y0), dict(x=y0, q=lin[0], s=lin[1], y=y1)]
    # the barrier waits for one workgroup that does not exist; 2 ms bound
    chain = binding.GemmGroup(items, chained=True, wait_us=2000, phantom_workgroups=1)
    chain.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0x100, hex(chain.chain_status())
    # sticky: the next call on this workspace does nothing and the status stays
    chain.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0x100
    # after a reset the same workspace serves a proper chain again
    good = binding.GemmGroup(items, chained=True, mode=binding.CHAIN_PERSISTENT)
    good.chain_ws = chain.chain_ws
    good.chain_reset()
    good.run()
    torch.cuda.synchronize()
    assert good.chain_status() == 0
    ref = binding.mxfp4_woq_gemm(binding.mxfp4_woq_gemm(x, lin[0], lin[1]), lin[0], lin[1])
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), ref.view(torch.int16))


def test_chain_in_a_graph_replays():
    h, f = 1024, 1408
    items, chained, _, _ = decoder_chain(h, f, 4096, 26000)
    chain = binding.GemmGroup(items, chained=True, mode=binding.CHAIN_PERSISTENT)
    chain.run()
    torch.cuda.synchronize()
    want = [chained[1].clone(), chained[0].clone(), chain.ys[3][0].clone()]
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        chain.run()                                  # warm up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            chain.run()
    for rep in range(4):
        for t in chained:
            t.zero_()                               # eager work between the replays
        chain.ys[3][0].fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert chain.chain_status() == 0
        assert torch.equal(chained[1].view(torch.int16), want[0].view(torch.int16)), rep
        assert torch.equal(chained[0].view(torch.int16), want[1].view(torch.int16)), rep
        assert torch.equal(chain.ys[3][0], want[2]), rep


def test_bad_descriptors_launch_nothing():
    h = 1024
    lin = make_linear(h, h, 27000)
    x = synth.activations_gaussian(2, h, seed=27001).to(DEV)
    y = torch.full((2, h), 7.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.GemmGroup([dict(x=x[:1], q=lin[0], s=lin[1], y=y[:1]), dict(x=x, q=lin[0], s=lin[1], y=y)],
                          chained=True).run()
    assert e.value.code == 6 and "descriptor 1" in str(e.value)
    with pytest.raises(binding.Mxfp4Error) as e:
        binding.GemmGroup([dict(x=x[:1], q=lin[0], s=lin[1], argmax=True), dict(x=x[:1], q=lin[0], s=lin[1], y=y[:1])],
                          chained=True).run()
    assert "last product" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)
