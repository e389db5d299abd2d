"""GPU checks of mxfp4_woq_gemm_grouped: a sequence of products in one call gives the bits of the
single calls (and with them the oracle's product), in order on the stream, and launches nothing
when a descriptor is invalid (arXiv 2503.13565, sections 3.1 and 3.4: a step is a fixed chain of
contractions with fused operators around them)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_cast_bit_exact, assert_gemm_close  # noqa: E402

NONE, SWIGLU = binding.ACT_NONE, binding.ACT_SWIGLU


def make_linear(n, k, seed):
    w = synth.weights_student_t(n, k, seed=seed)
    q, s, q_ref, s_ref = assert_cast_bit_exact(w)
    return q, s, q_ref, s_ref


def bf16_randn(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("m", [1, 2, 4, 8, 16])
def test_grouped_equals_single_calls_and_oracle(m):
    # a small layer: qkv-like, o-like with residual, gate+up with the gate, down with bias and residual
    h, f = 2048, 2816
    shapes = [(3 * h, h), (h, h), (2 * f, h), (h, f)]
    lins = [make_linear(n, k, 11000 + i) for i, (n, k) in enumerate(shapes)]
    xs = [synth.activations_outlier_channels(m, k, seed=11100 + i + m) for i, (_, k) in enumerate(shapes)]
    res = bf16_randn((m, h), 5, 0.5)
    bias = bf16_randn((h,), 6, 0.5)
    xg = [x.to(DEV) for x in xs]
    items = [
        dict(x=xg[0], q=lins[0][0], s=lins[0][1]),
        dict(x=xg[1], q=lins[1][0], s=lins[1][1], residual=res.to(DEV)),
        dict(x=xg[2], q=lins[2][0], s=lins[2][1], act=SWIGLU),
        dict(x=xg[3], q=lins[3][0], s=lins[3][1], bias=bias.to(DEV), residual=res.to(DEV)),
    ]
    group = binding.GemmGroup(items)
    group.run()
    torch.cuda.synchronize()
    ws = group.workspace
    for i, it in enumerate(items):
        if len(it) == 3:
            single = binding.mxfp4_woq_gemm(it["x"], it["q"], it["s"], workspace=ws)
        else:
            single = binding.mxfp4_woq_gemm_fused(it["x"], it["q"], it["s"], bias=it.get("bias"),
                                                  act=it.get("act", NONE), residual=it.get("residual"), workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(group.ys[i].view(torch.int16), single.view(torch.int16)), "descriptor %d M=%d" % (i, m)
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(xs[i]), lins[i][2], lins[i][3])
        out_ref, a_out = oracle.epilogue(
            y_ref, a_ref, synth.to_bits(bias) if "bias" in it else None,
            synth.to_bits(res) if "residual" in it else None, it.get("act", NONE))
        assert_gemm_close(group.ys[i], out_ref, a_out, "grouped descriptor %d M=%d" % (i, m))


@pytest.mark.parametrize("m", [1, 2, 5, 16])
def test_grouped_step_ends_with_the_fused_pick(m):
    # two products and the LM-head pick in one call, one workspace for all three
    h, vocab = 2048, 8192
    l0, head = make_linear(h, h, 11500), make_linear(vocab, h, 11501)
    x = synth.activations_outlier_channels(m, h, seed=11510 + m)
    xg = x.to(DEV)
    group = binding.GemmGroup([dict(x=xg, q=l0[0], s=l0[1]), dict(x=xg, q=head[0], s=head[1], argmax=True),
                               dict(x=xg, q=l0[0], s=l0[1], act=SWIGLU)])
    group.run()
    torch.cuda.synchronize()
    idx, val = group.ys[1]
    ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, vocab, h),), dtype=torch.uint8, device=DEV)
    idx1, val1 = binding.mxfp4_woq_gemm_argmax(xg, head[0], head[1], workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx1) and torch.equal(val.view(torch.int32), val1.view(torch.int32))
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), head[2], head[3])
    assert_argmax_ok(idx, val, y_ref, a_ref, "grouped pick M=%d" % m)
    single = binding.mxfp4_woq_gemm(xg, l0[0], l0[1])
    assert torch.equal(group.ys[0].view(torch.int16), single.view(torch.int16))


def test_grouped_chain_reads_what_an_earlier_descriptor_wrote():
    # y0 = x W0^T, y1 = y0 W1^T in one call; the second product's input is the first one's output
    m, h = 4, 2048
    l0, l1 = make_linear(h, h, 11200), make_linear(h, h, 11201)
    x = synth.activations_outlier_channels(m, h, seed=11210)
    y0 = torch.zeros((m, h), dtype=torch.bfloat16, device=DEV)
    group = binding.GemmGroup([dict(x=x.to(DEV), q=l0[0], s=l0[1], y=y0), dict(x=y0, q=l1[0], s=l1[1])])
    group.run()
    group.run()                                       # a second run gives the same bits
    torch.cuda.synchronize()
    y0_ref, a0 = oracle.woq_gemm(synth.to_bits(x), l0[2], l0[3])
    assert_gemm_close(group.ys[0], y0_ref, a0, "chain first")
    y1_ref, a1 = oracle.woq_gemm(synth.to_bits(group.ys[0].cpu()), l1[2], l1[3])
    assert_gemm_close(group.ys[1], y1_ref, a1, "chain second")


def test_grouped_launches_nothing_when_a_descriptor_is_invalid():
    m, h = 1, 2048
    l0 = make_linear(h, h, 11300)
    x = synth.activations_outlier_channels(m, h, seed=11310).to(DEV)
    y = torch.full((m, h), 7.0, dtype=torch.bfloat16, device=DEV)
    group = binding.GemmGroup([dict(x=x, q=l0[0], s=l0[1], y=y), dict(x=x, q=l0[0], s=l0[1])])
    group._descs[1].K = 40                             # not a multiple of 32
    with pytest.raises(binding.Mxfp4Error) as err:
        group.run()
    torch.cuda.synchronize()
    assert err.value.code == 2 and "descriptor 1: " in str(err.value)
    assert bool((y == 7.0).all())                      # the valid first product did not run either


@pytest.mark.parametrize("independent", [False, True])
def test_grouped_in_a_graph_replays_identically(independent):
    # (independent: the two products share one launch, captured as one kernel node)
    m, h = 1, 4096
    l0, l1 = make_linear(h, h, 11400), make_linear(h, h, 11401)
    x = synth.activations_outlier_channels(m, h, seed=11410).to(DEV)
    group = binding.GemmGroup([dict(x=x, q=l0[0], s=l0[1], independent=independent),
                               dict(x=x, q=l1[0], s=l1[1], independent=independent)])
    group.run()
    torch.cuda.synchronize()
    eager = [y.clone() for y in group.ys]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            group.run()
        for _ in range(3):
            for y in group.ys:
                y.zero_()
            g.replay()
            torch.cuda.synchronize()
            for y, e in zip(group.ys, eager):
                assert torch.equal(y.view(torch.int16), e.view(torch.int16))


def test_grouped_decode_step_at_full_7b_sizes_equals_single_calls():
    # the launch configuration the benchmark times: the five 7B linears at one row, the pick on the
    # LM head, one call; the single calls are checked against the oracle at these sizes elsewhere
    shape = synth.LLAMA_7B
    g = torch.Generator(device=DEV).manual_seed(11600)
    items, singles = [], []
    for name, n, k in shape.linears():
        q = torch.randint(0, 256, (n, k // 2), dtype=torch.uint8, device=DEV, generator=g)
        s = torch.randint(112, 130, (n, k // 32), dtype=torch.uint8, device=DEV, generator=g)
        x = synth.activations_outlier_channels(1, k, seed=11610 + n, device=DEV)
        if name == "lm_head":
            items.append(dict(x=x, q=q, s=s, argmax=True))
            ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(1, n, k),), dtype=torch.uint8, device=DEV)
            singles.append(binding.mxfp4_woq_gemm_argmax(x, q, s, workspace=ws))
        else:
            items.append(dict(x=x, q=q, s=s))
            singles.append(binding.mxfp4_woq_gemm(x, q, s))
    group = binding.GemmGroup(items)
    for _ in range(2):
        group.run()
    torch.cuda.synchronize()
    for y, ref in zip(group.ys, singles):
        if isinstance(y, tuple):
            assert torch.equal(y[0], ref[0]) and torch.equal(y[1].view(torch.int32), ref[1].view(torch.int32))
        else:
            assert torch.equal(y.view(torch.int16), ref.view(torch.int16))


@pytest.mark.parametrize("m", [3, 8, 16])
def test_grouped_on_tile_major_weights(m):
    # plain (whole K and K split through the workspace), fused and the pick, all on the tile-major copy
    h, f, vocab = 2048, 11008, 4096
    shapes = [(2 * h, h), (h, f), (2 * h, h), (vocab, h)]
    lins = [make_linear(n, k, 11700 + i) for i, (n, k) in enumerate(shapes)]
    tws = [binding.mxfp4_tile_repack(l[0], l[1]) for l in lins]
    xs = [synth.activations_outlier_channels(m, k, seed=11710 + i + m) for i, (_, k) in enumerate(shapes)]
    xg = [x.to(DEV) for x in xs]
    res = bf16_randn((m, h), 7, 0.5)
    group = binding.GemmGroup([
        dict(x=xg[0], w=tws[0]),
        dict(x=xg[1], w=tws[1]),
        dict(x=xg[2], w=tws[2], act=SWIGLU, residual=res.to(DEV)),
        dict(x=xg[3], w=tws[3], argmax=True),
    ])
    group.run()
    torch.cuda.synchronize()
    refs = [oracle.woq_gemm(synth.to_bits(xs[i]), lins[i][2], lins[i][3]) for i in range(4)]
    assert_gemm_close(group.ys[0], refs[0][0], refs[0][1], "tiled grouped plain M=%d" % m)
    assert_gemm_close(group.ys[1], refs[1][0], refs[1][1], "tiled grouped long K M=%d" % m)
    out_ref, a_out = oracle.epilogue(refs[2][0], refs[2][1], None, synth.to_bits(res), SWIGLU)
    assert_gemm_close(group.ys[2], out_ref, a_out, "tiled grouped fused M=%d" % m)
    assert_argmax_ok(group.ys[3][0], group.ys[3][1], refs[3][0], refs[3][1], "tiled grouped pick M=%d" % m)
    single = binding.mxfp4_woq_gemm_tiled(xg[1], tws[1], workspace=group.workspace)
    torch.cuda.synchronize()
    assert torch.equal(group.ys[1].view(torch.int16), single.view(torch.int16))


def _independent_items(shapes, k, seed, argmax_at=None):
    lins = [make_linear(n, k, seed + i) for i, n in enumerate(shapes)]
    xs = [synth.activations_outlier_channels(1, k, seed=seed + 50 + i) for i in range(len(shapes))]
    items = []
    for i, (lin, x) in enumerate(zip(lins, xs)):
        it = dict(x=x.to(DEV), q=lin[0], s=lin[1], independent=True)
        if i == argmax_at:
            it["argmax"] = True
        items.append(it)
    return lins, xs, items


def _check_against_single_calls_and_oracle(group, items, lins, xs, what):
    for i, it in enumerate(items):
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(xs[i]), lins[i][2], lins[i][3])
        if it.get("argmax"):
            n, k = lins[i][0].shape[0], lins[i][0].shape[1] * 2
            ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(1, n, k),), dtype=torch.uint8, device=DEV)
            idx1, val1 = binding.mxfp4_woq_gemm_argmax(it["x"], it["q"], it["s"], workspace=ws)
            torch.cuda.synchronize()
            idx, val = group.ys[i]
            assert torch.equal(idx, idx1) and torch.equal(val.view(torch.int32), val1.view(torch.int32)), (what, i)
            assert_argmax_ok(idx, val, y_ref, a_ref, "%s pick %d" % (what, i))
        else:
            single = binding.mxfp4_woq_gemm(it["x"], it["q"], it["s"])
            torch.cuda.synchronize()
            assert torch.equal(group.ys[i].view(torch.int16), single.view(torch.int16)), (what, i)
            assert_gemm_close(group.ys[i], y_ref, a_ref, "%s product %d" % (what, i))


@pytest.mark.parametrize("k", [2048, 4096, 6144, 8192])
def test_independent_products_in_one_launch(k):
    # one token, one K (two or four steps, whole and ragged), rows that are odd, a pick in the
    # middle: the products marked independent share a launch and keep the bits of the single calls
    shapes = [2048, 4104, 2817, 8192, 2056]
    lins, xs, items = _independent_items(shapes, k, 12000 + k, argmax_at=3)
    group = binding.GemmGroup(items)
    for _ in range(2):                                 # the second run must not depend on what the first left
        for y in group.ys:
            if not isinstance(y, tuple):
                y.fill_(3.0)
        group.run()
    torch.cuda.synchronize()
    _check_against_single_calls_and_oracle(group, items, lins, xs, "one launch K=%d" % k)


def test_independent_runs_split_where_the_products_cannot_share_a_launch():
    # eleven products: the run of independent ones is cut by a second pick, by a product of two
    # rows, by one with an activation and by the limit of eight per launch
    k = 4096
    shapes = [2048] * 11
    lins, xs, items = _independent_items(shapes, k, 12100, argmax_at=1)
    items[2]["argmax"] = True                          # a second pick: starts a new run
    x2 = synth.activations_outlier_channels(2, k, seed=12190)
    items[4]["x"] = x2.to(DEV)                         # two rows: runs on its own
    items[6]["act"] = SWIGLU                           # an epilogue: runs on its own
    group = binding.GemmGroup(items)
    group.run()
    torch.cuda.synchronize()
    for i in (4, 6):
        it = items[i]
        x_cpu = x2 if i == 4 else xs[i]
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x_cpu), lins[i][2], lins[i][3])
        out_ref, a_out = oracle.epilogue(y_ref, a_ref, None, None, it.get("act", NONE))
        assert_gemm_close(group.ys[i], out_ref, a_out, "split runs product %d" % i)
    keep = [i for i in range(11) if i not in (4, 6)]
    _check_against_single_calls_and_oracle(
        type("G", (), {"ys": [group.ys[i] for i in keep]}), [items[i] for i in keep], [lins[i] for i in keep],
        [xs[i] for i in keep], "split runs")


def test_independent_decode_step_at_full_7b_sizes_equals_single_calls():
    # the 7B linears at one row, all marked independent: the five share one launch, the pick
    # among them
    shape = synth.LLAMA_7B
    g = torch.Generator(device=DEV).manual_seed(12200)
    by_name = {}
    for name, n, k in shape.linears():
        q = torch.randint(0, 256, (n, k // 2), dtype=torch.uint8, device=DEV, generator=g)
        s = torch.randint(112, 130, (n, k // 32), dtype=torch.uint8, device=DEV, generator=g)
        x = synth.activations_outlier_channels(1, k, seed=12210 + n, device=DEV)
        by_name[name] = dict(x=x, q=q, s=s, independent=True)
    by_name["lm_head"]["argmax"] = True
    order = ["down", "qkv", "o", "gate_up", "lm_head"]
    group = binding.GemmGroup([by_name[n] for n in order])
    for _ in range(2):
        group.run()
    torch.cuda.synchronize()
    for name, y in zip(order, group.ys):
        it = by_name[name]
        if isinstance(y, tuple):
            n, k = it["q"].shape[0], it["q"].shape[1] * 2
            ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(1, n, k),), dtype=torch.uint8, device=DEV)
            ref = binding.mxfp4_woq_gemm_argmax(it["x"], it["q"], it["s"], workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(y[0], ref[0]) and torch.equal(y[1].view(torch.int32), ref[1].view(torch.int32))
        else:
            ref = binding.mxfp4_woq_gemm(it["x"], it["q"], it["s"])
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), ref.view(torch.int16)), name


@pytest.mark.parametrize("pick", [None, 2, 5])
def test_independent_products_of_different_k(pick):
    # one launch for products whose K differ (one step to fourteen, ragged last steps, K beyond
    # 8192): the activation rows stay in LDS, padded with zeros
    shapes = [(2048, 4096), (2100, 11008), (2817, 128), (4104, 8192), (2056, 28672), (8192, 4224)]
    lins = [make_linear(n, k, 12300 + i) for i, (n, k) in enumerate(shapes)]
    xs = [synth.activations_outlier_channels(1, k, seed=12350 + i) for i, (_, k) in enumerate(shapes)]
    items = []
    for i, (lin, x) in enumerate(zip(lins, xs)):
        item = dict(x=x.to(DEV), q=lin[0], s=lin[1], independent=True)
        if i == pick:
            item["argmax"] = True
        items.append(item)
    group = binding.GemmGroup(items)
    for _ in range(2):
        for y in group.ys:
            if not isinstance(y, tuple):
                y.fill_(3.0)
        group.run()
    torch.cuda.synchronize()
    _check_against_single_calls_and_oracle(group, items, lins, xs, "different K pick=%s" % pick)
