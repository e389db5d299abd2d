"""A seeded sweep over random valid shapes: every product entry point through the C ABI against the
CPU oracle (casts bit-exact, products within the stated tolerance, picks by the argmax rule).  The
shapes are drawn so that every kernel family and its ragged cases come up: K any multiple of 32 or
of 128, N below and above what the decode-step kernels take, one to 17 activation rows
(arXiv 2503.13565, section 3.4.3 for the layer, section 4.4 for the row counts)."""
import random

import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_cast_bit_exact, assert_gemm_close  # noqa: E402

KINDS = ["mx", "fused", "tiled", "grouped", "e4m3", "e2m3", "bf16", "e5m2", "e3m2", "t2", "rows"]


def draw(kind, rng):
    m = rng.choice([1, 1, 2, 3, 4, 5, 7, 8, 9, 16, 17])
    if kind == "e2m3":                                   # the 6-bit product needs K % 128 == 0
        k = 128 * rng.randint(1, 96)
        n = rng.choice([rng.randint(1, 300), rng.randint(2040, 2600), rng.randint(300, 5000)])
    elif kind == "tiled":
        k, n = 128 * rng.randint(1, 100), rng.randint(1, 3000)
    elif kind == "rows":                                 # the product along the rows: K is a head dimension
        k, n, m = 32 * rng.randint(1, 64), rng.randint(1, 9000), min(m, 9)
    else:
        k = 32 * rng.randint(1, 400) if rng.random() < 0.5 else 128 * rng.randint(1, 100)
        n = rng.choice([rng.randint(1, 300), rng.randint(2040, 2600), rng.randint(300, 5000)])
    if kind == "bf16":
        k = max(8, k // 8 * 8)
    if n * k * m > 1.2e8:
        m = max(1, int(1.2e8 // (n * k)))
    return n, k, m


@pytest.mark.parametrize("kind", KINDS)
def test_random_shapes(kind):
    rng = random.Random(KINDS.index(kind) + 100)
    for case in range(12):
        n, k, m = draw(kind, rng)
        tag = "%s case %d N=%d K=%d M=%d" % (kind, case, n, k, m)
        seed = rng.randint(0, 10 ** 6)
        w = synth.weights_student_t(n, k, seed=seed)
        x = synth.activations_outlier_channels(m, k, seed=seed + 1)
        xg = x.to(DEV)
        if kind == "rows":
            q, s, q_ref, s_ref = assert_cast_bit_exact(w, tag)
            p = synth.activations_outlier_channels(m, n, seed=seed + 2)
            y_ref, a_ref = oracle.woq_gemm_t(synth.to_bits(p), q_ref, s_ref)
            y = binding.mxfp4_woq_gemm_t(p.to(DEV), q, s)
            torch.cuda.synchronize()
            assert_gemm_close(y, y_ref, a_ref, tag)
            continue
        if kind in ("e5m2", "e3m2", "t2"):
            fmt = {"e5m2": binding.FMT_E5M2, "e3m2": binding.FMT_E3M2, "t2": binding.FMT_T2}[kind]
            q_ref, s_ref = oracle.mx_direct_cast(fmt, synth.to_bits(w))
            q, s = binding.mxfp4_fmt_direct_cast(fmt, w.to(DEV))
            assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref), tag
            y_ref, a_ref = oracle.mx_woq_gemm(fmt, synth.to_bits(x), q_ref, s_ref)
            y = binding.mxfp4_fmt_woq_gemm(fmt, xg, q, s)
            idx, val = binding.mxfp4_fmt_woq_gemm_argmax(fmt, xg, q, s)
        elif kind == "bf16":
            y_ref, a_ref = oracle.bf16_gemm(synth.to_bits(x), synth.to_bits(w))
            y = binding.mxfp4_bf16_gemm(xg, w.to(DEV))
            idx, val = binding.mxfp4_bf16_gemm_argmax(xg, w.to(DEV))
        elif kind in ("e4m3", "e2m3"):
            cast_ref = oracle.e4m3_direct_cast if kind == "e4m3" else oracle.e2m3_direct_cast
            cast = binding.mxfp4_e4m3_direct_cast if kind == "e4m3" else binding.mxfp4_e2m3_direct_cast
            q_ref, s_ref = cast_ref(synth.to_bits(w))
            q, s = cast(w.to(DEV))
            assert np.array_equal(q.cpu().numpy(), q_ref) and np.array_equal(s.cpu().numpy(), s_ref), tag
            if kind == "e4m3":
                y_ref, a_ref = oracle.e4m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
                y = binding.mxfp4_e4m3_woq_gemm(xg, q, s)
                idx, val = binding.mxfp4_e4m3_woq_gemm_argmax(xg, q, s)
            else:
                y_ref, a_ref = oracle.e2m3_woq_gemm(synth.to_bits(x), q_ref, s_ref)
                y = binding.mxfp4_e2m3_woq_gemm(xg, q, s)
                idx, val = binding.mxfp4_e2m3_woq_gemm_argmax(xg, q, s)
        else:
            q, s, q_ref, s_ref = assert_cast_bit_exact(w, tag)
            y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
            ws_bytes = binding.mxfp4_woq_gemm_workspace_bytes(m, n, k)
            ws = torch.empty((max(ws_bytes, 8),), dtype=torch.uint8, device=DEV)
            if kind == "mx":
                y = binding.mxfp4_woq_gemm(xg, q, s, workspace=ws if ws_bytes and rng.random() < 0.5 else None)
                idx, val = binding.mxfp4_woq_gemm_argmax(xg, q, s)
            elif kind == "tiled":
                tw = binding.mxfp4_tile_repack(q, s)
                y = binding.mxfp4_woq_gemm_tiled(xg, tw, workspace=ws)
                idx, val = binding.mxfp4_woq_gemm_tiled_argmax(xg, tw)
            else:
                act = rng.choice([0, 1]) if n % 2 == 0 else 0
                c = n // 2 if act else n
                g = torch.Generator().manual_seed(seed)
                bias = (torch.randn(n, generator=g) * 0.3).to(torch.bfloat16) if rng.random() < 0.6 else None
                res = (torch.randn(m, c, generator=g) * 0.3).to(torch.bfloat16) if rng.random() < 0.6 else None
                out_ref, a_out = oracle.epilogue(y_ref, a_ref, None if bias is None else synth.to_bits(bias),
                                                 None if res is None else synth.to_bits(res), act)
                bg = None if bias is None else bias.to(DEV)
                rg = None if res is None else res.to(DEV)
                if kind == "fused":
                    yf = binding.mxfp4_woq_gemm_fused(xg, q, s, bias=bg, act=act, residual=rg,
                                                      workspace=ws if ws_bytes else None)
                    torch.cuda.synchronize()
                    assert_gemm_close(yf, out_ref, a_out, tag)
                    continue
                group = binding.GemmGroup([dict(x=xg, q=q, s=s, bias=bg, act=act, residual=rg),
                                           dict(x=xg, q=q, s=s), dict(x=xg, q=q, s=s, argmax=True)])
                group.run()
                torch.cuda.synchronize()
                assert_gemm_close(group.ys[0], out_ref, a_out, tag)
                y, (idx, val) = group.ys[1], group.ys[2]
        torch.cuda.synchronize()
        assert_gemm_close(y, y_ref, a_ref, tag)
        assert_argmax_ok(idx, val, y_ref, a_ref, tag)


def test_random_independent_groups():
    # grouped calls of two to ten one-token products, of one K or each of its own, most of them
    # flagged independent (so that runs of every length up to the limit of eight form and break,
    # also where the activation rows no longer fit the LDS together), at most one pick
    rng = random.Random(900)
    for case in range(12):
        k, count = 128 * rng.randint(1, 64), rng.randint(2, 10)
        ks = [k] * count if case % 2 == 0 else [128 * rng.randint(1, 100) for _ in range(count)]
        ns = [rng.randint(2048, 3000) for _ in range(count)]
        pick = rng.choice([None] + list(range(count)))
        tag = "independent case %d K=%s N=%s pick=%s" % (case, ks, ns, pick)
        seed = rng.randint(0, 10 ** 6)
        items, refs = [], []
        for i, (n, k) in enumerate(zip(ns, ks)):
            w = synth.weights_student_t(n, k, seed=seed + i)
            x = synth.activations_outlier_channels(1, k, seed=seed + 100 + i)
            q, s, q_ref, s_ref = assert_cast_bit_exact(w, tag)
            refs.append(oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref))
            item = dict(x=x.to(DEV), q=q, s=s, independent=rng.random() < 0.9)
            if i == pick:
                item["argmax"] = True
            items.append(item)
        group = binding.GemmGroup(items)
        group.run()
        torch.cuda.synchronize()
        for i, item in enumerate(items):
            if item.get("argmax"):
                assert_argmax_ok(group.ys[i][0], group.ys[i][1], refs[i][0], refs[i][1], tag)
            else:
                assert_gemm_close(group.ys[i], refs[i][0], refs[i][1], tag)
