"""Shared pieces of the GPU parity tests: run the HIP path through the C-ABI binding, run the
CPU oracle on the same seeded inputs, compare to the stated bars.

Bars (from the project's north star): packed nibbles and scale bytes bit-exact; products
within |y_gpu - y_ref| <= 1e-3 * sum_k |x_k w_k| + 1 BF16 ulp of |y_ref|; an argmax index g is
correct iff y_ref[g] >= max_n y_ref[n] - (tol[g] + tol[n*]) (several indices can be correct
when the top gap is inside the tolerance); on exact ties of identical weight rows only the
lowest index is correct.
"""
import numpy as np
import torch

import oracle
from paper_2503_13565_amd import binding, synth

DEV = "cuda:0"
ALL_VALU = [binding.PATH_VALU_BITS, binding.PATH_VALU_CVT, binding.PATH_VALU_LUT]


def oracle_cast_t(w: torch.Tensor, threads: int = 0):
    return oracle.direct_cast(synth.to_bits(w), threads=threads)


def gpu_cast(w: torch.Tensor):
    """The cast as the product path runs it; the integer-rule variant must give the same bits."""
    wg = w.to(DEV)
    q, s = binding.mxfp4_direct_cast(wg)
    q2, s2 = binding.mxfp4_direct_cast(wg, integer_rule=True)
    torch.cuda.synchronize()
    assert torch.equal(q, q2) and torch.equal(s, s2), "convert instruction and integer rule disagree"
    return q, s


def assert_cast_bit_exact(w: torch.Tensor, what=""):
    q_ref, s_ref = oracle_cast_t(w)
    q, s = gpu_cast(w)
    qg, sg = q.cpu().numpy(), s.cpu().numpy()
    bad_s = np.argwhere(sg != s_ref)
    assert bad_s.size == 0, "%s: %d scale bytes differ, first at %r: gpu %d ref %d" % (
        what, len(bad_s), tuple(bad_s[0]), sg[tuple(bad_s[0])], s_ref[tuple(bad_s[0])])
    bad_q = np.argwhere(qg != q_ref)
    assert bad_q.size == 0, "%s: %d packed bytes differ, first at %r: gpu %#x ref %#x" % (
        what, len(bad_q), tuple(bad_q[0]), qg[tuple(bad_q[0])], q_ref[tuple(bad_q[0])])
    return q, s, q_ref, s_ref


def assert_gemm_close(y_gpu: torch.Tensor, y_ref: np.ndarray, a_ref: np.ndarray, what=""):
    yg = y_gpu.to(torch.float64).cpu().numpy()
    assert yg.shape == y_ref.shape, (yg.shape, y_ref.shape)
    tol = oracle.tolerance(y_ref, a_ref)
    err = np.abs(yg - y_ref)
    bad = np.argwhere(~(err <= tol))
    assert bad.size == 0, "%s: %d of %d outputs out of tolerance; first at %r: gpu %r ref %r tol %r" % (
        what, len(bad), yg.size, tuple(bad[0]), yg[tuple(bad[0])], y_ref[tuple(bad[0])], tol[tuple(bad[0])])
    return float((err / tol).max())


def assert_argmax_ok(idx_gpu: torch.Tensor, val_gpu: torch.Tensor, y_ref: np.ndarray, a_ref: np.ndarray,
                     what=""):
    ig = idx_gpu.cpu().numpy()
    vg = val_gpu.to(torch.float64).cpu().numpy()
    tol = oracle.tolerance(y_ref, a_ref)
    ref_idx, ref_val = oracle.argmax(y_ref)
    for m in range(y_ref.shape[0]):
        g = int(ig[m])
        assert 0 <= g < y_ref.shape[1], "%s: row %d index %d out of range" % (what, m, g)
        slack = tol[m, g] + tol[m, ref_idx[m]]
        assert y_ref[m, g] >= ref_val[m] - slack, "%s: row %d picked %d (%r) but %d holds %r" % (
            what, m, g, y_ref[m, g], ref_idx[m], ref_val[m])
        # the reported maximum is the FP32 accumulator of the picked column
        assert abs(vg[m] - y_ref[m, g]) <= 1e-3 * a_ref[m, g] + abs(y_ref[m, g]) * 2.0 ** -20 + 1e-30, (what, m)
    return ig


def run_gemm_case(w: torch.Tensor, x: torch.Tensor, paths, what="", argmax=False, threads=0):
    """Cast on the GPU (bit-exact check), then the product on every requested path."""
    q, s, q_ref, s_ref = assert_cast_bit_exact(w, what)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref, threads=threads)
    xg = x.to(DEV)
    worst = {}
    for p in paths:
        y = binding.mxfp4_woq_gemm(xg, q, s, path=p)
        torch.cuda.synchronize()
        worst[p] = assert_gemm_close(y, y_ref, a_ref, "%s path %d" % (what, p))
        ws_bytes = binding.mxfp4_woq_gemm_workspace_bytes(x.shape[0], w.shape[0], w.shape[1])
        if ws_bytes and p in (binding.PATH_AUTO, binding.PATH_MFMA, binding.PATH_MFMA_GENERAL):
            # with a workspace K is split across workgroups and a second kernel adds the phases; the
            # call above, without one, split K in time inside the kernel (or ran narrower passes)
            ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=DEV)
            y2 = binding.mxfp4_woq_gemm(xg, q, s, path=p, workspace=ws)
            torch.cuda.synchronize()
            worst[(p, "ws")] = assert_gemm_close(y2, y_ref, a_ref, "%s path %d with workspace" % (what, p))
        if argmax:
            idx, val = binding.mxfp4_woq_gemm_argmax(xg, q, s, path=p)
            torch.cuda.synchronize()
            assert_argmax_ok(idx, val, y_ref, a_ref, "%s argmax path %d" % (what, p))
    return worst
