"""GPU parity at the full sizes of the benchmark configurations that do not fit a full CPU
check: the 32-layer 7B-shaped stack (3.5 GB of MXFP4) and the 80-layer 70B-shaped stack (36.9 GB,
held resident).  Weights are drawn
on the device layer by layer (the BF16 source of a layer is dropped once it is cast); the oracle
checks full tensors where it is cheap and sampled rows / output columns elsewhere, on host
copies of exactly the tensors the GPU used.  Every call goes through the C ABI in the launch
configuration the benchmark uses (AUTO dispatch)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_13565_amd import binding, synth

pytestmark = pytest.mark.gpu

from helpers import DEV, assert_argmax_ok, assert_gemm_close  # noqa: E402


def cast_layer(shape, layer, linear_index, seed=0):
    name, n, k = shape.linears()[linear_index]
    w = synth.weights_student_t(n, k, seed=synth.tensor_seed(seed, layer, linear_index), device=DEV)
    q, s = binding.mxfp4_direct_cast(w)
    return name, n, k, w, q, s


def check_cast_rows(w, q, s, rows):
    """Bit-exact check of the cast on the given rows (host copy of the same BF16 data)."""
    rows_t = torch.as_tensor(rows, device=w.device)
    q_ref, s_ref = oracle.direct_cast(synth.to_bits(w[rows_t]))
    assert np.array_equal(q[rows_t].cpu().numpy(), q_ref)
    assert np.array_equal(s[rows_t].cpu().numpy(), s_ref)
    return q_ref, s_ref


def check_columns(x, q, s, cols, what, argmax_full=False):
    """Product on the GPU for all columns, oracle on the sampled output columns only."""
    y = binding.mxfp4_woq_gemm(x, q, s)
    torch.cuda.synchronize()
    cols_t = torch.as_tensor(cols, device=q.device)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q[cols_t].cpu().numpy(), s[cols_t].cpu().numpy())
    assert_gemm_close(y[:, cols_t], y_ref, a_ref, what)


@pytest.mark.parametrize("m", [1, 8])
def test_llama7b_full_stack_sampled(m):
    shape = synth.LLAMA_7B
    rng = np.random.default_rng(123 + m)
    total_bytes = 0
    for layer in range(shape.layers):
        for li in range(4):
            name, n, k, w, q, s = cast_layer(shape, layer, li)
            total_bytes += q.numel() + s.numel()
            x = synth.activations_outlier_channels(m, k, seed=synth.tensor_seed(0, layer, li) + 8, device=DEV)
            full = layer in (0, shape.layers - 1) and m == 1
            rows = np.arange(n) if full else np.sort(rng.choice(n, size=256, replace=False))
            check_cast_rows(w, q, s, rows)
            del w
            check_columns(x, q, s, rows, "7B layer %d %s M=%d" % (layer, name, m))
            del q, s
    name, n, k, w, q, s = cast_layer(shape, 0, 4)
    total_bytes += q.numel() + s.numel()
    q_ref, s_ref = check_cast_rows(w, q, s, np.arange(n))
    del w
    x = synth.activations_outlier_channels(m, k, seed=99, device=DEV)
    y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), q_ref, s_ref)
    idx, val = binding.mxfp4_woq_gemm_argmax(x, q, s)
    torch.cuda.synchronize()
    assert_argmax_ok(idx, val, y_ref, a_ref, "7B lm_head M=%d" % m)
    assert abs(total_bytes - 3.510e9) < 0.01e9                   # the stack is 3.51 GB of MXFP4


@pytest.fixture(scope="module")
def stack70b():
    """The fifth configuration's weights, resident: 80 layers x (qkv, o, gate_up, down) + the LM head,
    36.9 GB of MXFP4, generated and cast layer by layer (a layer's BF16 source is dropped once it is
    cast).  Beside every tensor: 256 seed-chosen rows whose cast has been checked bit for bit against
    the oracle on the same BF16 data (all rows for layer 0 and the LM head), and the oracle's bytes of
    those rows, which the product checks use."""
    shape = synth.LLAMA_70B
    rng = np.random.default_rng(70)
    stack = []
    total = 0
    for layer in range(shape.layers + 1):
        for li, (name, n, k) in enumerate(shape.linears()):
            if (layer < shape.layers) == (name == "lm_head"):
                continue
            _, n, k, w, q, s = cast_layer(shape, layer if name != "lm_head" else 0, li)
            full = layer == 0 or name == "lm_head"
            rows = np.arange(n) if full else np.sort(rng.choice(n, size=256, replace=False))
            q_ref, s_ref = check_cast_rows(w, q, s, rows)
            del w
            total += q.numel() + s.numel()
            stack.append(dict(layer=layer, name=name, n=n, k=k, q=q, s=s, rows=rows, q_ref=q_ref, s_ref=s_ref))
    assert abs(total - 36.92e9) < 0.02e9                         # the stack is 36.9 GB of MXFP4
    yield stack
    stack.clear()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("m", [1, 4, 16])
def test_llama70b_resident_stack(stack70b, m):
    """Every linear of the resident stack at M rows through the AUTO dispatch the benchmark uses: all
    output columns on the GPU, the oracle on the checked rows (256 per linear, all of layer 0), and the
    LM head's fused pick against the oracle's full product."""
    xs = {}
    for t in stack70b:
        key = (t["name"], t["k"])
        if key not in xs:
            xs[key] = synth.activations_outlier_channels(m, t["k"], seed=5000 + 16 * m + len(xs), device=DEV)
    ws_bytes = max(binding.mxfp4_woq_gemm_workspace_bytes(m, t["n"], t["k"]) for t in stack70b)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=DEV) if ws_bytes else None
    for t in stack70b:
        x = xs[(t["name"], t["k"])]
        what = "70B layer %d %s M=%d" % (t["layer"], t["name"], m)
        if t["name"] == "lm_head":
            y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), t["q_ref"], t["s_ref"])
            idx, val = binding.mxfp4_woq_gemm_argmax(x, t["q"], t["s"])
            torch.cuda.synchronize()
            assert_argmax_ok(idx, val, y_ref, a_ref, what)
            continue
        y = binding.mxfp4_woq_gemm(x, t["q"], t["s"], workspace=ws)
        torch.cuda.synchronize()
        y_ref, a_ref = oracle.woq_gemm(synth.to_bits(x), t["q_ref"], t["s_ref"])
        assert_gemm_close(y[:, torch.as_tensor(t["rows"], device=DEV)], y_ref, a_ref, what)


def test_llama70b_stack_chained_equals_single_launches(stack70b):
    """The whole resident stack as chained persistent launches (321 products, M = 1) against the
    same products launched one by one: the same bits in every output and the same pick."""
    xs, items = {}, []
    for t in stack70b:
        key = (t["name"], t["k"])
        if key not in xs:
            xs[key] = synth.activations_outlier_channels(1, t["k"], seed=5100 + len(xs), device=DEV)
        if t["name"] == "lm_head":
            items.append(dict(x=xs[key], q=t["q"], s=t["s"], argmax=True))
        else:
            items.append(dict(x=xs[key], q=t["q"], s=t["s"]))
    chain = binding.GemmGroup(items, chained=True, mode=binding.CHAIN_PERSISTENT)
    chain.run()
    torch.cuda.synchronize()
    assert chain.chain_status() == 0
    for i, (t, it) in enumerate(zip(stack70b, items)):
        if t["name"] == "lm_head":
            idx, val = binding.mxfp4_woq_gemm_argmax(it["x"], t["q"], t["s"])
            torch.cuda.synchronize()
            assert torch.equal(chain.ys[i][0], idx) and torch.equal(chain.ys[i][1].view(torch.int32), val.view(torch.int32))
        elif t["layer"] % 8 == 0:
            y = binding.mxfp4_woq_gemm(it["x"], t["q"], t["s"])
            torch.cuda.synchronize()
            assert torch.equal(chain.ys[i].view(torch.int16), y.view(torch.int16)), (t["layer"], t["name"])
