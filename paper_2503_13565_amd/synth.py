"""Seeded synthetic inputs with the shapes and value structure of the paper's
workloads (Llama2-7B-style decoder linears, section 4.1; a 70B-shaped variant).

The paper's models and prompt sets are not available here; these tensors stand
in for them: heavy-tailed weights, activations with a few outlier channels.
This module only draws random numbers and names shapes -- it holds none of the
method's arithmetic and is shared by the tests of the CPU oracle and of the HIP
path.  Everything is BF16 obtained by rounding FP32 samples to nearest-even.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import torch


@dataclass(frozen=True)
class ModelShape:
    name: str
    hidden: int
    mlp: int
    kv: int          # total width of K (and of V) projections
    vocab: int
    layers: int

    def linears(self) -> List[Tuple[str, int, int]]:
        """(name, N = out features, K = in features) of one decoder layer's linears,
        with Q/K/V and gate/up fused, followed by the LM head."""
        return [
            ("qkv", self.hidden + 2 * self.kv, self.hidden),
            ("o", self.hidden, self.hidden),
            ("gate_up", 2 * self.mlp, self.hidden),
            ("down", self.hidden, self.mlp),
            ("lm_head", self.vocab, self.hidden),
        ]


LLAMA_7B = ModelShape("llama-7b", hidden=4096, mlp=11008, kv=4096, vocab=32000, layers=32)
LLAMA_70B = ModelShape("llama-70b", hidden=8192, mlp=28672, kv=1024, vocab=128256, layers=80)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def weights_gaussian_outliers(n: int, k: int, seed: int = 0, device="cpu",
                              gen: torch.Generator = None) -> torch.Tensor:
    """W = 0.02 * N(0,1); an independent Bernoulli(0.001) mask multiplies entries by 20."""
    g = gen if gen is not None else _gen(seed, device)
    w = torch.randn(n, k, generator=g, device=device, dtype=torch.float32) * 0.02
    mask = torch.rand(n, k, generator=g, device=device, dtype=torch.float32) < 0.001
    w = torch.where(mask, w * 20.0, w)
    return w.to(torch.bfloat16)


def weights_student_t(n: int, k: int, seed: int = 0, device="cpu", nu: int = 4,
                      scale: float = 0.02, rows_per_chunk: int = 4096) -> torch.Tensor:
    """W = scale * StudentT(nu) = scale * N(0,1) / sqrt(chi2_nu / nu), drawn in row chunks."""
    g = _gen(seed, device)
    out = torch.empty(n, k, device=device, dtype=torch.bfloat16)
    for r0 in range(0, n, rows_per_chunk):
        r1 = min(n, r0 + rows_per_chunk)
        z = torch.randn(r1 - r0, k, generator=g, device=device, dtype=torch.float32)
        c = torch.zeros_like(z)
        for _ in range(nu):
            c += torch.randn(r1 - r0, k, generator=g, device=device, dtype=torch.float32).square_()
        out[r0:r1] = (z * scale / (c / nu).sqrt_()).to(torch.bfloat16)
    return out


def activations_gaussian(m: int, k: int, seed: int = 0, device="cpu",
                         gen: torch.Generator = None) -> torch.Tensor:
    g = gen if gen is not None else _gen(seed, device)
    return torch.randn(m, k, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def activations_outlier_channels(m: int, k: int, seed: int = 0, device="cpu",
                                 n_outliers: int = 8, factor: float = 50.0) -> torch.Tensor:
    """x = N(0,1); the same `n_outliers` seed-chosen K-indices are multiplied by `factor`
    in every row."""
    g = _gen(seed, device)
    x = torch.randn(m, k, generator=g, device=device, dtype=torch.float32)
    idx = torch.randperm(k, generator=g, device=device)[:n_outliers]
    x[:, idx] *= factor
    return x.to(torch.bfloat16)


def config0(device="cpu") -> Dict[str, torch.Tensor]:
    """Single linear: W [4096,4096] Gaussian with x20 outliers, x [1,4096] ~ N(0,1); seed 0;
    draw order W normal, W mask, x."""
    g = _gen(0, device)
    w = weights_gaussian_outliers(4096, 4096, device=device, gen=g)
    x = activations_gaussian(1, 4096, device=device, gen=g)
    return {"w": w, "x": x}


def tensor_seed(base: int, layer: int, linear_index: int) -> int:
    """Distinct seed per (layer, linear) from a base seed."""
    return int(base) * 1_000_003 + int(layer) * 16 + int(linear_index)


def llama_linear(shape: ModelShape, linear: str, m: int, layer: int = 0, seed: int = 0,
                 device="cpu") -> Dict[str, torch.Tensor]:
    """Student-t(4)*0.02 weights and outlier-channel activations for one named linear."""
    names = [nm for nm, _, _ in shape.linears()]
    li = names.index(linear)
    _, n, k = shape.linears()[li]
    w = weights_student_t(n, k, seed=tensor_seed(seed, layer, li), device=device)
    x = activations_outlier_channels(m, k, seed=tensor_seed(seed, layer, li) + 8, device=device)
    return {"w": w, "x": x}


def to_bits(t: torch.Tensor):
    """BF16 tensor -> numpy uint16 array of its bit patterns (host copy)."""
    import numpy as np
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def from_bits(a, device="cpu") -> torch.Tensor:
    """numpy uint16 bit patterns -> BF16 tensor."""
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)
