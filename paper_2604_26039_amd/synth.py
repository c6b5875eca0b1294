"""Seeded synthetic inputs: layer tensors and router outputs.

This module only draws random inputs.  It contains none of the method's
arithmetic and is the one piece that both the GPU path's tests/benchmark and
the CPU oracle's tests consume.

Shapes follow the model families the paper evaluates (Tab. 4): OLMoE-, Qwen3-,
Mixtral- and DeepSeek-V3-shaped experts.  The paper's routing traces are not
available, so routing skew is synthesised: each token draws its k experts from
a seeded subset holding a fraction beta of the experts (the paper's "only
8-14 % of experts active" regime, Sec. 3.1, corresponds to beta ~ 0.1), or
from a Zipf popularity law.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Shape:
    name: str
    H: int      # hidden size (K of the up-projection)
    I: int      # expert intermediate size
    E: int      # experts
    k: int      # top-k


SHAPES = {
    "tiny": Shape("tiny", 256, 512, 16, 2),
    "olmoe": Shape("olmoe", 2048, 1024, 64, 8),
    "qwen3": Shape("qwen3", 2048, 768, 128, 8),
    "mixtral": Shape("mixtral", 4096, 14336, 8, 2),
    "dsv3": Shape("dsv3", 7168, 2048, 256, 8),
}

SWEEPS = {
    "tiny": dict(T=[16], beta=[1.0, 0.2]),
    "olmoe": dict(T=[1, 16, 64, 256, 1024, 4096], beta=[1.0, 0.5, 0.2, 0.1]),
    "qwen3": dict(T=[1, 32, 128, 512, 2048, 8192], beta=[1.0, 0.3, 0.14, 0.08]),
    "mixtral": dict(T=[1, 16, 128, 1024, 8192], beta=[1.0, "zipf1.2"]),
    "dsv3": dict(T=[1, 64, 512, 2048, 8192], beta=[1.0, 0.2, 0.1]),
}


def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.default_rng([int(seed) & 0x7FFFFFFF, int(tag)])


def _softmax_gates(rng: np.random.Generator, T: int, k: int) -> np.ndarray:
    logits = rng.standard_normal((T, k))
    logits -= logits.max(axis=1, keepdims=True)
    p = np.exp(logits)
    p /= p.sum(axis=1, keepdims=True)
    return p.astype(np.float32)


def routing_subset(T: int, k: int, E: int, beta: float, seed: int):
    """Each token draws k distinct experts uniformly from a seeded subset of
    max(k, ceil(beta*E)) experts; gate weights are the softmax of N(0,1) logits
    over the chosen k.  Returns (ids int32 [T,k], w float32 [T,k])."""
    rng = _rng(seed, 1)
    m = max(k, int(math.ceil(beta * E - 1e-9)))
    m = min(m, E)
    subset = rng.permutation(E)[:m]
    keys = rng.random((T, m))
    pick = np.argsort(keys, axis=1, kind="stable")[:, :k]
    ids = subset[pick].astype(np.int32)
    return ids, _softmax_gates(rng, T, k)


def routing_zipf(T: int, k: int, E: int, s: float, seed: int):
    """Expert popularity proportional to rank^-s over a seeded permutation;
    each token draws k distinct experts without replacement in proportion to
    popularity (Gumbel top-k).  Returns (ids, w) as routing_subset."""
    rng = _rng(seed, 2)
    perm = rng.permutation(E)
    logp = -s * np.log(np.arange(1, E + 1, dtype=np.float64))
    gumbel = -np.log(-np.log(rng.random((T, E))))
    pick = np.argsort(-(logp[None, :] + gumbel), axis=1, kind="stable")[:, :k]
    ids = perm[pick].astype(np.int32)
    return ids, _softmax_gates(rng, T, k)


def routing(T: int, shape: Shape, beta, seed: int):
    """beta: a float (subset fraction) or the string 'zipf<s>'."""
    if isinstance(beta, str):
        assert beta.startswith("zipf")
        return routing_zipf(T, shape.k, shape.E, float(beta[4:]), seed)
    return routing_subset(T, shape.k, shape.E, float(beta), seed)


def histogram_subset(T: int, k: int, E: int, beta: float, seed: int) -> np.ndarray:
    """Expert histogram of routing_subset without materialising weights."""
    ids, _ = routing_subset(T, k, E, beta, seed)
    return np.bincount(ids.reshape(-1), minlength=E).astype(np.int32)


def _normal_bf16(shape, std: float, gen: torch.Generator, device) -> torch.Tensor:
    return (torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * std).to(torch.bfloat16)


def layer_tensors(shape: Shape, T: int, seed: int, device="cpu", x_std: float | None = None):
    """X [T,H], W_gate/W_up [E,H,I], W_down [E,I,H], all bf16 ~ N(0, 1/sqrt(fan_in)),
    generated expert by expert on `device` so the largest layer never needs an
    fp32 copy.  x_std overrides the activation scale (default 1/sqrt(H))."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    H, I, E = shape.H, shape.I, shape.E
    gen.manual_seed(1000003 * int(seed) + 17)
    X = _normal_bf16((T, H), (1.0 / math.sqrt(H)) if x_std is None else x_std, gen, dev)
    Wg = torch.empty((E, H, I), dtype=torch.bfloat16, device=dev)
    Wu = torch.empty((E, H, I), dtype=torch.bfloat16, device=dev)
    Wd = torch.empty((E, I, H), dtype=torch.bfloat16, device=dev)
    for e in range(E):
        gen.manual_seed(1000003 * int(seed) + 101 + e)
        Wg[e] = _normal_bf16((H, I), 1.0 / math.sqrt(H), gen, dev)
        Wu[e] = _normal_bf16((H, I), 1.0 / math.sqrt(H), gen, dev)
        Wd[e] = _normal_bf16((I, H), 1.0 / math.sqrt(I), gen, dev)
    return X, Wg, Wu, Wd


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 array of its bit patterns (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> exact float64 values."""
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
