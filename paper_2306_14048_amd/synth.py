"""Seeded synthetic inputs shaped like the paper's workloads.

The throughput experiments of the paper already run on synthetic prompts padded
to one length with a fixed generation length (Sec. 5.3) on OPT-6.7B / OPT-30B
shaped attention (32 / 56 heads of dimension 128); the heavy-tailed per-token
key scale stands in for the power-law accumulated scores and the > 95 %
attention sparsity it observes (Sec. 3).  This module only draws random
numbers: it contains none of the method's arithmetic and is shared by the
tests (GPU path and CPU oracle both consume the tensors made here) and the
benchmark.

Recipe: every element of Q, K, V is N(0, 1) in fp32 from a torch generator
seeded by (seed, layer, step, tensor id); each key row is multiplied by
exp(sigma * g) with one g ~ N(0, 1) per (batch, head, token); the result is
rounded to the storage dtype.  Values are generated on the device they are
requested on; a checker must always consume the materialised tensors (copied
to the host), never a regeneration on another device.
"""
from __future__ import annotations

import dataclasses
import math

import torch

BASE_SEED = 20230614
_TENSOR_ID = {"q": 0, "k": 1, "v": 2, "kscale": 3}
PROMPT_STEP = 0xFFFFF          # "step" slot of the seed used for prompt tensors


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    head_dim: int
    prompt: int
    steps: int
    heavy: int
    recent: int
    dtype: torch.dtype
    sigma: float
    layers: int = 1

    @property
    def budget(self) -> int:
        return self.heavy + self.recent


def split_budget(prompt: int, frac: float):
    """Budget rule: k = round(frac * prompt), heavy = ceil(k / 2), recent = k - heavy."""
    k = int(round(frac * prompt))
    heavy = (k + 1) // 2
    return heavy, k - heavy


def _wl(name, batch, heads, d, prompt, steps, frac, dtype, sigma, layers=1):
    h, r = split_budget(prompt, frac)
    return Workload(name, batch, heads, d, prompt, steps, h, r, dtype, sigma, layers)


# The five workload definitions this build is measured and checked on.
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", 1, 8, 64, 256, 64, 32, 32, torch.float32, 0.75),
    "opt6.7b_layer_f16": _wl("opt6.7b_layer_f16", 16, 32, 128, 2048, 256, 0.20, torch.float16, 1.0),
    "prefill_bf16": _wl("prefill_bf16", 4, 32, 128, 4096, 0, 0.20, torch.bfloat16, 1.0),
    "opt30b_layer_f16": _wl("opt30b_layer_f16", 64, 56, 128, 1024, 1024, 0.20, torch.float16, 1.0),
    "stack32_f16": _wl("stack32_f16", 128, 32, 128, 8192, 128, 0.05, torch.float16, 1.25, layers=32),
}


def _generator(device, seed: int, layer: int, step: int, tensor: str) -> torch.Generator:
    g = torch.Generator(device=device)
    mixed = (seed * 1000003 + layer) * 1000003 + step
    mixed = (mixed * 8 + _TENSOR_ID[tensor]) % (2 ** 63 - 1)
    g.manual_seed(mixed)
    return g


def _draw(shape, device, seed, layer, step, tensor):
    return torch.randn(shape, generator=_generator(device, seed, layer, step, tensor),
                       device=device, dtype=torch.float32)


def make_prompt(batch, heads, n, d, dtype, sigma, device, seed=BASE_SEED, layer=0,
                batch_chunk=None):
    """Q, K, V of shape [batch, heads, n, d] in `dtype`.  Large prompts are drawn
    one batch chunk at a time to bound the fp32 staging memory."""
    device = torch.device(device)
    if batch_chunk is None:
        per = heads * n * d * 4
        batch_chunk = max(1, min(batch, (1 << 31) // max(per, 1)))
    Q = torch.empty((batch, heads, n, d), dtype=dtype, device=device)
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)
    for b0 in range(0, batch, batch_chunk):
        b1 = min(batch, b0 + batch_chunk)
        shp = (b1 - b0, heads, n, d)
        step = PROMPT_STEP + b0          # distinct stream per chunk
        Q[b0:b1] = _draw(shp, device, seed, layer, step, "q").to(dtype)
        ks = torch.exp(sigma * _draw(shp[:3] + (1,), device, seed, layer, step, "kscale"))
        K[b0:b1] = (_draw(shp, device, seed, layer, step, "k") * ks).to(dtype)
        V[b0:b1] = _draw(shp, device, seed, layer, step, "v").to(dtype)
    return Q, K, V


def make_steps(batch, heads, d, steps, dtype, sigma, device, seed=BASE_SEED, layer=0,
               first_step=0):
    """q, k, v for `steps` generation steps, each [steps, batch, heads, d]: the
    new token's query/key/value come from the same distribution as the prompt."""
    device = torch.device(device)
    qs, ks, vs = [], [], []
    for s in range(first_step, first_step + steps):
        shp = (batch, heads, d)
        qs.append(_draw(shp, device, seed, layer, s, "q").to(dtype))
        sc = torch.exp(sigma * _draw(shp[:2] + (1,), device, seed, layer, s, "kscale"))
        ks.append((_draw(shp, device, seed, layer, s, "k") * sc).to(dtype))
        vs.append(_draw(shp, device, seed, layer, s, "v").to(dtype))
    if not qs:
        e = torch.empty((0, batch, heads, d), dtype=dtype, device=device)
        return e, e.clone(), e.clone()
    return torch.stack(qs), torch.stack(ks), torch.stack(vs)


def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)
