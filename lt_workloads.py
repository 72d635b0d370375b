"""Seeded synthetic inputs for the LightTransfer hot path.

This module only makes inputs: shapes, seeds, random tensors and the planted key/query
bias that gives some layers a lazy attention pattern.  It holds none of the method's
arithmetic (no softmax, no lazy ratio, no selection) and is the one module that both
the GPU tests/benchmark and the CPU oracle tests may share.

The paper measures on LongBench, Ruler and math benchmarks with LLaMA / Mistral / Qwen
weights; none of that is available here and the cost of the path depends only on shapes.
These workloads take the attention shapes of those model families and the paper's
context lengths, with i.i.d. N(0,1) bf16 values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 13846


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # position in the benchmark's list of configurations
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int               # prompt length n
    w_sink: int
    w_recent: int
    n_lazy: int
    decode_steps: int
    w_last: int = 64
    bias: str = "none"         # "none" | "planted" (chosen layers get magnitude 3.0) | "spread" (every layer, U[0,3])
    bias_magnitude: float = 3.0
    bias_recent: int = 256     # the last bias_recent prompt keys (and the first w_sink) carry the bias

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def max_tokens(self) -> int:
        return self.context + self.decode_steps

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (used by CPU tests that need the oracle to finish quickly)."""
        return replace(self, **kw)


WORKLOADS = {
    # 2 layers (layer 0 full, layer 1 streaming), the correctness configuration
    "tiny": Workload("tiny", 0, 2, 1, 32, 8, 128, 4096, 4, 1020, 1, 16),
    # Llama-3-8B-shaped stack, 16 planted lazy layers: the configuration the metric is quoted on
    "llama3_8b_32k": Workload("llama3_8b_32k", 1, 32, 8, 32, 8, 128, 32768, 4, 2044, 16, 128, bias="planted"),
    # Mistral-7B-shaped sweep over the lazy fraction (n_lazy set per sweep point)
    "mistral_7b_16k": Workload("mistral_7b_16k", 2, 32, 32, 32, 8, 128, 16384, 4, 2044, 16, 64, bias="spread"),
    # QwQ-32B-shaped long generation, fixed mask (pre-selected layers)
    "qwq_32b_gen": Workload("qwq_32b_gen", 3, 64, 4, 40, 8, 128, 1024, 4, 2044, 32, 31744),
    # 128K context, Llama-3.1-8B-shaped
    "llama31_8b_128k_b1": Workload("llama31_8b_128k_b1", 4, 32, 1, 32, 8, 128, 131072, 4, 4092, 16, 32, bias="planted"),
    "llama31_8b_128k_b16": Workload("llama31_8b_128k_b16", 4, 32, 16, 32, 8, 128, 131072, 4, 4092, 16, 32, bias="planted"),
    # a group of eight query heads per KV head (Llama-3-70B-shaped attention): not one of the benchmark's
    # configurations, but the shape where the decode kernels differ most
    # multi-head attention (one query head per KV head, LLaMA2-7B-shaped stack at its 4K context, the paper's default
    # 4 + 1020 window): the other end of the group sizes the paper's models have (1, 4, 5, 8)
    "llama2_7b_4k": Workload("llama2_7b_4k", 6, 32, 32, 32, 32, 128, 4096, 4, 1020, 16, 64, bias="planted"),
    "llama3_70b_32k": Workload("llama3_70b_32k", 5, 80, 4, 64, 8, 128, 32768, 4, 2044, 40, 64, bias="planted"),
}


def seed_for(wl: Workload, layer: int, step: Optional[int] = None, stream: int = 0) -> int:
    """One seed per (configuration, layer, decode step, tensor stream)."""
    s = BASE_SEED + 1000 * wl.index + layer + 7919 * stream
    if step is not None:
        s += 100000 * (step + 1)
    return s


def randn_bf16(shape, seed: int, device="cpu") -> torch.Tensor:
    """N(0,1) drawn in fp32 from a seeded generator on `device`, rounded to bf16 (nearest even)."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a bf16 tensor as uint16 bit patterns (exact, what the oracle consumes)."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_bf16(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """Inverse of bf16_bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def planted_lazy_layers(wl: Workload) -> List[int]:
    """The seeded choice of layers that are built to look lazy (sorted)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 1000 * wl.index + 999)
    perm = torch.randperm(wl.n_layers, generator=g).tolist()
    return sorted(perm[: wl.n_lazy])


def layer_bias_magnitude(wl: Workload, layer: int) -> float:
    """Mean logit shift given to the first w_sink and last bias_recent prompt keys of a layer."""
    if wl.bias == "planted":
        return wl.bias_magnitude if layer in planted_lazy_layers(wl) else 0.0
    if wl.bias == "spread":
        g = torch.Generator(device="cpu")
        g.manual_seed(BASE_SEED + 1000 * wl.index + 998)
        mags = torch.rand(wl.n_layers, generator=g) * wl.bias_magnitude
        return float(mags[layer])
    return 0.0


def _bias_direction(wl: Workload, layer: int, device) -> torch.Tensor:
    """Seeded unit vector per (sequence, KV head): [B, Hkv, d] fp32."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed_for(wl, layer, stream=5))
    u = torch.randn(wl.batch, wl.n_kv_heads, wl.head_dim, generator=g)
    u = u / u.norm(dim=-1, keepdim=True)
    return u.to(device)


def _bias_coeff(wl: Workload, layer: int) -> float:
    """c with c*c*scale = magnitude: adding c*u to a query and to a key shifts their logit by `magnitude`."""
    return math.sqrt(layer_bias_magnitude(wl, layer) / wl.scale)


def prefill_kv(wl: Workload, layer: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Prompt keys and values of a layer: bf16 [B, Hkv, n, d] each."""
    shape = (wl.batch, wl.n_kv_heads, wl.context, wl.head_dim)
    k = randn_bf16(shape, seed_for(wl, layer, stream=1), device)
    v = randn_bf16(shape, seed_for(wl, layer, stream=2), device)
    c = _bias_coeff(wl, layer)
    if c > 0.0:
        u = (_bias_direction(wl, layer, device) * c).unsqueeze(2)       # [B,Hkv,1,d]
        ns, nr = min(wl.w_sink, wl.context), min(wl.bias_recent, wl.context)
        k[:, :, :ns] = (k[:, :, :ns].float() + u).to(torch.bfloat16)
        k[:, :, wl.context - nr:] = (k[:, :, wl.context - nr:].float() + u).to(torch.bfloat16)
    return k, v


def _bias_queries(wl: Workload, layer: int, q: torch.Tensor) -> torch.Tensor:
    """q [B, Hq, ..., d]: add the layer's bias direction of each head's KV group."""
    c = _bias_coeff(wl, layer)
    if c == 0.0:
        return q
    u = _bias_direction(wl, layer, q.device) * c                           # [B,Hkv,d]
    u = u.repeat_interleave(wl.group, dim=1)                                # [B,Hq,d]
    while u.dim() < q.dim():
        u = u.unsqueeze(-2)
    return (q.float() + u).to(torch.bfloat16)


def last_queries(wl: Workload, layer: int, device="cpu", w_last: Optional[int] = None) -> torch.Tensor:
    """Queries of the last w_last prompt positions: bf16 [B, Hq, w, d]."""
    w = wl.w_last if w_last is None else w_last
    q = randn_bf16((wl.batch, wl.n_q_heads, w, wl.head_dim), seed_for(wl, layer, stream=3), device)
    return _bias_queries(wl, layer, q)


def prefill_queries(wl: Workload, layer: int, device="cpu") -> torch.Tensor:
    """Queries of every prompt position: bf16 [B, Hq, n, d]; the last w_last rows are last_queries()."""
    w = min(wl.w_last, wl.context)
    q = randn_bf16((wl.batch, wl.n_q_heads, wl.context, wl.head_dim), seed_for(wl, layer, stream=4), device)
    q = _bias_queries(wl, layer, q)
    q[:, :, wl.context - w:] = last_queries(wl, layer, device, w)
    return q


def decode_qkv(wl: Workload, layer: int, step: int, device="cpu"):
    """Query, key and value of the token generated at `step`: q [B,Hq,d], k/v [B,Hkv,1,d], bf16."""
    q = randn_bf16((wl.batch, wl.n_q_heads, wl.head_dim), seed_for(wl, layer, step, stream=3), device)
    k = randn_bf16((wl.batch, wl.n_kv_heads, 1, wl.head_dim), seed_for(wl, layer, step, stream=1), device)
    v = randn_bf16((wl.batch, wl.n_kv_heads, 1, wl.head_dim), seed_for(wl, layer, step, stream=2), device)
    return _bias_queries(wl, layer, q), k, v


def decode_qkv_block(wl: Workload, layer: int, first_step: int, n_steps: int, device="cpu"):
    """Inputs of n_steps consecutive decode steps of one layer, drawn in one go (benchmark use):
    q [S,B,Hq,d], k/v [S,B,Hkv,1,d], bf16.  Not the same numbers as decode_qkv."""
    q = randn_bf16((n_steps, wl.batch, wl.n_q_heads, wl.head_dim), seed_for(wl, layer, first_step, stream=13), device)
    k = randn_bf16((n_steps, wl.batch, wl.n_kv_heads, 1, wl.head_dim), seed_for(wl, layer, first_step, stream=11), device)
    v = randn_bf16((n_steps, wl.batch, wl.n_kv_heads, 1, wl.head_dim), seed_for(wl, layer, first_step, stream=12), device)
    c = _bias_coeff(wl, layer)
    if c > 0.0:
        u = (_bias_direction(wl, layer, device) * c).repeat_interleave(wl.group, dim=1)     # [B,Hq,d]
        q = (q.float() + u.unsqueeze(0)).to(torch.bfloat16)
    return q, k, v


def kv_bytes_per_step(wl: Workload, is_lazy, total_tokens: int) -> int:
    """Algorithmic K+V bytes one decode step reads: every stored entry once (2 tensors, bf16)."""
    per_token = 2 * wl.n_kv_heads * wl.head_dim * 2
    window = wl.w_sink + wl.w_recent
    total = 0
    for lazy in is_lazy:
        stored = min(total_tokens, window) if lazy else total_tokens
        total += wl.batch * per_token * stored
    return total
