"""Seeded synthetic workloads shaped like the Activated-LoRA inference experiment.

This module only draws random tensors and lengths.  It holds none of the method's
arithmetic (no projections, no rotary embedding, no attention, no normalisation), so
that the CPU oracle and the HIP path can both be fed from it without sharing code.

Shapes follow the timing experiment of the paper (Section "Inference timing results",
Appendix "Inference Timing Performance Evaluation Details"): a long base-model prefix
whose keys/values are already cached, a short adapter-activated suffix, rank 8-64
adapters on the q/k/v projections, several adapters sharing a batch, and short
generations.  Value distributions: x ~ N(0,1); W ~ N(0,1/d); A ~ N(0,1/d);
B ~ N(0,0.02^2); RMSNorm gain ~ N(1,0.1^2) so that a dropped gain is visible.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Optional

import numpy as np
import torch

BASE_SEED = 20250412


@dataclasses.dataclass(frozen=True)
class LayerShape:
    d: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rank: int
    n_adapters: int
    dtype: str = "bf16"          # "bf16" or "f32": storage type of x, W, A, B, cache, outputs
    rmsnorm: bool = True
    intermediate: int = 0        # SwiGLU width; 0 = attention block only
    adapt_rest: bool = False     # adapters on W_o and the MLP linears too (needs intermediate > 0)
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    scale: float = 2.0

    @property
    def n_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def n_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n_qkv(self) -> int:
        return self.n_q + 2 * self.n_kv

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


SHAPE_TINY = LayerShape(d=256, n_q_heads=4, n_kv_heads=4, head_dim=64, rank=8, n_adapters=1,
                        dtype="f32", rmsnorm=False)
SHAPE_8B = LayerShape(d=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=32, n_adapters=1)
SHAPE_8B_4AD = dataclasses.replace(SHAPE_8B, n_adapters=4)
SHAPE_8B_STACK = dataclasses.replace(SHAPE_8B, rank=64, intermediate=14336)


class Rng:
    """Named, seeded normal draws.  Every tensor gets a stream of its own derived from its
    name, so adding a tensor never shifts the values of another.  On the CPU the stream is
    numpy's counter-based Philox; on a GPU it is torch's device generator (used for the
    multi-gigabyte bench tensors, which nothing needs to reproduce on the host bit for bit:
    whoever wants them on the host copies them back)."""

    def __init__(self, seed: int, device: str = "cpu"):
        self.seed = int(seed)
        self.device = torch.device(device)

    def _key(self, name: str) -> int:
        return (self.seed << 32) ^ zlib.crc32(name.encode())

    def normal(self, name: str, shape, std: float = 1.0, mean: float = 0.0,
               dtype: torch.dtype = torch.float32) -> torch.Tensor:
        shape = tuple(int(s) for s in shape)
        if self.device.type == "cpu":
            g = np.random.Generator(np.random.Philox(key=self._key(name)))
            a = g.standard_normal(size=shape, dtype=np.float32)
            t = torch.from_numpy(a)
            t = t.mul_(std).add_(mean)
            return t.to(dtype)
        g = torch.Generator(device=self.device)
        g.manual_seed(self._key(name) & ((1 << 63) - 1))
        n = int(np.prod(shape)) if shape else 1
        out = torch.empty(shape, dtype=dtype, device=self.device)
        flat = out.view(-1)
        step = 1 << 26                       # bounded fp32 staging for very large tensors
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            chunk = torch.randn(hi - lo, generator=g, device=self.device, dtype=torch.float32)
            flat[lo:hi] = chunk.mul_(std).add_(mean).to(dtype)
        return out

    def integers(self, name: str, low: int, high_inclusive: int, n: int) -> List[int]:
        g = np.random.Generator(np.random.Philox(key=self._key(name)))
        return [int(v) for v in g.integers(low, high_inclusive + 1, size=n)]

    def permutation(self, name: str, n: int) -> List[int]:
        g = np.random.Generator(np.random.Philox(key=self._key(name)))
        return [int(v) for v in g.permutation(n)]


def make_layer(shape: LayerShape, rng: Rng, tag: str = "L0") -> Dict[str, Optional[torch.Tensor]]:
    """Random-init weights of one decoder layer, in the storage dtype of `shape`.

    W_qkv [N_q+2N_kv, d] (rows: q | k | v); A [n_ad, 3, r, d]; B_q [n_ad, N_q, r];
    B_k, B_v [n_ad, N_kv, r]; scale: python list [n_ad]; rms_gain [d] or None.
    With shape.intermediate > 0 also W_o [d, N_q], rms2_gain [d], W_gate, W_up [I, d],
    W_down [d, I]; with shape.adapt_rest their adapters A_o [n_ad, r, N_q], B_o [n_ad, d, r],
    A_gu [n_ad, 2, r, d], B_gate, B_up [n_ad, I, r], A_down [n_ad, r, I], B_down [n_ad, d, r]."""
    dt = shape.torch_dtype
    d, r, na = shape.d, shape.rank, shape.n_adapters
    sd = 1.0 / np.sqrt(d)
    L: Dict[str, Optional[torch.Tensor]] = {}
    L["W_qkv"] = rng.normal(f"{tag}.W_qkv", (shape.n_qkv, d), sd, dtype=dt)
    L["A"] = rng.normal(f"{tag}.A", (na, 3, r, d), sd, dtype=dt)
    L["B_q"] = rng.normal(f"{tag}.B_q", (na, shape.n_q, r), 0.02, dtype=dt)
    L["B_k"] = rng.normal(f"{tag}.B_k", (na, shape.n_kv, r), 0.02, dtype=dt)
    L["B_v"] = rng.normal(f"{tag}.B_v", (na, shape.n_kv, r), 0.02, dtype=dt)
    L["scale"] = [float(shape.scale)] * na
    L["rms_gain"] = rng.normal(f"{tag}.rms_gain", (d,), 0.1, 1.0, dtype=dt) if shape.rmsnorm else None
    if shape.intermediate:
        I = shape.intermediate
        L["W_o"] = rng.normal(f"{tag}.W_o", (d, shape.n_q), 1.0 / np.sqrt(shape.n_q), dtype=dt)
        L["rms2_gain"] = rng.normal(f"{tag}.rms2_gain", (d,), 0.1, 1.0, dtype=dt)
        L["W_gate"] = rng.normal(f"{tag}.W_gate", (I, d), sd, dtype=dt)
        L["W_up"] = rng.normal(f"{tag}.W_up", (I, d), sd, dtype=dt)
        L["W_down"] = rng.normal(f"{tag}.W_down", (d, I), 1.0 / np.sqrt(I), dtype=dt)
        if shape.adapt_rest:
            L["A_o"] = rng.normal(f"{tag}.A_o", (na, r, shape.n_q), 1.0 / np.sqrt(shape.n_q), dtype=dt)
            L["B_o"] = rng.normal(f"{tag}.B_o", (na, d, r), 0.02, dtype=dt)
            L["A_gu"] = rng.normal(f"{tag}.A_gu", (na, 2, r, d), sd, dtype=dt)
            L["B_gate"] = rng.normal(f"{tag}.B_gate", (na, I, r), 0.02, dtype=dt)
            L["B_up"] = rng.normal(f"{tag}.B_up", (na, I, r), 0.02, dtype=dt)
            L["A_down"] = rng.normal(f"{tag}.A_down", (na, r, I), 1.0 / np.sqrt(I), dtype=dt)
            L["B_down"] = rng.normal(f"{tag}.B_down", (na, d, r), 0.02, dtype=dt)
    return L


def make_hidden(rng: Rng, name: str, n_tokens: int, shape: LayerShape) -> torch.Tensor:
    return rng.normal(name, (n_tokens, shape.d), 1.0, dtype=shape.torch_dtype)


def make_random_kv(rng: Rng, name: str, n_tokens: int, shape: LayerShape):
    """Stand-in cache contents for prefixes too long for a CPU base pass: with W ~ N(0,1/d)
    and unit-variance inputs the true keys and values are N(0,1) per element."""
    k = rng.normal(name + ".K", (n_tokens, shape.n_kv_heads, shape.head_dim), 1.0, dtype=shape.torch_dtype)
    v = rng.normal(name + ".V", (n_tokens, shape.n_kv_heads, shape.head_dim), 1.0, dtype=shape.torch_dtype)
    return k, v


@dataclasses.dataclass
class Batch:
    """Per-sequence lengths of one call: P = tokens already cached, S = new tokens,
    k = 0-based absolute position of the first adapted token, adapter = id or -1."""
    shape: LayerShape
    P: List[int]
    S: List[int]
    k: List[int]
    adapter: List[int]
    name: str = ""
    seed: int = BASE_SEED

    @property
    def n_seqs(self) -> int:
        return len(self.P)

    @property
    def T(self) -> int:
        return int(sum(self.S))

    @property
    def cu_seqlens(self) -> List[int]:
        out = [0]
        for s in self.S:
            out.append(out[-1] + int(s))
        return out


def config1() -> Batch:
    """Single attention block, fp32, 64 cached base tokens + 16 adapted tokens."""
    return Batch(SHAPE_TINY, P=[64], S=[16], k=[64], adapter=[0], name="c1", seed=BASE_SEED + 1)


def config2() -> Batch:
    """One 8B-class layer, bf16, 4096 cached base tokens + 256 adapted tokens."""
    return Batch(SHAPE_8B, P=[4096], S=[256], k=[4096], adapter=[0], name="c2", seed=BASE_SEED + 2)


def regime2():
    """Second cache-reuse regime of Section 2 ("Cache reuse patterns"): an adapter call over 4096 tokens of context that the
    base model has not cached (k = 4096 > P = 0) plus 256 adapted tokens, then a base-model turn of
    256 tokens that reuses the 4096 base rows the adapter call left behind."""
    seed = BASE_SEED + 6
    first = Batch(SHAPE_8B, P=[0], S=[4096 + 256], k=[4096], adapter=[0], name="r2.adapter_call", seed=seed)
    then = Batch(SHAPE_8B, P=[4096], S=[256], k=[0], adapter=[-1], name="r2.base_turn", seed=seed)
    return first, then


def config3() -> Batch:
    """Mixed batch: 16 sequences, 4 adapters, 3 sequences base-only."""
    seed = BASE_SEED + 3
    rng = Rng(seed)
    P = rng.integers("c3.P", 512, 8192, 16)
    S = rng.integers("c3.S", 32, 512, 16)
    ad = rng.integers("c3.adapter", 0, 3, 16)
    for b in rng.permutation("c3.base_only", 16)[:3]:
        ad[b] = -1
    return Batch(SHAPE_8B_4AD, P=P, S=S, k=list(P), adapter=ad, name="c3", seed=seed)


def config4() -> Batch:
    """Decode step: 64 sequences, 16384 base tokens + 64 adapted tokens cached, 1 new token."""
    n = 64
    return Batch(SHAPE_8B_4AD, P=[16384 + 64] * n, S=[1] * n, k=[16384] * n,
                 adapter=[b % 4 for b in range(n)], name="c4", seed=BASE_SEED + 4)


def regime3(n_contexts: int = 16, per_context: int = 4, context: int = 16384, own: int = 64):
    """Third cache-reuse regime of Section 2, "Cache reuse patterns" (N adapters on one context, Proposition 2's N-adapter
    clause) as a decode step: the c4 batch regrouped into 16 contexts of 16384 base tokens, each
    read by 4 sequences with different adapters that hold 64 adapted rows of their own.  Returns
    the batch and, per sequence, the index of its context."""
    n = n_contexts * per_context
    batch = Batch(SHAPE_8B_4AD, P=[context + own] * n, S=[1] * n, k=[context] * n,
                  adapter=[b % per_context % 4 for b in range(n)], name="r3", seed=BASE_SEED + 7)
    return batch, [b // per_context for b in range(n)], context


def regime3_prefill(n_contexts: int = 4, per_context: int = 8, context: int = 16384, invocation: int = 16):
    """The same regime at the moment the adapters are invoked (Section 2, "Cache reuse patterns"; the invocation
    sequences of the appendix "Invocation sequences" are three or four tokens, Proposition 2's T_new counts them and
    what follows): 4 contexts of 16384 base tokens, each invoked by 8 adapter calls
    whose 16-token invocation sequences are prefilled in one call.  Returns the batch and, per sequence, the index
    of its context."""
    n = n_contexts * per_context
    batch = Batch(SHAPE_8B_4AD, P=[context] * n, S=[invocation] * n, k=[context] * n,
                  adapter=[b % per_context % 4 for b in range(n)], name="r3p", seed=BASE_SEED + 8)
    return batch, [b // per_context for b in range(n)], context


def config5(full_lora: bool = False) -> Batch:
    """32-layer stack shape: 32768 cached tokens + 128 adapted tokens (aLoRA), or the same
    32896 tokens recomputed from scratch with the adapter on everywhere (k = 0)."""
    if full_lora:
        return Batch(SHAPE_8B_STACK, P=[0], S=[32768 + 128], k=[0], adapter=[0], name="c5_k0",
                     seed=BASE_SEED + 5)
    return Batch(SHAPE_8B_STACK, P=[32768], S=[128], k=[32768], adapter=[0], name="c5",
                 seed=BASE_SEED + 5)


N_LAYERS_STACK = 32


def evaluators_on_one_context(n_evaluators: int = 8, context: int = 32768, invocation: int = 128):
    """Config 5 with N adapters instead of one (Proposition 2: N adapters invoked on one context cost N small
    prefills, not N recomputations; Section 3's pipeline runs several evaluators on one base answer): N sequences of
    128 adapted tokens each, every one with an adapter of its own, all reading the same 32768 cached base tokens."""
    shape = dataclasses.replace(SHAPE_8B_STACK, n_adapters=n_evaluators)
    n = n_evaluators
    return Batch(shape, P=[context] * n, S=[invocation] * n, k=[context] * n, adapter=list(range(n)), name="c5n",
                 seed=BASE_SEED + 9)
