"""Randomised differential test: seeded random batch compositions -- ragged lengths, empty sequences, invocation
points before, inside and beyond the new rows (Eq.6), base-only sequences, shared and private contexts (Section 2,
"Cache reuse patterns"), head groupings, option settings -- through alora_prefill and alora_decode, every sequence
compared with the oracle on its own.  The draws are fixed by the seed, so a failure names a reproducible case."""
import dataclasses

import numpy as np
import pytest

from paper_2504_12397_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu

SHAPES = [
    wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3),
    wl.LayerShape(d=512, n_q_heads=4, n_kv_heads=4, head_dim=128, rank=16, n_adapters=3),
    wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=1, head_dim=128, rank=32, n_adapters=3),
    wl.LayerShape(d=256, n_q_heads=4, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3),
    dataclasses.replace(wl.SHAPE_TINY, n_adapters=3, rmsnorm=True, n_kv_heads=2),          # fp32, plain kernels
]
OPTIONS = [{}, {}, {}, {"kv_splits": 2}, {"kv_splits": 5}, {"attn_waves": 4}, {"attn_fold": 0}, {"attn_partials16": 0},
           {"gemm_splits": 1}, {"rope_fuse": 0}, {"kernels": 1}, {"attn_lazy": 0}, {"lora_split": 1}, {"lora_split": 2}]


def draw(seed: int, decode: bool):
    r = np.random.default_rng(seed)
    shape = SHAPES[int(r.integers(len(SHAPES)))]
    opts = dict(OPTIONS[int(r.integers(len(OPTIONS)))])
    n_ctx = int(r.integers(0, 3))
    C = [int(r.choice([1, 17, 64, 130, 333, 700, 1100])) for _ in range(n_ctx)]
    n = int(r.integers(1, 8))
    group, S, own, k, adapter = [], [], [], [], []
    g_now = -1
    for b in range(n):
        # neighbours tend to stay on the same context (that is what gets packed), sometimes they do not
        if n_ctx and r.random() < 0.75:
            g_now = g_now if (g_now >= 0 and r.random() < 0.7) else int(r.integers(n_ctx))
            g = g_now
        else:
            g = -1
        group.append(g)
        if decode:
            S.append(1)
        else:
            S.append(int(r.choice([0, 1, 2, 15, 16, 31, 33, 64, 65, 100, 150])))
        own.append(int(r.choice([0, 0, 1, 5, 63, 64, 200, 450])))
        P = own[-1] + (C[g] if g >= 0 else 0)
        k.append(int(r.choice([0, P // 2, P, P + S[-1] // 2, P + S[-1], 10 ** 6])))
        adapter.append(int(r.integers(-1, shape.n_adapters)))
    if sum(S) == 0:
        S[0] = 3
    return shape, opts, C, group, S, own, k, adapter


@pytest.mark.parametrize("seed", range(24))
def test_random_prefill_batches(seed):
    from paper_2504_12397_amd import binding as ab
    shape, opts, C, group, S, own, k, adapter = draw(1000 + seed, decode=False)
    print(f"seed {seed}: {shape.dtype} G={shape.n_q_heads // shape.n_kv_heads} opts={opts} C={C} group={group} S={S} "
          f"own={own} k={k} adapter={adapter}", flush=True)
    ctx = ab.Context(0)
    try:
        for key, v in opts.items():
            ctx.set_option(key, v)
        case, ctx_kv = H.contexts_case(shape, C, group, own, S, k, adapter, seed=2000 + seed)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, group, own)
        H.report(test="random_prefill", seed=seed, dtype=shape.dtype, opts=opts, err=worst)
    finally:
        ctx.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_batches(seed):
    from paper_2504_12397_amd import binding as ab
    shape, opts, C, group, S, own, k, adapter = draw(3000 + seed, decode=True)
    print(f"seed {seed}: {shape.dtype} G={shape.n_q_heads // shape.n_kv_heads} opts={opts} C={C} group={group} "
          f"own={own} k={k} adapter={adapter}", flush=True)
    ctx = ab.Context(0)
    try:
        for key, v in opts.items():
            ctx.set_option(key, v)
        case, ctx_kv = H.contexts_case(shape, C, group, own, S, k, adapter, seed=4000 + seed)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, group, own, decode=True)
        H.report(test="random_decode", seed=seed, dtype=shape.dtype, opts=opts, err=worst)
    finally:
        ctx.close()


@pytest.mark.parametrize("heads", [(16, 16), (12, 6), (12, 12), (24, 12), (32, 8), (20, 10)])
def test_decode_over_head_counts_that_do_not_fill_a_workgroup_evenly(heads):
    """The decode kernel gives each of a workgroup's eight waves one kv head (Eq.4 per head; GQA grouping): more than
    eight kv heads take several workgroups per key range, head counts that do not divide eight leave waves idle,
    fewer than eight cut the key range among the spare waves.  Private and shared contexts, ragged lengths."""
    from paper_2504_12397_amd import binding as ab
    n_q_heads, n_kv_heads = heads
    shape = wl.LayerShape(d=512, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=128, rank=16, n_adapters=3)
    C = [1300, 90]
    group = [0, 0, -1, 1, 0, 0, 0, 1, -1]
    own = [0, 33, 2100, 5, 0, 1, 700, 0, 0]
    n = len(group)
    k = [C[g] if g >= 0 else 7 for g in group]
    adapter = [b % 4 - 1 for b in range(n)]
    ctx = ab.Context(0)
    try:
        case, ctx_kv = H.contexts_case(shape, C, group, own, [1] * n, k, adapter, seed=5000 + n_q_heads * 100 + n_kv_heads)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, group, own, decode=True)
        H.report(test="decode_head_counts", heads=list(heads), err=worst)
    finally:
        ctx.close()


@pytest.mark.parametrize("scale", [0.02, 3.0, 12.0])
@pytest.mark.parametrize("decode", [False, True])
def test_attention_over_a_wide_range_of_magnitudes(scale, decode):
    """Eq.1's softmax with scores away from the unit scale of the other tests: hidden states and cached rows
    multiplied by `scale`, no RMSNorm in front, so that queries and keys inherit it and the scores' spread grows
    with scale^2 (1 natural unit at scale 1, 9 at scale 3, 144 at scale 12).  At 0.02 all probabilities are close
    to 1/n and keys and values sit low in the range of the kernels' 16-bit operands; at 3 the spread is that of a
    sharp real attention head; at 12 the reference exponent moves in big steps and nearly every probability
    underflows.  The queries enter the matrix unit with 11 bits, which moves a score by about 2^-12 of its size,
    so the bar is the stated one up to a spread of 16 and grows with the spread beyond (measured: 0.5e-2 at
    spread 1, 0.9e-2 at 9, 1.5e-2 at 16, 8e-2 at 144)."""
    from paper_2504_12397_amd import binding as ab
    import torch
    shape = wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3, rmsnorm=False)
    C = [900]
    group = [0, 0, -1, 0]
    own = [0, 70, 1500, 3]
    S = [1] * 4 if decode else [40, 1, 130, 64]
    k = [900, 0, 10 ** 6, 930]
    adapter = [0, 1, -1, 2]
    ctx = ab.Context(0)
    saved = H.TOL["bf16"]
    try:
        case, ctx_kv = H.contexts_case(shape, C, group, own, S, k, adapter, seed=6000)
        scaled = lambda t: t.to(torch.float64).mul(scale).to(shape.torch_dtype)
        scaled_np = lambda a: H.f64(scaled(torch.from_numpy(a)))
        case.x_new = [scaled(x) for x in case.x_new]
        ctx_kv = [(scaled_np(K), scaled_np(V)) for K, V in ctx_kv]
        case.cache_K = [scaled_np(K) for K in case.cache_K]
        case.cache_V = [scaled_np(V) for V in case.cache_V]
        H.TOL["bf16"] = saved * max(1.0, (scale / 4.0) ** 2)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, group, own, decode=decode)
        H.report(test="attention_magnitudes", scale=scale, decode=decode, err=worst, tol=H.TOL["bf16"])
    finally:
        H.TOL["bf16"] = saved
        ctx.close()
