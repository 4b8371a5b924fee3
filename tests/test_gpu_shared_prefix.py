"""Shared-prefix batching (Section 2, "Cache reuse patterns", third regime; Proposition 2 for N adapters on one
context): several sequences read ONE physical copy of the base model's prefix rows and keep only
their own suffix rows.  The oracle knows nothing of sharing -- every sequence is computed on its own
with its own copy of the prefix -- so agreement with it proves that sharing changes nothing."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import alora_oracle as orc
from paper_2504_12397_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ab():
    from paper_2504_12397_amd import binding
    return binding


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def shared_case(shape, C0, S, k, adapter, seed, own_prefix=()):
    """N sequences over one base context of C0 tokens; `own_prefix[b]` = extra cached rows of
    sequence b beyond the shared ones (e.g. an invocation already prefilled)."""
    n = len(S)
    own = list(own_prefix) or [0] * n
    base = H.make_case(shape, [C0 + max(own)], [1], [10 ** 6], [-1], seed=seed)       # base-model rows for the context
    rng = wl.Rng(seed + 1)
    xn = [wl.make_hidden(rng, f"shared.x_new{b}", S[b], shape) for b in range(n)]
    cK, cV, P = [], [], []
    for b in range(n):
        # own cached rows: taken from the same base pass (values do not matter for the comparison,
        # only that the GPU and the oracle hold the same ones)
        cK.append(base.cache_K[0][:C0 + own[b]])
        cV.append(base.cache_V[0][:C0 + own[b]])
        P.append(C0 + own[b])
    return H.Case(shape, base.tensors, base.layer, P, list(S), list(k), list(adapter), [None] * n, xn, cK, cV), own


def build_cache(ab, case, own, C0, shared_mask, extra=4, guard=3):
    """Own regions for the N sequences, then one region that holds the shared context rows."""
    n = len(case.P)
    shape = case.shape
    caps = [(own[b] if shared_mask[b] else case.P[b]) + case.S[b] + extra for b in range(n)] + [C0]
    cache = ab.KVCache(caps, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY, guard_rows=guard)
    ctx_off = int(cache.seq_offset[n])
    nkv = shape.n_kv_heads
    k0 = torch.from_numpy(case.cache_K[0][:C0]).to(shape.torch_dtype).view(C0, nkv, -1).cuda()
    v0 = torch.from_numpy(case.cache_V[0][:C0]).to(shape.torch_dtype).view(C0, nkv, -1).cuda()
    cache.k[ctx_off:ctx_off + C0] = k0
    cache.v[ctx_off:ctx_off + C0] = v0
    for b in range(n):
        o = int(cache.seq_offset[b])
        lo = C0 if shared_mask[b] else 0
        rows = case.P[b] - lo
        if rows:
            cache.k[o:o + rows] = torch.from_numpy(case.cache_K[b][lo:]).to(shape.torch_dtype).view(rows, nkv, -1).cuda()
            cache.v[o:o + rows] = torch.from_numpy(case.cache_V[b][lo:]).to(shape.torch_dtype).view(rows, nkv, -1).cuda()
        cache.seq_len[b] = case.P[b]
        if shared_mask[b]:
            cache.share_prefix(b, ctx_off, C0)
    if not any(shared_mask):
        cache._refresh()
    return cache, ctx_off


def check_shared(ab, ctx, case, own, C0, shared_mask, decode=False):
    tol = H.TOL[case.shape.dtype]
    n = len(case.P)
    cache, ctx_off = build_cache(ab, case, own, C0, shared_mask)
    layer = H.gpu_layer(case, case.shape)
    before_k, before_v = cache.k.clone(), cache.v.clone()
    x = case.x_packed.cuda().contiguous()
    if decode:
        out = ab.alora_decode(ctx, layer, cache, x, case.k, case.adapter)
    else:
        out = ab.alora_prefill(ctx, layer, cache, x, case.cu, case.k, case.adapter)
    torch.cuda.synchronize()
    ref_o, new_rows = H.oracle_prefill(case)
    err = H.rel_err(H.f64(out), ref_o)
    assert err <= tol, f"attention output off by {err:.3e}"
    written = torch.zeros(cache.pool_tokens, dtype=torch.bool)
    for b in range(n):
        lo = C0 if shared_mask[b] else 0
        o = int(cache.seq_offset[b]) + case.P[b] - lo
        written[o:o + case.S[b]] = True
        assert int(cache.seq_len[b]) == case.P[b] + case.S[b]
        if case.S[b]:
            gk = H.f64(cache.k[o:o + case.S[b]]).reshape(case.S[b], -1)
            gv = H.f64(cache.v[o:o + case.S[b]]).reshape(case.S[b], -1)
            assert H.rel_err(gk, new_rows[b][0]) <= tol and H.rel_err(gv, new_rows[b][1]) <= tol
    keep = ~written.cuda()
    assert torch.equal(bits(cache.k[keep]), bits(before_k[keep])), "rows outside the new ones changed (shared prefix included)"
    assert torch.equal(bits(cache.v[keep]), bits(before_v[keep]))
    return out


SHAPES = {
    "G4": wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3),
    "G1": wl.LayerShape(d=512, n_q_heads=4, n_kv_heads=4, head_dim=128, rank=16, n_adapters=3),
    "G8": wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=1, head_dim=128, rank=16, n_adapters=3),
    "f32": dataclasses.replace(wl.SHAPE_TINY, n_adapters=3, rmsnorm=True, n_kv_heads=2),
}


@pytest.mark.parametrize("name", ["G4", "G1", "G8", "f32"])
def test_prefill_over_one_shared_context(ab, name):
    """Five adapter invocations (three adapters, one base-only turn) on one cached context."""
    shape = SHAPES[name]
    ctx = ab.Context(0)
    try:
        C0 = 333
        S = [70, 33, 129, 1, 64]
        case, own = shared_case(shape, C0, S, [C0, C0, C0 + 5, C0, 0], [0, 1, 2, 1, -1], seed=900)
        check_shared(ab, ctx, case, own, C0, [True] * 5)
        # the same call with private copies of the context
        ctx.set_option("kv_splits", 1)
        out_sh = check_shared(ab, ctx, case, own, C0, [True] * 5)
        out_pr = check_shared(ab, ctx, case, own, C0, [False] * 5)
        if name == "f32":
            assert torch.equal(bits(out_sh), bits(out_pr))
        else:
            # the matrix-unit kernel walks a shared context in workgroups of its own and merges: another summation
            # order than the private copy's single walk, the same values to well inside the tolerance
            assert H.rel_err(H.f64(out_sh), H.f64(out_pr)) <= 0.5 * H.TOL["bf16"]
    finally:
        ctx.close()


def test_prefill_over_shared_context_with_folded_softmax(ab):
    """The attention variant that takes prescaled queries (option attn_fold) over a shared context."""
    ctx = ab.Context(0)
    try:
        ctx.set_option("attn_fold", 1)
        C0 = 333
        S = [70, 33, 129, 1, 64]
        case, own = shared_case(SHAPES["G4"], C0, S, [C0, C0, C0 + 5, C0, 0], [0, 1, 2, 1, -1], seed=900)
        check_shared(ab, ctx, case, own, C0, [True] * 5)
        check_shared(ab, ctx, case, own, C0, [True, False, True, False, True])
    finally:
        ctx.close()


@pytest.mark.parametrize("name,opts", [("G4", {}), ("G4", {"kv_splits": 3}), ("G1", {}), ("G8", {}), ("f32", {}),
                                       ("G4", {"kernels": 1})])
def test_decode_over_shared_contexts(ab, name, opts):
    """Decode steps of sequences that name shared prefixes: packed several to a workgroup for the
    prefix part (MFMA kernel), own rows separately; mixed with sequences that share nothing."""
    shape = SHAPES[name]
    ctx = ab.Context(0)
    try:
        for k_, v in opts.items():
            ctx.set_option(k_, v)
        C0 = 1100
        own = [40, 0, 17, 64, 5, 0, 33]            # rows each sequence already holds beyond the context
        n = len(own)
        case, own = shared_case(shape, C0, [1] * n, [C0, C0 + 1, C0, 0, C0 + 50, C0, 10], [0, 1, 2, -1, 1, 0, 2],
                                seed=910, own_prefix=own)
        check_shared(ab, ctx, case, own, C0, [True] * n, decode=True)
        # sequences 1, 4 and 6 keep private copies, the others share
        check_shared(ab, ctx, case, own, C0, [True, False, True, True, False, True, False], decode=True)
        check_shared(ab, ctx, case, own, C0, [True, False, True, True, False, True, False], decode=False)
    finally:
        ctx.close()


def test_two_different_shared_contexts_and_decode_steps(ab):
    """Two groups of sequences, each over its own shared context, through a run of decode steps."""
    shape = SHAPES["G4"]
    ctx = ab.Context(0)
    try:
        n_steps = 4
        C = [700, 260]
        group = [0, 0, 0, 1, 1, 0, 0, 0]           # six sequences on context 0 (two packs), two on context 1
        n = len(group)
        k = [700, 0, 702, 260, 100, 700, 700, 701]
        a = [0, 1, 2, 1, -1, 2, 0, 1]
        bases = [H.make_case(shape, [C[i]], [1], [10 ** 6], [-1], seed=920 + i) for i in range(2)]
        # both contexts must come from the same layer weights: reuse the first case's tensors
        lay, tensors = bases[0].layer, bases[0].tensors
        rng = wl.Rng(930)
        ctxK, ctxV = [], []
        for i in range(2):
            xb = wl.make_hidden(rng, f"ctx{i}", C[i], shape)
            pos = np.arange(C[i])
            xh = orc._normed(lay, H.f64(xb), shape.dtype)
            _, kk, vv = orc.project_qkv(lay, xh, pos, 10 ** 6, -1)
            ctxK.append(orc._store(orc.rope(kk, pos, lay.n_kv_heads, lay.head_dim, lay.rope_theta), shape.dtype))
            ctxV.append(orc._store(vv, shape.dtype))
        xn = [wl.make_hidden(rng, f"steps{b}", n_steps, shape) for b in range(n)]
        case = H.Case(shape, tensors, lay, [C[g] for g in group], [n_steps] * n, k, a, [None] * n, xn,
                      [ctxK[g] for g in group], [ctxV[g] for g in group])
        ref_o, new_rows = H.oracle_prefill(case)

        caps = [n_steps] * n + C
        cache = ab.KVCache(caps, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY, guard_rows=2)
        for i in range(2):
            o = int(cache.seq_offset[n + i])
            cache.k[o:o + C[i]] = torch.from_numpy(ctxK[i]).to(shape.torch_dtype).view(C[i], shape.n_kv_heads, -1).cuda()
            cache.v[o:o + C[i]] = torch.from_numpy(ctxV[i]).to(shape.torch_dtype).view(C[i], shape.n_kv_heads, -1).cuda()
        for b in range(n):
            cache.share_prefix(b, int(cache.seq_offset[n + group[b]]), C[group[b]])
        layer = H.gpu_layer(tensors, shape)
        x_steps = torch.stack([torch.stack([xn[b][t] for b in range(n)]) for t in range(n_steps)]).cuda().contiguous()
        out = ab.alora_decode_steps(ctx, layer, cache, x_steps, k, a)
        torch.cuda.synchronize()
        got = torch.cat([out[:, b] for b in range(n)])
        assert H.rel_err(H.f64(got), ref_o) <= H.TOL["bf16"]
        for b in range(n):
            assert int(cache.seq_len[b]) == C[group[b]] + n_steps
            o = int(cache.seq_offset[b])
            assert H.rel_err(H.f64(cache.k[o:o + n_steps]).reshape(n_steps, -1), new_rows[b][0]) <= H.TOL["bf16"]
        # one more step does not fit the own rows
        with pytest.raises(ab.AloraError):
            ab.alora_decode(ctx, layer, cache, x_steps[0], k, a)
    finally:
        ctx.close()


@pytest.mark.parametrize("name,opts", [("G4", {}), ("G4", {"kv_splits": 3}), ("G4", {"attn_waves": 4}),
                                       ("G4", {"attn_fold": 0}), ("G4", {"attn_partials16": 0}), ("G1", {}), ("G8", {}),
                                       ("G4", {"kernels": 1}), ("f32", {})])
def test_prefill_rows_of_neighbouring_sequences_walk_their_context_together(ab, name, opts):
    """Invocation sequences of several adapters on one context, packed into shared workgroups for the context's
    keys (Section 2, "Cache reuse patterns"; Proposition 2 with N adapters): runs longer and shorter than a
    workgroup's rows, a run cut by a sequence on another context, by one without context and by an empty one,
    own cached rows behind the context, a context shorter than a tile."""
    shape = SHAPES[name]
    ctx = ab.Context(0)
    try:
        for k_, v in opts.items():
            ctx.set_option(k_, v)
        C = [1500, 300, 40]
        #        run of 7 on context 0 (133 rows)      ctx 1      none  ctx 0 again   empty  ctx 2
        group = [0, 0, 0, 0, 0, 0, 0,                  1, 1,      -1,   0, 0,         0,     2, 2, 0]
        S =     [16, 16, 9, 40, 1, 33, 18,             70, 3,     50,   16, 16,       0,     5, 64, 12]
        own =   [0, 0, 7, 0, 64, 0, 130,               0, 20,     310,  0, 3,         0,     0, 1, 0]
        n = len(S)
        k = [C[g] + own[b] if g >= 0 else 100 for b, g in enumerate(group)]
        k[3] = C[0] + 10          # invocation point inside the new tokens
        k[7] = 0                  # adapter rows from the start
        adapter = [b % 3 for b in range(n)]
        adapter[5] = -1
        case, ctx_kv = H.contexts_case(shape, C, group, own, S, k, adapter, seed=940)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, group, own)
        H.report(test="prefill_shared_contexts", shape=name, opts=opts, err=worst)
    finally:
        ctx.close()


def test_prefill_of_many_short_invocations_on_one_long_context(ab):
    """The shape the packing is for: sixteen adapters' invocation sequences (a dozen tokens each) on one context
    of several thousand tokens, at the width of the 8B configuration's attention (32 query heads, 8 kv heads)."""
    shape = wl.LayerShape(d=1024, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=32, n_adapters=16)
    ctx = ab.Context(0)
    try:
        C = [6000]
        n = 16
        S = [12 + (b % 5) for b in range(n)]
        own = [0] * n
        case, ctx_kv = H.contexts_case(shape, C, [0] * n, own, S, [C[0]] * n, list(range(n)), seed=950)
        worst = H.run_contexts(ab, ctx, case, ctx_kv, C, [0] * n, own)
        H.report(test="prefill_many_invocations_one_context", err=worst)
    finally:
        ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_a_stack_of_adapters_on_one_context_the_base_model_prefilled(ab, dtype):
    """Section 3's pipeline through a layer stack with one copy of the context: the base model prefills the
    context (adapter -1) into a slot of its own, layer by layer; N sequences name those rows as their prefix and
    run N different adapters over their invocation tokens in ONE stack call (Proposition 2 with N adapters; Section
    2, "Cache reuse patterns"), then generate three tokens each with alora_stack_decode.  The oracle recomputes every
    sequence on its own -- context, invocation and generated rows -- with position-gated weights.  Asserted end to
    end for two layers at four times the per-layer tolerance (each layer's own bar is asserted elsewhere); the same
    run with a private copy of the context per sequence is held to the same bound against the shared one (an
    indexing mistake in either shows as an error of order one)."""
    if dtype == "bf16":
        shape = wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3, intermediate=1024)
    else:
        shape = dataclasses.replace(wl.SHAPE_TINY, n_adapters=3, rmsnorm=True, n_kv_heads=2, intermediate=320)
    n_layers, C, n_dec = 2, 210, 3
    S = [40, 7, 64, 1]
    adapter = [0, 2, 1, -1]
    n = len(S)
    rng = wl.Rng(970)
    tensors = [wl.make_layer(shape, rng, f"L{l}") for l in range(n_layers)]
    layers = [H.oracle_layer(t, shape) for t in tensors]
    x_ctx = wl.make_hidden(rng, "x_ctx", C, shape)
    x_own = [wl.make_hidden(rng, f"x{b}", S[b] + n_dec, shape) for b in range(n)]
    tol = H.TOL[shape.dtype]

    def run(shared):
        c = ab.Context(0)
        try:
            glayers = [H.gpu_layer(t, shape) for t in tensors]
            if shared:
                # the sequences hold their own rows only; slot n holds the context, prefilled once by the base model
                caps = [S[b] + n_dec for b in range(n)] + [C]
                caches = [ab.KVCache(caps, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda") for _ in range(n_layers)]
                ab.alora_stack_prefill(c, glayers, caches, x_ctx.cuda().contiguous(), [0] * (n + 1) + [C], [0] * (n + 1),
                                       [-1] * (n + 1))
                assert int(caches[0].seq_len[n]) == C and int(caches[n_layers - 1].seq_len[n]) == C
                for cache in caches:
                    for b in range(n):
                        cache.share_prefix(b, int(cache.seq_offset[n]), C)
            else:
                # every sequence has room for the context too and the base model prefills it n times
                caps = [C + S[b] + n_dec for b in range(n)]
                caches = [ab.KVCache(caps, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda") for _ in range(n_layers)]
                ab.alora_stack_prefill(c, glayers, caches, torch.cat([x_ctx] * n).cuda().contiguous(),
                                       [b * C for b in range(n + 1)], [0] * n, [-1] * n)
            assert [int(v) for v in caches[0].seq_len[:n]] == [C] * n
            cu = [0]
            for b in range(n):
                cu.append(cu[-1] + S[b])
            x_inv = torch.cat([x_own[b][:S[b]] for b in range(n)]).cuda().contiguous()
            # from here on the calls name the first n sequences only (the context slot is reached through the prefixes)
            out_inv = ab.alora_stack_prefill(c, glayers, caches, x_inv, cu, [C] * n, adapter)
            out_dec = []
            for t in range(n_dec):
                xt = torch.stack([x_own[b][S[b] + t] for b in range(n)]).cuda().contiguous()
                out_dec.append(ab.alora_stack_decode(c, glayers, caches, xt, [C] * n, adapter))
            torch.cuda.synchronize()
            assert [int(v) for v in caches[n_layers - 1].seq_len[:n]] == [C + S[b] + n_dec for b in range(n)]
            per_seq = [torch.cat([out_inv[cu[b]:cu[b + 1]]] + [o[b:b + 1] for o in out_dec]) for b in range(n)]
            return per_seq
        finally:
            c.close()

    shared, private = run(True), run(False)
    worst, worst_sp = 0.0, 0.0
    for b in range(n):
        x_all = np.concatenate([H.f64(x_ctx), H.f64(x_own[b])])
        want, _ = orc.ref_stack_full(layers, x_all, C, adapter[b], shape.dtype)
        e = H.rel_err(H.f64(shared[b]), want[C:])
        e_sp = H.rel_err(H.f64(shared[b]), H.f64(private[b]))
        worst, worst_sp = max(worst, e), max(worst_sp, e_sp)
        assert e <= 4 * tol, f"sequence {b}: {e:.3e} against the oracle"
        # (two roundings of the same two-layer run: the private batch prefills the context in a call of another
        # size, so its layer-0 attention is partitioned differently and layer 1 sees other bf16 neighbours)
        assert e_sp <= 4 * tol, f"sequence {b}: shared and private copies of the context differ by {e_sp:.3e}"
    H.report(check="stack of adapters on one shared context", dtype=shape.dtype, err_end_to_end=worst, shared_vs_private=worst_sp)
