"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Cache prefix bytes, written row indices and seq_len are bit-exact; floating-point
outputs are within 1e-4 (fp32) / 2e-2 (bf16 storage, fp32 accumulation) in helpers.rel_err."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import alora_oracle as orc
from paper_2504_12397_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu

SMALL_BF16 = wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3)
SMALL_F32 = dataclasses.replace(wl.SHAPE_TINY, n_adapters=2, rmsnorm=True, n_kv_heads=2)


@pytest.fixture(scope="module")
def ab():
    from paper_2504_12397_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(ab):
    c = ab.Context(0)
    yield c
    c.close()


def run_prefill(ab, ctx, case, decode=False):
    layer = H.gpu_layer(case, case.shape)
    cache = H.gpu_cache(case)
    bk, bv = cache.k.cpu().clone(), cache.v.cpu().clone()
    x = case.x_packed.cuda().contiguous()
    if decode:
        out = ab.alora_decode(ctx, layer, cache, x, case.k, case.adapter)
    else:
        out = ab.alora_prefill(ctx, layer, cache, x, case.cu, case.k, case.adapter)
    torch.cuda.synchronize()
    return out, cache, bk, bv


def check_case(ab, ctx, case, decode=False):
    tol = H.TOL[case.shape.dtype]
    out, cache, bk, bv = run_prefill(ab, ctx, case, decode)
    ref_o, new_rows = H.oracle_prefill(case)
    cache_err = H.check_cache_after(case, cache, bk, bv, new_rows, tol)
    err = H.rel_err(H.f64(out), ref_o)
    rec = dict(err=err, tol=tol, cache_err=cache_err, tokens=int(sum(case.S)), decode=decode)
    if case.shape.dtype == "bf16" and case.shape.rmsnorm:
        # the same comparison against the oracle whose normalised activations are NOT rounded to bf16
        ref_u, _ = H.oracle_prefill(case, act_dtype="f64")
        rec["err_vs_unrounded_activations"] = H.rel_err(H.f64(out), ref_u)
        rec["oracle_bf16_vs_unrounded"] = H.rel_err(ref_o, ref_u)
    H.report(**rec)
    assert err <= tol, f"attention output off by {err:.3e} > {tol}"
    return out, cache


# ------------------------------------------------------------------ config 1 (fp32 single block)
def test_config1_fp32_block(ab, ctx):
    b = wl.config1()
    case = H.make_case(b.shape, b.P, b.S, b.k, b.adapter, b.seed)
    check_case(ab, ctx, case)


@pytest.mark.parametrize("P,S,k,a", [(64, 16, 64, 0), (64, 16, 40, 1), (64, 16, 70, 0), (64, 16, 200, 1),
                                     (64, 16, 64, -1), (0, 33, 0, 1), (0, 33, 9, 0), (77, 1, 77, 0)])
def test_fp32_invocation_positions(ab, ctx, P, S, k, a):
    case = H.make_case(SMALL_F32, [P], [S], [k], [a], seed=100 + P + S + k)
    check_case(ab, ctx, case)


# ------------------------------------------------------------------ bf16, several tiles + ragged tails
@pytest.mark.parametrize("P,S,k,a", [(300, 77, 300, 0), (300, 77, 150, 2), (300, 77, 333, 1), (300, 77, 300, -1),
                                     (0, 201, 0, 1), (1, 130, 1, 0), (513, 1, 513, 2)])
def test_bf16_single_sequence(ab, ctx, P, S, k, a):
    case = H.make_case(SMALL_BF16, [P], [S], [k], [a], seed=200 + P + S + k)
    check_case(ab, ctx, case)


def test_bf16_mixed_batch_with_empty_sequence(ab, ctx):
    P = [257, 0, 64, 700, 31, 128]
    S = [65, 130, 0, 3, 97, 1]
    k = [257, 0, 64, 650, 60, 128]
    a = [0, 1, 2, -1, 2, 1]
    case = H.make_case(SMALL_BF16, P, S, k, a, seed=301)
    check_case(ab, ctx, case)


def test_decode_matches_oracle_and_prefill(ab, ctx):
    P = [400, 33, 1000, 64]
    k = [380, 33, 2000, 0]
    a = [0, 1, 2, -1]
    case = H.make_case(SMALL_BF16, P, [1] * 4, k, a, seed=302)
    out_d, _ = check_case(ab, ctx, case, decode=True)
    out_p, _ = check_case(ab, ctx, case, decode=False)
    assert H.rel_err(H.f64(out_d), H.f64(out_p)) <= 1e-2


def test_token_by_token_decode_chain(ab, ctx):
    """Proposition 1, second part: inference one token at a time with cache reuse."""
    shape = SMALL_BF16
    P, S, k, a = 90, 6, 90, 1
    case = H.make_case(shape, [P], [S], [k], [a], seed=303)
    layer = H.gpu_layer(case, shape)
    cache = H.gpu_cache(case, extra_capacity=0)
    outs = []
    for t in range(S):
        x = case.x_new[0][t:t + 1].cuda().contiguous()
        outs.append(ab.alora_decode(ctx, layer, cache, x, [k], [a]))
    torch.cuda.synchronize()
    assert int(cache.seq_len[0]) == P + S
    ref_o, _ = H.oracle_prefill(case)
    assert H.rel_err(H.f64(torch.cat(outs)), ref_o) <= H.TOL["bf16"]


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_F32], ids=["bf16", "fp32"])
def test_decode_steps_equals_oracle_and_decode_chain(ab, ctx, shape):
    """A staged run of decode steps: same cache rows and outputs as the oracle's prefill of the same
    tokens, with the invocation point falling before, inside and after the run."""
    n = 7
    P = [120, 33, 257, 64]
    k = [100, 36, 400, 0]          # active throughout / from the 4th step on / never / adapter-free
    a = [0, 1, 1, -1]
    case = H.make_case(shape, P, [n] * 4, k, a, seed=305)
    layer = H.gpu_layer(case, shape)
    x_steps = torch.stack([torch.stack([case.x_new[b][t] for b in range(4)]) for t in range(n)]).cuda().contiguous()
    ref_o, new_rows = H.oracle_prefill(case)
    tol = H.TOL[shape.dtype]

    cache = H.gpu_cache(case, extra_capacity=0)
    bk, bv = cache.k.cpu().clone(), cache.v.cpu().clone()
    out = ab.alora_decode_steps(ctx, layer, cache, x_steps, k, a)
    torch.cuda.synchronize()
    assert out.shape == (n, 4, shape.n_q)
    H.check_cache_after(case, cache, bk, bv, new_rows, tol)
    got = torch.cat([out[:, b] for b in range(4)])          # the oracle's packed order: sequence-major
    assert H.rel_err(H.f64(got), ref_o) <= tol

    chain_cache = H.gpu_cache(case, extra_capacity=0)
    chain = torch.stack([ab.alora_decode(ctx, layer, chain_cache, x_steps[t], k, a) for t in range(n)])
    torch.cuda.synchronize()
    assert np.array_equal(cache.seq_len, chain_cache.seq_len)
    assert torch.equal(cache.k, chain_cache.k) and torch.equal(cache.v, chain_cache.v)
    assert H.rel_err(H.f64(out.reshape(n * 4, -1)), H.f64(chain.reshape(n * 4, -1))) <= tol

    # one step too many for the capacity: rejected before anything is written
    full = H.gpu_cache(case, extra_capacity=0)
    with pytest.raises(ab.AloraError):
        ab.alora_decode_steps(ctx, layer, full, torch.cat([x_steps, x_steps[:1]]), k, a)
    assert [int(v) for v in full.seq_len] == P


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def test_regime2_adapter_call_creates_the_base_cache(ab, ctx):
    """Section 2 ("Cache reuse patterns"), second cache-reuse regime: an adapter call over context the base model has not
    seen yet (k > P: the call straddles its own invocation point) leaves base-model cache rows for
    that context, and a later base-only call reuses them.  With a fixed reduction split the rows
    before k are bit-identical whoever computes them and whatever else is in the batch."""
    shape = SMALL_BF16
    C0, inv, turn = 300, 40, 50            # uncached context, invocation + answer tokens, next base turn
    ctx.set_option("gemm_splits", 1)
    ctx.set_option("kv_splits", 1)
    try:
        case = H.make_case(shape, [0], [C0 + inv], [C0], [1], seed=306)
        layer = H.gpu_layer(case, shape)
        x = case.x_new[0].cuda().contiguous()

        # (i) the adapter call alone: creates rows [0, C0) with base weights, [C0, C0+inv) adapted
        c_ad = ab.KVCache([C0 + inv + turn], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
        out_ad = ab.alora_prefill(ctx, layer, c_ad, x, [0, C0 + inv], [C0], [1])
        ref_o, _ = H.oracle_prefill(case)
        assert H.rel_err(H.f64(out_ad), ref_o) <= H.TOL["bf16"]

        # (ii) the base model alone over the same context
        c_base = ab.KVCache([C0 + turn], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
        ab.alora_prefill(ctx, layer, c_base, x[:C0], [0, C0], [0], [-1])

        # (iii) the adapter call inside a mixed batch (other sequences before and after it)
        other = H.make_case(shape, [0, 0], [70, 129], [10, 0], [0, -1], seed=307)
        c_mix = ab.KVCache([70, C0 + inv, 129], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
        xm = torch.cat([other.x_new[0].cuda(), x, other.x_new[1].cuda()]).contiguous()
        out_mix = ab.alora_prefill(ctx, layer, c_mix, xm, [0, 70, 70 + C0 + inv, 70 + C0 + inv + 129], [10, C0, 0],
                                   [0, 1, -1])
        torch.cuda.synchronize()

        o_ad, o_base, o_mix = int(c_ad.seq_offset[0]), int(c_base.seq_offset[0]), int(c_mix.seq_offset[1])
        for pool in ("k", "v"):
            a_rows = _bits(getattr(c_ad, pool)[o_ad:o_ad + C0])
            assert torch.equal(a_rows, _bits(getattr(c_base, pool)[o_base:o_base + C0])), f"{pool}: adapter call vs base call"
            assert torch.equal(_bits(getattr(c_ad, pool)[o_ad:o_ad + C0 + inv]),
                               _bits(getattr(c_mix, pool)[o_mix:o_mix + C0 + inv])), f"{pool}: alone vs in a batch"
        assert torch.equal(_bits(out_ad), _bits(out_mix[70:70 + C0 + inv]))

        # the next base-model turn over the rows the adapter call created: drop the adapted rows, continue
        nxt = H.make_case(shape, [C0], [turn], [0], [-1], seed=308)
        x_turn = nxt.x_new[0].cuda().contiguous()
        c_ad.seq_len[0] = C0
        out_reuse = ab.alora_prefill(ctx, layer, c_ad, x_turn, [0, turn], [0], [-1])
        out_base = ab.alora_prefill(ctx, layer, c_base, x_turn, [0, turn], [0], [-1])
        torch.cuda.synchronize()
        assert torch.equal(_bits(out_reuse), _bits(out_base))
        # and against the oracle: base rows for the context, then the base turn
        lay = case.layer
        xh = orc._normed(lay, H.f64(case.x_new[0][:C0]), "bf16")
        pos = np.arange(C0)
        _, kk, vv = orc.project_qkv(lay, xh, pos, 0, -1)
        kk = orc._store(orc.rope(kk, pos, lay.n_kv_heads, lay.head_dim, lay.rope_theta), "bf16")
        ref_turn, _, _ = orc.ref_cached(lay, kk, orc._store(vv, "bf16"), C0, H.f64(nxt.x_new[0]), 0, -1, "bf16")
        assert H.rel_err(H.f64(out_reuse), ref_turn) <= H.TOL["bf16"]
    finally:
        ctx.set_option("gemm_splits", 0)
        ctx.set_option("kv_splits", 0)


# ------------------------------------------------------------------ invariants on the GPU
def test_recompute_with_gated_weights_equals_cache_reuse(ab, ctx):
    """The brute-force identity through the ABI: P=0, S=L, k=P0 recomputes everything with
    position-gated weights and must agree with the cache-reuse call on the last S0 rows."""
    shape = SMALL_BF16
    P0, S0, a = 200, 60, 1
    case = H.make_case(shape, [P0], [S0], [P0], [a], seed=304)
    layer = H.gpu_layer(case, shape)
    x_all = torch.cat([case.x_prefix[0], case.x_new[0]]).cuda().contiguous()
    full_case = dataclasses.replace(case, P=[0], S=[P0 + S0], x_new=[x_all.cpu()], cache_K=[np.zeros((0, shape.n_kv))],
                                    cache_V=[np.zeros((0, shape.n_kv))])
    cache_full = H.gpu_cache(full_case)
    out_full = ab.alora_prefill(ctx, layer, cache_full, x_all, [0, P0 + S0], [P0], [a])
    # base-only run on the prefix, then the adapter reuses that cache
    base_case = dataclasses.replace(case, P=[0], S=[P0], x_new=[case.x_prefix[0]], cache_K=[np.zeros((0, shape.n_kv))],
                                    cache_V=[np.zeros((0, shape.n_kv))])
    cache = H.gpu_cache(dataclasses.replace(base_case, S=[P0 + S0]))
    ab.alora_prefill(ctx, layer, cache, case.x_prefix[0].cuda().contiguous(), [0, P0], [0], [-1])
    out_reuse = ab.alora_prefill(ctx, layer, cache, case.x_new[0].cuda().contiguous(), [0, S0], [P0], [a])
    torch.cuda.synchronize()
    # prefix rows written by the gated recompute are bitwise the base model's rows (Prop.1, strong form)
    kf, vf = cache_full.rows(0, 0, P0)
    kb, vb = cache.rows(0, 0, P0)
    assert torch.equal(kf.view(torch.int16), kb.view(torch.int16))
    assert torch.equal(vf.view(torch.int16), vb.view(torch.int16))
    assert H.rel_err(H.f64(out_reuse), H.f64(out_full[P0:])) <= 1e-2
    ref_o, _ = H.oracle_prefill(case)
    assert H.rel_err(H.f64(out_reuse), ref_o) <= H.TOL["bf16"]
    assert H.rel_err(H.f64(out_full[P0:]), ref_o) <= H.TOL["bf16"]


def test_base_rows_bitwise_independent_of_batch_composition(ab, ctx):
    """Rows before k must not depend on which adapters or sequences share the batch."""
    shape = SMALL_BF16
    rng = wl.Rng(305)
    tensors = wl.make_layer(shape, rng)
    layer = H.gpu_layer(tensors, shape)
    x0 = wl.make_hidden(rng, "x0", 150, shape)
    x1 = wl.make_hidden(rng, "x1", 70, shape)

    def run(seqs, ks, ads):
        caps = [s.shape[0] for s in seqs]
        cache = ab.KVCache(caps, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")
        cu = [0]
        for s in seqs:
            cu.append(cu[-1] + s.shape[0])
        out = ab.alora_prefill(ctx, layer, cache, torch.cat(seqs).cuda().contiguous(), cu, ks, ads)
        torch.cuda.synchronize()
        return out, cache

    out_a, cache_a = run([x0], [100], [2])
    out_b, cache_b = run([x1, x0], [0, 100], [1, 0])
    out_c, cache_c = run([x0], [0], [-1])
    ka, va = cache_a.rows(0, 0, 100)
    kb, vb = cache_b.rows(1, 0, 100)
    kc, vc = cache_c.rows(0, 0, 100)
    for other_k, other_v in ((kb, vb), (kc, vc)):
        assert torch.equal(ka.view(torch.int16), other_k.view(torch.int16))
        assert torch.equal(va.view(torch.int16), other_v.view(torch.int16))
    # attention outputs of those rows agree too (bitwise only if the key split happens to match)
    assert H.rel_err(H.f64(out_a[:100]), H.f64(out_c[:100])) <= 1e-2
    assert H.rel_err(H.f64(out_b[70:170]), H.f64(out_c[:100])) <= 1e-2
    # rows from k on are adapter-private: they differ between adapters
    assert not torch.equal(cache_a.rows(0, 100, 150)[0], cache_b.rows(1, 100, 150)[0])


def test_base_rows_do_not_depend_on_the_number_of_rows_at_the_8b_width(ab):
    """Proposition 1, strong form, with DEFAULT options at d = 4096 (N = 6144): the key and value rows of
    positions before the invocation point are bit-identical whether a 700-row straddling adapter call, a
    650-row or a 256-row base call, a 64-row prefill or a 64-sequence decode step computed them -- the
    reduction axis of the projection is cut into the same segments, summed in the same order, in all of them
    (one workgroup per segment for few rows, one workgroup walking through the segments for many)."""
    shape = wl.SHAPE_8B_4AD
    c = ab.Context(0)
    try:
        rng = wl.Rng(311, "cuda")
        tensors = wl.make_layer(shape, rng)
        layer = ab.Layer(tensors, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps, shape.rope_theta)
        n, k_inv = 700, 600
        x = wl.make_hidden(rng, "x", n, shape)

        def prefill(rows, k, a):
            cache = ab.KVCache([rows], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
            out = ab.alora_prefill(c, layer, cache, x[:rows].contiguous(), [0, rows], [k], [a])
            torch.cuda.synchronize()
            return out, cache

        out_a, c_a = prefill(n, k_inv, 1)               # straddles its invocation point: rows < 600 are base rows
        ka, va = c_a.rows(0, 0, n)
        for rows in (650, 256, 64):       # 650: not a multiple of the 16-row tiles of row preparation
            _, c_b = prefill(rows, 0, -1)
            kb, vb = c_b.rows(0, 0, rows)
            m = min(rows, k_inv)
            assert torch.equal(_bits(ka[:m]), _bits(kb[:m])), f"keys: {n}-row adapter call vs {rows}-row base call"
            assert torch.equal(_bits(va[:m]), _bits(vb[:m])), f"values: {n}-row adapter call vs {rows}-row base call"
        # a decode step over 64 sequences: sequence b holds positions 0..b-1 and appends the token of position b
        nd = 64
        c_d = ab.KVCache([b + 1 for b in range(nd)], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
        for b in range(nd):
            o = int(c_d.seq_offset[b])
            c_d.k[o:o + b] = ka[:b]
            c_d.v[o:o + b] = va[:b]
            c_d.seq_len[b] = b
        out_d = ab.alora_decode(c, layer, c_d, x[:nd].contiguous(), [k_inv] * nd, [b % 4 for b in range(nd)])
        torch.cuda.synchronize()
        for b in range(nd):
            kd, vd = c_d.rows(b, b, b + 1)
            assert torch.equal(_bits(kd[0]), _bits(ka[b])) and torch.equal(_bits(vd[0]), _bits(va[b])), f"decode row {b}"
        # attention outputs of those rows agree within rounding (prefill and decode attention are different kernels)
        e_attn = H.rel_err(H.f64(out_d), H.f64(out_a[:nd]))
        assert e_attn <= 1e-2
        # rows from the invocation point on are the adapter's own: they differ from the base rows
        _, c_base = prefill(n, 0, -1)
        assert not torch.equal(_bits(c_base.rows(0, k_inv, n)[0]), _bits(ka[k_inv:]))
        # and the straddling call is right: the oracle on the same 700 rows
        host = {k_: (v.cpu() if isinstance(v, torch.Tensor) else v) for k_, v in tensors.items()}
        o_ref, K_ref, V_ref = orc.ref_full(H.oracle_layer(host, shape), H.f64(x), k_inv, 1, "bf16")
        e = H.rel_err(H.f64(out_a), o_ref)
        ek = max(H.rel_err(H.f64(ka).reshape(n, -1), K_ref), H.rel_err(H.f64(va).reshape(n, -1), V_ref))
        H.report(check="700-row straddling call at d=4096", err=e, cache_err=ek, decode_vs_prefill_attention=e_attn)
        assert e <= H.TOL["bf16"] and ek <= H.TOL["bf16"]
    finally:
        c.close()


def test_base_model_rows_are_normalised_to_the_same_bits_by_both_kernels(ab):
    """A call without adapters at d = 4096 normalises its rows either in the kernel that prepares 16 rows per
    workgroup or, from 512 rows on, in a row-per-wave kernel (option prep_split).  Both add the squares of a row
    in the same order, so everything downstream -- cache rows and outputs (Eq.1-3 on the base weights) -- must be
    the same bits; and the base rows an adapter call writes before its invocation point (Proposition 1) are those
    bits too."""
    shape = wl.SHAPE_8B_4AD
    rng = wl.Rng(313, "cuda")
    tensors = wl.make_layer(shape, rng)
    S = [70, 33, 1, 40]
    cu = [0]
    for n in S:
        cu.append(cu[-1] + n)
    x = wl.make_hidden(rng, "x", cu[-1], shape)
    got = {}
    for tag, split, k, a in (("one kernel", 0, [0] * 4, [-1] * 4), ("row per wave", 2, [0] * 4, [-1] * 4),
                             ("adapter call", 1, [50, 20, 1, 10 ** 6], [2, 0, 3, 1])):
        c = ab.Context(0)
        try:
            c.set_option("prep_split", split)
            layer = ab.Layer(tensors, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps, shape.rope_theta)
            cache = ab.KVCache(S, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
            out = ab.alora_prefill(c, layer, cache, x, cu, k, a)
            torch.cuda.synchronize()
            got[tag] = (out.clone(), [cache.rows(b, 0, S[b]) for b in range(len(S))], k)
        finally:
            c.close()
    assert torch.equal(_bits(got["one kernel"][0]), _bits(got["row per wave"][0])), "outputs differ"
    for b in range(len(S)):
        for t in (0, 1):
            assert torch.equal(_bits(got["one kernel"][1][b][t]), _bits(got["row per wave"][1][b][t])), f"sequence {b}"
            base = min(S[b], got["adapter call"][2][b])
            assert torch.equal(_bits(got["adapter call"][1][b][t][:base]), _bits(got["row per wave"][1][b][t][:base])), \
                f"sequence {b}: rows before the invocation point"
    host = {k_: (v.cpu() if isinstance(v, torch.Tensor) else v) for k_, v in tensors.items()}
    worst = 0.0
    for b in range(len(S)):
        o_ref, K_ref, V_ref = orc.ref_full(H.oracle_layer(host, shape), H.f64(x[cu[b]:cu[b + 1]]), 0, -1, "bf16")
        out, rows, _ = got["row per wave"]
        e = max(H.rel_err(H.f64(out[cu[b]:cu[b + 1]]), o_ref), H.rel_err(H.f64(rows[b][0]).reshape(S[b], -1), K_ref),
                H.rel_err(H.f64(rows[b][1]).reshape(S[b], -1), V_ref))
        worst = max(worst, e)
        assert e <= H.TOL["bf16"], f"sequence {b}: {e}"
    H.report(check="base-model rows, row-per-wave normalisation", err=worst)


def test_zero_delta_reproduces_base_model(ab, ctx):
    shape = SMALL_BF16
    case = H.make_case(shape, [120], [50], [120], [0], seed=306)
    zeroed = dict(case.tensors)
    for n in ("B_q", "B_k", "B_v"):
        zeroed[n] = torch.zeros_like(case.tensors[n])
    outs = []
    for tensors, scale, a in ((zeroed, None, 0), (case.tensors, 0.0, 0), (case.tensors, None, -1)):
        t = dict(tensors)
        if scale is not None:
            t["scale"] = [scale] * shape.n_adapters
        layer = H.gpu_layer(t, shape)
        cache = H.gpu_cache(case)
        outs.append(ab.alora_prefill(ctx, layer, cache, case.x_packed.cuda().contiguous(), case.cu, case.k, [a]))
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[2]) and torch.equal(outs[1], outs[2])


def test_deterministic_across_runs(ab, ctx):
    case = H.make_case(SMALL_BF16, [300, 10], [77, 40], [300, 20], [0, 2], seed=307)
    a, _, _, _ = run_prefill(ab, ctx, case)
    b, _, _, _ = run_prefill(ab, ctx, case)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ------------------------------------------------------------------ error handling through the ABI
def test_errors_leave_everything_untouched(ab, ctx):
    case = H.make_case(SMALL_BF16, [10], [5], [10], [0], seed=308)
    layer = H.gpu_layer(case, case.shape)
    cache = H.gpu_cache(case, extra_capacity=0)
    bk = cache.k.clone()
    x = case.x_packed.cuda().contiguous()
    with pytest.raises(ab.AloraError) as e:
        ab.alora_prefill(ctx, layer, cache, x, [0, 5], [10], [7])
    assert e.value.status == ab.ALORA_EADAPTER
    cache.seq_len[0] = 11
    with pytest.raises(ab.AloraError) as e:
        ab.alora_prefill(ctx, layer, cache, x, [0, 5], [10], [0])
    assert e.value.status == ab.ALORA_ECAPACITY
    cache.seq_len[0] = 10
    with pytest.raises(ab.AloraError) as e:
        ab.alora_prefill(ctx, layer, cache, x, [0, 5], [-1], [0])
    assert e.value.status == ab.ALORA_EINVAL
    torch.cuda.synchronize()
    assert torch.equal(cache.k, bk) and int(cache.seq_len[0]) == 10


# ------------------------------------------------------------------ layer stack (first-token pass)
def make_stack_case(shape, n_layers, P, S, seed):
    rng = wl.Rng(seed)
    tensors = [wl.make_layer(shape, rng, f"L{l}") for l in range(n_layers)]
    layers = [H.oracle_layer(t, shape) for t in tensors]
    x_all = wl.make_hidden(rng, "x_all", P + S, shape)
    return tensors, layers, x_all


def stack_layers_one_by_one(ab, c, shape, tensors, layers, x_all, P, a, label):
    """The per-layer check behind the stack tests.  Layer l of the GPU gets the oracle's own layer-l input
    (rounded to the storage dtype, and the oracle's layer l is evaluated on those rounded values too, so both
    sides see the same numbers): the base model prefills rows [0, P) of that layer, the adapter call reuses its
    cache for the rest, and every layer has to meet the stated tolerance on its own."""
    tol = H.TOL[shape.dtype]
    S = x_all.shape[0] - P
    x = H.f64(x_all)
    worst = 0.0
    for l, (t, L) in enumerate(zip(tensors, layers)):
        xin = orc._store(x, shape.dtype)
        want, _ = orc.ref_stack_full([L], xin, P, a, shape.dtype)
        xg = torch.from_numpy(xin).to(shape.torch_dtype).cuda().contiguous()
        gl = [H.gpu_layer(t, shape)]
        cache = [ab.KVCache([P + S], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")]
        base_out = ab.alora_stack_prefill(c, gl, cache, xg[:P].contiguous(), [0, P], [0], [-1])
        got = ab.alora_stack_prefill(c, gl, cache, xg[P:].contiguous(), [0, S], [P], [a])
        torch.cuda.synchronize()
        e_base, e_new = H.rel_err(H.f64(base_out), want[:P]), H.rel_err(H.f64(got), want[P:])
        H.report(check=label, layer=l, err_base_rows=e_base, err_adapted_rows=e_new, tol=tol)
        assert e_base <= tol and e_new <= tol, f"layer {l}: {e_base:.3e} / {e_new:.3e} > {tol}"
        worst = max(worst, e_base, e_new)
        x = want
    return worst


@pytest.mark.parametrize("shape", [
    dataclasses.replace(SMALL_BF16, intermediate=1024),
    dataclasses.replace(SMALL_F32, intermediate=320),
])
def test_stack_cache_reuse_against_oracle_recompute(ab, ctx, shape):
    """Proposition 1 through a stack: the base model prefills the prefix (adapter -1) layer by layer, the
    adapter then reuses those caches for the suffix; the oracle recomputes the whole sequence with
    position-gated weights.  Asserted layer by layer at the stated tolerance; the error of the two-layer
    run as a whole (rounding of layer 0's output feeds layer 1) is recorded next to it."""
    n_layers, P, S, a = 2, 150, 45, 1
    tensors, layers, x_all = make_stack_case(shape, n_layers, P, S, seed=400)
    stack_layers_one_by_one(ab, ctx, shape, tensors, layers, x_all, P, a, "stack")
    want, _ = orc.ref_stack_full(layers, H.f64(x_all), P, a, shape.dtype)
    glayers = [H.gpu_layer(t, shape) for t in tensors]
    caches = [ab.KVCache([P + S], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda") for _ in range(n_layers)]
    xg = x_all.cuda().contiguous()
    base_out = ab.alora_stack_prefill(ctx, glayers, caches, xg[:P].contiguous(), [0, P], [0], [-1])
    assert int(caches[0].seq_len[0]) == P
    got = ab.alora_stack_prefill(ctx, glayers, caches, xg[P:].contiguous(), [0, S], [P], [a])
    torch.cuda.synchronize()
    assert int(caches[0].seq_len[0]) == P + S and int(caches[1].seq_len[0]) == P + S
    e2e = max(H.rel_err(H.f64(base_out), want[:P]), H.rel_err(H.f64(got), want[P:]))
    H.report(check="stack end to end (recorded)", layers=n_layers, err=e2e)
    assert e2e <= 4 * H.TOL[shape.dtype]      # sanity bound on the compounded run; the bar is per layer, above


@pytest.mark.parametrize("adapt_rest", [False, True], ids=["qkv-adapters", "all-linears"])
def test_stack_prefill_of_many_rows(ab, ctx, adapt_rest):
    """The stack on calls of more than 512 rows (what the k = 0 recompute of a long context and a batch of several
    evaluators look like to the linears: many row tiles, the blocks and epilogues chosen for them): the base model
    prefills 650 rows, an adapter call adds 530 (Eq.6 on q, k, v, or on every linear).  Every layer against the
    oracle's recompute at the stated tolerance."""
    shape = dataclasses.replace(SMALL_BF16, intermediate=1024, adapt_rest=adapt_rest)
    n_layers, P, S, a = 2, 650, 530, 2
    tensors, layers, x_all = make_stack_case(shape, n_layers, P, S, seed=430)
    worst = stack_layers_one_by_one(ab, ctx, shape, tensors, layers, x_all, P, a, "stack, many rows")
    H.report(check="stack prefill of many rows", err=worst)


@pytest.mark.parametrize("shape,opts", [(dataclasses.replace(SMALL_BF16, intermediate=1024), {}),
                                        (dataclasses.replace(SMALL_BF16, intermediate=1024, adapt_rest=True), {}),
                                        (dataclasses.replace(SMALL_BF16, intermediate=1024, adapt_rest=True), {"kernels": 1}),
                                        (dataclasses.replace(SMALL_F32, intermediate=320), {})],
                         ids=["bf16", "bf16-all-linears", "bf16-plain", "fp32"])
def test_stack_decode_steps_continue_the_prefill(ab, shape, opts):
    """Eq.4 through the stack: after the base model's prefill of P rows and the adapter's prefill of S rows, three
    tokens are decoded one at a time with alora_stack_decode; the oracle recomputes the whole sequence with
    position-gated weights.  Asserted layer by layer (each layer gets the oracle's own input for that layer), the
    compounded two-layer figure is recorded; then a batch of three sequences of different lengths in one call."""
    c = ab.Context(0)
    try:
        for k_, v in opts.items():
            c.set_option(k_, v)
        tol = H.TOL[shape.dtype]
        n_layers, P, S, D, a = 2, 150, 20, 3, 1
        tensors, layers, x_all = make_stack_case(shape, n_layers, P, S + D, seed=420)
        x = H.f64(x_all)
        for l, (t, L) in enumerate(zip(tensors, layers)):
            xin = orc._store(x, shape.dtype)
            want, _ = orc.ref_stack_full([L], xin, P, a, shape.dtype)
            xg = torch.from_numpy(xin).to(shape.torch_dtype).cuda().contiguous()
            gl = [H.gpu_layer(t, shape)]
            cache = [ab.KVCache([P + S + D], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")]
            ab.alora_stack_prefill(c, gl, cache, xg[:P].contiguous(), [0, P], [0], [-1])
            ab.alora_stack_prefill(c, gl, cache, xg[P:P + S].contiguous(), [0, S], [P], [a])
            for t_ in range(D):
                row = P + S + t_
                got = ab.alora_stack_decode(c, gl, cache, xg[row:row + 1].contiguous(), [P], [a])
                torch.cuda.synchronize()
                assert int(cache[0].seq_len[0]) == row + 1
                e = H.rel_err(H.f64(got), want[row:row + 1])
                H.report(check="stack decode", layer=l, step=t_, err=e, tol=tol)
                assert e <= tol, f"layer {l}, step {t_}: {e:.3e} > {tol}"
            x = want
        # the whole stack, and three sequences at once (different cached lengths, one base-only)
        want, _ = orc.ref_stack_full(layers, H.f64(x_all), P, a, shape.dtype)
        glayers = [H.gpu_layer(t, shape) for t in tensors]
        Ps = [P + S, 37, P]
        ks = [P, 10, 0]
        ads = [a, 0, -1]
        caches = [ab.KVCache([p_ + D + 1 for p_ in Ps], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")
                  for _ in range(n_layers)]
        xg = x_all.cuda().contiguous()
        wants = [orc.ref_stack_full(layers, H.f64(x_all[:Ps[b] + D]), ks[b], ads[b], shape.dtype)[0] for b in range(3)]
        # fill the three caches by prefill calls with the same gating the oracle used
        ab.alora_stack_prefill(c, glayers, caches, torch.cat([xg[:Ps[0]], xg[:Ps[1]], xg[:Ps[2]]]).contiguous(),
                               [0, Ps[0], Ps[0] + Ps[1], sum(Ps)], ks, ads)
        worst = 0.0
        for t_ in range(D):
            xt = torch.stack([xg[Ps[b] + t_] for b in range(3)]).contiguous()
            got = ab.alora_stack_decode(c, glayers, caches, xt, ks, ads)
            torch.cuda.synchronize()
            for b in range(3):
                assert int(caches[0].seq_len[b]) == Ps[b] + t_ + 1 and int(caches[1].seq_len[b]) == Ps[b] + t_ + 1
                worst = max(worst, H.rel_err(H.f64(got[b:b + 1]), wants[b][Ps[b] + t_:Ps[b] + t_ + 1]))
        H.report(check="stack decode end to end, three sequences (recorded)", layers=n_layers, err=worst)
        assert worst <= 4 * tol      # sanity bound on the compounded run; the bar is per layer, above
    finally:
        c.close()


REST_BF16 = dataclasses.replace(SMALL_BF16, intermediate=1024, adapt_rest=True)
REST_F32 = dataclasses.replace(SMALL_F32, intermediate=320, adapt_rest=True)


@pytest.mark.parametrize("shape,opts", [(REST_BF16, {}), (REST_BF16, {"gemm_splits": 1}), (REST_BF16, {"kernels": 1}),
                                        (REST_BF16, {"gemm_tile": 1}), (REST_BF16, {"gemm_tile": 4}),
                                        (REST_BF16, {"gemm_tile": 5}), (REST_F32, {})],
                         ids=["bf16", "bf16-unsplit", "bf16-plain", "bf16-4waves", "bf16-128x64", "bf16-8waves-32x64", "fp32"])
def test_stack_with_adapters_on_every_linear(ab, shape, opts):
    """Eq.6 applied to W_o and the MLP linears as well (Section 2's remark on MLP blocks): cache reuse
    over a base prefix, then a mixed batch whose sequences straddle their invocation points.  Every layer
    meets the stated tolerance on the oracle's own layer input; the compounded two-layer error is recorded."""
    c = ab.Context(0)
    try:
        for k_, v in opts.items():
            c.set_option(k_, v)
        n_layers, P, S, a = 2, 150, 45, 1
        tensors, layers, x_all = make_stack_case(shape, n_layers, P, S, seed=410)
        want, _ = orc.ref_stack_full(layers, H.f64(x_all), P, a, shape.dtype)
        stripped = [dataclasses.replace(L, A_o=None, A_gu=None, A_down=None) for L in layers]
        without, _ = orc.ref_stack_full(stripped, H.f64(x_all), P, a, shape.dtype)
        assert H.rel_err(without[P:], want[P:]) > 0.05          # the adapters of the tail matter in this case
        stack_layers_one_by_one(ab, c, shape, tensors, layers, x_all, P, a, "stack, adapters on every linear")
        glayers = [H.gpu_layer(t, shape) for t in tensors]
        tol = H.TOL[shape.dtype]
        caches = [ab.KVCache([P + S], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda") for _ in range(n_layers)]
        xg = x_all.cuda().contiguous()
        base_out = ab.alora_stack_prefill(c, glayers, caches, xg[:P].contiguous(), [0, P], [0], [-1])
        got = ab.alora_stack_prefill(c, glayers, caches, xg[P:].contiguous(), [0, S], [P], [a])
        torch.cuda.synchronize()
        e2e = max(H.rel_err(H.f64(base_out), want[:P]), H.rel_err(H.f64(got), want[P:]))
        H.report(check="stack end to end (recorded)", layers=n_layers, err=e2e)
        assert e2e <= 4 * tol

        # mixed batch from empty caches: adapter 0 from position 40 on, a base-only sequence, the last adapter from
        # the start -- one layer at a time on the oracle's layer input, like above
        lens, ks, ads = [90, 33, 140], [40, 0, 0], [0, -1, shape.n_adapters - 1]
        rng = wl.Rng(411)
        xs = [H.f64(wl.make_hidden(rng, f"mix{b}", lens[b], shape)) for b in range(3)]
        cu = [0, lens[0], lens[0] + lens[1], sum(lens)]
        for l in range(n_layers):
            xin = [orc._store(xb, shape.dtype) for xb in xs]
            refs = [orc.ref_stack_full([layers[l]], xin[b], ks[b], ads[b], shape.dtype)[0] for b in range(3)]
            cache = [ab.KVCache(lens, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")]
            xg = torch.from_numpy(np.concatenate(xin)).to(shape.torch_dtype).cuda().contiguous()
            out = ab.alora_stack_prefill(c, [glayers[l]], cache, xg, cu, ks, ads)
            torch.cuda.synchronize()
            for b in range(3):
                e = H.rel_err(H.f64(out[cu[b]:cu[b + 1]]), refs[b])
                H.report(check="mixed batch", layer=l, sequence=b, err=e, tol=tol)
                assert e <= tol, f"layer {l}, sequence {b}: {e:.3e}"
            xs = refs
    finally:
        c.close()


@pytest.mark.parametrize("adapter,adapt_rest", [(-1, False), (0, False), (0, True)], ids=["base", "qkv-adapter", "all-linears"])
def test_one_layer_of_the_first_token_stack_at_full_width(ab, ctx, adapter, adapt_rest):
    """The shape the 32-layer first-token workload runs per layer (Proposition 2: the MLP and the projections
    scale with the number of new rows): d = 4096, 32/8 heads, I = 14336, rank 64, 128 new tokens over a
    2048-token cache -- the output projection, gate/up and down projections take their split-reduction paths
    here.  One layer against the oracle at the stated tolerance."""
    shape = dataclasses.replace(wl.SHAPE_8B_STACK, adapt_rest=adapt_rest)
    P, S = 2048, 128
    case = H.make_case(shape, [P], [S], [P], [adapter], seed=430 + adapter + int(adapt_rest), prefix="random")
    layer = H.gpu_layer(case, shape)
    cache = H.gpu_cache(case)
    bk, bv = cache.k.cpu().clone(), cache.v.cpu().clone()
    x = case.x_packed.cuda().contiguous()
    out = ab.alora_stack_prefill(ctx, [layer], [cache], x, case.cu, case.k, case.adapter)
    torch.cuda.synchronize()
    xs = H.f64(case.x_packed)
    o, kn, vn = orc.ref_cached(case.layer, case.cache_K[0], case.cache_V[0], P, xs, P, adapter, "bf16")
    want = orc.layer_tail(case.layer, xs, o, "bf16", P + np.arange(S), P, adapter)
    H.check_cache_after(case, cache, bk, bv, [(kn, vn)], H.TOL["bf16"])
    err = H.rel_err(H.f64(out), want)
    H.report(check="one layer, d=4096, I=14336, T=128", adapter=adapter, adapt_rest=adapt_rest, err=err, tol=H.TOL["bf16"])
    assert err <= H.TOL["bf16"], f"layer output off by {err:.3e}"
    if adapter >= 0:
        # and the adapter does something at this shape: the base model's output differs visibly
        ob, _, _ = orc.ref_cached(case.layer, case.cache_K[0], case.cache_V[0], P, xs, P, -1, "bf16")
        e_base = H.rel_err(orc.layer_tail(case.layer, xs, ob, "bf16"), want)
        assert e_base > 2 * H.TOL["bf16"], f"base model within {e_base:.3e} of the adapted output"


# ------------------------------------------------------------------ full-size configurations
def test_config2_full_size(ab, ctx):
    """One 8B-class layer: 4096 cached base tokens (cache from the oracle's base pass), 256 adapted tokens."""
    b = wl.config2()
    case = H.make_case(b.shape, b.P, b.S, b.k, b.adapter, b.seed)
    check_case(ab, ctx, case)


def test_config3_mixed_batch_all_sequences(ab, ctx):
    """16 sequences, 4 adapters, 3 base-only; the oracle checks every sequence."""
    b = wl.config3()
    case = H.make_case(b.shape, b.P, b.S, b.k, b.adapter, b.seed, prefix="random")
    out, cache, bk, bv = run_prefill(ab, ctx, case)
    cu = case.cu
    worst = 0.0
    for i in range(b.n_seqs):
        o, kn, vn = orc.ref_cached(case.layer, case.cache_K[i], case.cache_V[i], b.P[i], H.f64(case.x_new[i]),
                                   b.k[i], b.adapter[i], "bf16")
        e = H.rel_err(H.f64(out[cu[i]:cu[i + 1]]), o)
        worst = max(worst, e)
        assert e <= H.TOL["bf16"], f"sequence {i}: {e:.3e}"
        gk, gv = cache.rows(i, b.P[i], b.P[i] + b.S[i])
        assert H.rel_err(H.f64(gk).reshape(b.S[i], -1), kn) <= H.TOL["bf16"]
        assert H.rel_err(H.f64(gv).reshape(b.S[i], -1), vn) <= H.TOL["bf16"]
    H.report(check="config 3, all 16 sequences", err=worst, tol=H.TOL["bf16"], tokens=b.T)
    # indexing over the whole pool: only rows [P_b, P_b + S_b) changed
    written = torch.zeros(cache.pool_tokens, dtype=torch.bool)
    for i in range(b.n_seqs):
        o = int(cache.seq_offset[i])
        written[o + b.P[i]:o + b.P[i] + b.S[i]] = True
        assert int(cache.seq_len[i]) == b.P[i] + b.S[i]
    assert torch.equal(cache.k.cpu()[~written].view(torch.int16), bk[~written].view(torch.int16))
    assert torch.equal(cache.v.cpu()[~written].view(torch.int16), bv[~written].view(torch.int16))


def test_config4_decode_all_sequences(ab, ctx):
    """64 sequences x 16448 cached tokens, one new token each; the oracle checks every sequence."""
    b = wl.config4()
    shape = b.shape
    rng = wl.Rng(b.seed, "cuda")
    tensors = wl.make_layer(shape, rng)
    layer = ab.Layer(tensors, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps, shape.rope_theta)
    cache = ab.KVCache([p + 1 for p in b.P], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")
    for i, P in enumerate(b.P):
        k_, v_ = wl.make_random_kv(rng, f"kv{i}", P, shape)
        o = int(cache.seq_offset[i])
        cache.k[o:o + P] = k_
        cache.v[o:o + P] = v_
        cache.seq_len[i] = P
    x = wl.make_hidden(rng, "x", b.T, shape)
    out = ab.alora_decode(ctx, layer, cache, x, b.k, b.adapter)
    torch.cuda.synchronize()
    host = {k_: (v.cpu() if isinstance(v, torch.Tensor) else v) for k_, v in tensors.items()}
    L = H.oracle_layer(host, shape)
    worst = 0.0
    for i in range(b.n_seqs):
        kc, vc = cache.rows(i, 0, b.P[i])
        o, kn, vn = orc.ref_cached(L, H.f64(kc).reshape(b.P[i], -1), H.f64(vc).reshape(b.P[i], -1), b.P[i],
                                   H.f64(x[i:i + 1]), b.k[i], b.adapter[i], "bf16")
        e = H.rel_err(H.f64(out[i:i + 1]), o)
        worst = max(worst, e)
        assert e <= H.TOL["bf16"], f"sequence {i}: {e:.3e}"
        gk, gv = cache.rows(i, b.P[i], b.P[i] + 1)
        assert H.rel_err(H.f64(gk).reshape(1, -1), kn) <= H.TOL["bf16"]
        assert H.rel_err(H.f64(gv).reshape(1, -1), vn) <= H.TOL["bf16"]
        assert int(cache.seq_len[i]) == b.P[i] + 1
    H.report(check="config 4, all 64 sequences", err=worst, tol=H.TOL["bf16"])


def test_config5_one_layer_full_length(ab, ctx):
    """The first-token shape on one layer: 128 adapted tokens over a 32768-token cache, rank 64."""
    b = wl.config5()
    shape = dataclasses.replace(b.shape, intermediate=0)
    case = H.make_case(shape, b.P, b.S, b.k, b.adapter, b.seed, prefix="random")
    check_case(ab, ctx, case)


def test_config5_three_layers_at_full_size_and_a_generated_token(ab, ctx):
    """The call bench.py times, on three of its 32 layers: d = 4096, 32/8 heads, I = 14336, rank 64, 128 adapted tokens
    over 32768 cached base tokens per layer (Section 3's first-token measurement), then one token through
    alora_stack_decode on the caches that call left behind (the first step of the evaluator's answer).  Every layer is
    checked on its own at the stated tolerance -- layer l of the GPU gets the oracle's layer-l input -- and the
    three-layer call as a whole is recorded (and bounded at four times that)."""
    b = wl.config5()
    shape = b.shape
    P, S, a = b.P[0], b.S[0], b.adapter[0]
    n_layers = 3
    tol = H.TOL["bf16"]
    cases = [H.make_case(shape, b.P, b.S, b.k, b.adapter, b.seed + 10 * l, prefix="random") for l in range(n_layers)]
    glayers = [H.gpu_layer(c, shape) for c in cases]
    caches = [H.gpu_cache(c) for c in cases]
    x0 = cases[0].x_packed
    rng = wl.Rng(b.seed + 99)
    x_tok = wl.make_hidden(rng, "x_tok", 1, shape)
    out = ab.alora_stack_prefill(ctx, glayers, caches, x0.cuda().contiguous(), cases[0].cu, b.k, b.adapter)
    out_tok = ab.alora_stack_decode(ctx, glayers, caches, x_tok.cuda().contiguous(), b.k, b.adapter)
    torch.cuda.synchronize()
    assert int(caches[0].seq_len[0]) == P + S + 1 and int(caches[n_layers - 1].seq_len[0]) == P + S + 1

    x, xt = H.f64(x0), H.f64(x_tok)
    pos = P + np.arange(S)
    for l, c in enumerate(cases):
        xin, xtin = orc._store(x, "bf16"), orc._store(xt, "bf16")
        o, kn, vn = orc.ref_cached(c.layer, c.cache_K[0], c.cache_V[0], P, xin, P, a, "bf16")
        want = orc.layer_tail(c.layer, xin, o, "bf16", pos, P, a)
        # the generated token reads the cached rows and the 128 rows the prefill appended
        K1, V1 = np.concatenate([c.cache_K[0], kn]), np.concatenate([c.cache_V[0], vn])
        ot, _, _ = orc.ref_cached(c.layer, K1, V1, P + S, xtin, P, a, "bf16")
        want_tok = orc.layer_tail(c.layer, xtin, ot, "bf16", np.asarray([P + S]), P, a)
        # layer l alone on the oracle's layer input
        cache_l = H.gpu_cache(c, extra_capacity=5)
        got = ab.alora_stack_prefill(ctx, [glayers[l]], [cache_l], torch.from_numpy(xin).to(torch.bfloat16).cuda(), c.cu, b.k, b.adapter)
        got_tok = ab.alora_stack_decode(ctx, [glayers[l]], [cache_l], torch.from_numpy(xtin).to(torch.bfloat16).cuda(), b.k, b.adapter)
        torch.cuda.synchronize()
        e, et = H.rel_err(H.f64(got), want), H.rel_err(H.f64(got_tok), want_tok)
        H.report(check="config 5, layer by layer", layer=l, err_first_tokens=e, err_generated_token=et, tol=tol)
        assert e <= tol and et <= tol, f"layer {l}: {e:.3e} / {et:.3e} > {tol}"
        x, xt = want, want_tok
    e2e, e2e_tok = H.rel_err(H.f64(out), x), H.rel_err(H.f64(out_tok), xt)
    H.report(check="config 5, three layers in one call (recorded)", err_first_tokens=e2e, err_generated_token=e2e_tok)
    assert e2e <= 4 * tol and e2e_tok <= 4 * tol


# ------------------------------------------------------------------ shapes off the main path and kernel options
@pytest.mark.parametrize("hq,hkv,h,r", [(4, 4, 128, 16), (8, 4, 128, 32), (16, 2, 128, 16), (8, 2, 64, 16), (6, 2, 96, 8),
                                         (8, 8, 128, 64)])
def test_bf16_head_layouts(ab, ctx, hq, hkv, h, r):
    """GQA group sizes 1, 2, 4, 8 on the MFMA kernels; head sizes and ranks they do not cover fall back to
    the plain kernels -- every combination must still match the oracle."""
    shape = wl.LayerShape(d=512, n_q_heads=hq, n_kv_heads=hkv, head_dim=h, rank=r, n_adapters=2)
    case = H.make_case(shape, [130, 0, 65], [70, 40, 1], [130, 7, 60], [1, 0, 1], seed=500 + hq + h + r)
    check_case(ab, ctx, case)
    dcase = H.make_case(shape, [200, 31], [1, 1], [150, 31], [0, 1], seed=600 + hq + h + r)
    check_case(ab, ctx, dcase, decode=True)


@pytest.mark.parametrize("rank", [16, 32, 64])
def test_full_width_rows_mixed_adapters(ab, ctx, rank):
    """Hidden size 4096 (the widest row-preparation variant) with every supported rank, several adapters
    and base-only rows inside one 16-row tile."""
    shape = wl.LayerShape(d=4096, n_q_heads=4, n_kv_heads=1, head_dim=128, rank=rank, n_adapters=3)
    case = H.make_case(shape, [40, 0, 9, 17], [21, 13, 7, 30], [40, 5, 0, 30], [2, 0, -1, 1], seed=520 + rank)
    check_case(ab, ctx, case)
    dcase = H.make_case(shape, [33, 5, 12, 20, 8], [1, 1, 1, 1, 1], [30, 5, 20, 0, 8], [0, 1, 2, -1, 1], seed=530 + rank)
    check_case(ab, ctx, dcase, decode=True)


@pytest.mark.parametrize("opts", [{"kernels": 1}, {"kv_splits": 1}, {"kv_splits": 5}, {"gemm_splits": 1}, {"gemm_splits": 4},
                                  {"gemm_tile": 1}, {"gemm_tile": 2}, {"gemm_tile": 3}, {"gemm_tile": 4}, {"gemm_tile": 5}, {"gemm_tile": 6}, {"attn_waves": 4}, {"attn_lazy": 0}, {"attn_lazy": 8},
                                  {"attn_fold": 0}, {"attn_fold": 0, "kv_splits": 3}, {"attn_fold": 0, "attn_waves": 4},
                                  {"attn_fold": 0, "attn_lazy": 0},
                                  {"attn_partials16": 0}, {"attn_partials16": 0, "kv_splits": 3}, {"attn_waves": 4, "kv_splits": 3}])
def test_kernel_options_do_not_change_results(ab, opts):
    c = ab.Context(0)
    try:
        for k_, v in opts.items():
            c.set_option(k_, v)
        case = H.make_case(SMALL_BF16, [700, 10], [150, 33], [700, 20], [0, 2], seed=700)
        check_case(ab, c, case)
        dcase = H.make_case(SMALL_BF16, [900, 64, 3], [1, 1, 1], [100, 64, 0], [1, -1, 2], seed=701)
        check_case(ab, c, dcase, decode=True)
        if "attn_lazy" in opts or "attn_fold" in opts or "attn_partials16" in opts or "attn_waves" in opts:
            # ragged mix for the prefill attention variants: empty prefix, one-token suffix, tile edges
            rag = H.make_case(SMALL_BF16, [0, 63, 64, 1000, 129], [65, 1, 64, 193, 31], [0, 63, 80, 990, 129],
                              [1, 0, -1, 2, 1], seed=705)
            check_case(ab, c, rag)
            for G in (1, 8):
                shp = wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=8 // G, head_dim=128, rank=16, n_adapters=2)
                check_case(ab, c, H.make_case(shp, [300, 0], [100, 70], [300, 5], [1, 0], seed=706 + G))
    finally:
        c.close()


@pytest.mark.parametrize("fold", [0, 1])
def test_rotation_in_the_projection_epilogue_gives_the_same_bits(ab, fold):
    """With many rows the QKV projection rotates and appends in its own epilogue (option rope_fuse, default
    on); the separate rotary kernel must produce the same Q, cache rows and outputs bit for bit (also when
    the queries are premultiplied for the folded softmax)."""
    case = H.make_case(SMALL_BF16, [300, 0, 64], [330, 290, 77], [310, 0, 100], [1, 2, -1], seed=708)
    res = []
    for fuse in (1, 0):
        c = ab.Context(0)
        try:
            c.set_option("attn_fold", fold)
            c.set_option("rope_fuse", fuse)
            out, cache = check_case(ab, c, case)
            res.append((out.clone(), cache.k.clone(), cache.v.clone()))
        finally:
            c.close()
    for a, b in zip(res[0], res[1]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_many_short_sequences(ab, ctx):
    """More sequences than a workgroup has threads (600): the per-sequence loops of the metadata and work-list
    code wrap around; prefill with one to three new tokens each, then a decode step for all of them."""
    rs = np.random.RandomState(77)
    n = 600
    P = [int(v) for v in rs.randint(0, 40, n)]
    S = [int(v) for v in rs.randint(1, 4, n)]
    k = [int(P[i] + rs.randint(-3, 3)) if rs.rand() < 0.7 else 0 for i in range(n)]
    k = [max(0, v) for v in k]
    a = [int(v) for v in rs.randint(-1, 3, n)]
    case = H.make_case(SMALL_BF16, P, S, k, a, seed=709, prefix="random")
    check_case(ab, ctx, case)
    Pd = [max(1, p) for p in P]
    dcase = H.make_case(SMALL_BF16, Pd, [1] * n, k, a, seed=710, prefix="random")
    check_case(ab, ctx, dcase, decode=True)


def test_long_positions_rotary_accuracy(ab, ctx):
    """Positions near 33k: the rotary table is evaluated in double, so late positions stay accurate."""
    shape = SMALL_BF16
    case = H.make_case(shape, [32800], [40], [32800], [1], seed=702, prefix="random")
    check_case(ab, ctx, case)


def test_workspace_regrowth_and_context_reuse(ab):
    """A small call, a larger one (workspace and rotary table regrow), then the small one again."""
    c = ab.Context(0)
    try:
        small = H.make_case(SMALL_BF16, [50], [20], [50], [0], seed=703)
        big = H.make_case(SMALL_BF16, [5000], [600], [5000], [1], seed=704, prefix="random")
        a1, _ = check_case(ab, c, small)
        check_case(ab, c, big)
        a2, _ = check_case(ab, c, small)
        assert torch.equal(a1.view(torch.int16), a2.view(torch.int16))
    finally:
        c.close()


def test_two_contexts_on_two_streams_do_not_disturb_each_other(ab):
    """A serving process runs several streams: two contexts, each on a stream of its own, enqueue prefill and decode
    calls alternately without waiting for each other (nothing in a context is shared with another: workspace,
    staging slots, rotary table).  Every result must be the bits the same call gives when it runs alone."""
    shape = SMALL_BF16
    pre = H.make_case(shape, [700, 10, 0], [150, 33, 64], [700, 20, 0], [0, 2, 1], seed=960, prefix="random")
    dec = H.make_case(shape, [900, 64, 3, 1500], [1, 1, 1, 1], [100, 64, 0, 10 ** 6], [1, -1, 2, 0], seed=961, prefix="random")
    layer_p, layer_d = H.gpu_layer(pre, shape), H.gpu_layer(dec, shape)
    xp, xd = pre.x_packed.cuda().contiguous(), dec.x_packed.cuda().contiguous()

    def alone(case, layer, x, decode):
        c = ab.Context(0)
        try:
            cache = H.gpu_cache(case)
            out = (ab.alora_decode(c, layer, cache, x, case.k, case.adapter) if decode
                   else ab.alora_prefill(c, layer, cache, x, case.cu, case.k, case.adapter))
            torch.cuda.synchronize()
            return out.clone(), cache.k.clone(), cache.v.clone()
        finally:
            c.close()

    ref_p, ref_d = alone(pre, layer_p, xp, False), alone(dec, layer_d, xd, True)
    ca, cb = ab.Context(0), ab.Context(0)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        torch.cuda.synchronize()
        rounds = 6
        caches_p = [H.gpu_cache(pre) for _ in range(rounds)]
        caches_d = [H.gpu_cache(dec) for _ in range(rounds)]
        outs_p = [torch.empty_like(ref_p[0]) for _ in range(rounds)]
        outs_d = [torch.empty_like(ref_d[0]) for _ in range(rounds)]
        torch.cuda.synchronize()
        for r in range(rounds):
            ab.alora_prefill(ca, layer_p, caches_p[r], xp, pre.cu, pre.k, pre.adapter, outs_p[r], stream=sa)
            ab.alora_decode(cb, layer_d, caches_d[r], xd, dec.k, dec.adapter, outs_d[r], stream=sb)
        sa.synchronize()
        sb.synchronize()
        for r in range(rounds):
            assert torch.equal(_bits(outs_p[r]), _bits(ref_p[0])) and torch.equal(_bits(caches_p[r].k), _bits(ref_p[1])) \
                and torch.equal(_bits(caches_p[r].v), _bits(ref_p[2])), f"prefill, round {r}"
            assert torch.equal(_bits(outs_d[r]), _bits(ref_d[0])) and torch.equal(_bits(caches_d[r].k), _bits(ref_d[1])) \
                and torch.equal(_bits(caches_d[r].v), _bits(ref_d[2])), f"decode, round {r}"
    finally:
        ca.close()
        cb.close()
