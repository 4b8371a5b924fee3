"""The entry point that allocates nothing (alora_decode_static) against alora_decode: same kernels, so the
outputs, the appended cache rows and seq_len must agree bit for bit; two calls in a row on the shared static
scratch, the second smaller than the first; requests beyond the scratch size are rejected before any launch; and,
since the entry point issues kernel launches only (no allocation, no staging copy, no event), a captured HIP graph of
it replays to the same bits, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2504_12397_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu

SMALL_BF16 = wl.LayerShape(d=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank=16, n_adapters=3)
SMALL_F32 = wl.LayerShape(d=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank=8, n_adapters=2, dtype="f32")


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def _both(ab, c, case):
    """The same decode step through alora_decode and alora_decode_static on identical caches."""
    layer = H.gpu_layer(case, case.shape)
    x = case.x_packed.cuda().contiguous()
    c_ref, c_sta = H.gpu_cache(case), H.gpu_cache(case)
    out_ref = ab.alora_decode(c, layer, c_ref, x, case.k, case.adapter)
    out_sta = torch.full_like(out_ref, 7.0)
    ab.alora_decode_static(c, layer, c_sta, x, case.k, case.adapter, out_sta)
    torch.cuda.synchronize()
    assert torch.equal(_bits(out_ref), _bits(out_sta)), "outputs differ from alora_decode"
    assert torch.equal(_bits(c_ref.k), _bits(c_sta.k)) and torch.equal(_bits(c_ref.v), _bits(c_sta.v))
    assert np.array_equal(c_ref.seq_len, c_sta.seq_len)
    ref_o, _ = H.oracle_prefill(case)
    err = H.rel_err(H.f64(out_sta), ref_o)
    H.report(check="alora_decode_static", err=err, tol=H.TOL[case.shape.dtype], sequences=len(case.P))
    assert err <= H.TOL[case.shape.dtype]


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_F32, wl.SHAPE_8B_4AD], ids=["bf16", "fp32", "8b-width"])
def test_two_calls_in_a_row_the_second_smaller(shape):
    from paper_2504_12397_amd import binding as ab
    c = ab.Context(0)
    try:
        big = H.make_case(shape, [1500, 33, 700, 64, 2100, 5, 129], [1] * 7, [1400, 33, 2000, 0, 2100, 0, 100],
                          [0, 1, 1, -1, 0, 1, 0], seed=901, prefix="random")
        small = H.make_case(shape, [40, 300], [1, 1], [40, 0], [1, -1], seed=902, prefix="random")
        _both(ab, c, big)
        _both(ab, c, small)
        _both(ab, c, big)            # and larger again: the scratch keeps whatever the last call left there
    finally:
        c.close()


def test_requests_beyond_the_scratch_and_shared_prefixes_are_rejected():
    from paper_2504_12397_amd import binding as ab
    c = ab.Context(0)
    try:
        shape = wl.SHAPE_8B_4AD
        n = 600                       # 600 rows of the 8B-class projection in fp32 partials alone exceed 32 MiB
        rng = wl.Rng(903, "cuda")
        layer = ab.Layer(wl.make_layer(shape, rng), shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps,
                         shape.rope_theta)
        cache = ab.KVCache([4] * n, shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda", fill=H.CANARY)
        cache.seq_len[:] = 3
        before = cache.k.clone()
        x = wl.make_hidden(rng, "x", n, shape)
        out = torch.zeros((n, shape.n_q), dtype=shape.torch_dtype, device="cuda")
        with pytest.raises(ab.AloraError) as e:
            ab.alora_decode_static(c, layer, cache, x, [0] * n, [0] * n, out)
        assert e.value.status == ab.ALORA_ECAPACITY and "scratch" in e.value.message
        torch.cuda.synchronize()
        assert torch.equal(cache.k, before) and int(cache.seq_len[0]) == 3 and float(out.abs().max()) == 0.0
        # the same call fits the ordinary entry point
        ab.alora_decode(c, layer, cache, x, [0] * n, [0] * n, out)
        torch.cuda.synchronize()
        assert int(cache.seq_len[0]) == 4
        # shared prefixes: not through the static entry point
        small = ab.KVCache([8, 8, 8], shape.n_kv_heads, shape.head_dim, shape.torch_dtype, "cuda")
        small.seq_len[:] = 4
        small.share_prefix(0, int(small.seq_offset[2]), 2)
        with pytest.raises(ab.AloraError) as e:
            ab.alora_decode_static(c, layer, small, x[:2].contiguous(), [0, 0], [0, 1], out[:2])
        assert e.value.status == ab.ALORA_EINVAL
    finally:
        c.close()


def test_replays_of_a_captured_static_decode_step_equal_the_eager_call():
    from paper_2504_12397_amd import binding as ab
    c = ab.Context(0)
    try:
        case = H.make_case(SMALL_BF16, [700, 33, 1500, 64, 5], [1] * 5, [600, 33, 2000, 0, 0], [0, 1, 1, -1, 2], seed=951,
                           prefix="random")
        layer = H.gpu_layer(case, SMALL_BF16)
        x = case.x_packed.cuda().contiguous()
        P = np.asarray(case.P, dtype=np.int32)

        def eager(xin):
            cache = H.gpu_cache(case)
            out = ab.alora_decode(c, layer, cache, xin, case.k, case.adapter)
            torch.cuda.synchronize()
            return out, cache

        ref_out, ref_cache = eager(x)                       # also loads every kernel before the capture
        warm = H.gpu_cache(case)
        out_g = torch.zeros_like(ref_out)
        ab.alora_decode_static(c, layer, warm, x, case.k, case.adapter, out_g)
        torch.cuda.synchronize()

        cache_g = H.gpu_cache(case)
        x_g = x.clone()
        out_g.zero_()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            ab.alora_decode_static(c, layer, cache_g, x_g, case.k, case.adapter, out_g)
        torch.cuda.synchronize()
        assert float(out_g.abs().max()) == 0.0, "capture must not execute anything"
        assert np.array_equal(cache_g.seq_len, P + 1)       # the host-side bookkeeping of the captured call

        for replay in range(4):
            print(f"replay {replay}", flush=True)
            if replay >= 2:                                  # new hidden states in the captured input buffer
                x_g.copy_(torch.roll(x, shifts=replay, dims=1))
                ref_out, ref_cache = eager(x_g.clone())
            out_g.fill_(3.0)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(_bits(out_g), _bits(ref_out)), f"replay {replay}: outputs differ from the eager call"
            assert torch.equal(_bits(cache_g.k), _bits(ref_cache.k)) and torch.equal(_bits(cache_g.v), _bits(ref_cache.v))
            # eager work of the same library between replays (shares the static scratch)
            other = H.gpu_cache(case)
            tmp = torch.empty_like(ref_out)
            ab.alora_decode_static(c, layer, other, x, case.k, case.adapter, tmp)
            torch.cuda.synchronize()
        H.report(check="alora_decode_static under graph capture", replays=4)
    finally:
        c.close()
