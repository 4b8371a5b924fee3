"""Pins for the CPU oracle: each test checks oracle/alora_oracle.py against something other
than itself -- a closed form, a library routine on a special case, a separately written
pure-loop brute force, or an invariant the paper proves (Proposition 1) -- chosen so that a
dropped term, a wrong sign or index, or a transposed operand fails at least one of them."""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

from oracle import alora_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_layer(seed, d=24, hq=4, hkv=2, h=6, r=3, n_ad=2, rms=True, scale=(2.0, 0.5), mlp=0, adapt_rest=False):
    g = np.random.default_rng(seed)
    nq, nkv = hq * h, hkv * h
    kw = {}
    if mlp:
        kw = dict(W_o=g.normal(size=(d, nq)) / math.sqrt(nq), rms2_gain=g.normal(1, 0.1, size=d),
                  W_gate=g.normal(size=(mlp, d)) / math.sqrt(d), W_up=g.normal(size=(mlp, d)) / math.sqrt(d),
                  W_down=g.normal(size=(d, mlp)) / math.sqrt(mlp))
    if adapt_rest:
        g2 = np.random.default_rng(seed + 1000)
        kw.update(A_o=g2.normal(size=(n_ad, r, nq)) / math.sqrt(nq), B_o=g2.normal(size=(n_ad, d, r)) * 0.3,
                  A_gu=g2.normal(size=(n_ad, 2, r, d)) / math.sqrt(d), B_gate=g2.normal(size=(n_ad, mlp, r)) * 0.3,
                  B_up=g2.normal(size=(n_ad, mlp, r)) * 0.3, A_down=g2.normal(size=(n_ad, r, mlp)) / math.sqrt(mlp),
                  B_down=g2.normal(size=(n_ad, d, r)) * 0.3)
    return orc.Layer(hq, hkv, h,
                     W_qkv=g.normal(size=(nq + 2 * nkv, d)) / math.sqrt(d),
                     A=g.normal(size=(n_ad, 3, r, d)) / math.sqrt(d),
                     B_q=g.normal(size=(n_ad, nq, r)) * 0.3,
                     B_k=g.normal(size=(n_ad, nkv, r)) * 0.3,
                     B_v=g.normal(size=(n_ad, nkv, r)) * 0.3,
                     scale=list(scale)[:n_ad],
                     rms_gain=g.normal(1, 0.1, size=d) if rms else None, **kw)


# ---------------------------------------------------------------------------- bf16 rounding
def test_round_to_bf16_matches_library_and_ties():
    g = np.random.default_rng(0)
    a32 = (g.normal(size=20000) * np.exp(g.normal(size=20000) * 4)).astype(np.float32)
    want = torch.from_numpy(a32).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(a32.astype(np.float64))
    assert np.array_equal(got, want)
    # exact ties between two bf16 neighbours go to the even one: 1 + 2^-8 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 0.0, 1.0])
    assert np.array_equal(orc.round_to_bf16(ties), np.array([1.0, 1 + 2.0 ** -6, -1.0, 0.0, 1.0]))
    # a float64 just above a tie must round up although float32 would first land on the tie
    assert orc.round_to_bf16(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1 + 2.0 ** -7


# ---------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_closed_forms():
    c, eps = 3.0, 1e-5
    gain = np.array([1.0, 2.0, -1.0, 0.5])
    out = orc.rmsnorm(np.full((1, 4), c), gain, eps)
    assert np.allclose(out[0], gain * c / math.sqrt(c * c + eps), rtol=1e-14)
    x = np.random.default_rng(1).normal(size=(5, 64)) * 7
    y = orc.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, rtol=1e-13)
    assert orc.rmsnorm(x, None, 1e-5) is not None and np.array_equal(orc.rmsnorm(x, None, 1e-5), x)


# ---------------------------------------------------------------------------- rotary embedding
def test_rope_two_dim_rotation_by_hand():
    u = np.array([[3.0, 4.0]])
    for p in (0, 1, 7):
        got = orc.rope(u, np.array([p]), 1, 2, 10000.0)[0]
        want = np.array([3 * math.cos(p) - 4 * math.sin(p), 4 * math.cos(p) + 3 * math.sin(p)])
        assert np.allclose(got, want, rtol=1e-14, atol=1e-14)


def test_rope_pairing_frequencies_identity_norm():
    h, theta = 8, 100.0
    u = np.random.default_rng(2).normal(size=(4, 2 * h))
    pos = np.array([0, 1, 5, 1000])
    r = orc.rope(u, pos, 2, h, theta)
    assert np.array_equal(r[0], u[0])                      # position 0 is the identity
    for i, p in enumerate(pos):
        for head in range(2):
            for c in range(h // 2):
                ang = p * theta ** (-2.0 * c / h)
                a, b = u[i, head * h + c], u[i, head * h + c + h // 2]
                assert math.isclose(r[i, head * h + c], a * math.cos(ang) - b * math.sin(ang), rel_tol=1e-12, abs_tol=1e-12)
                assert math.isclose(r[i, head * h + c + h // 2], b * math.cos(ang) + a * math.sin(ang), rel_tol=1e-12, abs_tol=1e-12)
    assert np.allclose(np.linalg.norm(r, axis=1), np.linalg.norm(u, axis=1), rtol=1e-13)


def test_rope_makes_attention_depend_on_relative_position_only():
    # <rope(q,m), rope(k,n)> depends on m-n only, so a cache-reuse call whose prefix keys and
    # new rows are ALL shifted by the same offset gives the same attention output.
    L = rand_layer(3, rms=False)
    g = np.random.default_rng(4)
    q = g.normal(size=(1, L.n_q))
    kk = g.normal(size=(6, L.n_kv))
    v = g.normal(size=(6, L.n_kv))
    outs = []
    for shift in (0, 11):
        qr = orc.rope(q, np.array([5 + shift]), L.n_q_heads, L.head_dim, L.rope_theta)
        kr = orc.rope(kk, np.arange(6) + shift, L.n_kv_heads, L.head_dim, L.rope_theta)
        outs.append(orc.causal_attention(qr, np.array([5]), kr, v, L.n_q_heads, L.n_kv_heads, L.head_dim))
    assert np.allclose(outs[0], outs[1], rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------- attention
def test_attention_matches_library_sdpa_with_gqa():
    hq, hkv, h, S, Lk = 6, 2, 8, 5, 9
    g = np.random.default_rng(5)
    q = g.normal(size=(S, hq * h))
    K = g.normal(size=(Lk, hkv * h))
    V = g.normal(size=(Lk, hkv * h))
    pos = np.array([4, 5, 6, 7, 8])
    got = orc.causal_attention(q, pos, K, V, hq, hkv, h)
    tq = torch.from_numpy(q).view(S, hq, h).transpose(0, 1)                      # [hq, S, h]
    tk = torch.from_numpy(K).view(Lk, hkv, h).transpose(0, 1).repeat_interleave(hq // hkv, dim=0)
    tv = torch.from_numpy(V).view(Lk, hkv, h).transpose(0, 1).repeat_interleave(hq // hkv, dim=0)
    mask = torch.arange(Lk)[None, :] <= torch.from_numpy(pos)[:, None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)
    want = want.transpose(0, 1).reshape(S, hq * h).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_closed_forms():
    hq, hkv, h = 4, 2, 4
    g = np.random.default_rng(6)
    K = g.normal(size=(7, hkv * h))
    V = g.normal(size=(7, hkv * h))
    pos = np.array([0, 3, 6])
    # zero queries: uniform weights over the visible rows -> mean of visible V rows per kv head
    o = orc.causal_attention(np.zeros((3, hq * h)), pos, K, V, hq, hkv, h).reshape(3, hq, h)
    Vh = V.reshape(7, hkv, h)
    for i, p in enumerate(pos):
        for head in range(hq):
            assert np.allclose(o[i, head], Vh[:p + 1, head // 2].mean(axis=0), rtol=1e-13)
    # a single visible key: output is that value row, whatever the query
    q = g.normal(size=(1, hq * h))
    o = orc.causal_attention(q, np.array([0]), K, V, hq, hkv, h).reshape(hq, h)
    for head in range(hq):
        assert np.allclose(o[head], Vh[0, head // 2], rtol=1e-14)
    # all value rows equal: output is that row
    Vc = np.tile(g.normal(size=(1, hkv * h)), (7, 1))
    o = orc.causal_attention(g.normal(size=(2, hq * h)), np.array([2, 6]), K, Vc, hq, hkv, h).reshape(2, hq, h)
    for head in range(hq):
        assert np.allclose(o[:, head], Vc.reshape(7, hkv, h)[0, head // 2], rtol=1e-13)
    # a key far more aligned with the query than the rest takes (almost) all the weight
    K2 = np.zeros((3, hkv * h)); K2[1] = 50.0
    qq = np.ones((1, hq * h))
    o = orc.causal_attention(qq, np.array([2]), K2, V[:3], hq, hkv, h).reshape(hq, h)
    assert np.allclose(o[0], Vh[1, 0], atol=1e-9)


# ---------------------------------------------------------------------------- gating (Eq.6, Prop.1)
def _x(seed, n, d):
    return np.random.default_rng(seed).normal(size=(n, d))


def test_zero_delta_or_late_invocation_is_the_base_model():
    L = rand_layer(7)
    x = _x(8, 9, 24)
    base = orc.ref_full(L, x, 0, -1)
    Lz = rand_layer(7); Lz.B_q[:] = 0; Lz.B_k[:] = 0; Lz.B_v[:] = 0
    for got in (orc.ref_full(Lz, x, 3, 0), orc.ref_full(rand_layer(7, scale=(0.0, 0.0)), x, 3, 1),
                orc.ref_full(L, x, 9, 0), orc.ref_full(L, x, 100, 1)):
        for a, b in zip(got, base):
            assert np.array_equal(a, b)
    assert not np.allclose(orc.ref_full(L, x, 3, 0)[0], base[0])


def test_invocation_at_start_is_standard_lora_with_merged_weights():
    # k = 0: Eq.6 reduces to Eq.5, i.e. plain attention with the dense W' = W + s B A
    L = rand_layer(9)
    x = _x(10, 8, 24)
    a = 1
    got_o, got_k, got_v = orc.ref_full(L, x, 0, a)
    s = L.scale[a]
    Wm = torch.from_numpy(L.W_qkv.copy())
    nq, nkv = L.n_q, L.n_kv
    for p, (B, lo) in enumerate(((L.B_q, 0), (L.B_k, nq), (L.B_v, nq + nkv))):
        Bt, At = torch.from_numpy(B[a]), torch.from_numpy(L.A[a, p])
        Wm[lo:lo + Bt.shape[0]] += s * (Bt @ At)
    Lm = rand_layer(9)
    Lm.W_qkv = Wm.numpy()
    want_o, want_k, want_v = orc.ref_full(Lm, x, 0, -1)
    assert np.allclose(got_o, want_o, rtol=1e-11, atol=1e-12)
    assert np.allclose(got_k, want_k, rtol=1e-11, atol=1e-12)
    assert np.allclose(got_v, want_v, rtol=1e-11, atol=1e-12)


def test_prefix_rows_identical_for_base_and_every_adapter_suffix_rows_differ():
    L = rand_layer(11)
    x = _x(12, 10, 24)
    k = 6
    ob, kb, vb = orc.ref_full(L, x, k, -1)
    o0, k0, v0 = orc.ref_full(L, x, k, 0)
    o1, k1, v1 = orc.ref_full(L, x, k, 1)
    for t in ((o0, k0, v0), (o1, k1, v1)):
        for a, b in zip(t, (ob, kb, vb)):
            assert np.array_equal(a[:k], b[:k])            # all states before k: bit-identical
    assert np.abs(k0[k:] - kb[k:]).min() > 0 and np.abs(v0[k:] - v1[k:]).min() > 0
    assert np.abs(o0[k:] - o1[k:]).max() > 1e-3


def test_low_rank_product_equals_dense_delta():
    L = rand_layer(13, rms=False)
    x = _x(14, 4, 24)
    q, kk, v = orc.project_qkv(L, x, np.arange(4), 0, 0)
    s = L.scale[0]
    for got, W, B, p in ((q, L.W_qkv[:L.n_q], L.B_q, 0), (kk, L.W_qkv[L.n_q:L.n_q + L.n_kv], L.B_k, 1),
                         (v, L.W_qkv[L.n_q + L.n_kv:], L.B_v, 2)):
        dense = W + s * (B[0] @ L.A[0, p])
        assert np.allclose(got, x @ dense.T, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------------------- cache reuse
@pytest.mark.parametrize("P,S,k", [(6, 4, 6), (6, 4, 3), (6, 4, 8), (6, 4, 10), (6, 4, 50), (0, 10, 0),
                                   (0, 10, 4), (9, 1, 9), (1, 9, 1)])
@pytest.mark.parametrize("cache_dtype", ["f64", "bf16"])
def test_cache_reuse_equals_recompute(P, S, k, cache_dtype):
    """The brute-force identity: recomputing the whole sequence with position-gated weights
    gives, on the new rows, what the cache-reuse path gives from the stored prefix."""
    L = rand_layer(15)
    x = _x(16, P + S, 24)
    a = 1
    of, Kf, Vf = orc.ref_full(L, x, k, a, cache_dtype)
    oc, kn, vn = orc.ref_cached(L, Kf[:P], Vf[:P], P, x[P:], k, a, cache_dtype)
    assert np.allclose(oc, of[P:], rtol=1e-11, atol=1e-12)
    # same rows, up to the summation order of the matrix products (a one-row and a many-row
    # product may differ in the last float64 bit, which can move a bf16 rounding by one step)
    tol = 1e-12 if cache_dtype == "f64" else 2.0 ** -7
    assert np.allclose(kn, Kf[P:], rtol=tol, atol=1e-13) and np.allclose(vn, Vf[P:], rtol=tol, atol=1e-13)
    assert np.mean(kn == Kf[P:]) > 0.99 or cache_dtype == "f64"
    assert kn.shape == (S, L.n_kv)                      # Prop.2: exactly S new cache rows
    if k >= P:
        # the prefix the adapter run reuses is the base model's own prefix (Prop.1)
        ob, Kb, Vb = orc.ref_full(L, x[:P], 0, -1, cache_dtype)
        assert np.allclose(Kb, Kf[:P], rtol=tol, atol=1e-13) and np.allclose(Vb, Vf[:P], rtol=tol, atol=1e-13)


def test_chunked_prefill_and_token_by_token_decode_agree():
    L = rand_layer(17)
    P, S, k, a = 5, 6, 5, 0
    x = _x(18, P + S, 24)
    _, Kb, Vb = orc.ref_full(L, x[:P], 0, -1)
    whole, kn, vn = orc.ref_cached(L, Kb, Vb, P, x[P:], k, a)
    # two chunks
    o1, k1, v1 = orc.ref_cached(L, Kb, Vb, P, x[P:P + 2], k, a)
    K2, V2 = np.concatenate([Kb, k1]), np.concatenate([Vb, v1])
    o2, k2, v2 = orc.ref_cached(L, K2, V2, P + 2, x[P + 2:], k, a)
    assert np.allclose(np.concatenate([o1, o2]), whole, rtol=1e-12, atol=1e-13)
    # one token at a time
    K, V, outs = Kb, Vb, []
    for t in range(S):
        o, kt, vt = orc.ref_cached(L, K, V, P + t, x[P + t:P + t + 1], k, a)
        K, V = np.concatenate([K, kt]), np.concatenate([V, vt])
        outs.append(o)
    assert np.allclose(np.concatenate(outs), whole, rtol=1e-12, atol=1e-13)
    assert np.allclose(K[P:], kn, rtol=1e-13) and np.allclose(V[P:], vn, rtol=1e-13)


def test_base_kv_is_the_cache_of_a_base_run():
    L = rand_layer(27)
    x = _x(28, 7, 24)
    for dt in ("f64", "bf16"):
        _, Kb, Vb = orc.ref_full(L, x, 0, -1, dt)
        K2, V2 = orc.base_kv(L, x, dt)
        assert np.array_equal(Kb, K2) and np.array_equal(Vb, V2)


def test_batch_is_a_loop_over_independent_sequences():
    L = rand_layer(19)
    P, S = [4, 0, 7], [3, 5, 1]
    k, ad = [4, 2, 3], [0, 1, -1]
    xs = [_x(20 + b, P[b] + S[b], 24) for b in range(3)]
    caches = []
    for b in range(3):
        _, Kb, Vb = orc.ref_full(L, xs[b][:P[b]], k[b], ad[b])
        caches.append((Kb, Vb))
    packed = np.concatenate([xs[b][P[b]:] for b in range(3)])
    cu = [0, 3, 8, 9]
    O, rows = orc.ref_prefill_batch(L, caches, P, packed, cu, k, ad)
    for b in range(3):
        of, Kf, Vf = orc.ref_full(L, xs[b], k[b], ad[b])
        assert np.allclose(O[cu[b]:cu[b + 1]], of[P[b]:], rtol=1e-11, atol=1e-12)
        assert np.allclose(rows[b][0], Kf[P[b]:], rtol=1e-12)


def test_inputs_and_cache_are_not_modified():
    L = rand_layer(21)
    x = _x(22, 8, 24)
    _, Kb, Vb = orc.ref_full(L, x[:5], 0, -1)
    canary_k = np.concatenate([Kb, np.full((3, L.n_kv), 777.0)])
    canary_v = np.concatenate([Vb, np.full((3, L.n_kv), -777.0)])
    ck, cv, cx = canary_k.copy(), canary_v.copy(), x.copy()
    orc.ref_cached(L, canary_k, canary_v, 5, x[5:], 5, 0)
    assert np.array_equal(ck, canary_k) and np.array_equal(cv, canary_v) and np.array_equal(cx, x)


# ---------------------------------------------------------------------------- pure-loop brute force
def _loops_full(L, x, k, a):
    """Everything again, scalar by scalar, with python loops and the math module only."""
    n, d = len(x), len(x[0])
    hq, hkv, h = L.n_q_heads, L.n_kv_heads, L.head_dim
    G = hq // hkv
    nq, nkv = hq * h, hkv * h
    rows = []
    for i in range(n):
        xi = list(x[i])
        if L.rms_gain is not None:
            ms = sum(c * c for c in xi) / d
            xi = [xi[c] * L.rms_gain[c] / math.sqrt(ms + L.rms_eps) for c in range(d)]
        y = [sum(L.W_qkv[o][c] * xi[c] for c in range(d)) for o in range(nq + 2 * nkv)]
        if a >= 0 and i >= k:
            for p, (B, lo, width) in enumerate(((L.B_q, 0, nq), (L.B_k, nq, nkv), (L.B_v, nq + nkv, nkv))):
                t = [sum(L.A[a][p][j][c] * xi[c] for c in range(d)) for j in range(L.A.shape[2])]
                for o in range(width):
                    y[lo + o] += L.scale[a] * sum(B[a][o][j] * t[j] for j in range(len(t)))
        for lo, heads in ((0, hq), (nq, hkv)):
            for hd in range(heads):
                for c in range(h // 2):
                    ang = i * L.rope_theta ** (-2.0 * c / h)
                    u, w = y[lo + hd * h + c], y[lo + hd * h + c + h // 2]
                    y[lo + hd * h + c] = u * math.cos(ang) - w * math.sin(ang)
                    y[lo + hd * h + c + h // 2] = w * math.cos(ang) + u * math.sin(ang)
        rows.append(y)
    out = []
    for i in range(n):
        oi = []
        for hd in range(hq):
            g = hd // G
            e = [sum(rows[i][hd * h + c] * rows[j][nq + g * h + c] for c in range(h)) / math.sqrt(h)
                 for j in range(i + 1)]
            m = max(e)
            w = [math.exp(v - m) for v in e]
            z = sum(w)
            oi += [sum(w[j] / z * rows[j][nq + nkv + g * h + c] for j in range(i + 1)) for c in range(h)]
        out.append(oi)
    K = [r[nq:nq + nkv] for r in rows]
    V = [r[nq + nkv:] for r in rows]
    return np.array(out), np.array(K), np.array(V)


@pytest.mark.parametrize("k,a", [(2, 0), (0, 1), (3, -1), (5, 1)])
def test_against_scalar_loop_brute_force(k, a):
    L = rand_layer(23, d=6, hq=2, hkv=1, h=4, r=2)
    x = _x(24, 5, 6)
    got = orc.ref_full(L, x, k, a)
    want = _loops_full(L, x.tolist(), k, a)
    for g_, w_ in zip(got, want):
        assert np.allclose(g_, w_, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------------------- hand-worked example
def test_two_token_example_worked_by_hand():
    """tests/golden/two_token_example.txt: d = 2, one head of width 2, two tokens, adapter on
    from the second token.  The expected values are closed forms derived there by hand."""
    txt = open(os.path.join(GOLDEN, "two_token_example.txt")).read()
    assert "Eq.6" in txt and "Eq.1" in txt
    L = orc.Layer(1, 1, 2,
                  W_qkv=np.array([[1.0, 2.0], [0.0, 1.0], [1.0, 0.0], [0.0, 1.0], [1.0, 0.0], [3.0, 1.0]]),
                  A=np.array([[[[0.0, 1.0]], [[0.0, 1.0]], [[0.0, 1.0]]]]),
                  B_q=np.array([[[1.0], [0.0]]]), B_k=np.array([[[0.0], [1.0]]]), B_v=np.array([[[0.0], [0.0]]]),
                  scale=[2.0], rms_gain=None)
    x = np.array([[1.0, 0.0], [0.0, 1.0]])
    c, s, r2 = math.cos(1.0), math.sin(1.0), math.sqrt(2.0)
    # adapter on at k = 1
    o, K, V = orc.ref_full(L, x, 1, 0)
    e0, e1 = (4 * c - s) / r2, 3 / r2
    p1 = 1 / (1 + math.exp(e0 - e1))
    assert np.allclose(o[0], [1.0, 3.0], rtol=1e-14)
    assert np.allclose(o[1], [(1 - p1) * 1.0, (1 - p1) * 3.0 + p1 * 1.0], rtol=1e-13)
    assert np.allclose(K, [[1.0, 0.0], [-3 * s, 3 * c]], rtol=1e-14, atol=1e-15)
    assert np.allclose(V, [[1.0, 3.0], [0.0, 1.0]], rtol=1e-14)
    # base model
    o, K, V = orc.ref_full(L, x, 1, -1)
    e0, e1 = (2 * c - s) / r2, 1 / r2
    p1 = 1 / (1 + math.exp(e0 - e1))
    assert np.allclose(o[1], [(1 - p1) * 1.0, (1 - p1) * 3.0 + p1 * 1.0], rtol=1e-13)
    assert np.allclose(K, [[1.0, 0.0], [-s, c]], rtol=1e-14, atol=1e-15)


# ---------------------------------------------------------------------------- storage points (bf16 activations)
A_BF16, B_BF16 = 0.84765625, 1.1328125          # (3, 4)/sqrt(12.5) rounded to bf16 by hand, see the golden file


def _storage_layer():
    """d = 2, one head of width 2, W_q = I, W_k = 2 I, W_v = [[1, 1], [1, -1]], unit gains, eps = 0, and a
    one-unit MLP; tests/golden/bf16_storage_points.txt works the numbers by hand."""
    return orc.Layer(1, 1, 2,
                     W_qkv=np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 0.0], [0.0, 2.0], [1.0, 1.0], [1.0, -1.0]]),
                     A=np.zeros((1, 3, 1, 2)), B_q=np.zeros((1, 2, 1)), B_k=np.zeros((1, 2, 1)), B_v=np.zeros((1, 2, 1)),
                     scale=[1.0], rms_gain=np.ones(2), rms_eps=0.0,
                     W_o=np.zeros((2, 2)), rms2_gain=np.ones(2), W_gate=np.array([[1.0, 1.0]]),
                     W_up=np.array([[1.0, 0.0]]), W_down=np.array([[1.0], [0.0]]))


def _two_token_closed_form(a, b):
    c, s, r2 = math.cos(1.0), math.sin(1.0), math.sqrt(2.0)
    e0 = 2 * (2 * a * b * c + (b * b - a * a) * s) / r2
    e1 = 2 * (a * a + b * b) / r2
    p1 = 1 / (1 + math.exp(e0 - e1))
    K = np.array([[2 * a, 2 * b], [2 * (b * c - a * s), 2 * (a * c + b * s)]])
    V = np.array([[a + b, a - b], [a + b, b - a]])
    o = np.array([[a + b, a - b], [a + b, (a - b) * (1 - 2 * p1)]])
    return o, K, V


def test_normalised_rows_are_rounded_to_bf16_before_the_projections():
    """tests/golden/bf16_storage_points.txt.  Fails if the rounding of the normalised hidden state is
    dropped, applied to x instead, or applied to the projections instead."""
    assert "0.84765625" in open(os.path.join(GOLDEN, "bf16_storage_points.txt")).read()
    L = _storage_layer()
    x = np.array([[3.0, 4.0], [4.0, 3.0]])
    # activations bf16, cache unrounded: q, k and v are exact products of the ROUNDED normalised rows
    o, K, V = orc.ref_full(L, x, 0, -1, cache_dtype="f64", act_dtype="bf16")
    wo, wK, wV = _two_token_closed_form(A_BF16, B_BF16)
    assert np.allclose(o, wo, rtol=1e-13, atol=1e-15) and np.array_equal(K[0], wK[0]) and np.array_equal(V, wV)
    assert np.allclose(K[1], wK[1], rtol=1e-14)
    # no rounding anywhere: the closed forms in (3, 4)/sqrt(12.5)
    r = math.sqrt(12.5)
    o64, K64, V64 = orc.ref_full(L, x, 0, -1, cache_dtype="f64", act_dtype="f64")
    wo, wK, wV = _two_token_closed_form(3 / r, 4 / r)
    assert np.allclose(o64, wo, rtol=1e-13) and np.allclose(K64, wK, rtol=1e-14) and np.allclose(V64, wV, rtol=1e-13)
    assert abs(o64[1, 1] - o[1, 1]) > 1e-4 and abs(V64[0, 0] - V[0, 0]) > 5e-4      # the two readings differ
    # bf16 cache on top: a + b = 1.98046875 is a tie and is stored as 254/128; without the rounding of the
    # normalised row (or with the projections rounded instead) the cache would hold 253/128
    _, Kc, Vc = orc.ref_full(L, x, 0, -1, cache_dtype="bf16")
    assert Vc[0, 0] == 1.984375 and Vc[1, 0] == 1.984375 and Kc[0, 0] == 1.6953125 and Kc[0, 1] == 2.265625
    _, _, Vu = orc.ref_full(L, x, 0, -1, cache_dtype="bf16", act_dtype="f64")
    assert Vu[0, 0] == 1.9765625
    # the cached method and the base-prefix helper round at the same point
    oc, kn, vn = orc.ref_cached(L, Kc[:1], Vc[:1], 1, x[1:], 0, -1, "bf16")
    assert vn[0, 0] == 1.984375 and np.array_equal(kn[0], Kc[1])
    Kb, Vb = orc.base_kv(L, x, "bf16")
    assert np.array_equal(Kb, Kc) and np.array_equal(Vb, Vc)
    ob, _ = orc.ref_prefill_batch(L, [(Kc[:1], Vc[:1])], [1], x[1:], [0, 1], [0], [-1], "bf16")
    assert np.array_equal(ob, oc)
    ob64, _ = orc.ref_prefill_batch(L, [(Kc[:1], Vc[:1])], [1], x[1:], [0, 1], [0], [-1], "bf16", act_dtype="f64")
    assert not np.array_equal(ob64, oc)


def test_layer_tail_rounds_the_normalised_row_and_nothing_else():
    """h = x = (3, 4) (W_o = 0): out = (3 + silu(g) u, 4) with g = a + b, u = a of the rounded normalised row.
    Fails if layer_tail drops the rounding, rounds h instead of its normalised value, or rounds more."""
    L = _storage_layer()
    x, attn = np.array([[3.0, 4.0]]), np.array([[0.5, -2.0]])
    silu = lambda z: z / (1 + math.exp(-z))
    got = orc.layer_tail(L, x, attn, "bf16")
    g, u = A_BF16 + B_BF16, A_BF16
    assert g == 1.98046875
    assert np.allclose(got, [[3 + silu(g) * u, 4.0]], rtol=1e-15)
    r = math.sqrt(12.5)
    got64 = orc.layer_tail(L, x, attn, "f64")
    assert np.allclose(got64, [[3 + silu(7 / r) * 3 / r, 4.0]], rtol=1e-15)
    assert abs(got64[0, 0] - got[0, 0]) > 5e-4
    # through the stack functions: the activation dtype reaches the tail (one layer, one token: h = x)
    out, caches = orc.ref_stack_full([L], x, 0, -1, "bf16")
    assert np.allclose(out, [[3 + silu(g) * u, 4.0]], rtol=1e-15) and caches[0][1][0, 0] == 1.984375
    out2, _ = orc.ref_stack_cached([L], [(np.zeros((0, 2)), np.zeros((0, 2)))], 0, x, 0, -1, "bf16")
    assert np.array_equal(out2, out)
    out64, _ = orc.ref_stack_full([L], x, 0, -1, "f64")
    assert np.allclose(out64, [[3 + silu(7 / r) * 3 / r, 4.0]], rtol=1e-15)


def test_lm_head_rounds_the_normalised_row():
    x, W = np.array([[3.0, 4.0]]), np.array([[1.0, 1.0]])
    assert orc.lm_head_logits(x, np.ones(2), 0.0, W, "bf16")[0, 0] == 1.98046875
    assert math.isclose(orc.lm_head_logits(x, np.ones(2), 0.0, W, "f64")[0, 0], 7 / math.sqrt(12.5), rel_tol=1e-15)


# ---------------------------------------------------------------------------- decoder-layer tail
def test_layer_tail_against_library_ops():
    L = rand_layer(25, mlp=40)
    g = np.random.default_rng(26)
    x = g.normal(size=(3, 24))
    attn = g.normal(size=(3, L.n_q))
    got = orc.layer_tail(L, x, attn)
    tx, ta = torch.from_numpy(x), torch.from_numpy(attn)
    hres = tx + torch.nn.functional.linear(ta, torch.from_numpy(L.W_o))
    hn = hres * torch.rsqrt(hres.pow(2).mean(-1, keepdim=True) + L.rms_eps) * torch.from_numpy(L.rms2_gain)
    m = torch.nn.functional.silu(torch.nn.functional.linear(hn, torch.from_numpy(L.W_gate))) * \
        torch.nn.functional.linear(hn, torch.from_numpy(L.W_up))
    want = hres + torch.nn.functional.linear(m, torch.from_numpy(L.W_down))
    assert np.allclose(got, want.numpy(), rtol=1e-12, atol=1e-13)


def test_stack_cache_reuse_equals_recompute():
    layers = [rand_layer(30 + i, mlp=32) for i in range(3)]
    P, S, k, a = 5, 3, 5, 0
    x = _x(33, P + S, 24)
    full, caches = orc.ref_stack_full(layers, x, k, a)
    # per-layer prefix caches are those of the base model run on the prefix alone (Prop.1:
    # all internal states before the invocation index agree)
    base_out, base_caches = orc.ref_stack_full(layers, x[:P], 0, -1)
    for (Kf, Vf), (Kb, Vb) in zip(caches, base_caches):
        assert np.allclose(Kf[:P], Kb, rtol=1e-12, atol=1e-13) and np.allclose(Vf[:P], Vb, rtol=1e-12, atol=1e-13)
    assert np.allclose(full[:P], base_out, rtol=1e-12, atol=1e-13)
    got, rows = orc.ref_stack_cached(layers, base_caches, P, x[P:], k, a)
    assert np.allclose(got, full[P:], rtol=1e-10, atol=1e-11)
    assert all(kn.shape[0] == S for kn, _ in rows)


# ------------------------------------------------------------------ adapters on the other linears
def _merged_tail_layer(L, a):
    """The same layer with Delta folded into the weights of adapter a: W + s B A (Eq.5 for every linear)."""
    s = L.scale[a]
    return dataclasses.replace(
        L, W_o=L.W_o + s * L.B_o[a] @ L.A_o[a], W_gate=L.W_gate + s * L.B_gate[a] @ L.A_gu[a, 0],
        W_up=L.W_up + s * L.B_up[a] @ L.A_gu[a, 1], W_down=L.W_down + s * L.B_down[a] @ L.A_down[a],
        A_o=None, B_o=None, A_gu=None, B_gate=None, B_up=None, A_down=None, B_down=None)


def test_adapted_tail_rows_after_k_use_merged_weights_rows_before_k_the_base():
    L = rand_layer(40, mlp=40, adapt_rest=True)
    g = np.random.default_rng(41)
    x, attn = g.normal(size=(6, 24)), g.normal(size=(6, L.n_q))
    pos, k, a = 10 + np.arange(6), 13, 1
    got = orc.layer_tail(L, x, attn, "f64", pos, k, a)
    base = orc.layer_tail(dataclasses.replace(L, A_o=None, A_gu=None, A_down=None), x, attn)
    merged = orc.layer_tail(_merged_tail_layer(L, a), x, attn)
    assert np.allclose(got[:3], base[:3], rtol=1e-13, atol=1e-14)            # positions 10, 11, 12 < k
    assert np.allclose(got[3:], merged[3:], rtol=1e-11, atol=1e-12)          # positions 13.. >= k
    assert not np.allclose(got[3:], base[3:], atol=1e-3)                     # and the adapter does something
    # no adapter / no positions: the base layer
    assert np.array_equal(orc.layer_tail(L, x, attn, "f64", pos, k, -1), base)
    assert np.array_equal(orc.layer_tail(L, x, attn), base)
    # only one of the linears adapted: the others stay base (each term is separate)
    only_o = dataclasses.replace(L, A_gu=None, A_down=None)
    h_diff = orc.layer_tail(only_o, x, attn, "f64", pos, 0, a) - orc.layer_tail(_merged_tail_layer(
        dataclasses.replace(L, B_gate=L.B_gate * 0, B_up=L.B_up * 0, B_down=L.B_down * 0), a), x, attn)
    assert np.abs(h_diff).max() < 1e-11


def test_adapted_tail_against_scalar_loops():
    L = rand_layer(42, d=6, hq=2, hkv=1, h=4, r=2, mlp=5, adapt_rest=True)
    g = np.random.default_rng(43)
    x, attn = g.normal(size=(2, 6)), g.normal(size=(2, L.n_q))
    a, s = 0, L.scale[0]
    got = orc.layer_tail(L, x, attn, "f64", np.array([4, 5]), 5, a)

    def lin(z, W, A, B, on):
        out = []
        for o in range(W.shape[0]):
            v = sum(W[o, c] * z[c] for c in range(len(z)))
            if on:
                v += s * sum(B[o, j] * sum(A[j, c] * z[c] for c in range(len(z))) for j in range(A.shape[0]))
            out.append(v)
        return out

    for i, on in enumerate([False, True]):
        h = [x[i, c] + v for c, v in enumerate(lin(list(attn[i]), L.W_o, L.A_o[a], L.B_o[a], on))]
        ms = sum(v * v for v in h) / len(h)
        hn = [h[c] / math.sqrt(ms + L.rms_eps) * L.rms2_gain[c] for c in range(len(h))]
        gate = lin(hn, L.W_gate, L.A_gu[a, 0], L.B_gate[a], on)
        up = lin(hn, L.W_up, L.A_gu[a, 1], L.B_up[a], on)
        act = [gv / (1 + math.exp(-gv)) * uv for gv, uv in zip(gate, up)]
        want = [h[c] + v for c, v in enumerate(lin(act, L.W_down, L.A_down[a], L.B_down[a], on))]
        assert np.allclose(got[i], want, rtol=1e-12, atol=1e-13)


def test_stack_with_adapted_tail_cache_reuse_equals_recompute():
    """Proposition 1 with adapters on every linear: rows before k are the base model's in every layer, so the
    base caches can be reused."""
    layers = [rand_layer(50 + i, mlp=32, adapt_rest=True) for i in range(3)]
    P, S, k, a = 5, 4, 5, 1
    x = _x(53, P + S, 24)
    full, caches = orc.ref_stack_full(layers, x, k, a)
    base_out, base_caches = orc.ref_stack_full(layers, x[:P], 0, -1)
    for (Kf, Vf), (Kb, Vb) in zip(caches, base_caches):
        assert np.allclose(Kf[:P], Kb, rtol=1e-12, atol=1e-13) and np.allclose(Vf[:P], Vb, rtol=1e-12, atol=1e-13)
    got, _ = orc.ref_stack_cached(layers, base_caches, P, x[P:], k, a)
    assert np.allclose(got, full[P:], rtol=1e-10, atol=1e-11)
    # and the tail adapters matter: stripping them changes the adapted rows
    stripped = [dataclasses.replace(L, A_o=None, A_gu=None, A_down=None) for L in layers]
    plain, _ = orc.ref_stack_cached(stripped, base_caches, P, x[P:], k, a)
    assert not np.allclose(plain, got, atol=1e-3)


# ------------------------------------------------------------------ output head (first token)
def test_lm_head_worked_by_hand():
    """x = (3, 4): mean square 12.5, so RMSNorm gives (3, 4)/sqrt(12.5); against the rows (1,0), (0,1), (1,1),
    (-1,-1) the logits are 3/s, 4/s, 7/s, -7/s with s = sqrt(12.5): token 2."""
    x = np.array([[3.0, 4.0]])
    W = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, -1.0]])
    lg = orc.lm_head_logits(x, np.ones(2), 0.0, W)
    s = np.sqrt(12.5)
    np.testing.assert_allclose(lg, [[3 / s, 4 / s, 7 / s, -7 / s]], rtol=1e-15)
    assert orc.greedy_token(lg).tolist() == [2]
    # the gain multiplies per feature: gain (2, 0) leaves only the first coordinate
    lg2 = orc.lm_head_logits(x, np.array([2.0, 0.0]), 0.0, W)
    np.testing.assert_allclose(lg2, [[6 / s, 0.0, 6 / s, -6 / s]], rtol=1e-15, atol=1e-15)
    assert orc.greedy_token(lg2).tolist() == [0]          # first of the equal maxima
    # no final norm: plain projection
    np.testing.assert_allclose(orc.lm_head_logits(x, None, 0.0, W), [[3.0, 4.0, 7.0, -7.0]])


def test_lm_head_against_scalar_loops():
    rng = np.random.default_rng(5)
    x, g, W = rng.standard_normal((3, 7)), rng.standard_normal(7), rng.standard_normal((11, 7))
    lg = orc.lm_head_logits(x, g, 1e-5, W)
    for b in range(3):
        ms = sum(float(v) ** 2 for v in x[b]) / 7
        xn = [float(x[b, c]) / np.sqrt(ms + 1e-5) * float(g[c]) for c in range(7)]
        for v in range(11):
            assert abs(lg[b, v] - sum(xn[c] * float(W[v, c]) for c in range(7))) < 1e-12
        assert orc.greedy_token(lg)[b] == max(range(11), key=lambda v: (lg[b, v], -v))
    # rounding the normalised row to bf16 is the only difference of the bf16 reading
    lg16 = orc.lm_head_logits(x, g, 1e-5, W, "bf16")
    xn16 = orc.round_to_bf16(orc.rmsnorm(x, g, 1e-5))
    np.testing.assert_allclose(lg16, xn16 @ W.T, rtol=1e-15)
