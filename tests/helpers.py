"""Shared test plumbing: building seeded cases, running them through the C ABI, error metrics.
Holds no arithmetic of the method: expected values always come from oracle/."""
from __future__ import annotations

import dataclasses
import json
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

from oracle import alora_oracle as orc
from paper_2504_12397_amd import workloads as wl

TOL = {"f32": 1e-4, "bf16": 2e-2}

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# where the parity tests record their measured errors (one JSON object per line)
REPORT_PATH = os.environ.get("ALORA_PARITY_REPORT", os.path.join(ROOT, "gpurun_out", "parity_report.jsonl"))


def report(**vals):
    """Prints and records measured errors of the running test: the asserted one (against the oracle as it
    stands, activations stored in bf16) next to the error against the oracle with unrounded activations."""
    rec = {"test": os.environ.get("PYTEST_CURRENT_TEST", "").split(" ")[0]}
    rec.update({k_: (float(v) if isinstance(v, (float, np.floating)) else v) for k_, v in vals.items()})
    print("parity:", json.dumps(rec))
    try:
        os.makedirs(os.path.dirname(REPORT_PATH), exist_ok=True)
        with open(REPORT_PATH, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass


def rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(row of i)): elementwise relative error, where an
    element smaller than the RMS of its own row (one token's output) is judged on that row's
    scale: a sum of signed terms has an absolute error set by the size of the terms, not by
    how close the sum happens to fall to zero, and rows differ in scale (a token that attends
    over few keys has a larger output than one that averages thousands)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    got = got.reshape(-1, got.shape[-1])
    ref = ref.reshape(-1, ref.shape[-1])
    floor = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    floor = np.where(floor > 0, floor, 1.0)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_layer(tensors: dict, shape: wl.LayerShape) -> orc.Layer:
    return orc.layer_from_tensors(tensors, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                                  shape.rms_eps, shape.rope_theta)


@dataclasses.dataclass
class Case:
    shape: wl.LayerShape
    tensors: dict                 # cpu torch tensors, storage dtype
    layer: orc.Layer              # same values, float64
    P: List[int]
    S: List[int]
    k: List[int]
    adapter: List[int]
    x_prefix: List[Optional[torch.Tensor]]   # hidden states of the cached tokens (None if cache is random)
    x_new: List[torch.Tensor]                # hidden states of the new tokens
    cache_K: List[np.ndarray]                # [P_b, N_kv] float64 values representable in the storage dtype
    cache_V: List[np.ndarray]

    @property
    def cu(self) -> List[int]:
        out = [0]
        for s in self.S:
            out.append(out[-1] + s)
        return out

    @property
    def x_packed(self) -> torch.Tensor:
        return torch.cat(self.x_new, dim=0) if self.x_new else torch.zeros((0, self.shape.d))


def make_case(shape: wl.LayerShape, P: Sequence[int], S: Sequence[int], k: Sequence[int], adapter: Sequence[int],
              seed: int, prefix: str = "oracle", prefix_k: Optional[Sequence[int]] = None) -> Case:
    """prefix = "oracle": cache rows come from the oracle's pass over seeded prefix hidden states with the
    same (k, adapter) gating (so k < P gives adapted rows in the cache); "random": N(0,1) keys/values."""
    rng = wl.Rng(seed)
    tensors = wl.make_layer(shape, rng)
    layer = oracle_layer(tensors, shape)
    xp, xn, cK, cV = [], [], [], []
    for b in range(len(P)):
        xn.append(wl.make_hidden(rng, f"x_new{b}", S[b], shape))
        if prefix == "oracle":
            xb = wl.make_hidden(rng, f"x_prefix{b}", P[b], shape)
            xp.append(xb)
            pos = np.arange(P[b])
            xh = orc._normed(layer, f64(xb), shape.dtype)
            _, kk, vv = orc.project_qkv(layer, xh, pos, k[b], adapter[b])
            kk = orc.rope(kk, pos, layer.n_kv_heads, layer.head_dim, layer.rope_theta)
            cK.append(orc._store(kk, shape.dtype))
            cV.append(orc._store(vv, shape.dtype))
        else:
            xp.append(None)
            K, V = wl.make_random_kv(rng, f"kv{b}", P[b], shape)
            cK.append(f64(K).reshape(P[b], shape.n_kv))
            cV.append(f64(V).reshape(P[b], shape.n_kv))
    return Case(shape, tensors, layer, list(P), list(S), list(k), list(adapter), xp, xn, cK, cV)


def oracle_prefill(case: Case, act_dtype: Optional[str] = None):
    """act_dtype = "f64": the reading in which the normalised hidden state is NOT rounded to the storage
    dtype before the projections (the cache keeps its dtype); used to report, never to assert."""
    caches = list(zip(case.cache_K, case.cache_V))
    return orc.ref_prefill_batch(case.layer, caches, case.P, f64(case.x_packed), case.cu, case.k, case.adapter,
                                 case.shape.dtype, act_dtype)


# ------------------------------------------------------------------------------ GPU side
def gpu_layer(case_or_tensors, shape: wl.LayerShape, device="cuda"):
    from paper_2504_12397_amd import binding as ab
    tensors = case_or_tensors.tensors if isinstance(case_or_tensors, Case) else case_or_tensors
    dev = {k_: (v.to(device).contiguous() if isinstance(v, torch.Tensor) else v) for k_, v in tensors.items()}
    return ab.Layer(dev, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rms_eps, shape.rope_theta,
                    shape.intermediate)


CANARY = 777.0


def gpu_cache(case: Case, extra_capacity: int = 5, guard_rows: int = 3, device="cuda"):
    """A pool with canary-filled guard rows between sequences and unused capacity behind each one."""
    from paper_2504_12397_amd import binding as ab
    caps = [case.P[b] + case.S[b] + extra_capacity for b in range(len(case.P))]
    cache = ab.KVCache(caps, case.shape.n_kv_heads, case.shape.head_dim, case.shape.torch_dtype, device,
                       fill=CANARY, guard_rows=guard_rows)
    for b in range(len(case.P)):
        cache.load_prefix(b, torch.from_numpy(case.cache_K[b]), torch.from_numpy(case.cache_V[b]))
    return cache


def check_cache_after(case: Case, cache, before_k: torch.Tensor, before_v: torch.Tensor, new_rows, tol: float):
    """Indexing is exact: only rows [P_b, P_b+S_b) of each sequence changed; they hold the new keys/values."""
    k_now, v_now = cache.k.cpu(), cache.v.cpu()
    written = torch.zeros(cache.pool_tokens, dtype=torch.bool)
    for b in range(len(case.P)):
        o = int(cache.seq_offset[b])
        written[o + case.P[b]:o + case.P[b] + case.S[b]] = True
        assert int(cache.seq_len[b]) == case.P[b] + case.S[b]
    keep = ~written
    assert torch.equal(k_now[keep].view(torch.int16 if k_now.dtype == torch.bfloat16 else torch.int32),
                       before_k[keep].view(torch.int16 if k_now.dtype == torch.bfloat16 else torch.int32)), \
        "cache rows outside [P, P+S) changed"
    assert torch.equal(v_now[keep].view(torch.int16 if v_now.dtype == torch.bfloat16 else torch.int32),
                       before_v[keep].view(torch.int16 if v_now.dtype == torch.bfloat16 else torch.int32))
    errs = []
    for b in range(len(case.P)):
        if case.S[b] == 0:
            continue
        o = int(cache.seq_offset[b]) + case.P[b]
        gk = f64(k_now[o:o + case.S[b]]).reshape(case.S[b], -1)
        gv = f64(v_now[o:o + case.S[b]]).reshape(case.S[b], -1)
        errs.append(rel_err(gk, new_rows[b][0]))
        errs.append(rel_err(gv, new_rows[b][1]))
    worst = max(errs) if errs else 0.0
    assert worst <= tol, f"new cache rows off by {worst:.3e} > {tol}"
    return worst


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


# ------------------------------------------------------------------------------ sequences over shared contexts
def contexts_case(shape, C, group, own, S, k, adapter, seed):
    """Sequences over several base contexts: sequence b reads context group[b] (C[group[b]] rows, -1: none) and
    holds own[b] cached rows of its own behind it.  All cached values are random: the comparison needs only that
    the GPU and the oracle hold the same ones."""
    rng = wl.Rng(seed)
    tensors = wl.make_layer(shape, rng)
    layer = oracle_layer(tensors, shape)
    ctx_kv = []
    for i, c in enumerate(C):
        K, V = wl.make_random_kv(rng, f"context{i}", c, shape)
        ctx_kv.append((f64(K).reshape(c, shape.n_kv), f64(V).reshape(c, shape.n_kv)))
    xn, cK, cV, P = [], [], [], []
    for b in range(len(S)):
        xn.append(wl.make_hidden(rng, f"x_new{b}", S[b], shape))
        K, V = wl.make_random_kv(rng, f"own{b}", own[b], shape)
        K, V = f64(K).reshape(own[b], shape.n_kv), f64(V).reshape(own[b], shape.n_kv)
        if group[b] >= 0:
            K, V = np.concatenate([ctx_kv[group[b]][0], K]), np.concatenate([ctx_kv[group[b]][1], V])
        cK.append(K)
        cV.append(V)
        P.append(len(K))
    case = Case(shape, tensors, layer, P, list(S), list(k), list(adapter), [None] * len(S), xn, cK, cV)
    return case, ctx_kv


def run_contexts(ab, ctx, case, ctx_kv, C, group, own, decode=False):
    shape = case.shape
    n = len(case.S)
    nkv = shape.n_kv_heads
    caps = [own[b] + case.S[b] + 2 for b in range(n)] + list(C)
    cache = ab.KVCache(caps, nkv, shape.head_dim, shape.torch_dtype, "cuda", fill=CANARY, guard_rows=2)

    def put(o, K, V):
        r = len(K)
        if r:
            cache.k[o:o + r] = torch.from_numpy(K).to(shape.torch_dtype).view(r, nkv, -1).cuda()
            cache.v[o:o + r] = torch.from_numpy(V).to(shape.torch_dtype).view(r, nkv, -1).cuda()

    for i in range(len(C)):
        put(int(cache.seq_offset[n + i]), *ctx_kv[i])
    for b in range(n):
        lo = C[group[b]] if group[b] >= 0 else 0
        put(int(cache.seq_offset[b]), case.cache_K[b][lo:], case.cache_V[b][lo:])
        cache.seq_len[b] = case.P[b]
        if group[b] >= 0:
            cache.share_prefix(b, int(cache.seq_offset[n + group[b]]), lo)
    cache._refresh()
    before_k, before_v = cache.k.clone(), cache.v.clone()
    layer = gpu_layer(case, shape)
    if decode:
        out = ab.alora_decode(ctx, layer, cache, case.x_packed.cuda().contiguous(), case.k, case.adapter)
    else:
        out = ab.alora_prefill(ctx, layer, cache, case.x_packed.cuda().contiguous(), case.cu, case.k, case.adapter)
    torch.cuda.synchronize()
    ref_o, new_rows = oracle_prefill(case)
    tol = TOL[shape.dtype]
    # row by row, so that a row that took another sequence's context shows up under its own number
    cu = case.cu
    worst = 0.0
    for b in range(n):
        if case.S[b] == 0:
            continue
        e = rel_err(f64(out[cu[b]:cu[b + 1]]), ref_o[cu[b]:cu[b + 1]])
        assert e <= tol, f"sequence {b}: attention output off by {e:.3e}"
        worst = max(worst, e)
    written = torch.zeros(cache.pool_tokens, dtype=torch.bool)
    for b in range(n):
        o = int(cache.seq_offset[b]) + own[b]
        written[o:o + case.S[b]] = True
        assert int(cache.seq_len[b]) == case.P[b] + case.S[b]
        if case.S[b]:
            assert rel_err(f64(cache.k[o:o + case.S[b]]).reshape(case.S[b], -1), new_rows[b][0]) <= tol
            assert rel_err(f64(cache.v[o:o + case.S[b]]).reshape(case.S[b], -1), new_rows[b][1]) <= tol
    keep = ~written.cuda()
    assert torch.equal(_bits(cache.k[keep]), _bits(before_k[keep])), "rows outside the new ones changed (contexts included)"
    assert torch.equal(_bits(cache.v[keep]), _bits(before_v[keep]))
    return worst
