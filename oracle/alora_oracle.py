"""CPU oracle for the Activated-LoRA attention hot path.  TEST INFRASTRUCTURE ONLY.

This file is the checker, not the product: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP path and
imports nothing from the package.

Everything is evaluated in float64 with numpy, straight from the definitions:

* Eq.1 (softmax attention), Eq.2 (Q/K/V projections), Eq.3-4 (one-token step over a KV
  cache), Eq.5 (LoRA) and Eq.6 (Activated LoRA: rows before the invocation index use the
  base weights alone, rows from it on use the adapted weights) of the paper.
* `ref_full` is the definition on a whole sequence; `ref_cached` is the method of
  Section 2 / Proposition 1: only the new rows are computed, the prefix keys and values
  come from the cache unchanged.

Readings of points the paper leaves open (all also listed in the design notes):
index base (k is the 0-based absolute position of the first adapted row, k = t_invoke-1);
Delta = s * B A with W stored [out, in], A [r, in], B [out, r]; softmax scale
1/sqrt(head_dim); causal attention includes the current token (Eq.4 attends K_{1:t});
rotary embedding in the "rotate-half" pairing (c, c + h/2) with absolute positions,
applied to q and k before caching; grouped-query attention with contiguous groups
(kv head = q head // G); RMSNorm before the projections.  Storage points: the data path
keeps activations and the cache in the storage dtype ("bf16 weights/activations with fp32
accumulation"), so the two tensors it materialises between steps -- the normalised hidden
state and the cached keys/values -- are rounded to that dtype here; every product and sum
is exact float64 and the attention output is left unrounded.

Pins: every function here is pinned by tests/test_oracle_pins.py (closed forms, library
special cases, a pure-loop brute force written separately, Proposition-1 invariants, two
hand-worked examples under tests/golden/: a two-token attention block, and the storage
points -- which tensor is rounded to bf16, and where -- of the block, the layer tail and the
output head).  `act_dtype="f64"` switches the activation rounding off (the cache keeps its
own dtype); the parity tests report the GPU's error against that reading as well.  No
function is "parity unpinned".
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# storage rounding (what a bf16 KV cache holds)
# --------------------------------------------------------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (8-bit significand, ties to even) and
    return them as float64.  Done directly on the float64 bit pattern, so there is no
    double rounding through float32.  Values are assumed to lie in bfloat16's normal range
    (true for everything this path produces); zero, inf and nan pass through."""
    a = np.ascontiguousarray(a, dtype=F64)
    bits = a.view(np.uint64)
    drop = np.uint64(52 - 7)                       # float64 keeps 52 fraction bits, bf16 keeps 7
    lsb = (bits >> drop) & np.uint64(1)
    rounded = bits + (np.uint64((1 << 44) - 1) + lsb)
    rounded &= ~np.uint64((1 << 45) - 1)
    out = rounded.view(F64).copy()
    special = ~np.isfinite(a)
    out[special] = a[special]
    return out


def _store(a: np.ndarray, cache_dtype: str) -> np.ndarray:
    if cache_dtype == "bf16":
        return round_to_bf16(a)
    if cache_dtype == "f32":
        return a.astype(np.float32).astype(F64)
    if cache_dtype == "f64":
        return np.array(a, dtype=F64)
    raise ValueError(cache_dtype)


# --------------------------------------------------------------------------------------
# layer description
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class Layer:
    """Weights of one decoder layer as float64 arrays.  W_qkv [N_q+2N_kv, d] rows q|k|v;
    A [n_ad, 3, r, d]; B_q [n_ad, N_q, r]; B_k, B_v [n_ad, N_kv, r]; scale [n_ad]."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    W_qkv: np.ndarray
    A: np.ndarray
    B_q: np.ndarray
    B_k: np.ndarray
    B_v: np.ndarray
    scale: Sequence[float]
    rms_gain: Optional[np.ndarray] = None
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    # the rest of the decoder layer (unadapted), only for the layer-stack functions
    W_o: Optional[np.ndarray] = None
    rms2_gain: Optional[np.ndarray] = None
    W_gate: Optional[np.ndarray] = None
    W_up: Optional[np.ndarray] = None
    W_down: Optional[np.ndarray] = None
    # optional adapters of the other linears (Section 2: "adaptations for the MLP blocks ... via
    # directly corresponding equations"), same rank and scales as A / B_q.. above:
    # A_o [n_ad, r, N_q], B_o [n_ad, d, r]; A_gu [n_ad, 2, r, d] (gate, up), B_gate, B_up [n_ad, I, r];
    # A_down [n_ad, r, I], B_down [n_ad, d, r]
    A_o: Optional[np.ndarray] = None
    B_o: Optional[np.ndarray] = None
    A_gu: Optional[np.ndarray] = None
    B_gate: Optional[np.ndarray] = None
    B_up: Optional[np.ndarray] = None
    A_down: Optional[np.ndarray] = None
    B_down: Optional[np.ndarray] = None

    @property
    def n_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def n_kv(self) -> int:
        return self.n_kv_heads * self.head_dim


def layer_from_tensors(t: dict, n_q_heads: int, n_kv_heads: int, head_dim: int,
                       rms_eps: float = 1e-5, rope_theta: float = 10000.0) -> Layer:
    """Build a Layer from a dict of torch tensors / arrays (any float dtype): the stored
    values are converted exactly to float64."""
    def f(x):
        if x is None:
            return None
        if hasattr(x, "detach"):
            x = x.detach().cpu().double().numpy()
        return np.ascontiguousarray(x, dtype=F64)
    return Layer(n_q_heads, n_kv_heads, head_dim, f(t["W_qkv"]), f(t["A"]), f(t["B_q"]), f(t["B_k"]),
                 f(t["B_v"]), [float(s) for s in t["scale"]], f(t.get("rms_gain")), rms_eps, rope_theta,
                 f(t.get("W_o")), f(t.get("rms2_gain")), f(t.get("W_gate")), f(t.get("W_up")),
                 f(t.get("W_down")), f(t.get("A_o")), f(t.get("B_o")), f(t.get("A_gu")), f(t.get("B_gate")),
                 f(t.get("B_up")), f(t.get("A_down")), f(t.get("B_down")))


# --------------------------------------------------------------------------------------
# the steps
# --------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: Optional[np.ndarray], eps: float) -> np.ndarray:
    """x_hat_i = x_i * g / sqrt(mean_c x_ic^2 + eps); identity when there is no gain."""
    x = np.asarray(x, dtype=F64)
    if gain is None:
        return x
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * gain / np.sqrt(ms + eps)


def project_qkv(layer: Layer, xh: np.ndarray, pos: np.ndarray, k: int, adapter: int
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq.6: every row gets W_p x; rows at absolute position >= k of a sequence with an
    adapter additionally get s * B_p (A_p x).  Rows before k, and all rows when
    adapter < 0, get nothing added (they are the base model's rows)."""
    y = xh @ layer.W_qkv.T
    nq, nkv = layer.n_q, layer.n_kv
    q, kk, v = y[:, :nq].copy(), y[:, nq:nq + nkv].copy(), y[:, nq + nkv:].copy()
    if adapter >= 0:
        on = np.asarray(pos) >= k
        if np.any(on):
            s = layer.scale[adapter]
            xa = xh[on]
            for out, p, Bp in ((q, 0, layer.B_q), (kk, 1, layer.B_k), (v, 2, layer.B_v)):
                t = xa @ layer.A[adapter, p].T            # [rows, r]
                out[on] += s * (t @ Bp[adapter].T)
    return q, kk, v


def rope(u: np.ndarray, pos: np.ndarray, n_heads: int, head_dim: int, theta: float) -> np.ndarray:
    """Rotary position embedding, rotate-half pairing: within each head, element c < h/2 is
    paired with element c + h/2 and the pair is rotated by pos * theta^(-2c/h)."""
    S = u.shape[0]
    h2 = head_dim // 2
    w = u.reshape(S, n_heads, head_dim)
    c = np.arange(h2, dtype=F64)
    ang = np.asarray(pos, dtype=F64)[:, None] * theta ** (-2.0 * c / head_dim)[None, :]
    cs, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = w[:, :, :h2], w[:, :, h2:]
    out = np.empty_like(w)
    out[:, :, :h2] = lo * cs - hi * sn
    out[:, :, h2:] = hi * cs + lo * sn
    return out.reshape(S, n_heads * head_dim)


def causal_attention(q: np.ndarray, pos: np.ndarray, K: np.ndarray, V: np.ndarray,
                     n_q_heads: int, n_kv_heads: int, head_dim: int) -> np.ndarray:
    """Eq.1 / Eq.4 with the causal mask: the row at absolute position p attends over cache
    rows 0..p inclusive.  q [S, N_q]; K, V [L, N_kv] (row index = absolute position)."""
    S = q.shape[0]
    G = n_q_heads // n_kv_heads
    L = K.shape[0]
    if S == 0:
        return np.zeros((0, n_q_heads * head_dim), dtype=F64)
    qh = q.reshape(S, n_q_heads, head_dim)
    Kh = K.reshape(L, n_kv_heads, head_dim)
    Vh = V.reshape(L, n_kv_heads, head_dim)
    visible = np.arange(L)[None, :] <= np.asarray(pos)[:, None]          # [S, L]
    out = np.empty((S, n_q_heads, head_dim), dtype=F64)
    for hq in range(n_q_heads):
        g = hq // G
        e = (qh[:, hq, :] @ Kh[:, g, :].T) / np.sqrt(head_dim)
        e = np.where(visible, e, -np.inf)
        e = e - e.max(axis=1, keepdims=True)
        p = np.exp(e)
        p /= p.sum(axis=1, keepdims=True)
        out[:, hq, :] = p @ Vh[:, g, :]
    return out.reshape(S, n_q_heads * head_dim)


# --------------------------------------------------------------------------------------
# attention block: the definition and the cached method
# --------------------------------------------------------------------------------------
def ref_full(layer: Layer, x_all: np.ndarray, k: int, adapter: int, cache_dtype: str = "f64",
             act_dtype: Optional[str] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The definition on one whole sequence of L tokens (positions 0..L-1): Eq.6 rows, rotary
    embedding, then causal attention of every row over rows 0..i.  Returns O [L, N_q] and the
    keys (after rotation) and values as a cache of `cache_dtype` would hold them; attention
    reads those stored values."""
    x_all = np.asarray(x_all, dtype=F64)
    L = x_all.shape[0]
    pos = np.arange(L)
    xh = _normed(layer, x_all, act_dtype or cache_dtype)
    q, kk, v = project_qkv(layer, xh, pos, k, adapter)
    q = rope(q, pos, layer.n_q_heads, layer.head_dim, layer.rope_theta)
    kk = rope(kk, pos, layer.n_kv_heads, layer.head_dim, layer.rope_theta)
    Kc, Vc = _store(kk, cache_dtype), _store(v, cache_dtype)
    o = causal_attention(q, pos, Kc, Vc, layer.n_q_heads, layer.n_kv_heads, layer.head_dim)
    return o, Kc, Vc


def _normed(layer: Layer, x: np.ndarray, act_dtype: str) -> np.ndarray:
    """RMSNorm output as the data path stores it (rounded to the activation dtype)."""
    if layer.rms_gain is None:
        return x
    return _store(rmsnorm(x, layer.rms_gain, layer.rms_eps), act_dtype)


def base_kv(layer: Layer, x_all: np.ndarray, cache_dtype: str = "f64", act_dtype: Optional[str] = None
            ) -> Tuple[np.ndarray, np.ndarray]:
    """Keys (rotated) and values the base model stores for a whole prefix at positions 0..L-1:
    the first three steps of `ref_full` with no adapter, without the attention step."""
    x_all = np.asarray(x_all, dtype=F64)
    pos = np.arange(x_all.shape[0])
    xh = _normed(layer, x_all, act_dtype or cache_dtype)
    _, kk, v = project_qkv(layer, xh, pos, 0, -1)
    kk = rope(kk, pos, layer.n_kv_heads, layer.head_dim, layer.rope_theta)
    return _store(kk, cache_dtype), _store(v, cache_dtype)


def ref_cached(layer: Layer, cache_K: np.ndarray, cache_V: np.ndarray, P: int, x_suffix: np.ndarray,
               k: int, adapter: int, cache_dtype: str = "f64", act_dtype: Optional[str] = None
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The method: cache rows [0, P) are taken as they are; the S new rows at positions
    P..P+S-1 are projected (Eq.6), rotated, stored behind the prefix, and each attends over
    rows 0..its own position.  cache_K/V: [>=P, N_kv].  Returns O [S, N_q] and the S new
    cache rows K_new, V_new [S, N_kv].  The inputs are not modified."""
    x_suffix = np.asarray(x_suffix, dtype=F64)
    S = x_suffix.shape[0]
    pos = P + np.arange(S)
    xh = _normed(layer, x_suffix, act_dtype or cache_dtype)
    q, kk, v = project_qkv(layer, xh, pos, k, adapter)
    q = rope(q, pos, layer.n_q_heads, layer.head_dim, layer.rope_theta)
    kk = rope(kk, pos, layer.n_kv_heads, layer.head_dim, layer.rope_theta)
    K_new, V_new = _store(kk, cache_dtype), _store(v, cache_dtype)
    K = np.concatenate([np.asarray(cache_K, dtype=F64)[:P].reshape(P, layer.n_kv), K_new], axis=0)
    V = np.concatenate([np.asarray(cache_V, dtype=F64)[:P].reshape(P, layer.n_kv), V_new], axis=0)
    o = causal_attention(q, pos, K, V, layer.n_q_heads, layer.n_kv_heads, layer.head_dim)
    return o, K_new, V_new


def ref_prefill_batch(layer: Layer, caches: List[Tuple[np.ndarray, np.ndarray]], P: Sequence[int],
                      x_packed: np.ndarray, cu_seqlens: Sequence[int], k: Sequence[int],
                      adapter: Sequence[int], cache_dtype: str = "f64", act_dtype: Optional[str] = None):
    """A packed batch is a loop over its sequences: they do not interact.  Returns the packed
    O [T, N_q] and, per sequence, its new cache rows."""
    outs, new_rows = [], []
    for b in range(len(P)):
        xs = x_packed[cu_seqlens[b]:cu_seqlens[b + 1]]
        o, kn, vn = ref_cached(layer, caches[b][0], caches[b][1], P[b], xs, k[b], adapter[b], cache_dtype, act_dtype)
        outs.append(o)
        new_rows.append((kn, vn))
    return np.concatenate(outs, axis=0), new_rows


# --------------------------------------------------------------------------------------
# the rest of the decoder layer (unadapted), for the first-token latency workload
# --------------------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def gated_linear(z: np.ndarray, W: np.ndarray, A: Optional[np.ndarray], B: Optional[np.ndarray], s: float,
                 m: Optional[np.ndarray]) -> np.ndarray:
    """Eq.6 for any linear of the layer: row i gets W z_i, plus s * B (A z_i) where m_i = 1."""
    y = z @ W.T
    if A is not None and m is not None and m.any():
        y = y + m[:, None] * (s * ((z @ A.T) @ B.T))
    return y


def layer_tail(layer: Layer, x: np.ndarray, attn: np.ndarray, act_dtype: str = "f64",
               pos: Optional[np.ndarray] = None, k: int = 0, adapter: int = -1) -> np.ndarray:
    """Output projection + residual, then RMSNorm + SwiGLU MLP + residual, all per token.  With
    the base weights, unless the layer carries adapters for these linears: then rows at positions
    >= k (pos given) of a sequence with an adapter use W + Delta exactly as the q/k/v projections
    do (Section 2, the remark after Eq.6 on MLP blocks)."""
    m = None
    a = adapter
    if a >= 0 and pos is not None:
        m = (np.asarray(pos) >= k).astype(F64)
    s = float(layer.scale[a]) if a >= 0 else 0.0
    pick = lambda t, *idx: None if (t is None or a < 0) else t[(a,) + idx]
    h = x + gated_linear(attn, layer.W_o, pick(layer.A_o), pick(layer.B_o), s, m)
    hn = _store(rmsnorm(h, layer.rms2_gain, layer.rms_eps), act_dtype)
    gate = gated_linear(hn, layer.W_gate, pick(layer.A_gu, 0), pick(layer.B_gate), s, m)
    up = gated_linear(hn, layer.W_up, pick(layer.A_gu, 1), pick(layer.B_up), s, m)
    act = silu(gate) * up
    return h + gated_linear(act, layer.W_down, pick(layer.A_down), pick(layer.B_down), s, m)


def ref_stack_full(layers: List[Layer], x_all: np.ndarray, k: int, adapter: int, cache_dtype: str = "f64",
                   act_dtype: Optional[str] = None):
    """All layers on a whole sequence.  Returns the final hidden states [L, d] and the list of
    per-layer caches (K, V)."""
    x = np.asarray(x_all, dtype=F64)
    caches = []
    for layer in layers:
        o, Kc, Vc = ref_full(layer, x, k, adapter, cache_dtype, act_dtype)
        caches.append((Kc, Vc))
        x = layer_tail(layer, x, o, act_dtype or cache_dtype, np.arange(x.shape[0]), k, adapter)
    return x, caches


def ref_stack_cached(layers: List[Layer], caches: List[Tuple[np.ndarray, np.ndarray]], P: int,
                     x_suffix: np.ndarray, k: int, adapter: int, cache_dtype: str = "f64",
                     act_dtype: Optional[str] = None):
    """All layers on the new rows only, each layer reading its own prefix cache.  Returns the
    final hidden states of the new rows [S, d] and the new cache rows per layer."""
    x = np.asarray(x_suffix, dtype=F64)
    new_rows = []
    for layer, (cK, cV) in zip(layers, caches):
        o, kn, vn = ref_cached(layer, cK, cV, P, x, k, adapter, cache_dtype, act_dtype)
        new_rows.append((kn, vn))
        x = layer_tail(layer, x, o, act_dtype or cache_dtype, P + np.arange(x.shape[0]), k, adapter)
    return x, new_rows


# --------------------------------------------------------------------------------------
# the first token itself (Section 3 measures the time to it): final norm, vocabulary
# projection, greedy choice
# --------------------------------------------------------------------------------------
def lm_head_logits(x_last: np.ndarray, final_gain: Optional[np.ndarray], eps: float, W_vocab: np.ndarray,
                   act_dtype: str = "f64") -> np.ndarray:
    """logits[b, v] = <RMSNorm(x_last[b]; final_gain), W_vocab[v]> -- the standard output head of
    the decoder the paper adapts (its Background section; the head itself is never adapted)."""
    xn = np.asarray(x_last, dtype=F64)
    if final_gain is not None:
        xn = rmsnorm(xn, np.asarray(final_gain, dtype=F64), eps)
    xn = _store(xn, act_dtype)
    return xn @ np.asarray(W_vocab, dtype=F64).T


def greedy_token(logits: np.ndarray) -> np.ndarray:
    """Index of the largest logit of every row, the lowest index among equals."""
    return np.argmax(np.asarray(logits, dtype=F64), axis=-1).astype(np.int64)
