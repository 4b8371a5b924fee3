"""ctypes binding of libalora (include/alora.h).  Argument marshalling only: torch supplies
device memory and streams, every step of the path runs in the library's HIP kernels.
There is no fallback: if the shared library is missing, importing this module raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ALORA_LIB: another build of the same library (kernel experiments); the default is the in-tree one
LIB_PATH = os.environ.get("ALORA_LIB") or os.path.join(_HERE, "libalora.so")

ALORA_OK, ALORA_EINVAL, ALORA_ESHAPE, ALORA_ECAPACITY, ALORA_EADAPTER, ALORA_EDTYPE, ALORA_EHIP = range(7)
ALORA_F32, ALORA_BF16 = 0, 1

EXPORTS = ["alora_create", "alora_destroy", "alora_last_error", "alora_status_string", "alora_set_option",
           "alora_profile_read", "alora_profile_reset", "alora_prefill", "alora_decode", "alora_decode_static", "alora_decode_steps", "alora_stack_prefill", "alora_stack_decode", "alora_lm_head"]
KERNELS = ["lm_head", "lm_argmax", "prep_rows", "qkv_gemm", "rope_append", "attn_prefill", "attn_decode", "attn_merge", "o_proj",
           "mlp_norm", "gate_up", "silu_mul", "down_proj"]


class LayerDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("rank", C.c_int32), ("n_adapters", C.c_int32), ("dtype", C.c_int32), ("intermediate", C.c_int32),
                ("W_qkv", C.c_void_p), ("A", C.c_void_p), ("B_q", C.c_void_p), ("B_k", C.c_void_p),
                ("B_v", C.c_void_p), ("scale", C.POINTER(C.c_float)), ("rms_gain", C.c_void_p),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("W_o", C.c_void_p), ("rms2_gain", C.c_void_p), ("W_gate", C.c_void_p), ("W_up", C.c_void_p),
                ("W_down", C.c_void_p),
                ("A_o", C.c_void_p), ("B_o", C.c_void_p), ("A_gu", C.c_void_p), ("B_gate", C.c_void_p),
                ("B_up", C.c_void_p), ("A_down", C.c_void_p), ("B_down", C.c_void_p)]


class KVCacheDesc(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("pool_tokens", C.c_int64),
                ("seq_offset", C.POINTER(C.c_int64)), ("seq_capacity", C.POINTER(C.c_int32)),
                ("seq_len", C.POINTER(C.c_int32)),
                ("prefix_offset", C.POINTER(C.c_int64)), ("prefix_len", C.POINTER(C.c_int32))]


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_12397_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.alora_create.restype = C.c_int
    lib.alora_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.alora_destroy.restype = None
    lib.alora_destroy.argtypes = [C.c_void_p]
    lib.alora_last_error.restype = C.c_char_p
    lib.alora_last_error.argtypes = [C.c_void_p]
    lib.alora_status_string.restype = C.c_char_p
    lib.alora_status_string.argtypes = [C.c_int]
    lib.alora_set_option.restype = C.c_int
    lib.alora_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int]
    lib.alora_profile_read.restype = C.c_int
    lib.alora_profile_read.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.alora_profile_reset.restype = C.c_int
    lib.alora_profile_reset.argtypes = [C.c_void_p]
    i32p = C.POINTER(C.c_int32)
    lib.alora_prefill.restype = C.c_int
    lib.alora_prefill.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.POINTER(KVCacheDesc), C.c_void_p, i32p, i32p,
                                  i32p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.alora_decode.restype = C.c_int
    lib.alora_decode.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.POINTER(KVCacheDesc), C.c_void_p, i32p, i32p,
                                 C.c_int32, C.c_void_p, C.c_void_p]
    lib.alora_decode_static.restype = C.c_int
    lib.alora_decode_static.argtypes = lib.alora_decode.argtypes
    lib.alora_decode_steps.restype = C.c_int
    lib.alora_decode_steps.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.POINTER(KVCacheDesc), C.c_void_p, i32p, i32p,
                                       C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.alora_lm_head.restype = C.c_int
    lib.alora_lm_head.argtypes = [C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p,
                                  C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.alora_stack_prefill.restype = C.c_int
    lib.alora_stack_prefill.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.c_int32, C.POINTER(KVCacheDesc),
                                        C.c_void_p, i32p, i32p, i32p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.alora_stack_decode.restype = C.c_int
    lib.alora_stack_decode.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.c_int32, C.POINTER(KVCacheDesc), C.c_void_p,
                                       C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p]
    return lib


_lib = load_library()


class AloraError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_lib.alora_status_string(status).decode()}: {message}")
        self.status = status
        self.message = message


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "libalora takes contiguous row-major buffers"
    return t.data_ptr()


def _i32(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class Layer:
    """Holds the device tensors of one decoder layer and the C descriptor that points at them."""

    def __init__(self, tensors: Dict[str, Optional[torch.Tensor]], n_q_heads: int, n_kv_heads: int, head_dim: int,
                 rms_eps: float = 1e-5, rope_theta: float = 10000.0, intermediate: int = 0):
        self.t = tensors
        W = tensors["W_qkv"]
        dt = {torch.float32: ALORA_F32, torch.bfloat16: ALORA_BF16}[W.dtype]
        A = tensors.get("A")
        n_ad = int(A.shape[0]) if A is not None else 0
        rank = int(A.shape[2]) if A is not None else 0
        self.scale = np.ascontiguousarray(np.asarray(tensors.get("scale") or [], dtype=np.float32))
        g = tensors.get
        self.desc = LayerDesc(int(W.shape[1]), n_q_heads, n_kv_heads, head_dim, rank, n_ad, dt, int(intermediate),
                              _ptr(W), _ptr(A), _ptr(g("B_q")), _ptr(g("B_k")), _ptr(g("B_v")),
                              self.scale.ctypes.data_as(C.POINTER(C.c_float)) if n_ad else None,
                              _ptr(g("rms_gain")), float(rms_eps), float(rope_theta),
                              _ptr(g("W_o")), _ptr(g("rms2_gain")), _ptr(g("W_gate")), _ptr(g("W_up")),
                              _ptr(g("W_down")), _ptr(g("A_o")), _ptr(g("B_o")), _ptr(g("A_gu")), _ptr(g("B_gate")),
                              _ptr(g("B_up")), _ptr(g("A_down")), _ptr(g("B_down")))
        self.n_q = n_q_heads * head_dim
        self.d = int(W.shape[1])
        self.dtype = W.dtype
        self.device = W.device


class KVCache:
    """A flat pool of token rows [pool_tokens, n_kv_heads, head_dim] for keys and for values, plus the
    host-side table that says which rows belong to which sequence and how many are valid."""

    def __init__(self, capacities: Sequence[int], n_kv_heads: int, head_dim: int, dtype: torch.dtype, device,
                 fill: Optional[float] = None, guard_rows: int = 0):
        caps = [int(c) for c in capacities]
        self.seq_capacity = _i32(caps)
        offs, o = [], guard_rows
        for c in caps:
            offs.append(o)
            o += c + guard_rows
        self.seq_offset = np.ascontiguousarray(np.asarray(offs, dtype=np.int64))
        self.pool_tokens = int(o)
        self.seq_len = np.zeros(len(caps), dtype=np.int32)
        self.prefix_offset = None        # set by share_prefix
        self.prefix_len = None
        shape = (self.pool_tokens, n_kv_heads, head_dim)
        if fill is None:
            self.k = torch.zeros(shape, dtype=dtype, device=device)
            self.v = torch.zeros(shape, dtype=dtype, device=device)
        else:
            self.k = torch.full(shape, fill, dtype=dtype, device=device)
            self.v = torch.full(shape, -fill, dtype=dtype, device=device)
        self._refresh()

    def _refresh(self):
        self.desc = KVCacheDesc(self.k.data_ptr(), self.v.data_ptr(), self.pool_tokens,
                                self.seq_offset.ctypes.data_as(C.POINTER(C.c_int64)),
                                self.seq_capacity.ctypes.data_as(C.POINTER(C.c_int32)),
                                self.seq_len.ctypes.data_as(C.POINTER(C.c_int32)),
                                None if self.prefix_len is None else self.prefix_offset.ctypes.data_as(C.POINTER(C.c_int64)),
                                None if self.prefix_len is None else self.prefix_len.ctypes.data_as(C.POINTER(C.c_int32)))

    def share_prefix(self, b: int, pool_row: int, n: int):
        """Positions 0..n-1 of sequence b are read from pool rows pool_row.. (one copy that several sequences
        may name); its own rows then start at position n.  seq_len[b] becomes n if it was smaller."""
        if self.prefix_len is None:
            self.prefix_offset = np.zeros(len(self.seq_len), dtype=np.int64)
            self.prefix_len = np.zeros(len(self.seq_len), dtype=np.int32)
        self.prefix_offset[b] = int(pool_row)
        self.prefix_len[b] = int(n)
        self.seq_len[b] = max(int(self.seq_len[b]), int(n))
        self._refresh()

    def rows(self, b: int, lo: int, hi: int):
        o = int(self.seq_offset[b])
        return self.k[o + lo:o + hi], self.v[o + lo:o + hi]

    def load_prefix(self, b: int, K: torch.Tensor, V: torch.Tensor):
        """Copy already-computed cache rows (e.g. the base model's) for positions 0..n-1 of sequence b."""
        n = K.shape[0]
        o = int(self.seq_offset[b])
        self.k[o:o + n] = K.to(self.k.dtype).view(n, *self.k.shape[1:]).to(self.k.device)
        self.v[o:o + n] = V.to(self.v.dtype).view(n, *self.v.shape[1:]).to(self.v.device)
        self.seq_len[b] = n


class Context:
    def __init__(self, device: int = 0):
        h = C.c_void_p()
        st = _lib.alora_create(C.byref(h), int(device))
        if st != ALORA_OK:
            raise AloraError(st, f"alora_create on device {device} failed")
        self._h = h
        self.device = int(device)

    def close(self):
        if getattr(self, "_h", None):
            _lib.alora_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != ALORA_OK:
            raise AloraError(st, _lib.alora_last_error(self._h).decode())

    def set_option(self, key: str, value: int):
        self._check(_lib.alora_set_option(self._h, key.encode(), int(value)))

    def profile_reset(self):
        self._check(_lib.alora_profile_reset(self._h))

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        """{kernel: {"ms": total, "launches": n}} for every kernel family that ran."""
        out = {}
        for name in KERNELS:
            ms, n = C.c_double(), C.c_int64()
            self._check(_lib.alora_profile_read(self._h, name.encode(), C.byref(ms), C.byref(n)))
            if n.value:
                out[name] = {"ms": ms.value, "launches": int(n.value)}
        return out


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def alora_prefill(ctx: Context, layer: Layer, cache: KVCache, x_suffix: torch.Tensor, cu_seqlens: Sequence[int],
                  k_per_seq: Sequence[int], adapter_per_seq: Sequence[int], attn_out: Optional[torch.Tensor] = None,
                  stream=None) -> torch.Tensor:
    cu, kk, ad = _i32(cu_seqlens), _i32(k_per_seq), _i32(adapter_per_seq)
    B = len(kk)
    if attn_out is None:
        attn_out = torch.empty((x_suffix.shape[0], layer.n_q), dtype=layer.dtype, device=layer.device)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_prefill(ctx._h, C.byref(layer.desc), C.byref(cache.desc), _ptr(x_suffix),
                            cu.ctypes.data_as(p), kk.ctypes.data_as(p), ad.ctypes.data_as(p), B,
                            _ptr(attn_out), _stream_ptr(stream))
    ctx._check(st)
    return attn_out


def alora_decode(ctx: Context, layer: Layer, cache: KVCache, x_tok: torch.Tensor, k_per_seq: Sequence[int],
                 adapter_per_seq: Sequence[int], attn_out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    kk, ad = _i32(k_per_seq), _i32(adapter_per_seq)
    B = len(kk)
    if attn_out is None:
        attn_out = torch.empty((B, layer.n_q), dtype=layer.dtype, device=layer.device)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_decode(ctx._h, C.byref(layer.desc), C.byref(cache.desc), _ptr(x_tok), kk.ctypes.data_as(p),
                           ad.ctypes.data_as(p), B, _ptr(attn_out), _stream_ptr(stream))
    ctx._check(st)
    return attn_out


def alora_decode_static(ctx: Context, layer: Layer, cache: KVCache, x_tok: torch.Tensor, k_per_seq: Sequence[int],
                        adapter_per_seq: Sequence[int], attn_out: torch.Tensor, stream=None) -> torch.Tensor:
    """alora_decode through the entry point that allocates nothing; the caller brings the output buffer."""
    kk, ad = _i32(k_per_seq), _i32(adapter_per_seq)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_decode_static(ctx._h, C.byref(layer.desc), C.byref(cache.desc), _ptr(x_tok), kk.ctypes.data_as(p),
                                  ad.ctypes.data_as(p), len(kk), _ptr(attn_out), _stream_ptr(stream))
    ctx._check(st)
    return attn_out


def alora_decode_steps(ctx: Context, layer: Layer, cache: KVCache, x_steps: torch.Tensor, k_per_seq: Sequence[int],
                       adapter_per_seq: Sequence[int], attn_out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x_steps [n_steps, B, d] -> attn_out [n_steps, B, N_q]: n_steps decode steps staged once."""
    kk, ad = _i32(k_per_seq), _i32(adapter_per_seq)
    B = len(kk)
    n_steps = int(x_steps.shape[0])
    if attn_out is None:
        attn_out = torch.empty((n_steps, B, layer.n_q), dtype=layer.dtype, device=layer.device)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_decode_steps(ctx._h, C.byref(layer.desc), C.byref(cache.desc), _ptr(x_steps), kk.ctypes.data_as(p),
                                 ad.ctypes.data_as(p), B, n_steps, _ptr(attn_out), _stream_ptr(stream))
    ctx._check(st)
    return attn_out


def alora_lm_head(ctx: Context, x_last: torch.Tensor, final_gain: Optional[torch.Tensor], rms_eps: float,
                  W_vocab: torch.Tensor, want_logits: bool = False, stream=None):
    """x_last [B, d], W_vocab [V, d] -> greedy token ids [B] (int32), and the fp32 logits [B, V] if asked for."""
    B, d = int(x_last.shape[0]), int(x_last.shape[1])
    V = int(W_vocab.shape[0])
    dt = ALORA_BF16 if x_last.dtype == torch.bfloat16 else ALORA_F32
    token = torch.empty((B,), dtype=torch.int32, device=x_last.device)
    logits = torch.empty((B, V), dtype=torch.float32, device=x_last.device) if want_logits else None
    st = _lib.alora_lm_head(ctx._h, dt, d, V, _ptr(x_last), _ptr(final_gain) if final_gain is not None else None,
                            float(rms_eps), _ptr(W_vocab), B, _ptr(logits) if logits is not None else None, _ptr(token),
                            _stream_ptr(stream))
    ctx._check(st)
    return (token, logits) if want_logits else token


def alora_stack_prefill(ctx: Context, layers: List[Layer], caches: List[KVCache], x: torch.Tensor,
                        cu_seqlens: Sequence[int], k_per_seq: Sequence[int], adapter_per_seq: Sequence[int],
                        out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    cu, kk, ad = _i32(cu_seqlens), _i32(k_per_seq), _i32(adapter_per_seq)
    B = len(kk)
    n = len(layers)
    descs = (LayerDesc * n)(*[l.desc for l in layers])
    cdescs = (KVCacheDesc * n)(*[c.desc for c in caches])
    if out is None:
        out = torch.empty_like(x)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_stack_prefill(ctx._h, descs, n, cdescs, _ptr(x), cu.ctypes.data_as(p), kk.ctypes.data_as(p),
                                  ad.ctypes.data_as(p), B, _ptr(out), _stream_ptr(stream))
    ctx._check(st)
    # the library updated the seq_len array that caches[0] points at; mirror it to the others
    for c in caches[1:]:
        if c.seq_len is not caches[0].seq_len:
            c.seq_len[:] = caches[0].seq_len
    return out


def alora_stack_decode(ctx: Context, layers: List[Layer], caches: List[KVCache], x_tok: torch.Tensor,
                       k_per_seq: Sequence[int], adapter_per_seq: Sequence[int], out: Optional[torch.Tensor] = None,
                       stream=None) -> torch.Tensor:
    kk, ad = _i32(k_per_seq), _i32(adapter_per_seq)
    B = len(kk)
    n = len(layers)
    descs = (LayerDesc * n)(*[l.desc for l in layers])
    cdescs = (KVCacheDesc * n)(*[c.desc for c in caches])
    if out is None:
        out = torch.empty_like(x_tok)
    p = C.POINTER(C.c_int32)
    st = _lib.alora_stack_decode(ctx._h, descs, n, cdescs, _ptr(x_tok), kk.ctypes.data_as(p), ad.ctypes.data_as(p), B,
                                 _ptr(out), _stream_ptr(stream))
    ctx._check(st)
    for c in caches[1:]:
        if c.seq_len is not caches[0].seq_len:
            c.seq_len[:] = caches[0].seq_len
    return out
