"""CPU-side checks of the boundary: the shared library loads, exports every entry point that
include/alora.h declares, and rejects bad arguments on the host before anything is launched
(through a validation-only context, device -1, which needs no GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ab():
    from paper_2504_12397_amd import binding
    return binding


def declared_entry_points():
    text = open(os.path.join(ROOT, "include", "alora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(alora_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(ab):
    names = declared_entry_points()
    assert set(names) == set(ab.EXPORTS)
    lib = C.CDLL(ab.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_header(ab):
    # natural alignment, no packing: 8 int32, then pointers / floats as declared
    assert C.sizeof(ab.LayerDesc) == 8 * 4 + 7 * 8 + 2 * 4 + 5 * 8 + 7 * 8
    assert ab.LayerDesc.W_qkv.offset == 32 and ab.LayerDesc.rms_eps.offset == 88 and ab.LayerDesc.W_o.offset == 96
    assert C.sizeof(ab.KVCacheDesc) == 64


def test_status_strings(ab):
    lib = ab._lib
    assert lib.alora_status_string(0) == b"ALORA_OK"
    assert lib.alora_status_string(3) == b"ALORA_ECAPACITY"


class FakeBuf:
    """Stands in for device memory in validation-only calls: never dereferenced."""
    PTR = 0x1000


def make_args(ab, **over):
    d = dict(d=64, n_q_heads=4, n_kv_heads=2, head_dim=16, rank=4, n_adapters=2, dtype=ab.ALORA_BF16, intermediate=0)
    d.update({k: v for k, v in over.items() if k in d})
    scale = np.ones(2, dtype=np.float32)
    p = FakeBuf.PTR
    desc = ab.LayerDesc(d["d"], d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["rank"], d["n_adapters"], d["dtype"],
                        d["intermediate"], p, p, p, p, p, scale.ctypes.data_as(C.POINTER(C.c_float)), p, 1e-5,
                        over.get("rope_theta", 10000.0), None, None, None, None, None)
    B = over.get("B", 2)
    off = np.asarray(over.get("seq_offset", [0, 100]), dtype=np.int64)
    cap = np.asarray(over.get("seq_capacity", [100, 100]), dtype=np.int32)
    ln = np.asarray(over.get("seq_len", [10, 20]), dtype=np.int32)
    cache = ab.KVCacheDesc(p, p, over.get("pool_tokens", 200), off.ctypes.data_as(C.POINTER(C.c_int64)),
                           cap.ctypes.data_as(C.POINTER(C.c_int32)), ln.ctypes.data_as(C.POINTER(C.c_int32)))
    cu = np.asarray(over.get("cu", [0, 3, 8]), dtype=np.int32)
    k = np.asarray(over.get("k", [10, 20]), dtype=np.int32)
    a = np.asarray(over.get("a", [0, -1]), dtype=np.int32)
    keep = (scale, off, cap, ln, cu, k, a)
    return desc, cache, cu, k, a, B, keep, ln


@pytest.fixture()
def vctx(ab):
    h = C.c_void_p()
    assert ab._lib.alora_create(C.byref(h), -1) == ab.ALORA_OK
    yield h
    ab._lib.alora_destroy(h)


def call(ab, h, desc, cache, cu, k, a, B):
    p = C.POINTER(C.c_int32)
    return ab._lib.alora_prefill(h, C.byref(desc), C.byref(cache), FakeBuf.PTR, cu.ctypes.data_as(p),
                                 k.ctypes.data_as(p), a.ctypes.data_as(p), B, FakeBuf.PTR, None)


@pytest.mark.parametrize("over,status", [
    (dict(dtype=7), "ALORA_EDTYPE"),
    (dict(n_q_heads=5), "ALORA_ESHAPE"),
    (dict(head_dim=15), "ALORA_ESHAPE"),
    (dict(head_dim=512), "ALORA_ESHAPE"),
    (dict(d=0), "ALORA_ESHAPE"),
    (dict(rank=0), "ALORA_ESHAPE"),
    (dict(rope_theta=0.0), "ALORA_ESHAPE"),
    (dict(B=0), "ALORA_EINVAL"),
    (dict(cu=[1, 3, 8]), "ALORA_EINVAL"),
    (dict(cu=[0, 5, 3]), "ALORA_EINVAL"),
    (dict(k=[-1, 0]), "ALORA_EINVAL"),
    (dict(seq_len=[-1, 0]), "ALORA_EINVAL"),
    (dict(a=[2, 0]), "ALORA_EADAPTER"),
    (dict(a=[-2, 0]), "ALORA_EADAPTER"),
    (dict(seq_len=[98, 20]), "ALORA_ECAPACITY"),
    (dict(seq_capacity=[100, 101]), "ALORA_ECAPACITY"),
    (dict(seq_offset=[0, -1]), "ALORA_ECAPACITY"),
])
def test_bad_arguments_are_rejected_before_launch(ab, vctx, over, status):
    desc, cache, cu, k, a, B, keep, ln = make_args(ab, **over)
    before = ln.copy()
    st = call(ab, vctx, desc, cache, cu, k, a, B)
    assert ab._lib.alora_status_string(st).decode() == status
    assert len(ab._lib.alora_last_error(vctx)) > 0
    assert np.array_equal(ln, before)          # seq_len untouched on error


def test_valid_arguments_pass_validation_and_empty_batch_is_a_noop(ab, vctx):
    desc, cache, cu, k, a, B, keep, ln = make_args(ab)
    st = call(ab, vctx, desc, cache, cu, k, a, B)
    # a validation-only context cannot launch: everything checked out, then it says so
    assert st == ab.ALORA_EHIP and b"validation-only" in ab._lib.alora_last_error(vctx)
    assert list(ln) == [10, 20]
    desc, cache, cu, k, a, B, keep, ln = make_args(ab, cu=[0, 0, 0])
    assert call(ab, vctx, desc, cache, cu, k, a, B) == ab.ALORA_OK
    assert list(ln) == [10, 20]


def test_null_pointers(ab, vctx):
    desc, cache, cu, k, a, B, keep, ln = make_args(ab)
    p = C.POINTER(C.c_int32)
    st = ab._lib.alora_prefill(vctx, None, C.byref(cache), FakeBuf.PTR, cu.ctypes.data_as(p), k.ctypes.data_as(p),
                               a.ctypes.data_as(p), B, FakeBuf.PTR, None)
    assert st == ab.ALORA_EINVAL
    st = ab._lib.alora_prefill(vctx, C.byref(desc), C.byref(cache), None, cu.ctypes.data_as(p), k.ctypes.data_as(p),
                               a.ctypes.data_as(p), B, FakeBuf.PTR, None)
    assert st == ab.ALORA_EINVAL
    assert ab._lib.alora_set_option(vctx, b"nonsense", 1) == ab.ALORA_EINVAL
    assert ab._lib.alora_set_option(vctx, b"kernels", 1) == ab.ALORA_OK
    assert ab._lib.alora_prefill(None, C.byref(desc), C.byref(cache), FakeBuf.PTR, cu.ctypes.data_as(p),
                                 k.ctypes.data_as(p), a.ctypes.data_as(p), B, FakeBuf.PTR, None) == ab.ALORA_EINVAL


def test_decode_steps_validation(ab, vctx):
    """A run of decode steps is checked as a whole: every step must fit the capacity."""
    p = C.POINTER(C.c_int32)

    def steps(n, **over):
        desc, cache, cu, k, a, B, keep, ln = make_args(ab, **over)
        st = ab._lib.alora_decode_steps(vctx, C.byref(desc), C.byref(cache), FakeBuf.PTR, k.ctypes.data_as(p),
                                        a.ctypes.data_as(p), B, n, FakeBuf.PTR, None)
        return ab._lib.alora_status_string(st).decode(), list(ln)

    assert steps(0) == ("ALORA_EINVAL", [10, 20])
    assert steps(-3) == ("ALORA_EINVAL", [10, 20])
    assert steps(4, B=0) == ("ALORA_EINVAL", [10, 20])
    # 20 cached + 81 steps > capacity 100; 80 steps fit (validation-only context then declines to launch)
    assert steps(81) == ("ALORA_ECAPACITY", [10, 20])
    assert steps(80) == ("ALORA_EHIP", [10, 20])
    assert steps(2, seq_len=[99, 20]) == ("ALORA_ECAPACITY", [99, 20])


def test_shared_prefix_validation(ab, vctx):
    """Shared-prefix fields of the cache descriptor: bounds, and the capacity counts own rows only."""
    p = C.POINTER(C.c_int32)
    p64 = C.POINTER(C.c_int64)

    def go(prefix_len, prefix_off, seq_len=(10, 20), cap=(100, 100), give_off=True):
        desc, cache, cu, k, a, B, keep, ln = make_args(ab, seq_len=list(seq_len), seq_capacity=list(cap))
        pl = np.asarray(prefix_len, dtype=np.int32)
        po = np.asarray(prefix_off, dtype=np.int64)
        cache.prefix_len = pl.ctypes.data_as(p)
        if give_off:
            cache.prefix_offset = po.ctypes.data_as(p64)
        st = call(ab, vctx, desc, cache, cu, k, a, B)
        return ab._lib.alora_status_string(st).decode(), list(ln)

    ok = "ALORA_EHIP"       # validation passed; the validation-only context then declines to launch
    assert go([0, 0], [0, 0]) == (ok, [10, 20])
    assert go([10, 5], [150, 150]) == (ok, [10, 20])
    assert go([11, 5], [150, 150])[0] == "ALORA_EINVAL"          # longer than what is cached
    assert go([-1, 5], [150, 150])[0] == "ALORA_EINVAL"
    assert go([10, 5], [195, 150])[0] == "ALORA_ECAPACITY"       # rows 195..204 leave the pool of 200
    assert go([10, 5], [-1, 150])[0] == "ALORA_ECAPACITY"
    assert go([10, 5], [0, 0], give_off=False)[0] == "ALORA_EINVAL"
    # 90 cached rows of which 80 are shared: 10 own + 3 new fit a capacity of 13, not of 12
    assert go([80, 0], [20, 0], seq_len=(90, 20), cap=(13, 100)) == (ok, [90, 20])
    assert go([80, 0], [20, 0], seq_len=(90, 20), cap=(12, 100))[0] == "ALORA_ECAPACITY"
    # the shared rows [100, 180) are rows sequence 1 is about to write ([120, 125)): rejected
    assert go([80, 0], [100, 0], seq_len=(90, 20), cap=(13, 100))[0] == "ALORA_ECAPACITY"
    # reading another sequence's already valid rows as a prefix is fine (the base model's own sequence in the batch)
    assert go([15, 0], [100, 0], seq_len=(18, 20), cap=(13, 100)) == (ok, [18, 20])


def test_overlapping_sequence_regions_are_rejected(ab, vctx):
    """Two sequences of one call may not own the same pool rows: both would write them."""
    for off, cap, want in (([0, 100], [100, 100], "ALORA_EHIP"), ([0, 99], [100, 100], "ALORA_ECAPACITY"),
                           ([100, 0], [100, 100], "ALORA_EHIP"), ([50, 0], [100, 100], "ALORA_ECAPACITY"),
                           ([0, 0], [100, 100], "ALORA_ECAPACITY"), ([0, 0], [100, 0], "ALORA_ECAPACITY")):
        desc, cache, cu, k, a, B, keep, ln = make_args(ab, seq_offset=off, seq_capacity=cap,
                                                       seq_len=[10, 0] if cap[1] == 0 else [10, 20],
                                                       cu=[0, 3, 3] if cap[1] == 0 else [0, 3, 8])
        st = ab._lib.alora_status_string(call(ab, vctx, desc, cache, cu, k, a, B)).decode()
        if cap[1] == 0:
            want = "ALORA_EHIP"          # an empty region overlaps nothing
        assert st == want, (off, cap, st)
        assert list(ln) == ([10, 0] if cap[1] == 0 else [10, 20])


def test_lm_head_validation(ab, vctx):
    f = ab._lib.alora_lm_head
    P = FakeBuf.PTR

    def go(dtype=ab.ALORA_BF16, d=64, vocab=1000, x=P, W=P, B=2, logits=P, token=P):
        return ab._lib.alora_status_string(f(vctx, dtype, d, vocab, x, P, 1e-5, W, B, logits, token, None)).decode()

    assert go() == "ALORA_EHIP"                      # everything checked out; a validation-only context cannot launch
    assert go(dtype=9) == "ALORA_EDTYPE"
    assert go(d=0) == "ALORA_ESHAPE"
    assert go(vocab=0) == "ALORA_ESHAPE"
    assert go(B=0) == "ALORA_EINVAL"
    assert go(x=None) == "ALORA_EINVAL"
    assert go(W=None) == "ALORA_EINVAL"
    assert go(logits=None, token=None) == "ALORA_EINVAL"
    assert go(logits=None) == "ALORA_EHIP" and go(token=None) == "ALORA_EHIP"
    assert f(None, ab.ALORA_BF16, 64, 1000, P, P, 1e-5, P, 2, P, P, None) == ab.ALORA_EINVAL


def test_tail_adapter_groups_are_checked_as_a_whole(ab, vctx):
    """Adapters of W_o / the MLP linears (layer stack only): each group is complete or absent."""
    p32 = C.POINTER(C.c_int32)

    def go(**fields):
        desc, cache, cu, k, a, B, keep, ln = make_args(ab, intermediate=128)
        for f in ("W_o", "rms2_gain", "W_gate", "W_up", "W_down"):
            setattr(desc, f, FakeBuf.PTR)
        for f, v in fields.items():
            setattr(desc, f, v)
        st = ab._lib.alora_stack_prefill(vctx, C.byref(desc), 1, C.byref(cache), FakeBuf.PTR, cu.ctypes.data_as(p32),
                                         k.ctypes.data_as(p32), a.ctypes.data_as(p32), B, FakeBuf.PTR, None)
        return ab._lib.alora_status_string(st).decode()

    P = FakeBuf.PTR
    assert go() == "ALORA_EHIP"                                     # valid, nothing to launch on
    assert go(A_o=P, B_o=P, A_gu=P, B_gate=P, B_up=P, A_down=P, B_down=P) == "ALORA_EHIP"
    assert go(A_o=P) == "ALORA_EINVAL"
    assert go(B_down=P) == "ALORA_EINVAL"
    assert go(A_gu=P, B_gate=P) == "ALORA_EINVAL"
    assert go(A_o=P, B_o=P, n_adapters=0, rank=0) == "ALORA_EINVAL"


def test_static_decode_rejects_what_its_scratch_cannot_hold(ab, vctx):
    """alora_decode_static checks its arguments like alora_decode and, on top, that the call fits the static
    scratch array (32 MiB); both before anything would be launched."""
    p = C.POINTER(C.c_int32)

    def go(B, **over):
        off = [100 * b for b in range(B)]
        desc, cache, cu, k, a, _, keep, ln = make_args(ab, B=B, seq_offset=off, seq_capacity=[100] * B, seq_len=[10] * B,
                                                       pool_tokens=100 * B, k=[0] * B, a=[0] * B, **over)
        st = ab._lib.alora_decode_static(vctx, C.byref(desc), C.byref(cache), FakeBuf.PTR, k.ctypes.data_as(p),
                                         a.ctypes.data_as(p), B, FakeBuf.PTR, None)
        return ab._lib.alora_status_string(st).decode(), ab._lib.alora_last_error(vctx).decode(), list(ln)

    assert go(2)[0] == "ALORA_EHIP"                       # valid; a validation-only context cannot launch
    st, msg, ln = go(3000, d=4096, n_q_heads=32, n_kv_heads=8, head_dim=128)
    assert st == "ALORA_ECAPACITY" and "scratch" in msg and ln == [10] * 3000
    assert go(5000)[0] == "ALORA_ECAPACITY"               # more than 4096 sequences
    assert go(0)[0] == "ALORA_EINVAL"
    assert go(2, dtype=9)[0] == "ALORA_EDTYPE"
