"""Host-side checks that need no GPU: the library loads, exports every declared entry point, and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_13319_amd import inputs as I
from paper_2605_13319_amd import nav

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            txt = open(os.path.join(ROOT, "include", fn)).read()
            txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
            names |= set(re.findall(r"\b(pipesd_[a-z0-9_]+)\s*\(", txt))
    return names


def test_every_declared_symbol_is_exported_and_bound():
    decl = _declared()
    assert len(decl) >= 15
    lib = C.CDLL(nav.LIB_PATH)
    for name in decl:
        assert hasattr(lib, name), name
    assert decl == set(nav.EXPORTS)


def test_strerror():
    for st in (0, -1, -2, -3, -4, -99):
        assert isinstance(nav._lib.pipesd_strerror(st), bytes)


def _create(shape, weights_ptr=None):
    h = C.c_void_p()
    cfg = nav.config_of(shape)
    return nav._lib.pipesd_model_create(C.byref(cfg), weights_ptr, C.byref(h)), h


@pytest.mark.parametrize("bad", [
    dict(n_layers=0), dict(n_q_heads=6, n_kv_heads=4), dict(head_dim=63), dict(head_dim=256, n_q_heads=2, n_kv_heads=2),
    dict(d_model=1000), dict(d_ffn=1000), dict(vocab=0), dict(dtype=7), dict(rope_base=0.0),
    dict(d_model=8704)])  # more than 512 partial sums of squares per row: beyond what the fused norm reads
def test_model_create_rejects_bad_shapes(bad):
    import dataclasses
    shape = dataclasses.replace(I.LLAMA_1B, **bad)
    rc, _ = _create(shape)
    assert rc == nav.EINVAL


def test_null_arguments():
    assert nav._lib.pipesd_model_create(None, None, None) == nav.EINVAL
    assert nav._lib.pipesd_model_destroy(None) == nav.EINVAL
    assert nav._lib.pipesd_kv_destroy(None) == nav.EINVAL
    assert nav._lib.pipesd_kv_block_bytes(None, 16) == 0
    n = C.c_int32()
    assert nav._lib.pipesd_kv_len(None, 0, C.byref(n)) == nav.EINVAL


def test_shape_only_handles_do_bookkeeping_but_refuse_compute():
    m = nav.Model(I.LLAMA_8B, None)
    assert nav._lib.pipesd_kv_block_bytes(m.handle, 16) == 32 * 2 * 8 * 128 * 16 * 2
    assert nav._lib.pipesd_kv_block_bytes(m.handle, 32) == 0
    kv = nav.KVCache(m, max_seqs=4, n_blocks=100, on_device=False)
    assert kv.free_blocks() == 100 and kv.length(3) == 0 and kv.seq_blocks(0) == 0
    with pytest.raises(nav.PipesdError) as e:
        kv.length(4)
    assert e.value.status == nav.EINVAL
    with pytest.raises(nav.PipesdError) as e:
        kv.rollback(0, 1)
    assert e.value.status == nav.ESTATE
    import numpy as np
    toks = np.arange(5, dtype=np.int32)
    rc = nav._lib.pipesd_prefill(m.handle, kv.handle, 0, toks.ctypes.data_as(nav._i32p), 5, None)
    assert rc == nav.ESTATE
    a, nx = C.c_int32(), C.c_int32()
    rc = nav._lib.pipesd_nav_verify(m.handle, kv.handle, 0, 5, toks.ctypes.data_as(nav._i32p), 4, None, None,
                                    C.byref(a), C.byref(nx), None)
    assert rc == nav.ESTATE
    # argument checks come first
    rc = nav._lib.pipesd_nav_verify(m.handle, kv.handle, 0, 5, toks.ctypes.data_as(nav._i32p), 0, None, None,
                                    C.byref(a), C.byref(nx), None)
    assert rc == nav.EINVAL
    rc = nav._lib.pipesd_nav_verify(m.handle, kv.handle, 0, 5, toks.ctypes.data_as(nav._i32p), 32, None, None,
                                    C.byref(a), C.byref(nx), None)
    assert rc == nav.EINVAL
    bad = np.array([1, 2, I.LLAMA_8B.vocab], dtype=np.int32)
    rc = nav._lib.pipesd_nav_verify(m.handle, kv.handle, 0, 5, bad.ctypes.data_as(nav._i32p), 3, None, None,
                                    C.byref(a), C.byref(nx), None)
    assert rc == nav.EINVAL
    assert kv.free_blocks() == 100
    # batched call: the same argument checks, plus distinct clients and a bounded count
    ip = nav._i32p
    ids = np.array([0, 1], dtype=np.int32)
    pl = np.array([5, 5], dtype=np.int32)
    ks = np.array([2, 2], dtype=np.int32)
    cat = np.array([1, 2, 3, 4], dtype=np.int32)
    out_a, out_n = np.zeros(2, dtype=np.int32), np.zeros(2, dtype=np.int32)

    def batch(n, ids_, ks_, cat_):
        return nav._lib.pipesd_nav_verify_batch(m.handle, kv.handle, n, ids_.ctypes.data_as(ip), pl.ctypes.data_as(ip),
                                                ks_.ctypes.data_as(ip), cat_.ctypes.data_as(ip), None, None,
                                                out_a.ctypes.data_as(ip), out_n.ctypes.data_as(ip), None)

    assert batch(2, ids, ks, cat) == nav.ESTATE          # shape-only handles refuse compute
    assert batch(0, ids, ks, cat) == nav.EINVAL
    assert batch(257, ids, ks, cat) == nav.EINVAL
    assert batch(2, np.array([1, 1], dtype=np.int32), ks, cat) == nav.EINVAL    # the same client twice
    assert batch(2, np.array([0, 4], dtype=np.int32), ks, cat) == nav.EINVAL    # no such client
    assert batch(2, ids, np.array([2, 0], dtype=np.int32), cat) == nav.EINVAL   # k out of range
    assert batch(2, ids, ks, np.array([1, 2, 3, -1], dtype=np.int32)) == nav.EINVAL
    assert nav._lib.pipesd_nav_verify_batch(m.handle, kv.handle, 2, None, None, None, None, None, None, None, None,
                                            None) == nav.EINVAL
    assert kv.free_blocks() == 100
    # chained rounds: the same checks for every round and for the guessed tokens in between
    ran = np.zeros(1, dtype=np.int32)

    def chain(n, ks_, cat_, seq=0):
        return nav._lib.pipesd_nav_verify_chain(m.handle, kv.handle, seq, 5, n, ks_.ctypes.data_as(ip),
                                                cat_.ctypes.data_as(ip), None, None, out_a.ctypes.data_as(ip),
                                                out_n.ctypes.data_as(ip), ran.ctypes.data_as(ip), None)

    cat2 = np.array([1, 2, 9, 3, 4], dtype=np.int32)  # round 0: 1 2; buffer: guess 9, drafts 3 4
    assert chain(2, ks, cat2) == nav.ESTATE              # shape-only handles refuse compute
    assert chain(0, ks, cat2) == nav.EINVAL
    assert chain(17, ks, cat2) == nav.EINVAL
    assert chain(2, ks, cat2, seq=4) == nav.EINVAL       # no such client
    assert chain(2, np.array([2, 32], dtype=np.int32), cat2) == nav.EINVAL
    assert chain(2, ks, np.array([1, 2, -1, 3, 4], dtype=np.int32)) == nav.EINVAL   # a guess outside the vocabulary
    assert chain(2, ks, np.array([1, 2, 9, 3, I.LLAMA_8B.vocab], dtype=np.int32)) == nav.EINVAL
    assert nav._lib.pipesd_nav_verify_chain(m.handle, kv.handle, 0, 5, 2, None, None, None, None, None, None, None,
                                            None) == nav.EINVAL
    assert kv.free_blocks() == 100
    kv.close()
    m.close()


def test_kv_create_argument_checks():
    m = nav.Model(I.TINY, None)
    h = C.c_void_p()
    bb = nav._lib.pipesd_kv_block_bytes(m.handle, 16)
    assert bb == 2 * 2 * 4 * 64 * 16 * 4
    assert nav._lib.pipesd_kv_create(m.handle, 0, 16, None, 10 * bb, C.byref(h)) == nav.EINVAL
    assert nav._lib.pipesd_kv_create(m.handle, 1, 8, None, 10 * bb, C.byref(h)) == nav.EINVAL
    assert nav._lib.pipesd_kv_create(m.handle, 1, 16, None, bb - 1, C.byref(h)) == nav.EINVAL
    assert nav._lib.pipesd_kv_create(m.handle, 1, 16, C.c_void_p(0x1010), 10 * bb, C.byref(h)) == nav.EINVAL
    # a device pool cannot be attached to a shape-only model
    assert nav._lib.pipesd_kv_create(m.handle, 1, 16, C.c_void_p(0x1000), 10 * bb, C.byref(h)) == nav.ESTATE
    m.close()


def test_two_half_verify_without_a_pass_begun():
    """pipesd_nav_verify_end / _done without a begin are state errors; null arguments are invalid."""
    rc, h = _create(I.LLAMA_1B)
    assert rc == nav.OK
    a, n, done = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    assert nav._lib.pipesd_nav_verify_end(h, C.byref(a), C.byref(n)) == nav.ESTATE
    assert nav._lib.pipesd_nav_verify_done(h, C.byref(done)) == nav.ESTATE
    assert nav._lib.pipesd_nav_verify_end(None, C.byref(a), C.byref(n)) == nav.EINVAL
    assert nav._lib.pipesd_nav_verify_end(h, None, C.byref(n)) == nav.EINVAL
    assert nav._lib.pipesd_nav_verify_done(h, None) == nav.EINVAL
    assert nav._lib.pipesd_nav_verify_begin(None, None, 0, 1, None, 1, None, None, None) == nav.EINVAL
    assert nav._lib.pipesd_model_destroy(h) == nav.OK
