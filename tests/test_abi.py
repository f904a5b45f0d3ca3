"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
and rejects bad arguments before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

import paper_2503_01840_amd as E
from paper_2503_01840_amd import binding as Bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(E.LIB_PATH):
        from paper_2503_01840_amd.build import build_library
        build_library()
    return E.lib()


def test_every_symbol_declared_in_the_header_is_exported(L):
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("eagle3.h", "eagle3_measure.h"))
    declared = set(re.findall(r"\b(eagle3_[a-z_]+)\s*\(", header))
    assert declared == set(E.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def _cfg(**over):
    c = Bd.Config()
    vals = dict(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, intermediate=688, vocab=2048, draft_vocab=2048,
                n_layers=4, dtype=Bd.EAGLE3_FP32, rope_theta=1e4, rms_eps=1e-5, max_batch=1, max_nodes=16, max_depth=3,
                max_topk=4, max_new=4)
    vals.update(over)
    for k, v in vals.items():
        setattr(c, k, v)
    c.tap_layers = (C.c_int32 * 3)(*over.get("taps", (1, 2, 3)))
    return c


def test_create_validates_the_configuration(L):
    h = C.c_void_p()
    assert L.eagle3_create(None, C.byref(h)) == -1
    for bad in (dict(max_nodes=65), dict(n_heads=3, n_kv_heads=2), dict(max_topk=17), dict(taps=(1, 2, 4)),
                dict(dtype=Bd.EAGLE3_BF16), dict(head_dim=63), dict(max_depth=20, max_topk=10), dict(hidden=0)):
        c = _cfg(**bad)
        assert L.eagle3_create(C.byref(c), C.byref(h)) == -2, bad
    c = _cfg()
    assert L.eagle3_create(C.byref(c), C.byref(h)) == 0
    need = C.c_size_t()
    assert L.eagle3_workspace_bytes(h, C.byref(need)) == 0 and need.value > 0
    # no workspace / weights yet: the step calls must refuse, and never touch the (bogus) pointers
    one = C.c_void_p(256)
    assert L.eagle3_set_workspace(h, one, 16) == -3
    assert L.eagle3_fuse_features(h, one, one, one, 1, one, None) == -3
    assert L.eagle3_accept(h, 1, 4, one, one, one, 0.0, None, one, one, one, None) == -3
    assert L.eagle3_fuse_features(h, None, one, one, 1, one, None) == -1
    assert L.eagle3_destroy(h) == 0
    assert L.eagle3_strerror(-2).decode().startswith("a size")


def test_bf16_configuration_limits(L):
    h = C.c_void_p()
    ok = _cfg(dtype=Bd.EAGLE3_BF16, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128, intermediate=1024)
    assert L.eagle3_create(C.byref(ok), C.byref(h)) == 0
    L.eagle3_destroy(h)
    for bad in (dict(hidden=500), dict(intermediate=1000), dict(head_dim=64), dict(vocab=1001, max_batch=4, max_nodes=32)):
        kw = dict(dtype=Bd.EAGLE3_BF16, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128, intermediate=1024)
        kw.update(bad)
        c = _cfg(**kw)
        assert L.eagle3_create(C.byref(c), C.byref(h)) == -2, bad
