"""Host-side checks of libpquant that need no GPU: the library loads, exports every function the
public header declares, and refuses bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2602_22592_amd import binding as pq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pq.LIB_PATH):
        from paper_2602_22592_amd.build import build
        build(verbose=False)
    return pq.lib()


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(pq_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_functions()
    assert {"pq_linear_fwd", "pq_linear_bwd", "pq_pack_sign", "pq_router_topk"} <= declared
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert set(pq.EXPORTS) <= declared
    assert lib.pq_version() >= 100


def test_bad_arguments_are_refused_on_the_host(lib):
    fake = C.c_void_p(0x1000)           # never dereferenced: validation fails first
    assert lib.pq_quant_act(fake, pq.PQ_BF16, 4, 48, fake, fake, None) == -2      # K % 32
    assert b"multiple of 32" in lib.pq_last_error_string()
    assert lib.pq_quant_act(fake, 7, 4, 64, fake, fake, None) == -3               # dtype
    assert lib.pq_quant_act(None, pq.PQ_BF16, 4, 64, fake, fake, None) == -1      # NULL
    assert lib.pq_quant_act(C.c_void_p(0x1004), pq.PQ_BF16, 4, 64, fake, fake, None) == -2   # alignment
    assert lib.pq_router_topk(fake, fake, pq.PQ_BF16, 4, 64, 8, 9, fake, fake, None, None) == -1
    assert lib.pq_pack_sign(fake, pq.PQ_BF16, 40, 64, fake, fake, fake, fake, C.c_size_t(1 << 20), None) == -2
    assert lib.pq_pack_sign(fake, pq.PQ_BF16, 64, 64, fake, None, fake, fake, C.c_size_t(8), None) == -4
    d = pq.make_desc(16, 48, 64)
    assert lib.pq_linear_ctx_bytes(C.byref(d)) == 0                               # d_in % 32
    d = pq.make_desc(16, 64, 64, hp_rank=8)
    nctx, nws = lib.pq_linear_ctx_bytes(C.byref(d)), lib.pq_linear_workspace_bytes(C.byref(d))
    assert nctx > 0 and nws > 0
    rc = lib.pq_linear_fwd(C.byref(d), fake, fake, None, fake, fake, None, fake, fake, C.c_size_t(8), fake,
                           C.c_size_t(nws), None)
    assert rc == -4 and b"ctx too small" in lib.pq_last_error_string()
    d2 = pq.make_desc(16, 64, 72, hp_rank=8)                                       # d_out % 32 for training
    rc = lib.pq_linear_bwd(C.byref(d2), fake, fake, fake, fake, fake, None, fake, C.c_size_t(1 << 30), fake, fake,
                           fake, fake, None, fake, fake, C.c_size_t(1 << 30), None)
    assert rc == -2


def test_zero_token_calls_launch_nothing(lib):
    fake = C.c_void_p(0x1000)
    assert lib.pq_quant_act(fake, pq.PQ_BF16, 0, 64, fake, fake, None) == 0
    assert lib.pq_router_topk(fake, fake, pq.PQ_BF16, 0, 64, 8, 2, fake, fake, None, None) == 0
    assert lib.pq_onebit_acc(fake, fake, 0, 64, 64, fake, None) == 0
