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


def test_public_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 (no C++ or torch types in it) and as C++."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no host C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "pquant.h"\nint main(void) { return (int)sizeof(pq_linear_desc) == 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    if shutil.which("g++") is not None:
        subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)


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
    assert lib.pq_pack_sign(fake, pq.PQ_BF16, 40, 42, fake, fake, fake, fake, C.c_size_t(1 << 20), None) == -2   # K % 4
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


def test_new_entry_points_validate_on_the_host(lib):
    fake = C.c_void_p(0x1000)
    big = C.c_size_t(1 << 40)
    # INT8 high-precision branch: bf16 only, multiples of 32, buffers sized by the queries
    lib.pq_hp_int8_ctx_bytes.restype = C.c_size_t
    assert lib.pq_hp_int8_ctx_bytes(16, 64, 64, 32) > 0 and lib.pq_hp_int8_ctx_bytes(16, 64, 64, 24) == 0
    assert lib.pq_hp_int8_fwd(fake, fake, fake, fake, pq.PQ_F32, 16, 64, 64, 32, C.c_float(1.0), fake, 0, fake, big, fake, big, None) == -3
    assert lib.pq_hp_int8_fwd(fake, fake, fake, fake, pq.PQ_BF16, 16, 64, 64, 32, C.c_float(1.0), fake, 0, fake, C.c_size_t(8), fake, big,
                              None) == -4
    # decode with INT8 experts: rank multiple of 32; batch > 1 only on the row-interleaved packing with r % 64 == 0
    d = pq.DecodeDesc(1, 256, 64, 16, 4, 2, 1, pq.PQ_PACKED_TILED64, 1.0)
    assert lib.pq_decode_gemv_int8(C.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, fake, big, None) == -2
    d = pq.DecodeDesc(4, 512, 64, 64, 4, 2, 1, pq.PQ_PACKED_ROWMAJOR, 1.0)
    assert lib.pq_decode_gemv_int8(C.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, fake, big, None) == -2
    # decode FFN: dimensions multiples of 128, a positive expert width
    lib.pq_decode_ffn_workspace_bytes.restype = C.c_size_t
    assert lib.pq_decode_ffn_workspace_bytes(C.byref(pq.DecodeFFNDesc(256, 384, 16, 4, 2, 2, 1.0))) > 0
    assert lib.pq_decode_ffn_workspace_bytes(C.byref(pq.DecodeFFNDesc(256, 400, 16, 4, 2, 2, 1.0))) == 0
    assert lib.pq_decode_ffn_workspace_bytes(C.byref(pq.DecodeFFNDesc(256, 384, 0, 4, 2, 2, 1.0))) == 0
    df = pq.DecodeFFNDesc(256, 384, 16, 4, 2, 2, 1.0)
    assert lib.pq_decode_ffn(C.byref(df), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, fake, C.c_size_t(8), None) == -4
