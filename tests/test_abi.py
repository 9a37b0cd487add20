"""The C-ABI library loads on a machine without a GPU, exports every function the header
declares, and rejects bad arguments on the host before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2510_17238_amd as st
    if not os.path.exists(st.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return st.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "st.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"st_rope_apply", "st_attn_prefill", "st_kv_append", "st_attn_decode_dual", "st_plan_create"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_version_and_error_string(lib):
    assert lib.st_version() >= 1
    assert lib.st_last_error() is not None


def test_host_side_argument_checks(lib):
    import paper_2510_17238_amd.binding as B
    # null pointers
    assert lib.st_rope_apply(None, None, None, 4, 2, 64, 1e6, B.ST_F32, None) == 1
    assert b"null" in lib.st_last_error()
    fake = C.c_void_p(0x1000)   # never dereferenced: the checks below fail first
    assert lib.st_rope_apply(fake, fake, fake, 4, 2, 80, 1e6, B.ST_F32, None) == 5      # head_dim
    assert lib.st_rope_apply(fake, fake, fake, 4, 2, 64, -1.0, B.ST_F32, None) == 1     # theta
    assert lib.st_rope_apply(C.c_void_p(0x1004), fake, fake, 4, 2, 64, 1e6, B.ST_F32, None) == 1   # alignment
    handle = C.c_void_p()
    assert lib.st_plan_create(C.byref(handle), None, None, None, None, 1, None, 0, 0, None) == 1
    cu = np.array([0, 5, 3], np.int32)
    assert lib.st_plan_create(C.byref(handle), fake, fake, fake, cu.ctypes.data, 2, None, 0, 0, None) == 3   # decreasing
    cu = np.array([1, 5], np.int32)
    assert lib.st_plan_create(C.byref(handle), fake, fake, fake, cu.ctypes.data, 1, None, 0, 0, None) == 3
    assert lib.st_plan_workspace_bytes(4, 16000) > 3 * 4 * 16000
    assert lib.st_attn_prefill(fake, None, fake, fake, fake, None, 4, 2, 64, 0.0, B.ST_BF16, None, 0, None) == 1
    lib.st_plan_destroy(None)   # ignored


def test_cache_argument_checks(lib):
    import paper_2510_17238_amd.binding as B
    fake = 0x1000

    def cache(**kw):
        base = dict(k_pool=fake, v_pool=fake, page_table=fake, appended_len=fake, max_pages_per_seq=4, n_pages=16,
                    page_size=16, n_kv_heads=2, head_dim=128, dtype=B.ST_BF16)
        base.update(kw)
        return B._KVCacheStruct(**base)

    good = B._DualCacheStruct(cache(), cache())
    fp = C.c_void_p(fake)
    # capacity: 4 pages x 16 tokens
    assert lib.st_kv_append(C.byref(good), B.ST_SOURCE, fp, fp, None, 8, 1, 65, None) == 4
    assert lib.st_kv_append(C.byref(good), 7, fp, fp, None, 8, 1, 64, None) == 1
    bad = B._DualCacheStruct(cache(page_size=32), cache())
    assert lib.st_kv_append(C.byref(bad), B.ST_SOURCE, fp, fp, None, 8, 1, 64, None) == 5
    bad = B._DualCacheStruct(cache(), cache(dtype=B.ST_F32))
    assert lib.st_kv_append(C.byref(bad), B.ST_REASONING, fp, fp, None, 8, 1, 64, None) == 5
    lens = B._DualLensStruct(fake, fake, 9, 64, 64)
    # q_len 9 x group 4 > 32 rows
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 5
    lens = B._DualLensStruct(fake, fake, 1, 64, 65)
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 4
    lens = B._DualLensStruct(fake, fake, 1, 64, 64)
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, C.c_void_p(0x1100), 16, None) == 4
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 7, 0.0, fp, 1 << 20, None) == 2
    need = lib.st_decode_workspace_bytes(1, 8, 2, 128, 1, 64, 64)
    assert need >= 2 * 4 * (128 + 2) * 4
    # the fused forms take the same checks, plus the rotation base
    assert lib.st_kv_append_rope(C.byref(good), B.ST_SOURCE, fp, fp, None, 8, 1, 65, 1.0e6, None) == 4
    assert lib.st_kv_append_rope(C.byref(good), B.ST_SOURCE, fp, fp, None, 8, 1, 64, 0.0, None) == 1
    assert b"theta" in lib.st_last_error() and b"st_kv_append_rope" in lib.st_last_error()
    assert lib.st_attn_decode_dual_rope(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, -2.0, fp, 1 << 20, None) == 1
    assert lib.st_attn_decode_dual_rope(fp, None, fp, C.byref(good), C.byref(lens), 1, 7, 0.0, 1.0e6, fp, 1 << 20, None) == 2
    assert lib.st_attn_source_chunk_rope(fp, None, fp, C.byref(good), fp, None, 8, 64, 1, 8, 0.0, 0.0, fp, 1 << 20, None) == 1
    assert lib.st_attn_source_chunk_rope(fp, None, fp, C.byref(good), fp, None, 8, 65, 1, 8, 0.0, 1.0e6, fp, 1 << 20, None) == 4
