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


def _declared_functions(header="st.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"st_rope_apply", "st_attn_prefill", "st_kv_append", "st_attn_decode_dual", "st_plan_create"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_probe_library_exports_its_header(lib):
    """The machine probes of the benchmark live in a library of their own; libst.so does not carry them."""
    import paper_2510_17238_amd as st
    probe = st.load_probe_library()
    names = _declared_functions("st_probe.h")
    assert names == ["st_probe_mfma_bf16", "st_probe_paged_read"]
    for name in names:
        assert hasattr(probe, name), name
        assert not hasattr(lib, name), name
    assert probe.st_probe_mfma_bf16(0, 1, None, None) == 1 and probe.st_probe_paged_read(None, 4096, 1, 1, 0, None, None) == 1


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
    assert lib.st_rope_apply_qk(fake, fake, 4, None, fake, 2, fake, 10, 64, 1.0e6, B.ST_BF16, None) == 1
    assert b"st_rope_apply_qk" in lib.st_last_error()
    assert lib.st_rope_apply_qk(fake, fake, 4, fake, fake, 2, fake, 10, 96, 1.0e6, B.ST_BF16, None) == 5
    assert lib.st_attn_prefill(fake, None, fake, fake, fake, None, 4, 2, 64, 0.0, B.ST_BF16, None, 0, None) == 1
    # the fused-rotation form: positions and a positive base are required, bf16 only
    assert lib.st_attn_prefill_rope(fake, None, fake, fake, fake, None, 1.0e6, None, 4, 2, 64, 0.0, B.ST_BF16, None, 0, None) == 1
    assert b"positions" in lib.st_last_error()
    assert lib.st_attn_prefill_rope(fake, None, fake, fake, fake, fake, 0.0, None, 4, 2, 64, 0.0, B.ST_BF16, None, 0, None) == 1
    assert b"theta" in lib.st_last_error()
    assert lib.st_attn_prefill_rope(fake, None, fake, fake, fake, fake, 1.0e6, None, 4, 2, 64, 0.0, B.ST_F32, None, 0, None) == 5
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
    lens = B._DualLensStruct(fake, fake, 9, 64, 64, 0)
    # q_len 9 x group 4 > 32 rows
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 5
    lens = B._DualLensStruct(fake, fake, 1, 64, 65, 0)
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 4
    lens = B._DualLensStruct(fake, fake, 1, 64, 64, 0)
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, C.c_void_p(0x1100), 16, None) == 4
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 7, 0.0, fp, 1 << 20, None) == 2
    need = lib.st_decode_workspace_bytes(1, 8, 2, 128, 1, 64, 64, 0)
    assert need >= 2 * 4 * (128 + 2) * 4
    # the work unit of the decode step is an argument: shorter units need more slots, a value that is no unit size gives 0
    # bytes (and ST_ERR_INVALID_ARG from the step), and the size by launch shrinks the unit for small launches
    w128 = lib.st_decode_workspace_bytes(32, 16, 8, 128, 1, 2048, 6144, 128)
    w1024 = lib.st_decode_workspace_bytes(32, 16, 8, 128, 1, 2048, 6144, 1024)
    auto_big = lib.st_decode_workspace_bytes(32, 16, 8, 128, 1, 2048, 6144, 0)
    auto_small = lib.st_decode_workspace_bytes(1, 16, 8, 128, 1, 2048, 6144, 0)
    # 512-token units are always provided for; 128-token units need about four times the slots
    assert w128 > 3 * w1024 and auto_big == w1024 and auto_small * 32 > 3 * auto_big
    assert lib.st_decode_workspace_bytes(32, 16, 8, 128, 1, 2048, 6144, 100) == 0
    lens = B._DualLensStruct(fake, fake, 1, 64, 64, 100)
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 1
    assert b"unit_tokens" in lib.st_last_error()
    # the fused forms take the same checks, plus the rotation base
    assert lib.st_kv_append_rope(C.byref(good), B.ST_SOURCE, fp, fp, None, 8, 1, 65, 1.0e6, None) == 4
    assert lib.st_kv_append_rope(C.byref(good), B.ST_SOURCE, fp, fp, None, 8, 1, 64, 0.0, None) == 1
    assert b"theta" in lib.st_last_error() and b"st_kv_append_rope" in lib.st_last_error()
    assert lib.st_attn_decode_dual_rope(fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, -2.0, fp, 1 << 20, None) == 1
    assert lib.st_attn_decode_dual_rope(fp, None, fp, C.byref(good), C.byref(lens), 1, 7, 0.0, 1.0e6, fp, 1 << 20, None) == 2
    assert lib.st_attn_source_chunk_rope(fp, None, fp, C.byref(good), fp, None, 8, 64, 1, 8, 0.0, 0.0, fp, 1 << 20, None) == 1
    assert lib.st_attn_source_chunk_rope(fp, None, fp, C.byref(good), fp, None, 8, 65, 1, 8, 0.0, 1.0e6, fp, 1 << 20, None) == 4
    # the whole decoding step in one call: one token, bf16 caches, a rotation base that is positive or 0
    ap = lib.st_attn_decode_dual_append
    assert ap(fp, None, fp, fp, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, -1.0, fp, 1 << 20, None) == 1
    assert ap(fp, None, fp, None, fp, C.byref(good), C.byref(lens), 1, 8, 0.0, 1.0e6, fp, 1 << 20, None) == 1
    assert b"st_attn_decode_dual_append" in lib.st_last_error()
    assert ap(fp, None, fp, fp, fp, C.byref(good), C.byref(lens), 1, 7, 0.0, 0.0, fp, 1 << 20, None) == 2
    two = B._DualLensStruct(fake, fake, 2, 64, 64, 0)
    assert ap(fp, None, fp, fp, fp, C.byref(good), C.byref(two), 1, 8, 0.0, 1.0e6, fp, 1 << 20, None) == 5
    # 8-bit caches: need their scale arrays; append (unfused) and decode up to 16 rows take them, nothing else does
    c8 = lambda **kw: cache(dtype=B.ST_FP8_E4M3, k_scale=fake, v_scale=fake, **kw)
    eight = B._DualCacheStruct(c8(), c8())
    assert lib.st_kv_append(C.byref(eight), B.ST_SOURCE, fp, fp, None, 8, 1, 65, None) == 4          # passes the dtype check
    assert ap(fp, None, fp, fp, fp, C.byref(eight), C.byref(lens), 1, 8, 0.0, 0.0, fp, 1 << 20, None) == 5
    assert lib.st_kv_append(C.byref(B._DualCacheStruct(cache(dtype=B.ST_FP8_E4M3), c8())), B.ST_SOURCE, fp, fp, None, 8, 1, 64, None) == 1
    assert b"scale" in lib.st_last_error()
    assert lib.st_kv_append_rope(C.byref(eight), B.ST_SOURCE, fp, fp, None, 8, 1, 64, 1.0e6, None) == 5
    assert lib.st_attn_source_chunk(fp, None, fp, C.byref(eight), fp, None, 8, 64, 1, 8, 0.0, fp, 1 << 20, None) == 5
    lens = B._DualLensStruct(fake, fake, 5, 64, 64, 0)                                                  # 5 x group 4 = 20 rows
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(eight), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 5
    assert b"16" in lib.st_last_error()
    lens = B._DualLensStruct(fake, fake, 1, 64, 64, 0)
    mixed = B._DualCacheStruct(c8(), cache())
    assert lib.st_attn_decode_dual(fp, None, fp, C.byref(mixed), C.byref(lens), 1, 8, 0.0, fp, 1 << 20, None) == 5


def test_stream_timeline_matches_oracle():
    """The scheduler's control logic (host model, no GPU) against the oracle's Alg. 1 timeline."""
    import paper_2510_17238_amd as st
    from oracle import streaming_attention as O
    rng = np.random.Generator(np.random.PCG64(1200))
    for trial in range(40):
        k = int(rng.integers(0, 9))
        arrival = np.cumsum(rng.uniform(0.0, 2.0, k)) * float(rng.integers(0, 2))       # sometimes everything at t = 0
        prefill = rng.uniform(0.0, 0.6, k)
        n_dec = rng.integers(0, 25, k)
        d = float(rng.uniform(0.0, 0.2))
        for mode, omode in ((st.ST_SCHED_STREAMING, O.STREAMING), (st.ST_SCHED_SERIAL, O.SERIAL), (st.ST_SCHED_BATCH, O.BATCH)):
            got = st.st_stream_timeline(mode, arrival, prefill, n_dec, d)
            want = O.alg1_timeline(arrival.tolist(), prefill.tolist(), n_dec.tolist(), d, omode)
            for name in ("prefill_done", "unit_start", "first_token", "unit_done"):
                assert np.allclose(got[name], np.asarray(want[name], dtype=np.float64), rtol=0, atol=1e-12), (trial, mode, name)
            for name in ("waited", "sliced"):
                assert got[name].tolist() == [bool(x) for x in want[name]], (trial, mode, name)
    # the worked example of the pins, through the library
    got = st.st_stream_timeline(st.ST_SCHED_STREAMING, [1.0, 2.0, 10.0], [1.0, 1.0, 1.0], [3, 2, 1], 1.0)
    assert got["unit_start"].tolist() == [2.0, 5.0, 11.0] and got["waited"].tolist() == [True, False, True]


def test_stream_argument_checks(lib):
    import paper_2510_17238_amd.binding as B
    a = np.array([1.0, 0.5]); p = np.array([0.1, 0.1]); n = np.array([1, 1], np.int32)
    assert lib.st_stream_timeline(0, 2, a.ctypes.data, p.ctypes.data, n.ctypes.data, 0.1, None, None, None, None, None, None) == 1   # decreasing
    a = np.array([0.5, 1.0])
    assert lib.st_stream_timeline(7, 2, a.ctypes.data, p.ctypes.data, n.ctypes.data, 0.1, None, None, None, None, None, None) == 1
    assert lib.st_stream_timeline(0, 2, a.ctypes.data, p.ctypes.data, n.ctypes.data, -1.0, None, None, None, None, None, None) == 1
    assert lib.st_stream_timeline(0, 2, a.ctypes.data, p.ctypes.data, n.ctypes.data, 0.1, None, None, None, None, None, None) == 0
    assert lib.st_stream_run(None, 0, None) == 1
    job = B._StreamJobStruct()
    rep = B._StreamReportStruct()
    assert lib.st_stream_run(C.byref(job), 5, C.byref(rep)) == 1
    assert lib.st_stream_run(C.byref(job), 0, C.byref(rep)) == 1 and b"sizes" in lib.st_last_error()


def test_bench_finds_its_traffic_figures_in_the_tracked_summary():
    """Every `traffic` key that bench.py asks for is a line of profiles/hbm_traffic_per_kernel.txt (so that no roofline
    object silently reports null), and the figures are plausible byte counts."""
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    src = open(os.path.join(root, "bench.py")).read()
    keys = set(re.findall(r'"([a-z0-9_]+@cfg[0-9a-z]+)"', src))
    keys |= {f"prefill_attn_kernel@{name}" for name in ("cfg4a", "cfg2")}
    assert len(keys) >= 8
    for key in sorted(keys):
        v = bench.measured_traffic(key)
        assert v is not None, f"no `traffic {key} ...` line in {bench.TRAFFIC_PROFILE}"
        assert 1e6 < v < 1e11
    assert bench.measured_traffic("no_such_kernel@cfg0") is None
