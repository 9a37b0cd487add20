"""ctypes binding of include/st.h.  Function names and argument order follow the header."""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))

ST_OK = 0
ST_F32, ST_BF16, ST_FP8_E4M3 = 0, 1, 2
ST_SOURCE, ST_REASONING = 0, 1
ST_TILE_SKIP, ST_TILE_FULL, ST_TILE_PARTIAL = 0, 1, 2
ST_BLOCK_SS, ST_BLOCK_RS, ST_BLOCK_RR = 0, 1, 2
PAGE = 16

_STATUS_NAMES = {1: "ST_ERR_INVALID_ARG", 2: "ST_ERR_SHAPE", 3: "ST_ERR_LAYOUT", 4: "ST_ERR_CAPACITY",
                 5: "ST_ERR_UNSUPPORTED", 6: "ST_ERR_RUNTIME"}


class StError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class _KVCacheStruct(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("page_table", C.c_void_p),
                ("appended_len", C.c_void_p), ("max_pages_per_seq", C.c_int32), ("n_pages", C.c_int32),
                ("page_size", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("k_scale", C.c_void_p), ("v_scale", C.c_void_p)]


class _DualCacheStruct(C.Structure):
    _fields_ = [("source", _KVCacheStruct), ("reasoning", _KVCacheStruct)]


class _StreamJobStruct(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_sentences", C.c_int32),
                ("caches", C.c_void_p), ("src_tokens", C.c_void_p), ("rsn_tokens", C.c_void_p), ("arrival_s", C.c_void_p),
                ("src_q", C.c_void_p), ("src_k", C.c_void_p), ("src_v", C.c_void_p), ("src_out", C.c_void_p),
                ("rsn_q", C.c_void_p), ("rsn_k", C.c_void_p), ("rsn_v", C.c_void_p), ("rsn_out", C.c_void_p),
                ("scale", C.c_float), ("theta_base", C.c_double),
                ("prefill_workspace", C.c_void_p), ("prefill_workspace_bytes", C.c_size_t),
                ("decode_workspace", C.c_void_p), ("decode_workspace_bytes", C.c_size_t),
                ("prefill_stream", C.c_void_p), ("decode_stream", C.c_void_p), ("decode_graph", C.c_int32)]


class _StreamReportStruct(C.Structure):
    _fields_ = [("prefill_done_s", C.c_void_p), ("first_token_s", C.c_void_p), ("unit_done_s", C.c_void_p),
                ("waited", C.c_void_p), ("sliced", C.c_void_p), ("total_s", C.c_double)]


class _DualLensStruct(C.Structure):
    _fields_ = [("src_visible_len", C.c_void_p), ("rsn_len", C.c_void_p), ("q_len", C.c_int32),
                ("max_src_len", C.c_int32), ("max_rsn_len", C.c_int32), ("unit_tokens", C.c_int32)]


_lib = None


def library_path():
    return os.path.join(HERE, "libst.so")


def load_library():
    """Load libst.so; raise if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2510_17238_amd.build` "
                           "(or __graft_entry__.build()); the HIP library is the only implementation")
    lib = C.CDLL(path)
    vp, i32, i64, f32, f64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_double, C.c_size_t
    lib.st_last_error.restype = C.c_char_p
    lib.st_last_error.argtypes = []
    lib.st_version.restype = i32
    lib.st_version.argtypes = []
    lib.st_plan_heads_per_workgroup.restype = i32
    lib.st_plan_heads_per_workgroup.argtypes = [vp, i32]
    lib.st_profile_enable.restype = None
    lib.st_profile_enable.argtypes = [i32]
    lib.st_profile_repeat.restype = i32
    lib.st_profile_repeat.argtypes = [i32]
    lib.st_profile_wave_trace.restype = i32
    lib.st_profile_wave_trace.argtypes = [vp, i32]
    lib.st_profile_read.restype = i32
    lib.st_profile_read.argtypes = [i32, C.POINTER(f64), C.POINTER(i32)]
    lib.st_rope_apply.restype = i32
    lib.st_rope_apply.argtypes = [vp, vp, vp, i64, i32, i32, f64, i32, vp]
    lib.st_rope_apply_qk.restype = i32
    lib.st_rope_apply_qk.argtypes = [vp, vp, i32, vp, vp, i32, vp, i64, i32, f64, i32, vp]
    lib.st_plan_workspace_bytes.restype = sz
    lib.st_plan_workspace_bytes.argtypes = [i32, i64]
    lib.st_plan_create.restype = i32
    lib.st_plan_create.argtypes = [C.POINTER(vp), vp, vp, vp, vp, i32, vp, sz, i32, vp]
    lib.st_plan_destroy.restype = None
    lib.st_plan_destroy.argtypes = [vp]
    lib.st_plan_tile_shape.restype = i32
    lib.st_plan_tile_shape.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    for name in ("st_plan_compact_index", "st_plan_visible_source", "st_plan_visible_pairs"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp, vp]
    lib.st_plan_stream_counts.restype = i32
    lib.st_plan_stream_counts.argtypes = [vp, vp, vp]
    lib.st_plan_tile_classes.restype = i32
    lib.st_plan_tile_classes.argtypes = [vp, i32, i32, vp, C.POINTER(i32), C.POINTER(i32)]
    lib.st_attn_prefill.restype = i32
    lib.st_attn_prefill.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.st_attn_prefill_rope.restype = i32
    lib.st_attn_prefill_rope.argtypes = [vp, vp, vp, vp, vp, vp, f64, vp, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.st_prefill_workspace_bytes.restype = sz
    lib.st_prefill_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.st_attn_prefill_ids.restype = i32
    lib.st_attn_prefill_ids.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, vp]
    lib.st_prefill_bwd_workspace_bytes.restype = sz
    lib.st_prefill_bwd_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.st_attn_prefill_bwd.restype = i32
    lib.st_attn_prefill_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.st_kv_append.restype = i32
    lib.st_kv_append.argtypes = [C.POINTER(_DualCacheStruct), i32, vp, vp, vp, i32, i32, i32, vp]
    lib.st_kv_append_rope.restype = i32
    lib.st_kv_append_rope.argtypes = [C.POINTER(_DualCacheStruct), i32, vp, vp, vp, i32, i32, i32, C.c_double, vp]
    lib.st_attn_decode_dual_rope.restype = i32
    lib.st_attn_decode_dual_rope.argtypes = [vp, vp, vp, C.POINTER(_DualCacheStruct), C.POINTER(_DualLensStruct), i32, i32,
                                             f32, C.c_double, vp, sz, vp]
    lib.st_attn_decode_dual_append.restype = i32
    lib.st_attn_decode_dual_append.argtypes = [vp, vp, vp, vp, vp, C.POINTER(_DualCacheStruct), C.POINTER(_DualLensStruct), i32, i32,
                                               f32, f64, vp, sz, vp]
    lib.st_decode_workspace_bytes.restype = sz
    lib.st_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32, i32]
    lib.st_attn_decode_dual.restype = i32
    lib.st_attn_decode_dual.argtypes = [vp, vp, vp, C.POINTER(_DualCacheStruct), C.POINTER(_DualLensStruct), i32, i32,
                                        f32, vp, sz, vp]
    lib.st_decode_static_scratch_bytes.restype = sz
    lib.st_decode_static_scratch_bytes.argtypes = []
    lib.st_attn_decode_dual_static.restype = i32
    lib.st_attn_decode_dual_static.argtypes = [vp, vp, vp, C.POINTER(_DualCacheStruct), C.POINTER(_DualLensStruct), i32, i32, f32, vp]
    lib.st_source_chunk_workspace_bytes.restype = sz
    lib.st_source_chunk_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.st_attn_source_chunk.restype = i32
    lib.st_attn_source_chunk.argtypes = [vp, vp, vp, C.POINTER(_DualCacheStruct), vp, vp, i32, i32, i32, i32, f32, vp, sz, vp]
    lib.st_attn_source_chunk_rope.restype = i32
    lib.st_attn_source_chunk_rope.argtypes = [vp, vp, vp, C.POINTER(_DualCacheStruct), vp, vp, i32, i32, i32, i32, f32, C.c_double,
                                              vp, sz, vp]
    lib.st_stream_run.restype = i32
    lib.st_stream_run.argtypes = [C.POINTER(_StreamJobStruct), i32, C.POINTER(_StreamReportStruct)]
    lib.st_stream_timeline.restype = i32
    lib.st_stream_timeline.argtypes = [i32, i32, vp, vp, vp, C.c_double, vp, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


def _check(status):
    if status != ST_OK:
        raise StError(status, load_library().st_last_error().decode())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return ST_F32
    if t.dtype == torch.bfloat16:
        return ST_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _temp_workspace(n_bytes, device, stream):
    """A workspace that lives only for one call: allocated ON the stream the kernels are launched on, so that the
    caching allocator does not hand the block to somebody else while they still run."""
    if stream is None or stream == torch.cuda.current_stream():
        return torch.empty(max(int(n_bytes), 256), dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(max(int(n_bytes), 256), dtype=torch.uint8, device=device)


def _dev_i32(t, name):
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int32 device tensor")
    return t


def st_version():
    return int(load_library().st_version())


def st_last_error():
    return load_library().st_last_error().decode()


ST_PROF_PREFILL_ATTN, ST_PROF_DECODE_SPLIT, ST_PROF_BWD_DQ, ST_PROF_BWD_DKV, ST_PROF_TILE_PACK, ST_PROF_SOURCE_CHUNK = 0, 1, 2, 3, 4, 5


_probe_lib = None


def load_probe_library():
    """libst_probe.so: the benchmark's machine probes (include/st_probe.h), not part of the path."""
    global _probe_lib
    if _probe_lib is None:
        path = os.path.join(HERE, "libst_probe.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2510_17238_amd.build`")
        lib = C.CDLL(path)
        lib.st_probe_paged_read.restype = C.c_int32
        lib.st_probe_paged_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_uint32, C.c_void_p, C.c_void_p]
        lib.st_probe_mfma_bf16.restype = C.c_int32
        lib.st_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        _probe_lib = lib
    return _probe_lib


def st_probe_paged_read(pool, n_waves, steps_per_wave, salt, sink, stream=None):
    """pool: uint8 device tensor whose size is a power of two; sink: uint32-sized device tensor."""
    rc = load_probe_library().st_probe_paged_read(_ptr(pool), pool.numel() * pool.element_size(), int(n_waves), int(steps_per_wave),
                                                  int(salt) & 0xFFFFFFFF, _ptr(sink), _stream(stream))
    if rc != ST_OK:
        raise StError(rc, "st_probe_paged_read")


def st_probe_mfma_bf16(n_workgroups, iterations, sink, stream=None):
    rc = load_probe_library().st_probe_mfma_bf16(int(n_workgroups), int(iterations), _ptr(sink), _stream(stream))
    if rc != ST_OK:
        raise StError(rc, "st_probe_mfma_bf16")


def st_profile_enable(on):
    load_library().st_profile_enable(1 if on else 0)


def st_profile_repeat(launches):
    _check(load_library().st_profile_repeat(int(launches)))


def st_profile_wave_trace(buffer):
    """buffer: int64 / uint64 device tensor of 2 n entries (n (start, end) pairs), or None to switch the timeline off."""
    if buffer is None:
        _check(load_library().st_profile_wave_trace(None, 0))
        return
    assert buffer.is_cuda and buffer.is_contiguous() and buffer.element_size() == 8
    _check(load_library().st_profile_wave_trace(_ptr(buffer), buffer.numel() // 2))


def st_profile_read(which):
    """(mean milliseconds, count) of the kernel launches recorded since the last read."""
    ms, n = C.c_double(), C.c_int32()
    _check(load_library().st_profile_read(which, C.byref(ms), C.byref(n)))
    return ms.value, n.value


# ------------------------------------------------------------------ RoPE --
def st_rope_apply(x, positions, theta_base=1.0e6, out=None, stream=None):
    """x[n_tokens, n_heads, head_dim] rotated by positions[n_tokens]; out defaults to in place."""
    lib = load_library()
    assert x.is_cuda and x.is_contiguous() and x.dim() == 3
    _dev_i32(positions, "positions")
    if out is None:
        out = x
    assert out.shape == x.shape and out.dtype == x.dtype and out.is_contiguous()
    n, h, d = x.shape
    _check(lib.st_rope_apply(_ptr(out), _ptr(x), _ptr(positions), n, h, d, float(theta_base), _dtype_code(x), _stream(stream)))
    return out


def st_rope_apply_qk(q, k, positions, theta_base=1.0e6, q_out=None, k_out=None, stream=None):
    """q[n_tokens, Hq, D] and k[n_tokens, Hkv, D] rotated by positions[n_tokens] in one launch; outs default to in place."""
    lib = load_library()
    assert q.is_cuda and q.is_contiguous() and q.dim() == 3 and k.is_contiguous() and k.dim() == 3 and k.dtype == q.dtype
    _dev_i32(positions, "positions")
    q_out = q if q_out is None else q_out
    k_out = k if k_out is None else k_out
    assert q_out.shape == q.shape and q_out.dtype == q.dtype and q_out.is_contiguous()
    assert k_out.shape == k.shape and k_out.dtype == k.dtype and k_out.is_contiguous()
    n, hq, d = q.shape
    assert k.shape[0] == n and k.shape[2] == d
    _check(lib.st_rope_apply_qk(_ptr(q_out), _ptr(q), hq, _ptr(k_out), _ptr(k), k.shape[1], _ptr(positions), n, d, float(theta_base),
                                _dtype_code(q), _stream(stream)))
    return q_out, k_out


# ------------------------------------------------------------------ plan --
def st_plan_workspace_bytes(batch, n_tokens):
    return int(load_library().st_plan_workspace_bytes(batch, n_tokens))


class Plan:
    """Owner of one st_plan handle."""

    def __init__(self, handle, batch, n_tokens, cu_seqlens, keep):
        self.handle = handle
        self.batch = batch
        self.n_tokens = n_tokens
        self.cu_seqlens = cu_seqlens
        self._keep = keep   # tensors the plan's kernels read / its workspace

    def destroy(self):
        if self.handle:
            load_library().st_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def heads_per_workgroup(self, heads):
        """0 = by problem size, 1 or 2 query heads of a KV head per workgroup of the bf16 attention kernel."""
        _check(load_library().st_plan_heads_per_workgroup(self.handle, int(heads)))
        return self

    def tile_shape(self):
        m, n = C.c_int32(), C.c_int32()
        _check(load_library().st_plan_tile_shape(self.handle, C.byref(m), C.byref(n)))
        return m.value, n.value

    def stream_counts(self):
        a = np.zeros(self.batch, np.int32); b = np.zeros(self.batch, np.int32)
        _check(load_library().st_plan_stream_counts(self.handle, a.ctypes.data, b.ctypes.data))
        return a, b

    def compact_index(self):
        a = np.zeros(self.n_tokens, np.int32)
        _check(load_library().st_plan_compact_index(self.handle, a.ctypes.data))
        return a

    def visible_source(self):
        a = np.zeros(self.n_tokens, np.int32)
        _check(load_library().st_plan_visible_source(self.handle, a.ctypes.data))
        return a

    def visible_pairs(self):
        a = np.zeros(self.batch, np.uint64)
        _check(load_library().st_plan_visible_pairs(self.handle, a.ctypes.data))
        return a

    def tile_classes(self, seq, block):
        tq, tk = C.c_int32(), C.c_int32()
        lib = load_library()
        _check(lib.st_plan_tile_classes(self.handle, seq, block, None, C.byref(tq), C.byref(tk)))
        out = np.zeros((tq.value, tk.value), np.uint8)
        if out.size:
            _check(lib.st_plan_tile_classes(self.handle, seq, block, out.ctypes.data, C.byref(tq), C.byref(tk)))
        return out


def st_plan_create(segment_ids, stream_ids, positions, cu_seqlens, workspace=None, validate=False, stream=None):
    """cu_seqlens: host sequence (list / numpy) of batch + 1 offsets.  Returns a Plan."""
    lib = load_library()
    for t, name in ((segment_ids, "segment_ids"), (stream_ids, "stream_ids"), (positions, "positions")):
        _dev_i32(t, name)
    cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
    batch = len(cu) - 1
    n_tokens = int(cu[-1]) if batch >= 0 and len(cu) else 0
    if not (segment_ids.numel() == stream_ids.numel() == positions.numel() == n_tokens):
        raise ValueError("metadata arrays must have cu_seqlens[-1] entries")
    handle = C.c_void_p()
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = _ptr(workspace), workspace.numel() * workspace.element_size()
    _check(lib.st_plan_create(C.byref(handle), _ptr(segment_ids), _ptr(stream_ids), _ptr(positions), cu.ctypes.data,
                              batch, ws_ptr, ws_bytes, 1 if validate else 0, _stream(stream)))
    return Plan(handle, batch, n_tokens, cu, (segment_ids, stream_ids, positions, workspace))


# --------------------------------------------------------------- prefill --
def st_prefill_workspace_bytes(plan, n_kv_heads, head_dim, dtype_code):
    return int(load_library().st_prefill_workspace_bytes(plan.handle, n_kv_heads, head_dim, dtype_code))


def st_attn_prefill(q, k, v, plan, scale=0.0, out=None, lse=None, workspace=None, stream=None, positions=None, rope_theta=None):
    """q[N, Hq, D], k, v[N, Hkv, D] -> out[N, Hq, D]; lse: fp32 [N, Hq] tensor to fill, or None.
    rope_theta: None for st_attn_prefill (rotated q, k); a base (with positions) for st_attn_prefill_rope."""
    lib = load_library()
    assert q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    assert q.dtype == k.dtype == v.dtype
    n, hq, d = q.shape
    assert k.shape == v.shape and k.shape[0] == n and k.shape[2] == d and n == plan.n_tokens
    hkv = k.shape[1]
    if out is None:
        out = torch.empty_like(q)
    if lse is not None:
        assert lse.dtype == torch.float32 and lse.shape == (n, hq) and lse.is_contiguous()
    ws_bytes = 0
    if workspace is None:
        need = st_prefill_workspace_bytes(plan, hkv, d, _dtype_code(q))
        if need:
            workspace = _temp_workspace(need, q.device, stream)
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    if rope_theta is None:
        _check(lib.st_attn_prefill(_ptr(out), _ptr(lse), _ptr(q), _ptr(k), _ptr(v), plan.handle, hq, hkv, d, float(scale),
                                   _dtype_code(q), _ptr(workspace), ws_bytes, _stream(stream)))
    else:
        _dev_i32(positions, "positions")
        assert positions.numel() == n
        _check(lib.st_attn_prefill_rope(_ptr(out), _ptr(lse), _ptr(q), _ptr(k), _ptr(v), _ptr(positions), float(rope_theta), plan.handle,
                                        hq, hkv, d, float(scale), _dtype_code(q), _ptr(workspace), ws_bytes, _stream(stream)))
    return out


def st_attn_prefill_rope(q, k, v, positions, theta_base, plan, **kw):
    """st_attn_prefill for UNROTATED q, k (rotated inside by positions[token], base theta_base); bf16 only."""
    return st_attn_prefill(q, k, v, plan, positions=positions, rope_theta=theta_base, **kw)


def st_attn_prefill_bwd(d_out, q, k, v, out, lse, plan, scale=0.0, workspace=None, stream=None):
    """Gradients (dq, dk, dv) of st_attn_prefill; `out` and `lse` are the forward's results."""
    lib = load_library()
    for t in (d_out, q, k, v, out):
        assert t.is_cuda and t.is_contiguous() and t.dtype == q.dtype and t.dim() == 3
    assert lse.dtype == torch.float32 and lse.is_contiguous()
    n, hq, d = q.shape
    hkv = k.shape[1]
    assert d_out.shape == q.shape == out.shape and k.shape == v.shape and tuple(lse.shape) == (n, hq)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    if workspace is None:
        workspace = _temp_workspace(int(lib.st_prefill_bwd_workspace_bytes(plan.handle, hq, hkv, d, _dtype_code(q))), q.device, stream)
    _check(lib.st_attn_prefill_bwd(_ptr(dq), _ptr(dk), _ptr(dv), _ptr(d_out), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                   plan.handle, hq, hkv, d, float(scale), _dtype_code(q), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)))
    return dq, dk, dv


def st_attn_prefill_ids(q, k, v, segment_ids, stream_ids, positions, cu_seqlens, scale=0.0, out=None, lse=None, stream=None):
    """One-off form taking the token metadata directly (builds and frees a plan; waits)."""
    lib = load_library()
    cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
    n, hq, d = q.shape
    hkv = k.shape[1]
    if out is None:
        out = torch.empty_like(q)
    _check(lib.st_attn_prefill_ids(_ptr(out), _ptr(lse), _ptr(q), _ptr(k), _ptr(v), _ptr(_dev_i32(segment_ids, "segment_ids")),
                                   _ptr(_dev_i32(stream_ids, "stream_ids")), _ptr(_dev_i32(positions, "positions")),
                                   cu.ctypes.data, len(cu) - 1, hq, hkv, d, float(scale), _dtype_code(q), _stream(stream)))
    return out


# ------------------------------------------------------------ KV caches --
class KVCache:
    """Caller-owned paged cache: pools, page table and length vector are torch tensors."""

    def __init__(self, n_pages, batch, max_pages_per_seq, n_kv_heads, head_dim, page_table, device="cuda", fill=None, fp8=False):
        self.n_pages, self.batch, self.max_pages_per_seq = n_pages, batch, max_pages_per_seq
        self.n_kv_heads, self.head_dim = n_kv_heads, head_dim
        self.fp8 = bool(fp8)
        shape_k = (n_pages, n_kv_heads, head_dim // 8, PAGE, 8)
        shape_v = (n_pages, n_kv_heads, head_dim, PAGE)
        self.k_scale = self.v_scale = None
        if self.fp8:
            # E4M3 codes as bytes; `fill` (a byte) pre-sets pools, and scales get NaN, to show what is never read
            self.k_pool = torch.full((n_pages, n_kv_heads, head_dim // 16, PAGE, 16), 0 if fill is None else int(fill), dtype=torch.uint8, device=device)
            self.v_pool = torch.full(shape_v, 0 if fill is None else int(fill), dtype=torch.uint8, device=device)
            self.k_scale = torch.full((n_pages, n_kv_heads, PAGE), float("nan") if fill is not None else 0.0, dtype=torch.float32, device=device)
            self.v_scale = self.k_scale.clone()
        elif fill is None:
            self.k_pool = torch.empty(shape_k, dtype=torch.bfloat16, device=device)
            self.v_pool = torch.empty(shape_v, dtype=torch.bfloat16, device=device)
        else:
            self.k_pool = torch.full(shape_k, fill, dtype=torch.bfloat16, device=device)
            self.v_pool = torch.full(shape_v, fill, dtype=torch.bfloat16, device=device)
        self.page_table = _dev_i32(page_table, "page_table")
        assert tuple(page_table.shape) == (batch, max_pages_per_seq)
        self.appended_len = torch.zeros(batch, dtype=torch.int32, device=device)

    def struct(self):
        return _KVCacheStruct(self.k_pool.data_ptr(), self.v_pool.data_ptr(), self.page_table.data_ptr(),
                              self.appended_len.data_ptr(), self.max_pages_per_seq, self.n_pages, PAGE,
                              self.n_kv_heads, self.head_dim, ST_FP8_E4M3 if self.fp8 else ST_BF16,
                              self.k_scale.data_ptr() if self.fp8 else None, self.v_scale.data_ptr() if self.fp8 else None)


class DualCache:
    """The source cache and the reasoning cache of one layer."""

    def __init__(self, source, reasoning):
        self.source, self.reasoning = source, reasoning
        self._struct = None

    def struct(self):
        # built once: the tensors behind a cache are fixed after construction (call refresh() otherwise)
        if self._struct is None:
            self._struct = _DualCacheStruct(self.source.struct(), self.reasoning.struct())
        return self._struct

    def refresh(self):
        self._struct = None


def k_pool_to_logical(k_pool):
    """[n_pages, Hkv, D/8, 16, 8] -> [n_pages, 16, Hkv, D] (a pure permutation of the pool)."""
    p, h, c, s, e = k_pool.shape
    return k_pool.permute(0, 3, 1, 2, 4).reshape(p, s, h, c * e)


def v_pool_to_logical(v_pool):
    """[n_pages, Hkv, D, 16] -> [n_pages, 16, Hkv, D]."""
    return v_pool.permute(0, 3, 1, 2)


def k_pool8_to_logical(k_pool):
    """8-bit key pool [n_pages, Hkv, D/16, 16, 16] -> [n_pages, 16, Hkv, D] (bytes)."""
    p, h, c, s, e = k_pool.shape
    return k_pool.permute(0, 3, 1, 2, 4).reshape(p, s, h, c * e)


def scale_to_logical(scale):
    """[n_pages, Hkv, 16] -> [n_pages, 16, Hkv]."""
    return scale.permute(0, 2, 1)


def k_pool_from_logical(x):
    """[n_pages, 16, Hkv, D] -> pool layout [n_pages, Hkv, D/8, 16, 8]."""
    p, s, h, d = x.shape
    return x.reshape(p, s, h, d // 8, 8).permute(0, 2, 3, 1, 4).contiguous()


def v_pool_from_logical(x):
    return x.permute(0, 2, 3, 1).contiguous()


def st_kv_append(caches, which, k_new, v_new, n_new=None, host_len_upper_bound=None, stream=None, rope_theta=None):
    """k_new, v_new: bf16 [batch, max_new, Hkv, D]; n_new: int32 [batch] device tensor or None.
    rope_theta: None for st_kv_append (keys already rotated), a base for st_kv_append_rope (unrotated keys)."""
    lib = load_library()
    assert k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    batch, max_new = k_new.shape[0], k_new.shape[1]
    cache = caches.source if which == ST_SOURCE else caches.reasoning
    if host_len_upper_bound is None:
        host_len_upper_bound = cache.max_pages_per_seq * PAGE
    if n_new is not None:
        _dev_i32(n_new, "n_new")
    st = caches.struct()
    if rope_theta is None:
        _check(lib.st_kv_append(C.byref(st), which, _ptr(k_new), _ptr(v_new), _ptr(n_new), max_new, batch,
                                int(host_len_upper_bound), _stream(stream)))
    else:
        _check(lib.st_kv_append_rope(C.byref(st), which, _ptr(k_new), _ptr(v_new), _ptr(n_new), max_new, batch,
                                     int(host_len_upper_bound), float(rope_theta), _stream(stream)))


def st_kv_append_rope(caches, which, k_new, v_new, theta_base, n_new=None, host_len_upper_bound=None, stream=None):
    """st_kv_append for UNROTATED keys: each key is rotated by its index in the cache on the way in."""
    st_kv_append(caches, which, k_new, v_new, n_new, host_len_upper_bound, stream, rope_theta=theta_base)


def st_decode_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, q_len, max_src_len, max_rsn_len, unit_tokens=0):
    return int(load_library().st_decode_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, q_len, max_src_len, max_rsn_len,
                                                        int(unit_tokens)))


def st_attn_decode_dual(q, caches, src_visible_len, rsn_len, max_src_len, max_rsn_len, scale=0.0, out=None, lse=None,
                        workspace=None, stream=None, rope_theta=None, unit_tokens=0):
    """q[batch, q_len, Hq, D] bf16 -> out of the same shape; lengths are int32 device tensors.
    rope_theta: None for st_attn_decode_dual (rotated queries), a base for st_attn_decode_dual_rope."""
    lib = load_library()
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch.bfloat16 and q.dim() == 4
    batch, q_len, hq, d = q.shape
    _dev_i32(src_visible_len, "src_visible_len"); _dev_i32(rsn_len, "rsn_len")
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = st_decode_workspace_bytes(batch, hq, caches.source.n_kv_heads, d, q_len, max_src_len, max_rsn_len, unit_tokens)
        workspace = _temp_workspace(need, q.device, stream)
    st = caches.struct()
    lens = _DualLensStruct(src_visible_len.data_ptr(), rsn_len.data_ptr(), q_len, int(max_src_len), int(max_rsn_len), int(unit_tokens))
    if rope_theta is None:
        _check(lib.st_attn_decode_dual(_ptr(out), _ptr(lse), _ptr(q), C.byref(st), C.byref(lens), batch, hq, float(scale),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    else:
        _check(lib.st_attn_decode_dual_rope(_ptr(out), _ptr(lse), _ptr(q), C.byref(st), C.byref(lens), batch, hq, float(scale),
                                            float(rope_theta), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream)))
    return out


def st_decode_static_scratch_bytes():
    return int(load_library().st_decode_static_scratch_bytes())


def st_attn_decode_dual_static(q, caches, src_visible_len, rsn_len, max_src_len, max_rsn_len, out, lse=None, scale=0.0, stream=None):
    """st_attn_decode_dual without a workspace (the library's own device array); `out` is the caller's: nothing is
    allocated here either."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch.bfloat16 and q.dim() == 4
    assert out.shape == q.shape and out.dtype == q.dtype and out.is_contiguous()
    batch, q_len, hq, d = q.shape
    _dev_i32(src_visible_len, "src_visible_len"); _dev_i32(rsn_len, "rsn_len")
    st = caches.struct()
    lens = _DualLensStruct(src_visible_len.data_ptr(), rsn_len.data_ptr(), q_len, int(max_src_len), int(max_rsn_len), 0)
    _check(load_library().st_attn_decode_dual_static(_ptr(out), _ptr(lse), _ptr(q), C.byref(st), C.byref(lens), batch, hq, float(scale),
                                                     _stream(stream)))
    return out


def st_attn_decode_dual_rope(q, caches, src_visible_len, rsn_len, max_src_len, max_rsn_len, theta_base, **kw):
    """st_attn_decode_dual for UNROTATED queries (rotated in the kernel by their index in the reasoning stream)."""
    return st_attn_decode_dual(q, caches, src_visible_len, rsn_len, max_src_len, max_rsn_len, rope_theta=theta_base, **kw)


def st_attn_decode_dual_append(q, k_new, v_new, caches, src_visible_len, rsn_len, max_src_len, max_rsn_len, theta_base=0.0, scale=0.0,
                               out=None, lse=None, workspace=None, stream=None, unit_tokens=0):
    """One decoding step: k_new / v_new [batch, 1, Hkv, D] go into the reasoning cache at index rsn_len - 1 and
    q [batch, 1, Hq, D] attends over both caches.  theta_base > 0: q and k_new are unrotated; 0: already rotated."""
    lib = load_library()
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch.bfloat16 and q.dim() == 4
    batch, q_len, hq, d = q.shape
    hkv = caches.source.n_kv_heads
    for t in (k_new, v_new):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16 and tuple(t.shape) == (batch, 1, hkv, d)
    _dev_i32(src_visible_len, "src_visible_len"); _dev_i32(rsn_len, "rsn_len")
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = st_decode_workspace_bytes(batch, hq, hkv, d, q_len, max_src_len, max_rsn_len, unit_tokens)
        workspace = _temp_workspace(need, q.device, stream)
    st = caches.struct()
    lens = _DualLensStruct(src_visible_len.data_ptr(), rsn_len.data_ptr(), q_len, int(max_src_len), int(max_rsn_len), int(unit_tokens))
    _check(lib.st_attn_decode_dual_append(_ptr(out), _ptr(lse), _ptr(q), _ptr(k_new), _ptr(v_new), C.byref(st), C.byref(lens), batch, hq,
                                          float(scale), float(theta_base), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                          _stream(stream)))
    return out


def st_source_chunk_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, max_new, max_src_len):
    return int(load_library().st_source_chunk_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, max_new, max_src_len))


def st_attn_source_chunk(q, caches, src_len, max_src_len, n_new=None, scale=0.0, out=None, lse=None, workspace=None, stream=None,
                         rope_theta=None):
    """q[batch, max_new, Hq, D] bf16: the newest source tokens attend causally over the source cache.
    rope_theta: None for st_attn_source_chunk (rotated queries), a base for st_attn_source_chunk_rope."""
    lib = load_library()
    assert q.is_cuda and q.is_contiguous() and q.dtype == torch.bfloat16 and q.dim() == 4
    batch, max_new, hq, d = q.shape
    _dev_i32(src_len, "src_len")
    if n_new is not None:
        _dev_i32(n_new, "n_new")
    if out is None:
        out = torch.zeros_like(q)
    if workspace is None:
        need = st_source_chunk_workspace_bytes(batch, hq, caches.source.n_kv_heads, d, max_new, max_src_len)
        workspace = _temp_workspace(need, q.device, stream)
    st = caches.struct()
    if rope_theta is None:
        _check(lib.st_attn_source_chunk(_ptr(out), _ptr(lse), _ptr(q), C.byref(st), _ptr(src_len), _ptr(n_new), max_new,
                                        int(max_src_len), batch, hq, float(scale), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))
    else:
        _check(lib.st_attn_source_chunk_rope(_ptr(out), _ptr(lse), _ptr(q), C.byref(st), _ptr(src_len), _ptr(n_new), max_new,
                                             int(max_src_len), batch, hq, float(scale), float(rope_theta), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def st_attn_source_chunk_rope(q, caches, src_len, max_src_len, theta_base, **kw):
    """st_attn_source_chunk for UNROTATED queries (rotated in the kernel by their index in the source stream)."""
    return st_attn_source_chunk(q, caches, src_len, max_src_len, rope_theta=theta_base, **kw)


# ------------------------------------------------------- Alg. 1 scheduler --
ST_SCHED_STREAMING, ST_SCHED_SERIAL, ST_SCHED_BATCH = 0, 1, 2


def st_stream_timeline(mode, arrival_s, prefill_s, n_decode, decode_s):
    """Event times of a schedule for given stage durations (host model, no GPU): dict of numpy arrays."""
    import numpy as np
    a = np.ascontiguousarray(arrival_s, dtype=np.float64); p = np.ascontiguousarray(prefill_s, dtype=np.float64)
    n = np.ascontiguousarray(n_decode, dtype=np.int32)
    k = len(a)
    assert len(p) == k and len(n) == k
    out = {name: np.zeros(k, np.float64) for name in ("prefill_done", "unit_start", "first_token", "unit_done")}
    flags = {name: np.zeros(k, np.int32) for name in ("waited", "sliced")}
    ptr = lambda x: x.ctypes.data if k else None
    _check(load_library().st_stream_timeline(int(mode), k, ptr(a), ptr(p), ptr(n), float(decode_s), ptr(out["prefill_done"]),
                                             ptr(out["unit_start"]), ptr(out["first_token"]), ptr(out["unit_done"]),
                                             ptr(flags["waited"]), ptr(flags["sliced"])))
    out.update({name: v.astype(bool) for name, v in flags.items()})
    return out


def st_stream_run(mode, layers, n_q_heads, src_tokens, rsn_tokens, src_q, src_k, src_v, rsn_q, rsn_k, rsn_v, theta_base=1.0e6,
                  arrival_s=None, scale=0.0, prefill_stream=None, decode_stream=None, decode_graph=True):
    """Run one streaming session (Alg. 1) over `layers` (a list of DualCache, all empty).

    src_*: flat bf16 device tensors in the sentence-major layout of st.h, rsn_*: [steps, batch, heads, D].
    Returns (src_out, rsn_out, report dict).  Blocks until the session is over."""
    import numpy as np
    lib = load_library()
    src_tokens = np.ascontiguousarray(src_tokens, dtype=np.int32); rsn_tokens = np.ascontiguousarray(rsn_tokens, dtype=np.int32)
    k = len(src_tokens)
    assert len(rsn_tokens) == k and len(layers) > 0
    arr = None if arrival_s is None else np.ascontiguousarray(arrival_s, dtype=np.float64)
    batch = layers[0].source.batch
    hkv, d = layers[0].source.n_kv_heads, layers[0].source.head_dim
    for t in (src_q, src_k, src_v, rsn_q, rsn_k, rsn_v):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16
    total_src, steps = int(src_tokens.sum()), int(rsn_tokens.sum())
    assert src_q.numel() == total_src * batch * n_q_heads * d and src_k.numel() == total_src * batch * hkv * d == src_v.numel()
    assert rsn_q.numel() == steps * batch * n_q_heads * d and rsn_k.numel() == steps * batch * hkv * d == rsn_v.numel()
    src_out = torch.zeros_like(src_q); rsn_out = torch.zeros_like(rsn_q)
    dev = rsn_q.device
    pws = torch.empty(max(256, st_source_chunk_workspace_bytes(batch, n_q_heads, hkv, d, max(1, int(src_tokens.max(initial=0))),
                                                               total_src)), dtype=torch.uint8, device=dev)
    dws = torch.empty(max(256, st_decode_workspace_bytes(batch, n_q_heads, hkv, d, 1, total_src, steps)), dtype=torch.uint8, device=dev)
    if prefill_stream is None:
        prefill_stream = torch.cuda.Stream(device=dev)
    if decode_stream is None:
        decode_stream = torch.cuda.Stream(device=dev)
    cache_arr = (_DualCacheStruct * len(layers))(*[c.struct() for c in layers])
    rep = {name: np.zeros(k, np.float64) for name in ("prefill_done", "first_token", "unit_done")}
    flags = {name: np.zeros(k, np.int32) for name in ("waited", "sliced")}
    ptr = lambda x: x.ctypes.data if (x is not None and len(x)) else None
    dp = lambda t: t.data_ptr()
    job = _StreamJobStruct(len(layers), batch, n_q_heads, k, C.addressof(cache_arr), ptr(src_tokens), ptr(rsn_tokens), ptr(arr),
                           dp(src_q), dp(src_k), dp(src_v), dp(src_out), dp(rsn_q), dp(rsn_k), dp(rsn_v), dp(rsn_out),
                           float(scale), float(theta_base), dp(pws), pws.numel(), dp(dws), dws.numel(),
                           prefill_stream.cuda_stream, decode_stream.cuda_stream, 1 if decode_graph else 0)
    report = _StreamReportStruct(ptr(rep["prefill_done"]), ptr(rep["first_token"]), ptr(rep["unit_done"]), ptr(flags["waited"]),
                                 ptr(flags["sliced"]), 0.0)
    torch.cuda.synchronize(dev)
    _check(lib.st_stream_run(C.byref(job), int(mode), C.byref(report)))
    rep.update({name: v.astype(bool) for name, v in flags.items()})
    rep["total_s"] = report.total_s
    return src_out, rsn_out, rep
