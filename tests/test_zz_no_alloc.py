"""The decode step for callers that cannot allocate (st_attn_decode_dual_static: partial results in a device array
of the library instead of a workspace) against st_attn_decode_dual on the same inputs -- same kernels, so the
outputs must agree bit for bit -- and against the fp64 oracle at the bf16 tolerance, on two calls in a row, the
second with a smaller input, so that whatever the first call left in the shared array is shown not to matter."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import streaming_attention as O
from gpu_helpers import DEV, make_cache, to_dev, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def st():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_17238_amd as st_
    st_.load_library()
    return st_


def _filled(st, rng, batch, hkv, d, src_lens, rsn_lens):
    """Both caches filled through st_kv_append; the oracle's contiguous copies beside them."""
    cs, _ = make_cache(batch, (int(src_lens.max()) + 15) // 16 + 1, hkv, d, rng, fill=float("nan"))
    cr, _ = make_cache(batch, (int(rsn_lens.max()) + 15) // 16 + 1, hkv, d, rng, fill=float("nan"))
    caches = st.DualCache(cs, cr)
    ref = {}
    for which, lens in ((st.ST_SOURCE, src_lens), (st.ST_REASONING, rsn_lens)):
        total = int(lens.max())
        kk = W.normal(rng, (batch, total, hkv, d), "bf16"); vv = W.normal(rng, (batch, total, hkv, d), "bf16")
        st.st_kv_append(caches, which, to_dev(kk, "bf16"), to_dev(vv, "bf16"), torch.from_numpy(lens.astype(np.int32)).to(DEV))
        ref[which] = (kk, vv)
    torch.cuda.synchronize()
    return caches, ref


def _one_call(st, seed, batch, hq, hkv, d, src_lens, rsn_lens, src_vis, q_len):
    rng = np.random.Generator(np.random.PCG64(seed))
    caches, ref = _filled(st, rng, batch, hkv, d, src_lens, rsn_lens)
    q = W.normal(rng, (batch, q_len, hq, d), "bf16")
    tq = to_dev(q, "bf16")
    vis_t = torch.from_numpy(src_vis.astype(np.int32)).to(DEV); rl_t = torch.from_numpy(rsn_lens.astype(np.int32)).to(DEV)
    ms, mr = int(src_lens.max()), int(rsn_lens.max())
    lse_ws = torch.empty((batch, q_len, hq), dtype=torch.float32, device=DEV)
    out_ws = st.st_attn_decode_dual(tq, caches, vis_t, rl_t, ms, mr, lse=lse_ws)
    out_st = torch.full_like(tq, float("nan")); lse_st = torch.full_like(lse_ws, float("nan"))
    torch.cuda.synchronize()
    print(f"no-alloc decode: seed {seed} batch {batch} heads {hq}/{hkv} d {d} q_len {q_len} bounds {ms}/{mr}", flush=True)
    st.st_attn_decode_dual_static(tq, caches, vis_t, rl_t, ms, mr, out_st, lse=lse_st)
    torch.cuda.synchronize()
    assert torch.equal(out_st.view(torch.int16), out_ws.view(torch.int16))
    assert torch.equal(lse_st.view(torch.int32), lse_ws.view(torch.int32))
    for b in range(batch):
        o_ref, l_ref = O.decode_dual_concat(q[b].astype(np.float64), ref[st.ST_SOURCE][0][b], ref[st.ST_SOURCE][1][b],
                                            ref[st.ST_REASONING][0][b], ref[st.ST_REASONING][1][b], int(src_vis[b]), int(rsn_lens[b]))
        assert np.abs(to_f64(out_st[b]) - o_ref).max() <= 2e-2, b
        assert np.abs(to_f64(lse_st[b]) - l_ref).max() <= 2e-2, b


def test_decode_static_scratch_two_calls_in_a_row(st):
    assert st.st_decode_static_scratch_bytes() == 64 << 20
    # first call: caches long enough for the split + merge kernels (partial results in the array), several units each
    _one_call(st, 9001, 6, 16, 8, 128, np.array([1500, 700, 33, 1024, 2047, 512]), np.array([3000, 1100, 2500, 17, 1025, 640]),
              np.array([1500, 0, 33, 1000, 2047, 511]), 1)
    # second call: fewer sequences, shorter caches, two query tokens -- the array still holds the first call's partials
    _one_call(st, 9002, 3, 8, 2, 64, np.array([1100, 40, 300]), np.array([200, 1300, 18]), np.array([1100, 16, 0]), 2)
    # and a short one that takes the single-launch kernel (no partial results at all)
    _one_call(st, 9003, 2, 4, 2, 128, np.array([100, 7]), np.array([60, 300]), np.array([100, 0]), 1)


def test_decode_static_scratch_rejects_what_does_not_fit(st):
    rng = np.random.Generator(np.random.PCG64(9010))
    batch, hq, hkv, d = 2, 16, 8, 128
    caches, _ = _filled(st, rng, batch, hkv, d, np.array([64, 64]), np.array([64, 64]))
    tq = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
    lens = torch.full((batch,), 64, dtype=torch.int32, device=DEV)
    out = torch.zeros_like(tq)
    # a batch far beyond the array (checked on the host before anything is launched; `batch` is only a number here)
    lib = st.load_library()
    import ctypes as C
    from paper_2510_17238_amd.binding import _DualLensStruct
    stc = caches.struct()
    ls = _DualLensStruct(lens.data_ptr(), lens.data_ptr(), 1, 64, 64)
    rc = lib.st_attn_decode_dual_static(C.c_void_p(out.data_ptr()), None, C.c_void_p(tq.data_ptr()), C.byref(stc), C.byref(ls),
                                        1 << 20, hq, 0.0, None)
    assert rc == 4 and "array holds" in st.st_last_error()       # ST_ERR_CAPACITY
    torch.cuda.synchronize()
    assert float(out.float().abs().max()) == 0.0
