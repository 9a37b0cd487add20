"""Parity at the benchmark configurations' FULL sizes, in the launch configuration bench.py times.
The oracle cannot run these whole, so outputs are checked on samples it computes row by row
(first / last rows of segments, rows next to tile boundaries, the final row), and the integer
metadata is checked in full against the dense-mask reduction or against closed forms.
Inputs are drawn on the device with a seeded generator and copied to the host for the oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import streaming_attention as O

pytestmark = pytest.mark.gpu

from gpu_helpers import DEV, ids_to_dev, to_f64  # noqa: E402


@pytest.fixture(scope="module")
def st():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_17238_amd as st_
    st_.load_library()
    return st_


def _device_normal(shape, seed):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    return torch.randn(shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)


def _sample_rows(cfg, b, tile_m, n_extra, rng):
    """Rows of sequence b (local indices): segment starts / ends, tile-boundary neighbours, last row, random."""
    s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
    n = e - s
    seg = cfg.segment_ids[s:e]; strm = cfg.stream_ids[s:e]
    change = np.nonzero((np.diff(seg) != 0) | (np.diff(strm) != 0))[0]
    rows = {0, n - 1}
    for c in change[:: max(1, len(change) // 12)]:
        rows.update({int(c), int(c) + 1})
    # rows whose stream-local position sits next to a query-tile boundary
    pos = cfg.positions[s:e]
    near = np.nonzero((pos % tile_m == 0) | (pos % tile_m == tile_m - 1))[0]
    rows.update(int(x) for x in near[:: max(1, len(near) // 12)])
    rows.update(int(x) for x in rng.integers(0, n, size=n_extra))
    return np.array(sorted(r for r in rows if 0 <= r < n))


def _prefill_full(st, cfg, meta_seqs, n_extra=24, heads=0):
    hq, hkv, d, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_tokens
    q = _device_normal((n, hq, d), cfg.seed); k = _device_normal((n, hkv, d), cfg.seed + 1); v = _device_normal((n, hkv, d), cfg.seed + 2)
    seg, strm, pos = ids_to_dev(cfg)
    st.st_rope_apply(q, pos, cfg.theta); st.st_rope_apply(k, pos, cfg.theta)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, validate=True).heads_per_workgroup(heads)
    lse = torch.empty((n, hq), dtype=torch.float32, device=DEV)
    out = st.st_attn_prefill(q, k, v, plan, lse=lse)
    torch.cuda.synchronize()
    bm, bn = plan.tile_shape()
    # --- metadata: pair counts for every sequence (closed form), full tables for `meta_seqs`
    assert [int(x) for x in plan.visible_pairs()] == cfg.closed_form_pairs()
    n_src, n_rsn = plan.stream_counts(); perm = plan.compact_index(); vis = plan.visible_source()
    for b in range(cfg.batch):
        assert n_src[b] == int(cfg.src_lens[b].sum()) and n_rsn[b] == int(cfg.rsn_lens[b].sum())
    for b in meta_seqs:
        s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
        md = O.canonical_metadata(cfg.stream_ids[s:e], cfg.segment_ids[s:e], cfg.positions[s:e], bm, bn)
        S = len(md["src_idx"])
        assert np.array_equal(perm[s:s + S] - s, md["src_idx"]) and np.array_equal(perm[s + S:e] - s, md["rsn_idx"])
        assert np.array_equal(vis[s + S:e], md["vis_src"]) and md["visible_pairs"] == cfg.closed_form_pairs()[b]
        for blk, name in ((st.ST_BLOCK_SS, "SS"), (st.ST_BLOCK_RS, "RS"), (st.ST_BLOCK_RR, "RR")):
            assert np.array_equal(plan.tile_classes(b, blk), md[name]), (b, name)
    # --- outputs on sampled rows, every head
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 77))
    worst = 0.0
    for b in range(cfg.batch):
        s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
        rows = _sample_rows(cfg, b, bm, n_extra, rng)
        ref, ref_lse = O.attention_dense(to_f64(q[s:e]), to_f64(k[s:e]), to_f64(v[s:e]), cfg.stream_ids[s:e],
                                         cfg.segment_ids[s:e], cfg.positions[s:e], rows=rows)
        idx = torch.from_numpy(rows + s).to(DEV)
        err = np.abs(to_f64(out[idx]) - ref).max()
        worst = max(worst, err)
        assert err <= 2e-2, (b, err)
        assert np.abs(to_f64(lse[idx]) - ref_lse).max() <= 2e-2
    return worst


def test_config4a_prefill_16k(st):
    """Qwen3-4B-shaped layer, 8 x 16,384 tokens: full metadata for two sequences, sampled rows for all."""
    _prefill_full(st, W.config4a(), meta_seqs=(0, 5))


def test_config4a_prefill_16k_one_head_kernel(st):
    """The same batch through the kernel the automatic choice does NOT take at this size."""
    _prefill_full(st, W.config4a(), meta_seqs=(), heads=1)


def test_config4b_prefill_128_pairs(st):
    """Count-pinned variant (128 pairs, about 37K tokens per sequence): full metadata for one sequence."""
    _prefill_full(st, W.config4b(), meta_seqs=(3,), n_extra=12)


def _decode_full(st, shp, q_len, check_seqs, seed, fp8=False, one_call=False):
    B, hq, hkv, d = shp.batch, shp.n_q_heads, shp.n_kv_heads, shp.head_dim
    rng = np.random.Generator(np.random.PCG64(seed))
    pages_s = (shp.max_src_len + 15) // 16; pages_r = (shp.max_rsn_len + 15) // 16
    tab_s = W.shuffled_page_table(rng, B, pages_s); tab_r = W.shuffled_page_table(rng, B, pages_r)
    cs = st.KVCache(B * pages_s, B, pages_s, hkv, d, torch.from_numpy(tab_s).to(DEV), fp8=fp8)
    cr = st.KVCache(B * pages_r, B, pages_r, hkv, d, torch.from_numpy(tab_r).to(DEV), fp8=fp8)
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    for c in (cs, cr):       # any bit pattern is a valid cache content: draw the pools directly
        if fp8:
            # any code but the two NaN codes (0x7f, 0xff), scales 2^-9 .. 2^-6 (values up to +-7)
            for pool in (c.k_pool, c.v_pool):
                pool.random_(0, 256, generator=g)
                pool[(pool & 0x7f) == 0x7f] = 0x3a
            for sc in (c.k_scale, c.v_scale):
                sc.copy_(torch.ldexp(torch.ones_like(sc), torch.randint(-9, -5, sc.shape, generator=g, device=DEV)))
        else:
            c.k_pool.normal_(generator=g); c.v_pool.normal_(generator=g)
    caches = st.DualCache(cs, cr)
    # the step itself: append the q_len new reasoning tokens, then attend
    rsn_before = (shp.rsn_len - q_len).astype(np.int32)
    cs.appended_len.copy_(torch.from_numpy(shp.src_visible_len)); cr.appended_len.copy_(torch.from_numpy(rsn_before))
    k_tok = _device_normal((B, q_len, hkv, d), seed + 1); v_tok = _device_normal((B, q_len, hkv, d), seed + 2)
    q = _device_normal((B, q_len, hq, d), seed + 3)
    if not one_call:
        st.st_kv_append(caches, st.ST_REASONING, k_tok, v_tok, host_len_upper_bound=int(shp.rsn_len.max()))
    # a source chunk arriving on a second stream while the decode runs (not yet visible)
    k_src = _device_normal((B, shp.src_append, hkv, d), seed + 4)
    side = torch.cuda.Stream(); side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.st_kv_append(caches, st.ST_SOURCE, k_src, k_src, host_len_upper_bound=shp.max_src_len, stream=side)
    vis = torch.from_numpy(shp.src_visible_len).to(DEV); rl = torch.from_numpy(shp.rsn_len).to(DEV)
    lse = torch.empty((B, q_len, hq), dtype=torch.float32, device=DEV)
    if one_call:     # the form bench.py times: store the token and attend in one call (rotated inputs: theta_base 0)
        out = st.st_attn_decode_dual_append(q, k_tok, v_tok, caches, vis, rl, int(shp.src_visible_len.max()), int(shp.rsn_len.max()), lse=lse)
    else:
        out = st.st_attn_decode_dual(q, caches, vis, rl, int(shp.src_visible_len.max()), int(shp.rsn_len.max()), lse=lse)
    torch.cuda.synchronize()
    assert cr.appended_len.cpu().tolist() == shp.rsn_len.tolist()
    assert cs.appended_len.cpu().tolist() == (shp.src_visible_len + shp.src_append).tolist()
    assert torch.isfinite(out).all()
    for b in check_seqs:
        def gather(cache, tab, length):
            ids = torch.from_numpy(tab[b, :(length + 15) // 16].astype(np.int64)).to(DEV)
            if fp8:          # stored values: code x scale
                kc = st.k_pool8_to_logical(cache.k_pool[ids]).reshape(-1, hkv, d)[:length].cpu().numpy()
                vc = st.v_pool_to_logical(cache.v_pool[ids]).reshape(-1, hkv, d)[:length].cpu().numpy()
                ks = st.scale_to_logical(cache.k_scale[ids]).reshape(-1, hkv)[:length].cpu().numpy().astype(np.float64)
                vs = st.scale_to_logical(cache.v_scale[ids]).reshape(-1, hkv)[:length].cpu().numpy().astype(np.float64)
                return O.e4m3_decode(kc) * ks[..., None], O.e4m3_decode(vc) * vs[..., None]
            kl = st.k_pool_to_logical(cache.k_pool[ids]).reshape(-1, hkv, d)[:length]
            vl = st.v_pool_to_logical(cache.v_pool[ids]).reshape(-1, hkv, d)[:length]
            return to_f64(kl), to_f64(vl)
        sk, sv = gather(cs, tab_s, int(shp.src_visible_len[b]))
        rk, rv = gather(cr, tab_r, int(shp.rsn_len[b]))
        # the appended tokens really are the last q_len rows of the reasoning cache
        if fp8:
            stored = lambda x: O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(to_f64(x)))
            assert np.array_equal(rk[-q_len:], stored(k_tok[b])) and np.array_equal(rv[-q_len:], stored(v_tok[b]))
            o_ref, l_ref = O.decode_dual_fp8(to_f64(q[b]), sk, sv, rk, rv, int(shp.src_visible_len[b]), int(shp.rsn_len[b]))
            assert np.abs(to_f64(out[b]) - o_ref).max() <= 2e-2 * max(1.0, np.abs(o_ref).max()), b
            assert np.abs(to_f64(lse[b]) - l_ref).max() <= 2e-2, b
            continue
        assert np.array_equal(rk[-q_len:], to_f64(k_tok[b])) and np.array_equal(rv[-q_len:], to_f64(v_tok[b]))
        o_ref, l_ref = O.decode_dual_concat(to_f64(q[b]), sk, sv, rk, rv, int(shp.src_visible_len[b]), int(shp.rsn_len[b]))
        assert np.abs(to_f64(out[b]) - o_ref).max() <= 2e-2, b
        assert np.abs(to_f64(lse[b]) - l_ref).max() <= 2e-2, b


def test_config3_decode_one_layer(st):
    """Qwen3-1.7B-shaped decode step (batch 32, 2K source + 1-6K reasoning), one of the 28 identical layers."""
    shp = W.config3()
    longest, shortest = int(np.argmax(shp.rsn_len)), int(np.argmin(shp.rsn_len))
    _decode_full(st, shp, 1, sorted({0, 7, longest, shortest}), seed=31)


def test_config3_decode_one_layer_in_one_call(st):
    """The same step the way bench.py issues it: st_attn_decode_dual_append stores the token and attends (512-token
    units chosen by launch size, the token through the split kernel's extra work unit); the whole output, all 32
    sequences, against the oracle."""
    shp = W.config3()
    _decode_full(st, shp, 1, range(shp.batch), seed=33, one_call=True)             # every row of all 32 sequences


def test_config5_decode_token_in_one_call(st):
    """One token of the Qwen3-8B-shaped streaming step (64 streams, caches up to 8K + 16K tokens: 1024-token units), one
    layer, issued as bench.py's streaming-step leg issues it; the whole output, all 64 streams, against the oracle."""
    shp = W.config5()
    _decode_full(st, shp, 1, range(shp.batch), seed=34, one_call=True)             # every row of all 64 streams


def test_config3_decode_one_layer_8bit_caches(st):
    """The same step over caches stored in 8 bits (codes drawn at random, the step's own token quantised by the append)."""
    shp = W.config3()
    longest, shortest = int(np.argmax(shp.rsn_len)), int(np.argmin(shp.rsn_len))
    _decode_full(st, shp, 1, sorted({3, longest, shortest}), seed=32, fp8=True)


def test_config2_prefill_backward(st):
    """Gradients of the attention stage on the benchmark batch (configs[1]) at full size, through the matrix-core
    kernels: every row of dQ and every key of dK / dV of two (sequence, KV head) picks against the oracle."""
    cfg = W.config2()
    hq, hkv, d, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_tokens
    q = _device_normal((n, hq, d), cfg.seed + 10); k = _device_normal((n, hkv, d), cfg.seed + 11)
    v = _device_normal((n, hkv, d), cfg.seed + 12); go = _device_normal((n, hq, d), cfg.seed + 13)
    seg, strm, pos = ids_to_dev(cfg)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    lse = torch.empty((n, hq), dtype=torch.float32, device=DEV)
    out = st.st_attn_prefill(q, k, v, plan, lse=lse)
    dq, dk, dv = st.st_attn_prefill_bwd(go, q, k, v, out, lse, plan)
    torch.cuda.synchronize()
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()
    group = hq // hkv
    for b, hk in ((0, 0), (cfg.batch - 1, hkv - 1)):
        s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
        hs = slice(hk * group, (hk + 1) * group)
        rq, rk, rv = O.attention_dense_backward(to_f64(q[s:e, hs]), to_f64(k[s:e, hk:hk + 1]), to_f64(v[s:e, hk:hk + 1]),
                                                to_f64(go[s:e, hs]), cfg.stream_ids[s:e], cfg.segment_ids[s:e], cfg.positions[s:e])
        for name, got, ref in (("dq", dq[s:e, hs], rq), ("dk", dk[s:e, hk:hk + 1], rk), ("dv", dv[s:e, hk:hk + 1], rv)):
            err = np.abs(to_f64(got) - ref).max()
            assert err <= 6e-2 * max(1.0, np.abs(ref).max()), (b, hk, name, err, np.abs(ref).max())


def test_config5_stream_step_one_layer(st):
    """Qwen3-8B-shaped streaming step (batch 64, caches to 8K / 16K, 32-token appends), one layer, q_len = 1."""
    shp = W.config5()
    longest = int(np.argmax(shp.rsn_len + shp.src_visible_len))
    _decode_full(st, shp, 1, sorted({1, 33, longest}), seed=51)


def test_config5_eight_tokens_in_one_call(st):
    """The same shape with the step's 8 reasoning tokens decoded in a single call (q_len = 8, causal among them)."""
    shp = W.config5(batch=16)
    _decode_full(st, shp, 8, [0, 9], seed=52)


def test_config5_source_chunk_one_layer(st):
    """Config 5's concurrent source side at full size: batch 64, 32-token chunks arriving on source caches of
    1-8K tokens (32 query heads, group 4 -> 128 rows = 4 blocks per sequence and KV head), one layer."""
    shp = W.config5()
    B, hq, hkv, d, n_new = shp.batch, shp.n_q_heads, shp.n_kv_heads, shp.head_dim, shp.src_append
    rng = np.random.Generator(np.random.PCG64(53))
    pages = (shp.max_src_len + 15) // 16
    tab = W.shuffled_page_table(rng, B, pages)
    cs = st.KVCache(B * pages, B, pages, hkv, d, torch.from_numpy(tab).to(DEV))
    cr = st.KVCache(B, B, 1, hkv, d, torch.arange(B, dtype=torch.int32, device=DEV).reshape(B, 1).contiguous())
    g = torch.Generator(device=DEV); g.manual_seed(53)
    cs.k_pool.normal_(generator=g); cs.v_pool.normal_(generator=g)
    caches = st.DualCache(cs, cr)
    cs.appended_len.copy_(torch.from_numpy(shp.src_visible_len))
    k_new = _device_normal((B, n_new, hkv, d), 54); v_new = _device_normal((B, n_new, hkv, d), 55); q = _device_normal((B, n_new, hq, d), 56)
    st.st_kv_append(caches, st.ST_SOURCE, k_new, v_new, host_len_upper_bound=shp.max_src_len)
    total = (shp.src_visible_len + n_new).astype(np.int32)
    lse = torch.empty((B, n_new, hq), dtype=torch.float32, device=DEV)
    out = st.st_attn_source_chunk(q, caches, torch.from_numpy(total).to(DEV), int(total.max()), lse=lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    for b in sorted({0, 21, int(np.argmax(total)), int(np.argmin(total))}):
        ids = torch.from_numpy(tab[b, :(int(total[b]) + 15) // 16].astype(np.int64)).to(DEV)
        kl = to_f64(st.k_pool_to_logical(cs.k_pool[ids]).reshape(-1, hkv, d)[:int(total[b])])
        vl = to_f64(st.v_pool_to_logical(cs.v_pool[ids]).reshape(-1, hkv, d)[:int(total[b])])
        assert np.array_equal(kl[-n_new:], to_f64(k_new[b]))
        o_ref, l_ref = O.source_chunk_attention(to_f64(q[b]), kl, vl, int(total[b]))
        assert np.abs(to_f64(out[b]) - o_ref).max() <= 2e-2, b
        assert np.abs(to_f64(lse[b]) - l_ref).max() <= 2e-2, b
