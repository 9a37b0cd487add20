"""GPU parity: every call goes through the C-ABI library and is compared with the fp64
oracle on the same seeded inputs.  Tolerances (max-abs): 1e-4 for fp32 inputs, 2e-2 for
bf16 inputs with fp32 accumulation; integer metadata bit-exact."""
import gc

import numpy as np
import pytest
import torch

import workloads as W
from oracle import streaming_attention as O

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def st():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_17238_amd as st_
    st_.load_library()
    return st_


from gpu_helpers import DEV, ids_to_dev, make_cache, to_dev, to_f64  # noqa: E402


# ------------------------------------------------------------------ RoPE --
@pytest.mark.parametrize("dtype,n,h,d,pmax", [("f32", 128, 2, 64, 64), ("f32", 77, 3, 128, 200000),
                                              ("bf16", 1000, 24, 128, 40000), ("bf16", 5, 1, 64, 7)])
def test_rope(st, dtype, n, h, d, pmax):
    rng = np.random.Generator(np.random.PCG64(100 + n))
    x = W.normal(rng, (n, h, d), dtype)
    pos = rng.integers(0, pmax, size=n).astype(np.int32)
    pos[0] = 0
    tx = to_dev(x, dtype)
    out = torch.empty_like(tx)
    st.st_rope_apply(tx, torch.from_numpy(pos).to(DEV), 1.0e6, out=out)
    ref = O.rope(x, pos, 1.0e6)
    tol = 2e-6 * max(1.0, np.abs(ref).max()) if dtype == "f32" else 2e-2
    assert np.abs(to_f64(out) - ref).max() <= tol
    if dtype == "bf16":
        # correctly rounded up to one bf16 ulp
        assert np.abs(to_f64(out) - ref).max() <= np.abs(ref).max() * 2.0 ** -8
    # in place gives the same bits
    st.st_rope_apply(tx, torch.from_numpy(pos).to(DEV), 1.0e6)
    assert torch.equal(tx, out)


# -------------------------------------------------------------- metadata --
def _check_metadata(st, cfg):
    seg, strm, pos = ids_to_dev(cfg)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, validate=True)
    bm, bn = plan.tile_shape()
    n_src, n_rsn = plan.stream_counts()
    perm = plan.compact_index(); vis = plan.visible_source(); pairs = plan.visible_pairs()
    closed = cfg.closed_form_pairs()
    for b in range(cfg.batch):
        s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
        md = O.canonical_metadata(cfg.stream_ids[s:e], cfg.segment_ids[s:e], cfg.positions[s:e], bm, bn)
        S = len(md["src_idx"])
        assert n_src[b] == S and n_rsn[b] == len(md["rsn_idx"])
        assert np.array_equal(perm[s:s + S] - s, md["src_idx"])
        assert np.array_equal(perm[s + S:e] - s, md["rsn_idx"])
        assert np.array_equal(vis[s + S:e], md["vis_src"])
        assert np.array_equal(vis[s:s + S], np.arange(1, S + 1))
        assert int(pairs[b]) == md["visible_pairs"] == closed[b]
        for blk, name in ((st.ST_BLOCK_SS, "SS"), (st.ST_BLOCK_RS, "RS"), (st.ST_BLOCK_RR, "RR")):
            got = plan.tile_classes(b, blk)
            assert got.shape == md[name].shape, (name, got.shape, md[name].shape)
            assert np.array_equal(got, md[name]), name
    plan.destroy()


def test_metadata_config1(st):
    _check_metadata(st, W.config1())
    _check_metadata(st, W.config1("grouped"))


def test_metadata_config2(st):
    _check_metadata(st, W.config2())


@pytest.mark.parametrize("seed", [201, 202, 203, 204])
def test_metadata_random_ragged(st, seed):
    # empty and 1-token segments, sequences shorter than one tile, several tiles with ragged tails
    _check_metadata(st, W.random_prefill(seed, 5, 9, (0, 70), (0, 90), 2, 1, 64, "f32"))


def test_metadata_edge_structures(st):
    # only sources / only reasoning / empty sequence in the middle of a batch
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1]))]
    cfg = W._assemble("edges", "f32", 2, 1, 64, lists, "interleaved", 7)
    _check_metadata(st, cfg)


def test_many_short_sequences_take_the_large_plan_paths(st):
    """2,800 sequences of a few tokens each: more than 64 sequences (segment tables copied to the device instead of
    passed by value) and more than 4,096 work items (items and their longest-first order built by the multi-workgroup
    kernels).  Metadata bit-exact, attention and its gradients against the oracle for both dtypes."""
    rng = np.random.Generator(np.random.PCG64(250))
    lists = [W.draw_pairs(rng, int(rng.integers(1, 2, endpoint=True)), (0, 3), (0, 3)) for _ in range(2800)]
    lists[7] = (np.array([150]), np.array([140]))            # one sequence with several tiles among them
    for dtype in ("f32", "bf16"):
        cfg = W._assemble("many-short", dtype, 2, 1, 64, lists, "interleaved", 250)
        assert cfg.batch == 2800
        items = sum(-(-int(sl.sum()) // 128) + -(-int(rl.sum()) // 128) for sl, rl in lists)
        assert items > 4096
        if dtype == "f32":
            _check_metadata(st, cfg)
        _run_prefill(st, cfg)
        _run_prefill_bwd(st, cfg)          # the backward walks the same tables (2,800 sequences, > 4,096 items)


def test_plan_validation_rejects_bad_metadata(st):
    cfg = W.config1()
    seg, strm, pos = ids_to_dev(cfg)
    bad = pos.clone(); bad[5] = 0          # positions no longer increase inside the source stream
    with pytest.raises(st.StError) as e:
        st.st_plan_create(seg, strm, bad, cfg.cu_seqlens, validate=True)
    assert e.value.status == 3
    bad = strm.clone(); bad[9] = 2
    with pytest.raises(st.StError):
        st.st_plan_create(seg, bad, pos, cfg.cu_seqlens, validate=True)
    bad = seg.clone(); bad[40] = 0         # segment ids decrease inside a stream
    with pytest.raises(st.StError):
        st.st_plan_create(bad, strm, pos, cfg.cu_seqlens, validate=True)


# --------------------------------------------------------------- prefill --
def _run_prefill(st, cfg, rope=True, check_lse=True, heads=0):
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = to_dev(q, cfg.dtype), to_dev(k, cfg.dtype), to_dev(v, cfg.dtype)
    if rope:
        st.st_rope_apply(tq, pos, cfg.theta)
        st.st_rope_apply(tk, pos, cfg.theta)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, validate=True).heads_per_workgroup(heads)
    lse = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV)
    out = st.st_attn_prefill(tq, tk, tv, plan, lse=lse)
    torch.cuda.synchronize()
    # the oracle takes the attention stage's actual inputs (rotated, in the storage dtype)
    ref, ref_lse = O.attention_varlen(to_f64(tq), to_f64(tk), to_f64(tv), cfg.stream_ids, cfg.segment_ids, cfg.positions,
                                      cfg.cu_seqlens)
    err = np.abs(to_f64(out) - ref).max()
    assert err <= TOL[cfg.dtype], err
    if check_lse:
        assert np.abs(to_f64(lse) - ref_lse).max() <= TOL[cfg.dtype]
    return tq, tk, tv, out, plan


def test_rope_queries_and_keys_in_one_launch(st):
    """st_rope_apply_qk gives the bits of two st_rope_apply calls (fp32 and bf16, both head dims, in place and not)."""
    rng = np.random.Generator(np.random.PCG64(140))
    for dt, d, hq, hkv, n in (("f32", 64, 2, 1, 131), ("bf16", 128, 16, 8, 1000), ("bf16", 64, 4, 4, 7), ("f32", 128, 3, 2, 257)):
        q = to_dev(W.normal(rng, (n, hq, d), dt), dt); k = to_dev(W.normal(rng, (n, hkv, d), dt), dt)
        pos = torch.from_numpy(rng.integers(0, 40000, n).astype(np.int32)).to(DEV)
        rq = st.st_rope_apply(q, pos, 1.0e6, out=torch.empty_like(q)); rk = st.st_rope_apply(k, pos, 1.0e6, out=torch.empty_like(k))
        oq, ok = st.st_rope_apply_qk(q, k, pos, 1.0e6, q_out=torch.empty_like(q), k_out=torch.empty_like(k))
        assert torch.equal(rq, oq) and torch.equal(rk, ok)
        q2, k2 = q.clone(), k.clone()
        st.st_rope_apply_qk(q2, k2, pos, 1.0e6)
        torch.cuda.synchronize()
        assert torch.equal(rq, q2) and torch.equal(rk, k2)


def test_prefill_config1_fp32(st):
    cfg = W.config1()
    tq, tk, tv, out, plan = _run_prefill(st, cfg)
    # chained check: rope + attention against the oracle's own rope (fp32 end to end)
    q, k, v = cfg.tensors()
    ref, _ = O.attention_dense(O.rope(q, cfg.positions, cfg.theta), O.rope(k, cfg.positions, cfg.theta), v,
                               cfg.stream_ids, cfg.segment_ids, cfg.positions)
    assert np.abs(to_f64(out) - ref).max() <= 1e-4
    # one-off form with ids gives the same bits
    seg, strm, pos = ids_to_dev(cfg)
    out2 = st.st_attn_prefill_ids(tq, tk, tv, seg, strm, pos, cfg.cu_seqlens)
    assert torch.equal(out, out2)


def test_prefill_config1_grouped_layout(st):
    _run_prefill(st, W.config1("grouped"))


def test_prefill_config1_as_bf16(st):
    cfg = W.config1()
    cfg.dtype = "bf16"
    _run_prefill(st, cfg)


@pytest.mark.parametrize("seed,d,dtype", [(301, 64, "bf16"), (302, 128, "bf16"), (303, 128, "f32"), (304, 64, "f32"),
                                          (305, 128, "bf16")])
def test_prefill_random_ragged(st, seed, d, dtype):
    cfg = W.random_prefill(seed, 3, 8, (0, 90), (0, 120), 4, 2, d, dtype)
    _run_prefill(st, cfg)


def test_prefill_edge_structures(st):
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1])), (np.array([64, 64]), np.array([128, 1]))]
    for dtype in ("bf16", "f32"):
        cfg = W._assemble("edges", dtype, 4, 4, 128, lists, "interleaved", 7)
        _run_prefill(st, cfg)


def test_prefill_config2_bf16_full(st):
    cfg = W.config2()
    tq, tk, tv, out, plan = _run_prefill(st, cfg)
    # determinism: a second launch gives identical bits
    out2 = st.st_attn_prefill(tq, tk, tv, plan)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("heads", [1, 2])
def test_prefill_each_bf16_kernel(st, heads):
    """Both forms of the bf16 attention kernel (one / two query heads per workgroup), pinned in turn through the plan,
    against the oracle: small tiles (head_dim 64), ragged random structures (two heads per KV head), degenerate
    structures, and the full configs[1] batch."""
    cfg = W.config1()
    cfg.dtype = "bf16"
    _run_prefill(st, cfg, heads=heads)
    for seed, d in ((301, 64), (302, 128), (305, 128)):
        _run_prefill(st, W.random_prefill(seed, 3, 8, (0, 90), (0, 120), 4, 2, d, "bf16"), heads=heads)
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1])), (np.array([64, 64]), np.array([128, 1]))]
    _run_prefill(st, W._assemble("edges", "bf16", 4, 2, 128, lists, "interleaved", 7), heads=heads)
    tq, tk, tv, out, plan = _run_prefill(st, W.config2(), heads=heads)
    with pytest.raises(st.StError) as e:                          # values other than 0, 1, 2 are refused, the plan keeps its setting
        plan.heads_per_workgroup(17)
    assert e.value.status == 1
    out2 = st.st_attn_prefill(tq, tk, tv, plan)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_prefill_reference_exponent_moves(st):
    """Scores that outgrow the first tile's maximum by far more than the kernel lets probabilities grow (keys whose
    magnitude doubles three times along the sequence, and a sequence of all-but-zero scores whose last quarter is
    large): the attention kernel has to move a row's reference exponent in the middle of the row, more than once,
    without losing what it has accumulated."""
    for heads in (1, 2):
        for d in (64, 128):
            cfg = W.random_prefill(331 + d, 2, 6, (40, 120), (50, 160), 4, 2, d, "bf16")
            q, k, v = cfg.tensors()
            n = cfg.n_tokens
            e1 = int(cfg.cu_seqlens[1])
            ramp = np.ones(n, np.float32)
            ramp[:e1] = np.ldexp(1.0, np.minimum(np.arange(e1) // 70, 3).astype(np.int32)).astype(np.float32)   # x1, x2, x4, x8
            ramp[e1:] = 1.0e-3
            ramp[e1 + (n - e1) * 3 // 4:] = 8.0
            k = W.bf16_round(k * ramp[:, None, None])
            seg, strm, pos = ids_to_dev(cfg)
            tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
            plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens).heads_per_workgroup(heads)
            lse = torch.empty((n, cfg.n_q_heads), dtype=torch.float32, device=DEV)
            out = st.st_attn_prefill(tq, tk, tv, plan, lse=lse)
            torch.cuda.synchronize()
            ref, ref_lse = O.attention_varlen(to_f64(tq), to_f64(tk), to_f64(tv), cfg.stream_ids, cfg.segment_ids, cfg.positions,
                                              cfg.cu_seqlens)
            assert ref_lse.max() > 25.0                               # the case is what it claims to be: rises of e^25 and more
            # The kernel's queries carry the softmax scale, rounded to bf16 once more (at most half a unit in the last
            # place of q); on scores of magnitude 40 that rounding alone moves probabilities by percents.  So the
            # bookkeeping is checked against the oracle on exactly the queries the kernel uses ...
            c = np.float32(np.float32(1.0) / np.sqrt(np.float32(d))) * np.float32(1.4426950408889634)
            q_used = W.bf16_round(to_f64(tq).astype(np.float32) * c).astype(np.float64) / np.float64(c)
            ref_u, lse_u = O.attention_varlen(q_used, to_f64(tk), to_f64(tv), cfg.stream_ids, cfg.segment_ids, cfg.positions,
                                              cfg.cu_seqlens)
            err_u = np.abs(to_f64(out) - ref_u).max()
            assert np.isfinite(to_f64(out)).all() and err_u <= 2e-2, (heads, d, err_u)
            assert np.abs(to_f64(lse) - lse_u).max() <= 2e-2, (heads, d)
            # ... and against the oracle on the given queries with the bound that perturbation allows
            assert np.abs(to_f64(out) - ref).max() <= 0.15 and np.abs(to_f64(lse) - ref_lse).max() <= 0.15, (heads, d)


@pytest.mark.parametrize("heads", [1, 2])
def test_prefill_rope_fused(st, heads):
    """UNROTATED q, k through st_attn_prefill_rope (keys rotated on their way into the key tiles, queries as the
    attention kernel loads them) against the oracle's rotate-then-attend on the same bf16 inputs, and against the
    unfused path (st_rope_apply twice, then st_attn_prefill), with both forms of the attention kernel."""
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1])), (np.array([64, 64]), np.array([128, 1]))]
    for cfg in (W.random_prefill(321, 3, 8, (0, 90), (0, 120), 4, 2, 64, "bf16"), W.random_prefill(322, 3, 8, (0, 90), (0, 120), 4, 2, 128, "bf16"),
                W._assemble("edges", "bf16", 4, 2, 128, lists, "interleaved", 7), W.config2()):
        q, k, v = cfg.tensors()
        seg, strm, pos = ids_to_dev(cfg)
        tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
        plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens).heads_per_workgroup(heads)
        lse = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV)
        out_f = st.st_attn_prefill_rope(tq, tk, tv, pos, cfg.theta, plan, lse=lse)
        rq, rk = st.st_rope_apply(tq, pos, cfg.theta, out=torch.empty_like(tq)), st.st_rope_apply(tk, pos, cfg.theta, out=torch.empty_like(tk))
        out_u = st.st_attn_prefill(rq, rk, tv, plan)
        torch.cuda.synchronize()
        ref, ref_lse = O.attention_varlen(O.rope(to_f64(tq), cfg.positions, cfg.theta), O.rope(to_f64(tk), cfg.positions, cfg.theta),
                                          to_f64(tv), cfg.stream_ids, cfg.segment_ids, cfg.positions, cfg.cu_seqlens)
        assert np.abs(to_f64(out_f) - ref).max() <= 2e-2, cfg.name
        assert np.abs(to_f64(lse) - ref_lse).max() <= 2e-2, cfg.name
        assert (out_f.float() - out_u.float()).abs().max().item() <= 2e-2, cfg.name
    cfg = W.config1()
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    with pytest.raises(st.StError) as e:                      # fp32 inputs keep the separate, fp64-accurate rotation
        st.st_attn_prefill_rope(to_dev(q, "f32"), to_dev(k, "f32"), to_dev(v, "f32"), pos, cfg.theta, plan)
    assert e.value.status == 5
    with pytest.raises(st.StError) as e:
        st.st_attn_prefill_rope(to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), pos, 0.0, plan)
    assert e.value.status == 1


def test_plan_built_on_one_stream_used_on_others(st):
    """A plan built (unvalidated, so nothing waits on the host) on stream A, the forward on stream B and the backward on
    stream C, each with the binding's temporary workspaces: the entry points order themselves against the build, and
    the results have the bits of the same calls on one stream."""
    cfg = W.config2()
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = to_dev(q, cfg.dtype), to_dev(k, cfg.dtype), to_dev(v, cfg.dtype)
    go = to_dev(W.normal(np.random.Generator(np.random.PCG64(77)), q.shape, cfg.dtype), cfg.dtype)
    plan0 = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    lse0 = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV)
    out0 = st.st_attn_prefill(tq, tk, tv, plan0, lse=lse0)
    g0 = st.st_attn_prefill_bwd(go, tq, tk, tv, out0, lse0, plan0)
    torch.cuda.synchronize()
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, stream=sa)
        lse1 = torch.empty_like(lse0)
        out1 = st.st_attn_prefill(tq, tk, tv, plan, lse=lse1, stream=sb)
        sc.wait_stream(sb)
        g1 = st.st_attn_prefill_bwd(go, tq, tk, tv, out1, lse1, plan, stream=sc)
        torch.cuda.synchronize()
        assert torch.equal(out0, out1) and torch.equal(lse0, lse1)
        for a, b in zip(g0, g1):
            assert torch.equal(a, b)
        plan.destroy()
    plan0.destroy()


def test_kernel_timing_with_repeated_launches_changes_no_result(st):
    """st_profile_enable + st_profile_repeat: the timed kernels are launched several times between their two events;
    outputs keep their bits, one reading per call comes back, and the state is the thread's own."""
    cfg = W.config2()
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = to_dev(q, cfg.dtype), to_dev(k, cfg.dtype), to_dev(v, cfg.dtype)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    lse0 = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV); lse1 = torch.empty_like(lse0)
    out0 = st.st_attn_prefill(tq, tk, tv, plan, lse=lse0)
    for which in (st.ST_PROF_PREFILL_ATTN, st.ST_PROF_TILE_PACK):
        st.st_profile_read(which)
    st.st_profile_repeat(4)
    st.st_profile_enable(True)
    try:
        out1 = st.st_attn_prefill(tq, tk, tv, plan, lse=lse1)
        out2 = st.st_attn_prefill(tq, tk, tv, plan)
    finally:
        st.st_profile_enable(False)
        st.st_profile_repeat(1)
    torch.cuda.synchronize()
    assert torch.equal(out0, out1) and torch.equal(out0, out2) and torch.equal(lse0, lse1)
    ms_attn, n_attn = st.st_profile_read(st.ST_PROF_PREFILL_ATTN)
    ms_pack, n_pack = st.st_profile_read(st.ST_PROF_TILE_PACK)
    assert n_attn == 2 and n_pack == 2
    assert 0.0 < ms_pack < ms_attn < 50.0
    assert st.st_profile_read(st.ST_PROF_PREFILL_ATTN) == (0.0, 0)           # read forgets
    with pytest.raises(st.StError):
        st.st_profile_repeat(0)
    plan.destroy()


def test_prefill_mfma_agrees_with_plain_kernel(st):
    """bf16 inputs through the MFMA kernel vs the same values through the fp32 kernel."""
    cfg = W.random_prefill(311, 2, 10, (10, 80), (10, 100), 4, 2, 128, "bf16")
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    o_b = st.st_attn_prefill(to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), plan)
    o_f = st.st_attn_prefill(to_dev(q, "f32"), to_dev(k, "f32"), to_dev(v, "f32"), plan)
    torch.cuda.synchronize()
    assert (o_b.float() - o_f).abs().max().item() <= 2e-2


# ------------------------------------------------------------- backward --
def _run_prefill_bwd(st, cfg, tol_scale=1.0):
    """Forward then backward through the library; gradients against the oracle's, element by element."""
    q, k, v = cfg.tensors()
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 77))
    g = W.normal(rng, q.shape, cfg.dtype)
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv, tg = (to_dev(x, cfg.dtype) for x in (q, k, v, g))
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    lse = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV)
    out = st.st_attn_prefill(tq, tk, tv, plan, lse=lse)
    dq, dk, dv = st.st_attn_prefill_bwd(tg, tq, tk, tv, out, lse, plan)
    torch.cuda.synchronize()
    rq, rk, rv = O.attention_varlen_backward(q, k, v, g, cfg.stream_ids, cfg.segment_ids, cfg.positions, cfg.cu_seqlens)
    # fp32: rounding of the sums only.  bf16: the forward's out / lse carry bf16 / MFMA rounding (2e-2 on out), and
    # the gradients are rounded to bf16; a gradient sums up to a few hundred terms of that accuracy.
    tol = (2e-4 if cfg.dtype == "f32" else 6e-2) * tol_scale
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = np.abs(to_f64(got) - ref).max()
        assert err <= tol * max(1.0, np.abs(ref).max()), (name, err, np.abs(ref).max())
    return dq, dk, dv


def test_prefill_bwd_config1_fp32(st):
    _run_prefill_bwd(st, W.config1())


@pytest.mark.parametrize("seed,d,dtype,hq,hkv", [(601, 64, "f32", 4, 2), (602, 128, "f32", 2, 1), (603, 128, "bf16", 4, 2),
                                                  (604, 64, "bf16", 4, 4)])
def test_prefill_bwd_random_ragged(st, seed, d, dtype, hq, hkv):
    _run_prefill_bwd(st, W.random_prefill(seed, 3, 8, (0, 90), (0, 120), hq, hkv, d, dtype))


def test_prefill_bwd_edge_structures(st):
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1])), (np.array([64, 64]), np.array([128, 1]))]
    _run_prefill_bwd(st, W._assemble("edges", "f32", 2, 1, 64, lists, "interleaved", 7))
    _run_prefill_bwd(st, W._assemble("edges", "f32", 2, 2, 128, lists, "grouped", 8))


def test_prefill_bwd_bf16_tiles(st):
    """The matrix-core path over several 64-row tiles and 128-row items per stream, both head sizes, grouped heads,
    the edge structures (empty streams, single tokens, exact tile multiples) and the small standard case."""
    lists = [(np.array([5, 130]), np.array([0, 0])), (np.array([0]), np.array([200])), (np.array([], int), np.array([], int)),
             (np.array([1]), np.array([1])), (np.array([64, 64]), np.array([128, 1]))]
    _run_prefill_bwd(st, W._assemble("edges", "bf16", 4, 2, 128, lists, "interleaved", 7))
    _run_prefill_bwd(st, W._assemble("edges", "bf16", 2, 2, 64, lists, "grouped", 8))
    _run_prefill_bwd(st, W.random_prefill(611, 2, 5, (40, 160), (60, 200), 8, 2, 128, "bf16"))
    _run_prefill_bwd(st, W.random_prefill(612, 2, 4, (100, 200), (30, 90), 2, 1, 64, "bf16"))
    cfg = W.config1()
    cfg.dtype = "bf16"
    _run_prefill_bwd(st, cfg)


def test_prefill_bwd_bf16_agrees_with_plain_kernels(st):
    """bf16 inputs through the matrix-core backward vs the same values through the fp32 one-thread-per-row kernels."""
    cfg = W.random_prefill(613, 2, 6, (30, 150), (30, 170), 4, 2, 128, "bf16")
    q, k, v = cfg.tensors()
    g = W.normal(np.random.Generator(np.random.PCG64(5)), q.shape, "bf16")
    seg, strm, pos = ids_to_dev(cfg)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    grads = {}
    for dt in ("bf16", "f32"):
        tq, tk, tv, tg = (to_dev(x, dt) for x in (q, k, v, g))
        lse = torch.empty((cfg.n_tokens, cfg.n_q_heads), dtype=torch.float32, device=DEV)
        out = st.st_attn_prefill(tq, tk, tv, plan, lse=lse)
        grads[dt] = st.st_attn_prefill_bwd(tg, tq, tk, tv, out, lse, plan)
    torch.cuda.synchronize()
    for a, b in zip(grads["bf16"], grads["f32"]):
        assert (a.float() - b).abs().max().item() <= 6e-2 * max(1.0, b.abs().max().item())


def test_prefill_bwd_is_deterministic_and_checks_arguments(st):
    cfg = W.random_prefill(605, 2, 6, (5, 60), (5, 70), 4, 2, 128, "bf16")
    a = _run_prefill_bwd(st, cfg)
    b = _run_prefill_bwd(st, cfg)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = (to_dev(x, "bf16") for x in (q, k, v))
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    lse = torch.zeros((cfg.n_tokens, 4), dtype=torch.float32, device=DEV)
    with pytest.raises(st.StError) as e:
        st.st_attn_prefill_bwd(tq, tq, tk, tv, tq, lse, plan, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.status == 4


# ------------------------------------------------- many random structures --
def test_forward_and_backward_over_many_random_structures(st):
    """Sixty seeded structures -- segment counts, empty and one-token segments, both layouts, both head sizes, grouped
    heads, tile multiples by chance, reasoning streams from a few to a few thousand tokens -- through the bf16 forward
    (both kernels) and backward, and a few in fp32."""
    rng = np.random.Generator(np.random.PCG64(9000))
    for trial in range(60):
        d = int(rng.choice([64, 128])); hkv = int(rng.choice([1, 2])); hq = hkv * int(rng.choice([1, 2, 4]))
        layout = "interleaved" if trial % 2 else "grouped"
        hi_s, hi_r = int(rng.choice([3, 40, 130, 300])), int(rng.choice([3, 50, 150, 500]))
        cfg = W.random_prefill(9100 + trial, int(rng.integers(1, 4)), int(rng.integers(1, 9)), (0, hi_s), (0, hi_r), hq, hkv, d,
                               "f32" if trial % 10 == 9 else "bf16", layout)
        if cfg.n_tokens == 0:
            continue
        _run_prefill(st, cfg, heads=2 if trial % 3 == 0 else 1)
        _run_prefill_bwd(st, cfg)


def test_decode_over_many_random_lengths(st):
    """Random cache lengths around page, step and unit boundaries, visible source prefixes from 0 to everything, one to
    eight query tokens, bf16 and 8-bit caches, short (fused single launch) and long (split + merge) caches."""
    rng = np.random.Generator(np.random.PCG64(9001))
    marks = np.array([0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 511, 512, 513, 1023, 1024, 1025, 1300])
    for trial in range(14):
        batch = int(rng.integers(1, 5)); d = int(rng.choice([64, 128])); hkv = int(rng.choice([1, 2])); group = int(rng.choice([1, 2, 4]))
        q_len = int(rng.choice([1, 1, 2, 4]))
        if q_len * group > 16:
            q_len = 16 // group
        short = trial % 2 == 0
        pool = marks[marks <= (400 if short else 1300)]
        src_lens = rng.choice(pool, batch); rsn_lens = np.maximum(rng.choice(pool, batch), q_len)
        src_vis = np.array([int(rng.integers(0, s + 1)) for s in src_lens])
        _check_decode(st, rng, batch, hkv * group, hkv, d, src_lens, rsn_lens, src_vis, q_len=q_len, fp8=(trial % 4 == 3))


# ------------------------------------------------------- append / decode --
def _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra=0, chunks=(1, 15, 17, 64, 3), rope_theta=None, fp8=False,
               row_exponents=None):
    """Fill both caches through st_kv_append in uneven chunks; returns caches and the oracle's contiguous copies.
    With rope_theta the keys go in UNROTATED through st_kv_append_rope, and the oracle's copy of K is what
    paged_append_rotated stores: RoPE(k, index in the cache), in fp64."""
    pages_s = (int(max(src_lens)) + src_extra + 15) // 16 + 1
    pages_r = (int(max(rsn_lens)) + 15) // 16 + 1
    # never-written slots keep a fill that would poison any result: NaN (0x7f is the E4M3 NaN code; scales get NaN too)
    cs, tab_s = make_cache(batch, pages_s, hkv, d, rng, fill=0x7f if fp8 else float("nan"), fp8=fp8)
    cr, tab_r = make_cache(batch, pages_r, hkv, d, rng, fill=0x7f if fp8 else float("nan"), fp8=fp8)
    caches = st.DualCache(cs, cr)
    ref = {}
    for which, lens, cache in ((st.ST_SOURCE, src_lens, cs), (st.ST_REASONING, rsn_lens, cr)):
        total = int(max(lens)) if len(lens) else 0
        kk = W.normal(rng, (batch, total, hkv, d), "bf16"); vv = W.normal(rng, (batch, total, hkv, d), "bf16")
        if row_exponents is not None:                        # rows of very different magnitude (exact: powers of two)
            kk = np.ldexp(kk, rng.integers(row_exponents[0], row_exponents[1] + 1, (batch, total, hkv, 1))).astype(np.float32)
            vv = np.ldexp(vv, rng.integers(row_exponents[0], row_exponents[1] + 1, (batch, total, hkv, 1))).astype(np.float32)
        ref[which] = (kk, vv)
        done = np.zeros(batch, np.int64); ci = 0
        while (done < lens).any():
            step = chunks[ci % len(chunks)]; ci += 1
            n_new = np.minimum(step, lens - done).astype(np.int32)
            kn = np.zeros((batch, step, hkv, d), np.float32); vn = np.zeros((batch, step, hkv, d), np.float32)
            for b in range(batch):
                kn[b, :n_new[b]] = kk[b, done[b]:done[b] + n_new[b]]
                vn[b, :n_new[b]] = vv[b, done[b]:done[b] + n_new[b]]
            st.st_kv_append(caches, which, to_dev(kn, "bf16"), to_dev(vn, "bf16"), torch.from_numpy(n_new).to(DEV),
                            rope_theta=rope_theta)
            done += n_new
        torch.cuda.synchronize()
        assert np.array_equal(cache.appended_len.cpu().numpy(), lens)
        if rope_theta is not None:
            tab = tab_s if which == st.ST_SOURCE else tab_r
            n_pages = batch * cache.max_pages_per_seq
            pk = np.zeros((n_pages, O.PAGE, hkv, d)); pv = np.zeros_like(pk)
            olen = np.zeros(batch, np.int64)
            rot = np.zeros(kk.shape, np.float64)
            for b in range(batch):
                O.paged_append_rotated(pk, pv, tab, olen, b, kk[b, :lens[b]].astype(np.float64), vv[b, :lens[b]].astype(np.float64),
                                       rope_theta)
                rot[b, :lens[b]] = O.paged_gather(pk, tab, b, int(lens[b]))
            ref[which] = (rot, vv)
    return caches, ref, (tab_s, tab_r)


def test_kv_append_matches_paged_model(st):
    rng = np.random.Generator(np.random.PCG64(400))
    batch, hkv, d = 3, 2, 128
    src_lens = np.array([70, 33, 16]); rsn_lens = np.array([5, 100, 48])
    caches, ref, (tab_s, tab_r) = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens)
    for cache, which, lens, tab in ((caches.source, st.ST_SOURCE, src_lens, tab_s), (caches.reasoning, st.ST_REASONING, rsn_lens, tab_r)):
        kl = st.k_pool_to_logical(cache.k_pool).float().cpu().numpy()
        vl = st.v_pool_to_logical(cache.v_pool).float().cpu().numpy()
        # the oracle's paged model, filled in one go from the same rows
        pool_k = np.full(kl.shape, np.nan, np.float32); pool_v = np.full(vl.shape, np.nan, np.float32)
        olen = np.zeros(batch, np.int64)
        for b in range(batch):
            O.paged_append(pool_k, tab, olen.copy(), b, ref[which][0][b, :lens[b]])
            O.paged_append(pool_v, tab, olen, b, ref[which][1][b, :lens[b]])
        # written slots are bit-identical, unwritten slots still hold the NaN fill
        assert np.array_equal(np.isnan(kl), np.isnan(pool_k)) and np.array_equal(np.isnan(vl), np.isnan(pool_v))
        assert np.array_equal(np.nan_to_num(kl), np.nan_to_num(pool_k))
        assert np.array_equal(np.nan_to_num(vl), np.nan_to_num(pool_v))
        for b in range(batch):
            assert np.array_equal(O.paged_gather(kl, tab, b, int(lens[b])), ref[which][0][b, :lens[b]])


def test_kv_append_capacity(st):
    rng = np.random.Generator(np.random.PCG64(401))
    cs, _ = make_cache(2, 2, 1, 64, rng); cr, _ = make_cache(2, 2, 1, 64, rng)
    caches = st.DualCache(cs, cr)
    kn = torch.zeros((2, 40, 1, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(st.StError) as e:
        st.st_kv_append(caches, st.ST_SOURCE, kn, kn, host_len_upper_bound=40)
    assert e.value.status == 4
    # a wrong host bound cannot make the device write past the page table: the overflow is dropped
    st.st_kv_append(caches, st.ST_SOURCE, kn, kn, host_len_upper_bound=32)
    torch.cuda.synchronize()
    assert cs.appended_len.cpu().tolist() == [32, 32]


def _check_decode(st, rng, batch, hq, hkv, d, src_lens, rsn_lens, src_vis, q_len=1, src_extra=0, rope_theta=None, fp8=False, unit_tokens=0):
    if fp8:
        # 8-bit caches take rotated keys (the fused append is bf16 only); the fused QUERY rotation works on either
        caches, ref, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra, fp8=True, row_exponents=(-4, 1))
    else:
        caches, ref, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra, rope_theta=rope_theta)
    q = W.normal(rng, (batch, q_len, hq, d), "bf16")
    tq = to_dev(q, "bf16")
    lse = torch.empty((batch, q_len, hq), dtype=torch.float32, device=DEV)
    vis_t = torch.from_numpy(src_vis.astype(np.int32)).to(DEV); rl_t = torch.from_numpy(rsn_lens.astype(np.int32)).to(DEV)
    out = st.st_attn_decode_dual(tq, caches, vis_t, rl_t, int(max(src_lens)), int(max(rsn_lens)), lse=lse, rope_theta=rope_theta,
                                 unit_tokens=unit_tokens)
    torch.cuda.synchronize()
    for b in range(batch):
        args = (q[b].astype(np.float64), ref[st.ST_SOURCE][0][b], ref[st.ST_SOURCE][1][b], ref[st.ST_REASONING][0][b],
                ref[st.ST_REASONING][1][b], int(src_vis[b]), int(rsn_lens[b]))
        if fp8:
            if rope_theta is not None and rsn_lens[b] < q_len:
                continue
            qa = args[0] if rope_theta is None else O.rope(args[0], int(rsn_lens[b]) - q_len + np.arange(q_len), rope_theta)
            o_ref, l_ref = O.decode_dual_fp8(qa, *args[1:])
        elif rope_theta is None:
            o_ref, l_ref = O.decode_dual_concat(*args)
        elif rsn_lens[b] >= q_len:
            o_ref, l_ref = O.decode_dual_rotated(*args, rope_theta)
        else:
            continue          # fewer cached reasoning tokens than query rows: positions undefined
        # (the 8-bit cases scale value rows by up to 2, so outputs exceed 1: the bound follows the bf16 grid there)
        assert np.abs(to_f64(out[b]) - o_ref).max() <= 2e-2 * (max(1.0, np.abs(o_ref).max()) if fp8 else 1.0), b
        got_l = to_f64(lse[b])
        both = np.isfinite(l_ref)
        assert np.array_equal(np.isfinite(got_l), both)
        # (8-bit cases: key rows up to twice the unit scale, and the scores' rounding error with them)
        assert np.abs(got_l[both] - l_ref[both]).max(initial=0.0) <= 2e-2
    return caches, tq, out


def test_decode_small_ragged(st):
    rng = np.random.Generator(np.random.PCG64(410))
    src_lens = np.array([70, 33, 16, 300, 1]); rsn_lens = np.array([5, 100, 48, 257, 1])
    # visible source prefix: 0, page - 1, page, page + 1, everything
    src_vis = np.array([0, 15, 16, 17, 1])
    _check_decode(st, rng, 5, 4, 2, 128, src_lens, rsn_lens, src_vis)


def test_decode_head_dim_64_and_group_4(st):
    rng = np.random.Generator(np.random.PCG64(411))
    _check_decode(st, rng, 2, 8, 2, 64, np.array([100, 513]), np.array([700, 31]), np.array([100, 500]))


@pytest.mark.parametrize("q_len,hq,hkv,d,rope", [(1, 4, 2, 128, None), (4, 8, 2, 128, 1.0e6), (2, 16, 2, 64, None), (3, 4, 1, 64, 1.0e6)])
def test_decode_short_caches_one_workgroup_per_head(st, q_len, hq, hkv, d, rope):
    """Both caches together at most 1,024 tokens: one launch, the units dealt out to the waves of a workgroup and
    merged in LDS -- lengths with fewer units than waves, more units than waves, ragged ends, empty caches; up to 16
    rows (the largest LDS footprint)."""
    rng = np.random.Generator(np.random.PCG64(414 + q_len))
    src_lens = np.array([98, 0, 500, 64, 1, 130, 16]); rsn_lens = np.array([439, 5, 524, 3, 4, 890, 700])
    src_vis = np.array([98, 0, 449, 63, 0, 130, 16])
    _check_decode(st, rng, 7, hq, hkv, d, src_lens, rsn_lens, src_vis, q_len=q_len, rope_theta=rope)


def test_decode_q_len_8(st):
    rng = np.random.Generator(np.random.PCG64(412))
    _check_decode(st, rng, 3, 8, 2, 128, np.array([64, 10, 290]), np.array([8, 300, 40]), np.array([64, 0, 290]), q_len=8)


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("unit", [128, 256, 512, 1024])
def test_decode_every_unit_size(st, unit, fp8):
    """The work unit is chosen by launch size (small launches take short units); every size the rule can pick is
    pinned here on caches that span several units with ragged ends, and gives the same rows."""
    rng = np.random.Generator(np.random.PCG64(413))
    src_lens = np.array([1100, 129, 640]); rsn_lens = np.array([700, 1500, 127]); src_vis = np.array([1025, 128, 0])
    _check_decode(st, rng, 3, 4, 2, 128, src_lens, rsn_lens, src_vis, fp8=fp8, unit_tokens=unit)


# ------------------------------------------------------- 8-bit caches --
def test_kv_append_fp8_codes_and_scales_are_the_oracles(st):
    """Bytes and scales in the pools == the oracle's E4M3 codes and powers of two, bit for bit; untouched slots keep the fill."""
    rng = np.random.Generator(np.random.PCG64(440))
    for batch, hkv, d, src_lens, rsn_lens in ((3, 2, 128, np.array([70, 33, 16]), np.array([5, 100, 48])),
                                               (2, 3, 64, np.array([17, 1]), np.array([64, 31]))):
        caches, ref, (tab_s, tab_r) = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, fp8=True, row_exponents=(-14, 14))
        for which, cache, lens, tab in ((st.ST_SOURCE, caches.source, src_lens, tab_s), (st.ST_REASONING, caches.reasoning, rsn_lens, tab_r)):
            kl = st.k_pool8_to_logical(cache.k_pool).cpu().numpy(); vl = st.v_pool_to_logical(cache.v_pool).cpu().numpy()
            ksl = st.scale_to_logical(cache.k_scale).cpu().numpy(); vsl = st.scale_to_logical(cache.v_scale).cpu().numpy()
            written = np.zeros(kl.shape[:2], bool)
            for b in range(batch):
                n = int(lens[b])
                for name, pool, scl, rows in (("k", kl, ksl, ref[which][0][b, :n]), ("v", vl, vsl, ref[which][1][b, :n])):
                    codes, k = O.quantize_rows_e4m3(rows.astype(np.float64))
                    got_c = O.paged_gather(pool, tab, b, n); got_s = O.paged_gather(scl, tab, b, n)
                    # -0 and +0 are the same value: compare values where the oracle's code is a zero, bytes elsewhere
                    assert np.array_equal(got_c & 0x7f, codes & 0x7f), (which, b, name)
                    nz = (codes & 0x7f) != 0
                    assert np.array_equal(got_c[nz], codes[nz]), (which, b, name)
                    assert np.array_equal(got_s.astype(np.float64), np.ldexp(1.0, k)), (which, b, name)
                for p in range(n):
                    written[tab[b][p // 16], p % 16] = True
            assert np.all(kl[~written] == 0x7f) and np.all(vl[~written] == 0x7f)
            assert np.all(np.isnan(ksl[~written])) and np.all(np.isnan(vsl[~written]))
    # boundary rows: the largest magnitude exactly 448 2^k, just above it, 1.75 (mantissa boundary), an all-zero row
    cs, _ = make_cache(1, 2, 1, 64, rng, fp8=True); cr, _ = make_cache(1, 2, 1, 64, rng, fp8=True)
    rows = np.zeros((1, 5, 1, 64), np.float32)
    rows[0, 0, 0, :4] = [448.0, -3.0, 0.001953125, 13.0]; rows[0, 1, 0, :3] = [450.0, 1.0, -225.0]
    rows[0, 2, 0, :3] = [1.75, -1.0, 0.9375]; rows[0, 3, 0, :2] = [2.0 ** -40, 3 * 2.0 ** -44]
    dc = st.DualCache(cs, cr)
    st.st_kv_append(dc, st.ST_SOURCE, to_dev(rows, "bf16"), to_dev(-rows, "bf16"))
    torch.cuda.synchronize()
    tab = cs.page_table.cpu().numpy()
    codes, k = O.quantize_rows_e4m3(W.bf16_round(rows[0]).astype(np.float64))
    got = O.paged_gather(st.k_pool8_to_logical(cs.k_pool).cpu().numpy(), tab, 0, 5)
    assert np.array_equal(got & 0x7f, codes & 0x7f) and np.array_equal(got[(codes & 0x7f) != 0], codes[(codes & 0x7f) != 0])
    assert np.array_equal(O.paged_gather(st.scale_to_logical(cs.k_scale).cpu().numpy(), tab, 0, 5).astype(np.float64), np.ldexp(1.0, k))
    assert k[:, 0].tolist() == [0, 1, -8, -48, 0]
    gotv = O.paged_gather(st.v_pool_to_logical(cs.v_pool).cpu().numpy(), tab, 0, 5)
    assert np.array_equal(O.e4m3_decode(gotv), -O.e4m3_decode(got))


def test_decode_fp8_small_ragged(st):
    rng = np.random.Generator(np.random.PCG64(441))
    src_lens = np.array([70, 33, 16, 300, 1]); rsn_lens = np.array([5, 100, 48, 257, 1])
    src_vis = np.array([0, 15, 16, 17, 1])
    _check_decode(st, rng, 5, 4, 2, 128, src_lens, rsn_lens, src_vis, fp8=True)


def test_decode_fp8_head_dim_64_group_4_and_long_units(st):
    rng = np.random.Generator(np.random.PCG64(442))
    _check_decode(st, rng, 2, 8, 2, 64, np.array([100, 1100]), np.array([1500, 31]), np.array([100, 1030]), fp8=True)


@pytest.mark.parametrize("q_len,hq,hkv,d", [(8, 4, 2, 128), (1, 4, 2, 128), (3, 4, 1, 64)])
def test_decode_fp8_several_rows_and_fused_query_rotation(st, q_len, hq, hkv, d):
    rng = np.random.Generator(np.random.PCG64(443 + q_len + d))
    args = (3, hq, hkv, d, np.array([64, 10, 290]), np.array([8, 300, 40]), np.array([64, 0, 290]))
    _check_decode(st, rng, *args, q_len=q_len, fp8=True)
    _check_decode(st, rng, *args, q_len=q_len, fp8=True, rope_theta=1.0e6)


def test_decode_fp8_is_the_bf16_decode_of_the_stored_values(st):
    """Same tokens through an 8-bit and a bf16 cache pair holding the DEQUANTISED values: the two kernels agree to rounding."""
    rng = np.random.Generator(np.random.PCG64(447))
    batch, hq, hkv, d = 2, 4, 2, 128
    src_lens, rsn_lens = np.array([200, 77]), np.array([130, 600])
    state = rng.bit_generator.state
    c8, ref, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, fp8=True)
    rng.bit_generator.state = state
    c16, _, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens)
    rq = lambda a: O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(a.astype(np.float64))).astype(np.float32)
    for which, cache, lens in ((st.ST_SOURCE, c16.source, src_lens), (st.ST_REASONING, c16.reasoning, rsn_lens)):
        cache.appended_len.zero_()
        st.st_kv_append(c16, which, to_dev(rq(ref[which][0]), "bf16"), to_dev(rq(ref[which][1]), "bf16"),
                        torch.from_numpy(lens.astype(np.int32)).to(DEV))
    q = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
    sl = torch.from_numpy(src_lens.astype(np.int32)).to(DEV); rl = torch.from_numpy(rsn_lens.astype(np.int32)).to(DEV)
    o8 = st.st_attn_decode_dual(q, c8, sl, rl, 200, 600)
    o16 = st.st_attn_decode_dual(q, c16, sl, rl, 200, 600)
    torch.cuda.synchronize()
    assert (o8.float() - o16.float()).abs().max().item() <= 4e-3


def test_kv_append_rope_matches_oracle_and_unfused_path(st):
    """Rotate-on-append: stored keys == RoPE(k, index in the cache) of the oracle within one bf16 ulp, values
    bit-identical; and the unfused pair st_rope_apply + st_kv_append stores (almost always) the same bits."""
    rng = np.random.Generator(np.random.PCG64(420))
    theta = 1.0e6
    for batch, hkv, d, src_lens, rsn_lens in ((3, 2, 128, np.array([70, 33, 16]), np.array([5, 100, 48])),
                                               (2, 1, 64, np.array([40000, 1]), np.array([17, 3000]))):
        state = rng.bit_generator.state
        caches, ref, (tab_s, tab_r) = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, chunks=(1, 15, 17, 64, 3, 4096),
                                                 rope_theta=theta)
        rng.bit_generator.state = state                      # the same pools, tables and rows again
        caches_u, ref_u, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, chunks=(1, 15, 17, 64, 3, 4096))
        for which, cache, cache_u, lens, tab in ((st.ST_SOURCE, caches.source, caches_u.source, src_lens, tab_s),
                                                 (st.ST_REASONING, caches.reasoning, caches_u.reasoning, rsn_lens, tab_r)):
            kl = st.k_pool_to_logical(cache.k_pool).float().cpu().numpy()
            vl = st.v_pool_to_logical(cache.v_pool).float().cpu().numpy()
            for b in range(batch):
                n = int(lens[b])
                got = O.paged_gather(kl, tab, b, n).astype(np.float64)
                want = ref[which][0][b, :n]
                # one bf16 ulp (or more) of |want|, plus the fp32 rounding of the two products where they cancel
                ulp = np.abs(want) * 2.0 ** -7 + 4e-6
                assert (np.abs(got - want) <= ulp).all(), (which, b)
                assert (np.abs(got - want) <= 0.51 * ulp).mean() > 0.999          # round-to-nearest almost everywhere
                assert np.array_equal(O.paged_gather(vl, tab, b, n), ref[which][1][b, :n])
                # unfused: rotate the same rows with st_rope_apply, append with st_kv_append
                raw = to_dev(ref_u[which][0][b, :n], "bf16")
                pos = torch.arange(n, dtype=torch.int32, device=DEV)
                rot = st.st_rope_apply(raw, pos, theta).float().cpu().numpy().astype(np.float64) if n else np.zeros_like(got)
                assert (np.abs(got - rot) <= ulp).all() and (got == rot).mean() > 0.995
        assert np.array_equal(np.isnan(st.k_pool_to_logical(caches.source.k_pool).float().cpu().numpy()),
                              np.isnan(st.k_pool_to_logical(caches_u.source.k_pool).float().cpu().numpy()))


@pytest.mark.parametrize("q_len,hq,hkv,d", [(1, 4, 2, 128), (1, 8, 2, 64), (8, 8, 2, 128), (3, 4, 1, 64)])
def test_decode_rope_fused(st, q_len, hq, hkv, d):
    """Unrotated keys through st_kv_append_rope, unrotated queries through st_attn_decode_dual_rope, against the
    oracle's rotate-then-attend with position id = index in the stream."""
    rng = np.random.Generator(np.random.PCG64(430 + q_len + d))
    src_lens = np.array([70, 33, 600, 1]); rsn_lens = np.array([9, 100, 1500, 8])
    src_vis = np.array([64, 0, 600, 1])
    _check_decode(st, rng, 4, hq, hkv, d, src_lens, rsn_lens, src_vis, q_len=q_len, rope_theta=1.0e6)


@pytest.mark.parametrize("hq,hkv,d,theta,long", [(4, 2, 128, 1.0e6, False), (8, 2, 64, 1.0e6, False), (32, 8, 128, None, False),
                                                  (16, 1, 128, 1.0e6, False), (4, 2, 128, 1.0e6, True), (8, 2, 64, None, True),
                                                  (32, 1, 64, 1.0e6, True), (32, 8, 128, 1.0e6, True)])
def test_decode_append_in_one_call(st, hq, hkv, d, theta, long):
    """st_attn_decode_dual_append against the oracle (store the rotated key and the value at index rsn_len - 1, then
    attend), and against the two separate calls on a twin pair of caches: same pool bits, same lengths, rows that
    agree within rounding.  Short caches take the single fused launch; long ones the split kernel with one more slot
    for the token (up to 16 rows) or a token launch of its own (32 rows); one sequence starts with an empty reasoning
    cache, one is idle (rsn_len 0: nothing stored, source only)."""
    src_lens = np.array([98, 0, 500, 64, 1, 31]); rsn_lens = np.array([439, 7, 500, 3, 15, 0]); src_vis = np.array([98, 0, 449, 63, 0, 31])
    if long:
        src_lens = np.array([1198, 0, 500, 764, 1, 31]); rsn_lens = np.array([439, 1507, 1100, 3, 15, 0]); src_vis = np.array([1198, 0, 449, 700, 0, 31])
    batch, idle = len(src_lens), 3
    twins = []
    for _ in range(2):
        rng = np.random.Generator(np.random.PCG64(440 + d))
        twins.append(_fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra=0, rope_theta=theta))
    (ca, ref, _), (cb, _, _) = twins
    assert torch.equal(ca.reasoning.k_pool.view(torch.int16), cb.reasoning.k_pool.view(torch.int16))
    assert torch.equal(ca.reasoning.page_table, cb.reasoning.page_table)
    q = W.normal(rng, (batch, 1, hq, d), "bf16"); k_tok = W.normal(rng, (batch, 1, hkv, d), "bf16"); v_tok = W.normal(rng, (batch, 1, hkv, d), "bf16")
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k_tok, "bf16"), to_dev(v_tok, "bf16")
    new_len = rsn_lens + 1; new_len[idle] = 0
    n_new = np.ones(batch, np.int32); n_new[idle] = 0
    vis_t = torch.from_numpy(src_vis.astype(np.int32)).to(DEV); rl_t = torch.from_numpy(new_len.astype(np.int32)).to(DEV)
    max_s, max_r = int(src_lens.max()), int(new_len.max())
    lse_f = torch.empty((batch, 1, hq), dtype=torch.float32, device=DEV)
    out_f = st.st_attn_decode_dual_append(tq, tk, tv, ca, vis_t, rl_t, max_s, max_r, theta_base=theta or 0.0, lse=lse_f)
    st.st_kv_append(cb, st.ST_REASONING, tk, tv, torch.from_numpy(n_new).to(DEV), rope_theta=theta)
    out_u = st.st_attn_decode_dual(tq, cb, vis_t, rl_t, max_s, max_r, rope_theta=theta)
    torch.cuda.synchronize()
    want_len = rsn_lens + n_new
    assert ca.reasoning.appended_len.cpu().tolist() == want_len.tolist() == cb.reasoning.appended_len.cpu().tolist()
    # only slots below the lengths are defined (the rest keeps its NaN fill in both)
    for name in ("k_pool", "v_pool"):
        a, b_ = getattr(ca.reasoning, name), getattr(cb.reasoning, name)
        assert torch.equal(a.view(torch.int16), b_.view(torch.int16)), name
    assert np.abs(to_f64(out_f) - to_f64(out_u)).max() <= 1e-2
    for b in range(batch):
        L = int(rsn_lens[b])
        if b == idle:
            if theta is not None:
                continue                                  # no reasoning token: the query has no position id
            o_ref, l_ref = O.decode_dual_concat(q[b].astype(np.float64), ref[st.ST_SOURCE][0][b], ref[st.ST_SOURCE][1][b],
                                                ref[st.ST_REASONING][0][b], ref[st.ST_REASONING][1][b], int(src_vis[b]), 0)
        else:
            k_row = k_tok[b].astype(np.float64)
            if theta is not None:
                k_row = O.rope(k_row, np.array([L]), theta)
            kr = np.concatenate([ref[st.ST_REASONING][0][b][:L], k_row]); vr = np.concatenate([ref[st.ST_REASONING][1][b][:L], v_tok[b]])
            args = (q[b].astype(np.float64), ref[st.ST_SOURCE][0][b], ref[st.ST_SOURCE][1][b], kr, vr, int(src_vis[b]), L + 1)
            o_ref, l_ref = O.decode_dual_rotated(*args, theta) if theta is not None else O.decode_dual_concat(*args)
        assert np.abs(to_f64(out_f[b]) - o_ref).max() <= 2e-2, b
        assert np.abs(to_f64(lse_f[b]) - l_ref).max() <= 2e-2, b
    with pytest.raises(st.StError) as e:                  # one token per step
        st.st_attn_decode_dual_append(torch.cat([tq, tq], 1), tk, tv, ca, vis_t, rl_t, max_s, max_r)
    assert e.value.status == 5


def test_decode_append_in_one_call_random_lengths(st):
    """Twenty random shapes and length vectors around the page, unit and short-cache boundaries: the one-call step
    leaves the same pool bits and lengths as st_kv_append_rope + st_attn_decode_dual_rope on a twin pair of caches,
    and its rows agree with theirs within rounding (those calls are checked against the oracle elsewhere)."""
    rng = np.random.Generator(np.random.PCG64(450))
    specials = np.array([0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 511, 512, 513, 1023, 1024, 1025])
    for trial in range(20):
        hkv = int(rng.choice([1, 2])); group = int(rng.choice([1, 2, 4, 8, 16])); d = int(rng.choice([64, 128]))
        hq, batch = hkv * group, 4
        top = int(rng.choice([200, 900, 1500]))
        pick = lambda: np.where(rng.random(batch) < 0.5, rng.choice(specials[specials <= top], batch), rng.integers(0, top + 1, batch))
        src_lens, rsn_lens = pick(), pick()
        src_vis = np.minimum(src_lens, pick())
        theta = 1.0e6 if trial % 3 else None
        twins = []
        for _ in range(2):
            r2 = np.random.Generator(np.random.PCG64(4500 + trial))
            twins.append(_fill_dual(st, r2, batch, hkv, d, src_lens, rsn_lens, rope_theta=theta)[0])
        ca, cb = twins
        q = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
        tk = to_dev(W.normal(rng, (batch, 1, hkv, d), "bf16"), "bf16"); tv = to_dev(W.normal(rng, (batch, 1, hkv, d), "bf16"), "bf16")
        new_len = rsn_lens + 1
        vis_t = torch.from_numpy(src_vis.astype(np.int32)).to(DEV); rl_t = torch.from_numpy(new_len.astype(np.int32)).to(DEV)
        max_s, max_r = int(src_lens.max()), int(new_len.max())
        lse_f = torch.empty((batch, 1, hq), dtype=torch.float32, device=DEV); lse_u = torch.empty_like(lse_f)
        out_f = st.st_attn_decode_dual_append(q, tk, tv, ca, vis_t, rl_t, max_s, max_r, theta_base=theta or 0.0, lse=lse_f)
        st.st_kv_append(cb, st.ST_REASONING, tk, tv, rope_theta=theta)
        out_u = st.st_attn_decode_dual(q, cb, vis_t, rl_t, max_s, max_r, rope_theta=theta, lse=lse_u)
        torch.cuda.synchronize()
        tag = (trial, hq, hkv, d, src_lens.tolist(), rsn_lens.tolist())
        assert ca.reasoning.appended_len.cpu().tolist() == new_len.tolist() == cb.reasoning.appended_len.cpu().tolist(), tag
        for name in ("k_pool", "v_pool"):
            assert torch.equal(getattr(ca.reasoning, name).view(torch.int16), getattr(cb.reasoning, name).view(torch.int16)), (name, tag)
        assert (out_f.float() - out_u.float()).abs().max().item() <= 1e-2, tag
        assert (lse_f - lse_u).abs().max().item() <= 1e-2, tag


def test_decode_wave_timeline_changes_no_result(st):
    """st_profile_wave_trace: every workgroup of the split kernel's launch leaves a (start, end) pair of the wall clock in
    the caller's buffer; the step's output keeps its bits; without timing enabled nothing is written."""
    rng = np.random.Generator(np.random.PCG64(460))
    batch, hq, hkv, d = 3, 8, 2, 128
    src_lens = np.array([1500, 40, 700]); rsn_lens = np.array([900, 2100, 0])
    caches, _, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens)
    tq = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
    vis = torch.from_numpy(src_lens.astype(np.int32)).to(DEV); rl = torch.from_numpy(rsn_lens.astype(np.int32)).to(DEV)
    max_s, max_r = int(src_lens.max()), int(rsn_lens.max())
    ref = st.st_attn_decode_dual(tq, caches, vis, rl, max_s, max_r)
    buf = torch.zeros((4096, 2), dtype=torch.int64, device=DEV)
    st.st_profile_wave_trace(buf)
    out_off = st.st_attn_decode_dual(tq, caches, vis, rl, max_s, max_r)       # timing not enabled: no stamps
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0
    st.st_profile_enable(True)
    try:
        out_on = st.st_attn_decode_dual(tq, caches, vis, rl, max_s, max_r)
    finally:
        st.st_profile_enable(False)
        st.st_profile_wave_trace(None)
    torch.cuda.synchronize()
    st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    assert torch.equal(ref, out_off) and torch.equal(ref, out_on)
    a = buf.cpu().numpy()
    n = int((a[:, 1] > 0).sum())
    # one workgroup per (sequence, KV head, unit slot of either cache): a multiple of batch x heads, all stamped, contiguous
    assert n > 0 and n % (batch * hkv) == 0 and (a[:n, 1] > 0).all() and (a[n:] == 0).all()
    assert (a[:n, 1] >= a[:n, 0]).all()
    assert (a[:n, 1].max() - a[:n, 0].min()) < 100 * 1000 * 100             # the launch took less than 100 ms of the 100 MHz clock
    # a buffer shorter than the launch: only its pairs are written
    small = torch.zeros((16, 2), dtype=torch.int64, device=DEV)
    st.st_profile_wave_trace(small[:10])
    st.st_profile_enable(True)
    try:
        out_small = st.st_attn_decode_dual(tq, caches, vis, rl, max_s, max_r)
    finally:
        st.st_profile_enable(False)
        st.st_profile_wave_trace(None)
    torch.cuda.synchronize()
    st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    assert torch.equal(ref, out_small)
    b2 = small.cpu().numpy()
    assert (b2[:10, 1] > 0).all() and (b2[10:] == 0).all()


def test_decode_empty_row(st):
    """Both lengths zero: out = 0, lse = -inf."""
    rng = np.random.Generator(np.random.PCG64(413))
    cs, _ = make_cache(2, 2, 2, 128, rng, fill=float("nan")); cr, _ = make_cache(2, 2, 2, 128, rng, fill=float("nan"))
    caches = st.DualCache(cs, cr)
    kn = to_dev(W.normal(rng, (2, 3, 2, 128), "bf16"), "bf16")
    st.st_kv_append(caches, st.ST_REASONING, kn, kn, torch.tensor([3, 0], dtype=torch.int32, device=DEV))
    q = to_dev(W.normal(rng, (2, 1, 4, 128), "bf16"), "bf16")
    lse = torch.empty((2, 1, 4), dtype=torch.float32, device=DEV)
    zero = torch.zeros(2, dtype=torch.int32, device=DEV)
    out = st.st_attn_decode_dual(q, caches, zero, torch.tensor([3, 0], dtype=torch.int32, device=DEV), 32, 32, lse=lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out[1] == 0).all() and torch.isinf(lse[1]).all() and torch.isfinite(lse[0]).all()


def test_decode_ignores_poison_beyond_lens(st):
    """NaN bit patterns in slots that are not visible must not reach the output: the pools start
    NaN-filled, so the unwritten tail of each last page (source: slots 8..15 of page 2; reasoning:
    slots 1..15 / 7..15) is poison sitting right next to visible data."""
    rng = np.random.Generator(np.random.PCG64(414))
    src_lens = np.array([40, 64]); rsn_lens = np.array([33, 7]); src_vis = np.array([40, 48])
    caches, tq, out = _check_decode(st, rng, 2, 4, 2, 128, src_lens, rsn_lens, src_vis)
    assert torch.isfinite(out).all()


def test_decode_concurrent_append_is_bitwise_serial(st):
    """Source append on a second stream while decoding: same bits as the serial order."""
    rng = np.random.Generator(np.random.PCG64(415))
    batch, hq, hkv, d = 4, 4, 2, 128
    src_lens = np.array([200, 64, 130, 17]); rsn_lens = np.array([300, 50, 7, 260])
    caches, ref, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra=64)
    q = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
    vis = torch.from_numpy(src_lens.astype(np.int32)).to(DEV); rl = torch.from_numpy(rsn_lens.astype(np.int32)).to(DEV)
    serial = st.st_attn_decode_dual(q, caches, vis, rl, int(src_lens.max()), int(rsn_lens.max()))
    torch.cuda.synchronize()
    kn = to_dev(W.normal(rng, (batch, 64, hkv, d), "bf16"), "bf16")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.st_kv_append(caches, st.ST_SOURCE, kn, kn, stream=side)
    conc = st.st_attn_decode_dual(q, caches, vis, rl, int(src_lens.max()), int(rsn_lens.max()))
    torch.cuda.synchronize()
    assert torch.equal(serial, conc)
    assert caches.source.appended_len.cpu().tolist() == (src_lens + 64).tolist()


def test_decode_equals_last_prefill_row(st):
    """The two halves of the path agree: decode over caches filled from a prefill's K/V == that prefill's last row."""
    cfg = W.random_prefill(420, 1, 6, (5, 40), (5, 60), 4, 2, 128, "bf16", layout="grouped")
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    out = st.st_attn_prefill(tq, tk, tv, plan)
    S = int((cfg.stream_ids == O.SRC).sum()); R = cfg.n_tokens - S
    rng = np.random.Generator(np.random.PCG64(421))
    cs, _ = make_cache(1, (S + 15) // 16, 2, 128, rng); cr, _ = make_cache(1, (R + 15) // 16, 2, 128, rng)
    caches = st.DualCache(cs, cr)
    st.st_kv_append(caches, st.ST_SOURCE, tk[:S][None].contiguous(), tv[:S][None].contiguous())
    st.st_kv_append(caches, st.ST_REASONING, tk[S:][None].contiguous(), tv[S:][None].contiguous())
    one = lambda x: torch.tensor([x], dtype=torch.int32, device=DEV)
    dec = st.st_attn_decode_dual(tq[-1][None, None].contiguous(), caches, one(S), one(R), S, R)
    torch.cuda.synchronize()
    assert (dec[0, 0].float() - out[-1].float()).abs().max().item() <= 2e-2


def test_decode_workspace_reuse(st):
    """One workspace (never cleared, garbage at first) serves many calls of different shapes."""
    rng = np.random.Generator(np.random.PCG64(430))
    batch, hq, hkv, d = 3, 4, 2, 128
    src_lens = np.array([600, 40, 257]); rsn_lens = np.array([30, 900, 512])
    caches, ref, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens)
    need = st.st_decode_workspace_bytes(batch, hq, hkv, d, 1, 600, 900)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=DEV)
    q = W.normal(rng, (batch, 1, hq, d), "bf16")
    tq = to_dev(q, "bf16")
    for vis, rl in ((src_lens, rsn_lens), (np.array([100, 0, 256]), np.array([1, 700, 255])), (src_lens, rsn_lens)):
        out = st.st_attn_decode_dual(tq, caches, torch.from_numpy(vis.astype(np.int32)).to(DEV),
                                     torch.from_numpy(rl.astype(np.int32)).to(DEV), 600, 900, workspace=ws)
        torch.cuda.synchronize()
        for b in range(batch):
            o_ref, _ = O.decode_dual_concat(q[b], ref[st.ST_SOURCE][0][b], ref[st.ST_SOURCE][1][b], ref[st.ST_REASONING][0][b],
                                            ref[st.ST_REASONING][1][b], int(vis[b]), int(rl[b]))
            assert np.abs(to_f64(out[b]) - o_ref).max() <= 2e-2, b


def test_whole_step_replays_from_a_hip_graph(st):
    """Nothing on the path allocates or waits: plan build, rotation, prefill, appends, decode and the source chunk are
    recorded into one HIP graph; every replay -- with eager work of the same kind in between -- reproduces the eager
    step bit for bit."""
    rng = np.random.Generator(np.random.PCG64(431))
    cfg = W.random_prefill(432, 2, 5, (10, 70), (10, 90), 4, 2, 128, "bf16")
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    q0, k0, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    tq, tk = torch.empty_like(q0), torch.empty_like(k0)
    n, hq, hkv, d, batch = cfg.n_tokens, 4, 2, 128, 2
    plan_ws = torch.empty(st.st_plan_workspace_bytes(cfg.batch, n), dtype=torch.uint8, device=DEV)
    out = torch.empty_like(q0); lse = torch.empty((n, hq), dtype=torch.float32, device=DEV)
    src_lens = np.array([300, 37]); rsn_lens = np.array([129, 560])
    caches, _, _ = _fill_dual(st, rng, batch, hkv, d, src_lens, rsn_lens, src_extra=64)
    base_s, base_r = caches.source.appended_len.clone(), caches.reasoning.appended_len.clone()
    k_tok = to_dev(W.normal(rng, (batch, 1, hkv, d), "bf16"), "bf16"); v_tok = to_dev(W.normal(rng, (batch, 1, hkv, d), "bf16"), "bf16")
    q_tok = to_dev(W.normal(rng, (batch, 1, hq, d), "bf16"), "bf16")
    k_src = to_dev(W.normal(rng, (batch, 20, hkv, d), "bf16"), "bf16"); q_src = to_dev(W.normal(rng, (batch, 20, hq, d), "bf16"), "bf16")
    vis = torch.from_numpy(src_lens.astype(np.int32)).to(DEV); rl = torch.from_numpy((rsn_lens + 1).astype(np.int32)).to(DEV)
    sl = torch.from_numpy((src_lens + 20).astype(np.int32)).to(DEV)
    o_dec = torch.empty_like(q_tok); o_src = torch.empty_like(q_src)
    dws = torch.empty(st.st_decode_workspace_bytes(batch, hq, hkv, d, 1, 320, 561), dtype=torch.uint8, device=DEV)
    cws = torch.empty(st.st_source_chunk_workspace_bytes(batch, hq, hkv, d, 20, 320), dtype=torch.uint8, device=DEV)
    plan0 = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws)
    pws = torch.empty(st.st_prefill_workspace_bytes(plan0, hkv, d, st.ST_BF16), dtype=torch.uint8, device=DEV)
    plan0.destroy()
    plans = []

    def step():
        caches.source.appended_len.copy_(base_s); caches.reasoning.appended_len.copy_(base_r)
        plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws)
        plans.append(plan)
        st.st_rope_apply(q0, pos, cfg.theta, out=tq); st.st_rope_apply(k0, pos, cfg.theta, out=tk)
        st.st_attn_prefill(tq, tk, tv, plan, out=out, lse=lse, workspace=pws)
        # (a bound on the lengths from the host: no read-back of the device counters, which a capture forbids)
        st.st_kv_append(caches, st.ST_REASONING, k_tok, v_tok, rope_theta=cfg.theta, host_len_upper_bound=561)
        st.st_attn_decode_dual(q_tok, caches, vis, rl, 320, 561, out=o_dec, workspace=dws, rope_theta=cfg.theta)
        st.st_kv_append(caches, st.ST_SOURCE, k_src, k_src, rope_theta=cfg.theta, host_len_upper_bound=320)
        st.st_attn_source_chunk(q_src, caches, sl, 320, out=o_src, workspace=cws, rope_theta=cfg.theta)

    step(); torch.cuda.synchronize()
    want = [t.clone() for t in (out, lse, o_dec, o_src)]
    # (plans of earlier tests that own device memory free it when Python collects them: not during the capture)
    gc.collect()
    gc.disable()
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    finally:
        gc.enable()
    torch.cuda.synchronize()
    for _ in range(3):
        for t in (out, lse, o_dec, o_src):
            t.fill_(float("nan"))
        graph.replay(); torch.cuda.synchronize()
        for got, ref in zip((out, lse, o_dec, o_src), want):
            assert torch.equal(got, ref)
        step(); torch.cuda.synchronize()                  # eager work between the replays


# ------------------------------------------------- source-chunk prefill --
def _check_source_chunk(st, rng, batch, hq, hkv, d, src_before, n_new, max_new, rope_theta=None):
    """Append a ragged chunk to the source cache, then let its tokens attend over the cache.
    With rope_theta, keys and queries go in UNROTATED through the fused entry points."""
    src_before = np.asarray(src_before); n_new = np.asarray(n_new)
    total = src_before + n_new
    pages = (int(total.max()) + 15) // 16 + 1
    cs, _ = make_cache(batch, pages, hkv, d, rng, fill=float("nan")); cr, _ = make_cache(batch, 1, hkv, d, rng, fill=float("nan"))
    caches = st.DualCache(cs, cr)
    kk = W.normal(rng, (batch, int(total.max()), hkv, d), "bf16"); vv = W.normal(rng, (batch, int(total.max()), hkv, d), "bf16")
    # history first, then the chunk (two appends, as Alg. 1 does sentence by sentence)
    hist = int(src_before.max())
    if hist:
        st.st_kv_append(caches, st.ST_SOURCE, to_dev(kk[:, :hist], "bf16"), to_dev(vv[:, :hist], "bf16"),
                        torch.from_numpy(src_before.astype(np.int32)).to(DEV), rope_theta=rope_theta)
    kn = np.zeros((batch, max_new, hkv, d), np.float32); vn = np.zeros_like(kn)
    for b in range(batch):
        kn[b, :n_new[b]] = kk[b, src_before[b]:total[b]]; vn[b, :n_new[b]] = vv[b, src_before[b]:total[b]]
        kk[b, :total[b]] = np.concatenate([kk[b, :src_before[b]], kn[b, :n_new[b]]]); vv[b, :total[b]] = np.concatenate([vv[b, :src_before[b]], vn[b, :n_new[b]]])
    nn = torch.from_numpy(n_new.astype(np.int32)).to(DEV)
    st.st_kv_append(caches, st.ST_SOURCE, to_dev(kn, "bf16"), to_dev(vn, "bf16"), nn, rope_theta=rope_theta)
    q = W.normal(rng, (batch, max_new, hq, d), "bf16")
    tq = to_dev(q, "bf16")
    lse = torch.full((batch, max_new, hq), 7.0, dtype=torch.float32, device=DEV)
    out = torch.full_like(tq, 3.0)
    st.st_attn_source_chunk(tq, caches, torch.from_numpy(total.astype(np.int32)).to(DEV), int(total.max()), n_new=nn, out=out, lse=lse,
                            rope_theta=rope_theta)
    torch.cuda.synchronize()
    assert cs.appended_len.cpu().tolist() == total.tolist()
    for b in range(batch):
        nb = int(n_new[b])
        if nb and rope_theta is not None:
            k_rot = O.rope(kk[b, :total[b]].astype(np.float64), np.arange(total[b]), rope_theta)
            o_ref, l_ref = O.source_chunk_attention_rotated(q[b, :nb].astype(np.float64), k_rot, vv[b], int(total[b]), rope_theta)
            assert np.abs(to_f64(out[b, :nb]) - o_ref).max() <= 2e-2, b
            assert np.abs(to_f64(lse[b, :nb]) - l_ref).max() <= 2e-2, b
        elif nb:
            o_ref, l_ref = O.source_chunk_attention(q[b, :nb], kk[b], vv[b], int(total[b]))
            assert np.abs(to_f64(out[b, :nb]) - o_ref).max() <= 2e-2, b
            assert np.abs(to_f64(lse[b, :nb]) - l_ref).max() <= 2e-2, b
        # rows past n_new[b] are not written
        assert (out[b, nb:] == 3.0).all() and (lse[b, nb:] == 7.0).all()


def test_source_chunk_small_ragged(st):
    rng = np.random.Generator(np.random.PCG64(440))
    # first sentence (empty cache), mid-page starts, a chunk crossing the 512-token split, an empty chunk
    _check_source_chunk(st, rng, 5, 4, 2, 128, [0, 5, 500, 33, 100], [7, 16, 40, 0, 1], 40)


def test_source_chunk_many_row_blocks(st):
    """64 tokens x group 4 = 256 (token, head) rows = 8 blocks of 32; head_dim 64 as well."""
    rng = np.random.Generator(np.random.PCG64(441))
    _check_source_chunk(st, rng, 2, 8, 2, 128, [1000, 17], [64, 61], 64)
    _check_source_chunk(st, rng, 2, 4, 4, 64, [70, 0], [33, 64], 64)


def test_source_chunk_unit_order(st):
    """The work units of a launch go longest first (a rank worked out from the lengths by every workgroup) for up to
    256 (sequence, unit) pairs and in index order beyond: a batch on either side, lengths from empty to several
    units, equal lengths among them (ties)."""
    rng = np.random.Generator(np.random.PCG64(445))
    before = [0, 1500, 300, 300, 5000, 64, 4096, 300, 2047, 9]
    _check_source_chunk(st, rng, len(before), 4, 2, 128, before, [8] * len(before), 8)
    before = list(rng.integers(0, 700, size=300))
    before[17] = 0; before[18] = before[19] = 333
    _check_source_chunk(st, rng, 300, 2, 1, 64, before, list(rng.integers(0, 5, size=300)), 4)


def test_source_chunk_rope_fused(st):
    """Unrotated keys and queries through st_kv_append_rope + st_attn_source_chunk_rope."""
    rng = np.random.Generator(np.random.PCG64(444))
    _check_source_chunk(st, rng, 5, 4, 2, 128, [0, 5, 500, 33, 100], [7, 16, 40, 0, 1], 40, rope_theta=1.0e6)
    _check_source_chunk(st, rng, 2, 4, 4, 64, [70, 0], [33, 64], 64, rope_theta=1.0e4)


def test_source_chunk_equals_prefill_source_rows(st):
    """The streaming path agrees with the batch path: chunk prefill over the cache == the same source rows of st_attn_prefill."""
    cfg = W.random_prefill(442, 1, 6, (20, 50), (5, 30), 4, 2, 128, "bf16", layout="interleaved")
    q, k, v = cfg.tensors()
    seg, strm, pos = ids_to_dev(cfg)
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    out = st.st_attn_prefill(tq, tk, tv, plan)
    src = torch.from_numpy(np.nonzero(cfg.stream_ids == O.SRC)[0]).to(DEV)
    S = len(src); last = int(cfg.src_lens[0][-1])         # the last sentence arrives as a chunk
    rng = np.random.Generator(np.random.PCG64(443))
    cs, _ = make_cache(1, (S + 15) // 16, 2, 128, rng); cr, _ = make_cache(1, 1, 2, 128, rng)
    caches = st.DualCache(cs, cr)
    st.st_kv_append(caches, st.ST_SOURCE, tk[src][None].contiguous(), tv[src][None].contiguous())
    one = torch.tensor([S], dtype=torch.int32, device=DEV)
    got = st.st_attn_source_chunk(tq[src[S - last:]][None].contiguous(), caches, one, S)
    torch.cuda.synchronize()
    assert (got[0].float() - out[src[S - last:]].float()).abs().max().item() <= 2e-2
