#!/usr/bin/env python3
"""Benchmark of the streaming-constrained attention path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
  plan build -> RoPE(q, k) -> tile packing + streaming-mask prefill attention   (configs[3]: Qwen3-4B-shaped layer,
  batch 8 x 16,384 tokens, 32/8 heads, D = 128, bf16, source segments of 64-192 and reasoning segments of 64-256 tokens)
  -> paged append of a 64-token source chunk (second stream) and of one reasoning token
  -> dual-cache decode of that token over the batch's own source / reasoning caches.
`value` is the effective (unmasked) prefill FLOPs divided by the WHOLE step time.  The decode half of the metric is
measured in the same run on configs[4] (Qwen3-8B-shaped streaming step: 36 layers, 64 streams, source caches to 8K and
reasoning caches to 16K tokens, a 32-token source chunk appended per layer beside 8 decoded tokens) and reported in the
"decode" object as GB/s of algorithmic cache bytes.

Further objects of the same line (all by default; --no-extras leaves out those marked *): "stages" (every stage of the
step timed alone, the HBM-bound ones with a roofline of their own), "prefill_small" (the same step on configs[1]),
"decode_small" (configs[2]: 28 layers, batch 32, with its concurrent source appends), "source_chunk" (Alg. 1's prefill loop
on the streaming shape), "decode_fp8"* (8-bit caches), "prefill_backward"* (gradients), "stream_session"* (Alg. 1 end to
end), "probes"* (what the machine sustains for the two kernels' access pattern / instruction).

Prints ONE JSON line.  All inputs are seeded, synthetic and resident in HBM before timing starts.
"""
import argparse
import contextlib
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E

# launches of a timed kernel between its two events (st_profile_repeat): a pair of events around a single launch adds
# several microseconds of dispatch and completion that are no part of the kernel and that a kernel trace does not count
PROF_REPEAT = 8
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_kernel.txt")


def measured_traffic(key):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by what the counters read for a plain copy) of one kernel on
    one workload, from the lines `traffic <key> fetch_bytes=.. write_bytes=..` of the tracked rocprofv3 summary; None if
    the summary has no such line.  The figure is from the profiled run that wrote the summary, not from this run."""
    try:
        for l in open(TRAFFIC_PROFILE):
            f = l.split()
            if len(f) >= 4 and f[0] == "traffic" and f[1] == key:
                kv = dict(x.split("=") for x in f[2:])
                return float(kv["fetch_bytes"]) + float(kv["write_bytes"])
    except OSError:
        pass
    return None


def _median(xs):
    return float(np.median(np.asarray(xs, dtype=np.float64)))


@contextlib.contextmanager
def _no_gc():
    """Around a graph capture: Python must not collect, inside it, an object whose destructor frees device memory
    (a plan that owns its workspace does) -- that would invalidate the capture."""
    gc.collect()
    was = gc.isenabled()
    gc.disable()
    try:
        yield
    finally:
        if was:
            gc.enable()


@contextlib.contextmanager
def _leg(line, name, torch):
    """An additional leg must not cost the line its main figures: a failure is reported in the leg's place."""
    try:
        yield
    except Exception as exc:                               # noqa: BLE001
        line[name] = {"error": f"{type(exc).__name__}: {exc}"}
        print(f"bench.py: leg '{name}' failed: {type(exc).__name__}: {exc}", file=sys.stderr)
        torch.cuda.empty_cache()


def _time_launch_modes(torch, steps, graph, eager_step):
    """Wall time per step of `steps` graph replays (if a verified graph is given) and of `steps` plain launches of the
    same step; returns ({launch mode: seconds per step}, the faster mode)."""
    times = {}
    for mode, run in (("hip-graph", graph.replay if graph is not None else None), ("eager", eager_step)):
        if run is None:
            continue
        run(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        times[mode] = (time.perf_counter() - t0) / steps
    return times, min(times, key=times.get)


def _event_ms(torch, fn, reps, warm=2):
    """Mean duration of fn() (a few launches on the current stream) over `reps` calls, from events on that stream."""
    for _ in range(warm):
        fn()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record(); torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def bench_prefill_step(st, torch, W, cfg, steps, warmup, use_graph=True, fused_rope=False, stage_reps=10):
    dev = "cuda"
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    n, batch = cfg.n_tokens, cfg.batch
    g = torch.Generator(device=dev); g.manual_seed(cfg.seed)
    q = torch.randn((n, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((n, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((n, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    seg = torch.from_numpy(cfg.segment_ids).to(dev); strm = torch.from_numpy(cfg.stream_ids).to(dev)
    pos = torch.from_numpy(cfg.positions).to(dev)
    q_rot = torch.empty_like(q); k_rot = torch.empty_like(k); out = torch.empty_like(q)
    plan_ws = torch.empty(st.st_plan_workspace_bytes(batch, n), dtype=torch.uint8, device=dev)

    # the batch's own caches: source / reasoning K, V of each sequence, paged with shuffled ids
    S = np.array([int(s.sum()) for s in cfg.src_lens]); R = np.array([int(r.sum()) for r in cfg.rsn_lens])
    chunk = 64
    pages_s = (int(S.max()) + chunk + 15) // 16; pages_r = (int(R.max()) + 1 + 15) // 16
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    cs = st.KVCache(batch * pages_s, batch, pages_s, hkv, d, torch.from_numpy(W.shuffled_page_table(rng, batch, pages_s)).to(dev))
    cr = st.KVCache(batch * pages_r, batch, pages_r, hkv, d, torch.from_numpy(W.shuffled_page_table(rng, batch, pages_r)).to(dev))
    caches = st.DualCache(cs, cr)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws, validate=True)
    st.st_rope_apply(k, pos, cfg.theta, out=k_rot)
    perm = torch.from_numpy(plan.compact_index().astype(np.int64)).to(dev)
    for which, lens, off in ((st.ST_SOURCE, S, 0), (st.ST_REASONING, R, 1)):
        mx = int(lens.max())
        kn = torch.zeros((batch, mx, hkv, d), dtype=torch.bfloat16, device=dev); vn = torch.zeros_like(kn)
        for b in range(batch):
            c0 = int(cfg.cu_seqlens[b]) + (0 if off == 0 else int(S[b]))
            idx = perm[c0:c0 + int(lens[b])]
            kn[b, :int(lens[b])] = k_rot[idx]; vn[b, :int(lens[b])] = v[idx]
        st.st_kv_append(caches, which, kn, vn, torch.from_numpy(lens.astype(np.int32)).to(dev))
        del kn, vn
    torch.cuda.synchronize()
    pairs = plan.visible_pairs()
    assert [int(x) for x in pairs] == cfg.closed_form_pairs()
    pre_ws = torch.empty(st.st_prefill_workspace_bytes(plan, hkv, d, st.ST_BF16), dtype=torch.uint8, device=dev)
    flops = 4.0 * d * hq * float(pairs.sum())
    two_heads = (n // batch >= 8192) and (hq // hkv) % 2 == 0            # the library's own choice (st_plan_heads_per_workgroup)
    plan.destroy()

    len_s0 = cs.appended_len.clone(); len_r0 = cr.appended_len.clone()
    src_vis = len_s0.clone(); rsn_len = (len_r0 + 1).contiguous()
    k_src_new = torch.randn((batch, chunk, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_src_new = torch.randn((batch, chunk, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q_tok = torch.randn((batch, 1, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_tok = torch.randn((batch, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_tok = torch.randn((batch, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out_tok = torch.empty_like(q_tok)
    max_s, max_r = int(S.max()), int(R.max()) + 1
    dec_ws = torch.empty(st.st_decode_workspace_bytes(batch, hq, hkv, d, 1, max_s, max_r), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()

    def step(i_timed):
        # (the stream the step is issued on: torch's current stream now -- under graph capture that is the capturing
        # stream, and only streams that wait on IT become part of the graph)
        main = torch.cuda.current_stream()
        cs.appended_len.copy_(len_s0); cr.appended_len.copy_(len_r0)      # same state every step
        side.wait_stream(main)
        with torch.cuda.stream(side):
            # the plan needs the ids only: it is built beside the rotation (the attention call orders itself against the
            # build); then the arriving source chunk (Alg. 1, prefill loop)
            p = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws, stream=side)
            st.st_kv_append(caches, st.ST_SOURCE, k_src_new, v_src_new, host_len_upper_bound=max_s + chunk, stream=side)
        if fused_rope:
            # rotation inside the attention call: keys on their way into the key tiles, queries as they are loaded
            st.st_attn_prefill_rope(q, k, v, pos, cfg.theta, p, out=out, workspace=pre_ws)
        else:
            st.st_rope_apply_qk(q, k, pos, cfg.theta, q_out=q_rot, k_out=k_rot)      # queries and keys in one launch
            st.st_attn_prefill(q_rot, k_rot, v, p, out=out, workspace=pre_ws)
        # the decoded token: key rotated on its way into the reasoning cache, query rotated inside the decode
        # kernel, both by the token's index in the reasoning stream (its position id)
        st.st_attn_decode_dual_append(q_tok, k_tok, v_tok, caches, src_vis, rsn_len, max_s, max_r, theta_base=cfg.theta, out=out_tok,
                                      workspace=dec_ws)
        main.wait_stream(side)
        return p

    plans = []
    for _ in range(warmup):
        plans.append(step(None))
    torch.cuda.synchronize()
    # kernel-only durations of the packing and the attention kernel (HIP events on their launch stream), from eager steps
    st.st_profile_enable(True)
    n_prof = min(steps, 10)
    for i in range(n_prof):
        plans.append(step(i))
    torch.cuda.synchronize()
    st.st_profile_enable(False)
    kern_ms, n_rec = st.st_profile_read(st.ST_PROF_PREFILL_ATTN)
    pack_ms, _ = st.st_profile_read(st.ST_PROF_TILE_PACK)
    st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    assert n_rec == n_prof
    # every stage alone (events on the stream; the launches of one stage back to back)
    p_stage = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws)
    plans.append(p_stage)
    stage_ms = {
        "plan": _event_ms(torch, lambda: plans.append(st.st_plan_create(seg, strm, pos, cfg.cu_seqlens, workspace=plan_ws)), stage_reps),
        "rope_qk": _event_ms(torch, lambda: st.st_rope_apply_qk(q, k, pos, cfg.theta, q_out=q_rot, k_out=k_rot), stage_reps),
        "append_source_chunk": _event_ms(torch, lambda: (cs.appended_len.copy_(len_s0),
                                                         st.st_kv_append(caches, st.ST_SOURCE, k_src_new, v_src_new, host_len_upper_bound=max_s + chunk)), stage_reps),
        "length_reset_only": _event_ms(torch, lambda: cs.appended_len.copy_(len_s0), stage_reps),
        "decode_token_with_append": _event_ms(torch, lambda: (cr.appended_len.copy_(len_r0),
                                                              st.st_attn_decode_dual_append(q_tok, k_tok, v_tok, caches, src_vis, rsn_len, max_s, max_r, theta_base=cfg.theta,
                                                                                            out=out_tok, workspace=dec_ws)), stage_reps),
        "tile_pack": pack_ms, "attention": kern_ms,
    }
    stage_ms["append_source_chunk"] = max(stage_ms["append_source_chunk"] - stage_ms.pop("length_reset_only"), 1e-6)
    # the timed steps, two ways: the whole step (two streams) recorded once into a HIP graph and replayed -- every
    # replay first checked against the eager step, side stream included -- and as plain launches; the faster one is
    # the step time, both are reported (graphs with a second branch replay slowly on this ROCm)
    mode, graph = "eager", None
    if use_graph:
        try:
            ref_out, ref_tok = out.clone(), out_tok.clone()
            graph = torch.cuda.CUDAGraph()
            with _no_gc(), torch.cuda.graph(graph):
                plans.append(step(None))
            for _ in range(3):
                out.zero_(); out_tok.zero_()
                graph.replay()
                torch.cuda.synchronize()
                if not (torch.equal(ref_out, out) and torch.equal(ref_tok, out_tok)):
                    raise RuntimeError("graph replay differs from the eager step")
                if not torch.equal(cs.appended_len, len_s0 + chunk):       # the side stream's append is part of the replay
                    raise RuntimeError("graph replay did not run the source append")
                plans.append(step(None))
                torch.cuda.synchronize()
            del ref_out, ref_tok
            mode = "hip-graph"
        except Exception as exc:                           # noqa: BLE001
            print(f"bench.py: HIP graph capture not used ({exc}); timing eager launches", file=sys.stderr)
            graph = None
    times, mode = _time_launch_modes(torch, steps, graph, lambda: plans.append(step(None)))
    for p in plans:
        p.destroy()
    elt = 2                                                 # bytes per bf16 element
    stage_bytes = {"rope_qk": 2.0 * n * (hq + hkv) * d * elt,                          # read + write of q and k
                   "tile_pack": 2.0 * 2.0 * n * hkv * d * elt,                          # k, v read; K tiles, V^T tiles written
                   "append_source_chunk": 2.0 * 2.0 * batch * chunk * hkv * d * elt}    # k, v rows read and stored
    return {"cfg": cfg, "flops": flops, "sec_per_step": times[mode], "prefill_kernel_ms": kern_ms, "n_tokens": n, "mode": mode,
            "sec_per_step_by_launch": times, "stage_ms": stage_ms, "stage_bytes": stage_bytes, "two_heads": two_heads}


def bench_prefill_zero_inputs(st, torch, W, reps):
    """The attention stage of configs[3] on random inputs and, the same launches, on ALL-ZERO inputs: the same instruction
    stream with no operand bits toggling -- how much of the time is the power limit and not the schedule."""
    dev = "cuda"
    cfg = W.config4a()
    hq, hkv, d, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_tokens
    g = torch.Generator(device=dev); g.manual_seed(cfg.seed)
    q = torch.randn((n, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((n, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((n, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    seg = torch.from_numpy(cfg.segment_ids).to(dev); strm = torch.from_numpy(cfg.stream_ids).to(dev)
    pos = torch.from_numpy(cfg.positions).to(dev)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    flops = 4.0 * d * hq * float(plan.visible_pairs().sum())
    out = torch.empty_like(q)
    ws = torch.empty(st.st_prefill_workspace_bytes(plan, hkv, d, st.ST_BF16), dtype=torch.uint8, device=dev)
    res = {}
    for name in ("random", "zero"):
        if name == "zero":
            q.zero_(); k.zero_(); v.zero_()
        for _ in range(2):
            st.st_attn_prefill(q, k, v, plan, out=out, workspace=ws)
        torch.cuda.synchronize()
        st.st_profile_read(st.ST_PROF_PREFILL_ATTN)
        st.st_profile_enable(True)
        for _ in range(reps):
            st.st_attn_prefill(q, k, v, plan, out=out, workspace=ws)
        torch.cuda.synchronize()
        st.st_profile_enable(False)
        res[name], _ = st.st_profile_read(st.ST_PROF_PREFILL_ATTN)
        st.st_profile_read(st.ST_PROF_TILE_PACK)
    plan.destroy()
    return {"kernel_ms": res["random"], "zero_input_kernel_ms": res["zero"], "flops": flops}


def bench_stream_session(st, torch, W, time_scale):
    """Alg. 1 end to end over the attention path: one stream shaped like the paper's efficiency experiment
    (Table 4: about 70 words read at 0.4 s per word in 4.65 sentences, 439 decoded tokens; Qwen3-4B-shaped layers),
    arrival times compressed by `time_scale`.  Streaming (two loops), alternating and batch schedules."""
    dev = "cuda"
    n_layers, hq, hkv, d, batch, theta = 36, 32, 8, 128, 1, 1.0e6
    words = [15, 15, 15, 15, 10]                       # 70 words, five sentences
    s = [int(round(1.3 * w)) + 1 for w in words]       # tokens: about 1.3 per word, plus the boundary token
    r = [94, 94, 94, 94, 63]                           # 439 decoded tokens
    arrival = (0.4 * np.cumsum(words) * time_scale).tolist()
    g = torch.Generator(device=dev); g.manual_seed(5)
    rnd = lambda *shape: torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    S, R = sum(s), sum(r)
    sq, sk, sv = rnd(S * batch * hq * d), rnd(S * batch * hkv * d), rnd(S * batch * hkv * d)
    rq, rk, rv = rnd(R, batch, hq, d), rnd(R, batch, hkv, d), rnd(R, batch, hkv, d)
    rng = np.random.Generator(np.random.PCG64(5))

    def layers():
        out = []
        for _ in range(n_layers):
            ps, pr = (S + 15) // 16 + 1, (R + 15) // 16 + 1
            cs = st.KVCache(batch * ps, batch, ps, hkv, d, torch.from_numpy(W.shuffled_page_table(rng, batch, ps)).to(dev))
            cr = st.KVCache(batch * pr, batch, pr, hkv, d, torch.from_numpy(W.shuffled_page_table(rng, batch, pr)).to(dev))
            out.append(st.DualCache(cs, cr))
        return out

    res = {}
    st.st_stream_run(st.ST_SCHED_SERIAL, layers(), hq, s, r, sq, sk, sv, rq, rk, rv, theta)          # warm-up
    for name, mode in (("streaming", st.ST_SCHED_STREAMING), ("alternating", st.ST_SCHED_SERIAL), ("batch", st.ST_SCHED_BATCH)):
        _, _, rep = st.st_stream_run(mode, layers(), hq, s, r, sq, sk, sv, rq, rk, rv, theta, arrival_s=arrival)
        res[name] = rep
    # the same alternating session with plain launches for every decoded token (no graph replay)
    _, _, plain = st.st_stream_run(st.ST_SCHED_SERIAL, layers(), hq, s, r, sq, sk, sv, rq, rk, rv, theta, arrival_s=arrival,
                                   decode_graph=False)
    per_token = lambda rep: float(np.mean([(rep["unit_done"][t] - rep["first_token"][t]) / max(r[t] - 1, 1) for t in range(len(r))]))
    # stage durations measured in the alternating run, then the schedule at the paper's real-time arrival
    alt = res["alternating"]
    dec_s = per_token(alt)
    pf_s = [max(float(alt["first_token"][t] - dec_s - max(arrival[t], alt["unit_done"][t - 1] if t else 0.0)), 0.0) for t in range(len(s))]
    real = (0.4 * np.cumsum(words)).tolist()
    model = {name: st.st_stream_timeline(mode, real, pf_s, r, dec_s) for name, mode in
             (("streaming", st.ST_SCHED_STREAMING), ("batch", st.ST_SCHED_BATCH))}
    return {"workload": "one stream shaped like the paper's efficiency experiment (70 words in 5 sentences at 0.4 s per word, "
                        f"{S} source tokens, {R} decoded tokens), 36 layers x (32 q / 8 kv heads, head_dim 128), attention path only; "
                        f"arrival times compressed x{time_scale}",
            "first_token_s": {k: round(float(v["first_token"][0]), 5) for k, v in res.items()},
            "total_s": {k: round(float(v["total_s"]), 4) for k, v in res.items()},
            "units_that_waited_for_prefill": {k: int(v["waited"].sum()) for k, v in res.items()},
            "decode_ms_per_token": round(dec_s * 1e3, 4), "decode_ms_per_token_plain_launches": round(per_token(plain) * 1e3, 4),
            "prefill_ms_per_sentence": [round(x * 1e3, 3) for x in pf_s],
            "at_150_words_per_minute": {"first_token_s": {k: round(float(v["first_token"][0]), 3) for k, v in model.items()},
                                        "note": "st_stream_timeline with the stage times measured above and uncompressed arrivals; "
                                                "the paper reports 6.231 s (streaming) vs 28.003 s (batch) for the whole model"}}


def bench_probes(st, torch):
    """What this GPU sustains for the decode kernel's access pattern and for the prefill kernel's MFMA instruction."""
    dev = "cuda"
    pool = torch.empty(1 << 34, dtype=torch.uint8, device=dev)       # 16 GiB: 64 times the memory-side cache
    pool.view(torch.int64).random_()
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    fsink = torch.zeros(4, dtype=torch.float32, device=dev)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    res = {}
    # the decode kernel's launch on configs[2]: about 2,800 one-wave units of up to 1024 tokens x 4 KB;
    # and a launch four times as large
    for name, waves, steps in (("paged_read_decode_sized", 2816, 16), ("paged_read_large", 11264, 16)):
        for i in range(3):
            st.st_probe_paged_read(pool, waves, steps, 1000 + i, sink)
        e0.record()
        for i in range(20):
            st.st_probe_paged_read(pool, waves, steps, i, sink)              # (other pages every launch)
        e1.record(); torch.cuda.synchronize()
        res[name] = {"bytes_per_launch": waves * steps * 16384, "GBps": round(waves * steps * 16384 * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)}
    st.st_probe_mfma_bf16(512, 2000, fsink)
    torch.cuda.synchronize()
    iters = 200000
    e0.record(); st.st_probe_mfma_bf16(512, iters, fsink); e1.record(); torch.cuda.synchronize()
    res["mfma_bf16_registers_only"] = {"ms": round(e0.elapsed_time(e1), 2),
                                       "TFLOPs": round(512 * 4 * iters * 8 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)}
    del pool
    return res


def bench_prefill_backward(st, torch, W, reps, zero_inputs=False):
    """Forward + backward of the attention stage on configs[1]; zero_inputs: the same launches on all-zero q, k, v, dO."""
    dev = "cuda"
    cfg = W.config2()
    hq, hkv, d, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_tokens
    g = torch.Generator(device=dev); g.manual_seed(cfg.seed + 9)
    rnd = lambda h: torch.randn((n, h, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, k, v, go = rnd(hq), rnd(hkv), rnd(hkv), rnd(hq)
    if zero_inputs:
        for t in (q, k, v, go):
            t.zero_()
    seg = torch.from_numpy(cfg.segment_ids).to(dev); strm = torch.from_numpy(cfg.stream_ids).to(dev)
    pos = torch.from_numpy(cfg.positions).to(dev)
    plan = st.st_plan_create(seg, strm, pos, cfg.cu_seqlens)
    flops_fwd = 4.0 * d * hq * float(plan.visible_pairs().sum())
    lse = torch.empty((n, hq), dtype=torch.float32, device=dev)
    out = st.st_attn_prefill(q, k, v, plan, lse=lse)
    st.st_attn_prefill_bwd(go, q, k, v, out, lse, plan)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        st.st_attn_prefill_bwd(go, q, k, v, out, lse, plan)
    e1.record(); torch.cuda.synchronize()
    # the per-kernel times come from a pass of their own: with kernel timing on, every timed kernel is launched
    # several times between its events, which must not count in the call's own time
    st.st_profile_read(st.ST_PROF_BWD_DQ); st.st_profile_read(st.ST_PROF_BWD_DKV)
    st.st_profile_enable(True)
    for _ in range(reps):
        st.st_attn_prefill_bwd(go, q, k, v, out, lse, plan)
    torch.cuda.synchronize()
    st.st_profile_enable(False)
    dq_ms, _ = st.st_profile_read(st.ST_PROF_BWD_DQ)
    dkv_ms, _ = st.st_profile_read(st.ST_PROF_BWD_DKV)
    plan.destroy()
    return {"ms": e0.elapsed_time(e1) / reps, "flops": 2.5 * flops_fwd, "dq_ms": dq_ms, "dkv_ms": dkv_ms, "flops_fwd": flops_fwd}


def _compact_page_table(rng, need_pages, max_pages):
    """[batch, max_pages] page ids: sequence b owns need_pages[b] distinct pages (shuffled over the pool); entries
    past them are never used by a step that stays within those pages and point at page 0.  Returns (table, n_pages)."""
    total = int(need_pages.sum())
    ids = rng.permutation(total).astype(np.int32)
    table = np.zeros((len(need_pages), max_pages), np.int32)
    off = 0
    for b, n in enumerate(need_pages):
        table[b, :n] = ids[off:off + n]; off += int(n)
    return table, total


def bench_stream_step(st, torch, W, steps, warmup, distinct_layers=None, use_graph=True):
    """configs[4], the end-to-end streaming step: 36 layers, 64 streams; per step every layer appends a 32-token source
    chunk (second stream) while 8 reasoning tokens are decoded one after the other, each through all layers (store the
    token, attend over the source cache and the reasoning cache).  Pools hold exactly the pages the drawn lengths need
    (about 3.6 GB per layer)."""
    dev = "cuda"
    shp = W.config5()
    B, L, hq, hkv, d = shp.batch, shp.n_layers, shp.n_q_heads, shp.n_kv_heads, shp.head_dim
    n_tok = 8
    rng = np.random.Generator(np.random.PCG64(shp.seed))
    src0 = shp.src_visible_len.astype(np.int64); rsn0 = shp.rsn_len.astype(np.int64) - 1      # cached before the step
    need_s = (src0 + shp.src_append + 15) // 16; need_r = (rsn0 + n_tok + 15) // 16
    pages_s = int(need_s.max()); pages_r = int(need_r.max())
    tab_s_np, n_pages_s = _compact_page_table(rng, need_s, pages_s)
    tab_r_np, n_pages_r = _compact_page_table(rng, need_r, pages_r)
    tab_s = torch.from_numpy(tab_s_np).to(dev); tab_r = torch.from_numpy(tab_r_np).to(dev)
    g = torch.Generator(device=dev); g.manual_seed(shp.seed)
    per_layer = (n_pages_s + n_pages_r) * 16 * hkv * d * 2 * 2
    free, _ = torch.cuda.mem_get_info()
    n_phys = L if distinct_layers is None else int(distinct_layers)
    n_phys = max(1, min(n_phys, L, int(free * 0.85) // per_layer))
    layers = []
    len_s_all = torch.zeros((n_phys, B), dtype=torch.int32, device=dev)
    for li in range(n_phys):
        cs = st.KVCache(n_pages_s, B, pages_s, hkv, d, tab_s); cr = st.KVCache(n_pages_r, B, pages_r, hkv, d, tab_r)
        cs.appended_len = len_s_all[li]
        for c in (cs, cr):
            c.k_pool.normal_(generator=g); c.v_pool.normal_(generator=g)
        layers.append(st.DualCache(cs, cr))
    src_vis = torch.from_numpy(shp.src_visible_len).to(dev)
    # reasoning length of every sequence while token t of the step is decoded, the token included
    rsn_len_t = [torch.from_numpy((rsn0 + t + 1).astype(np.int32)).to(dev) for t in range(n_tok)]
    q = torch.randn((n_tok, B, 1, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_tok = torch.randn((n_tok, B, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_tok = torch.randn((n_tok, B, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_src = torch.randn((B, shp.src_append, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_src = torch.randn((B, shp.src_append, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    max_s, max_r = int(src0.max()), int(rsn0.max()) + n_tok
    ws = torch.empty(st.st_decode_workspace_bytes(B, hq, hkv, d, 1, max_s, max_r), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()

    def step():
        main = torch.cuda.current_stream()                              # (under capture: the capturing stream)
        len_s_all.copy_(src_vis.expand(n_phys, B))                      # the source caches as they were before the step
        side.wait_stream(main)
        with torch.cuda.stream(side):                                   # prefill loop: the arriving chunk, every layer
            for li in range(L):
                if li < n_phys:                                         # (a cache standing for several layers takes it once)
                    st.st_kv_append_rope(layers[li], st.ST_SOURCE, k_src, v_src, 1.0e6, host_len_upper_bound=max_s + shp.src_append, stream=side)
        for t in range(n_tok):                                          # decoding loop: token after token, layer after layer
            for li in range(L):
                st.st_attn_decode_dual_append(q[t], k_tok[t], v_tok[t], layers[li % n_phys], src_vis, rsn_len_t[t], max_s, max_r,
                                              theta_base=1.0e6, out=out[t], workspace=ws)
        main.wait_stream(side)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    mode, graph = "eager", None
    ref = out.clone()
    step(); torch.cuda.synchronize()
    if not torch.equal(ref.view(torch.int16), out.view(torch.int16)):
        raise RuntimeError("stream step: two eager runs of the same step differ")
    if use_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with _no_gc(), torch.cuda.graph(graph):
                step()
            for _ in range(2):
                out.zero_()
                graph.replay(); torch.cuda.synchronize()
                if not torch.equal(ref.view(torch.int16), out.view(torch.int16)):
                    dd = (ref.float() - out.float()).abs()
                    raise RuntimeError(f"graph replay differs from the eager step (max abs difference {float(dd.max())})")
                if not torch.equal(len_s_all, (src_vis + shp.src_append).expand(n_phys, B)):
                    raise RuntimeError("graph replay did not run the source appends")
                step(); torch.cuda.synchronize()
            mode = "hip-graph"
        except Exception as exc:                           # noqa: BLE001
            print(f"bench.py: HIP graph capture not used ({exc}); timing eager launches", file=sys.stderr)
            graph = None
    times, mode = _time_launch_modes(torch, steps, graph, step)
    dt = times[mode]
    # kernel-only duration of the split kernel (HIP events on the launch stream), from one eager step; and the source
    # append of one layer alone
    st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    st.st_profile_enable(True)
    step(); torch.cuda.synchronize()
    st.st_profile_enable(False)
    split_ms, n_rec = st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    assert n_rec == n_tok * L
    append_ms = _event_ms(torch, lambda: (len_s_all[0].copy_(src_vis),
                                          st.st_kv_append_rope(layers[0], st.ST_SOURCE, k_src, v_src, 1.0e6, host_len_upper_bound=max_s + shp.src_append)), 20)
    append_ms -= _event_ms(torch, lambda: len_s_all[0].copy_(src_vis), 20)
    tokens_read = float(sum((src0 + rsn0 + t + 1).sum() for t in range(n_tok)))
    read_bytes = tokens_read * hkv * d * 2 * 2 * L
    append_bytes = float(B * (shp.src_append + n_tok) * hkv * d * 2 * 2 * 2 * L)
    del layers
    return {"sec_per_step": dt, "read_bytes": read_bytes, "append_bytes": append_bytes, "mode": mode, "distinct_layers": n_phys,
            "resident_gb": per_layer * n_phys / 1e9, "n_tok": n_tok, "sec_per_step_by_launch": times, "split_kernel_ms": split_ms,
            "bytes_per_launch": read_bytes / (n_tok * L), "append_layer_ms": max(append_ms, 1e-6),
            "append_layer_bytes": float(B * shp.src_append * hkv * d * 2 * 2 * 2), "n_layers": L, "batch": B}


def _wave_timeline(st, torch, launch, reset, n_pairs=1 << 16, bin_us=10.0):
    """One launch of the decode split kernel with st_profile_wave_trace on (one launch between the events): when its waves
    (one per work unit) start and end on the 100 MHz wall clock -- how many are in flight over the launch."""
    buf = torch.zeros((n_pairs, 2), dtype=torch.int64, device="cuda")
    reset(); launch(); torch.cuda.synchronize()
    st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    st.st_profile_repeat(1); st.st_profile_wave_trace(buf); st.st_profile_enable(True)
    try:
        reset(); launch(); torch.cuda.synchronize()
    finally:
        st.st_profile_enable(False); st.st_profile_wave_trace(None); st.st_profile_repeat(PROF_REPEAT)
    ev_ms, _ = st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    a = buf.cpu().numpy()
    a = a[a[:, 1] > 0]
    if not len(a):
        return None
    t0 = a[:, 0].min()
    start = (a[:, 0] - t0) / 100.0; end = (a[:, 1] - t0) / 100.0          # microseconds
    dur = end - start
    real = dur > 2.0                                                        # units past a cache's length (and the token's unit) end at once
    span = float(end.max())
    bins = []
    lo = 0.0
    while lo < span:
        bins.append(int(((start < lo + bin_us) & (end > lo) & real).sum()))
        lo += bin_us
    return {"note": "one launch, every workgroup (one wave, one work unit) stamped at start and end with the 100 MHz wall clock (st_profile_wave_trace)",
            "workgroups": int(len(a)), "units_with_tokens": int(real.sum()), "first_start_to_last_end_us": round(span, 1),
            "events_around_this_single_launch_us": round(ev_ms * 1e3, 1),
            "unit_duration_us": {"mean": round(float(dur[real].mean()), 1), "p10": round(float(np.percentile(dur[real], 10)), 1),
                                 "p90": round(float(np.percentile(dur[real], 90)), 1), "max": round(float(dur[real].max()), 1)},
            "last_unit_started_at_us": round(float(start[real].max()), 1),
            f"waves_in_flight_per_{int(bin_us)}us_bin": bins}


def bench_decode(st, torch, W, steps, warmup, n_layers=None, use_graph=True, fp8=False):
    dev = "cuda"
    shp = W.config3() if n_layers is None else W.config3(n_layers=n_layers)
    B, L, hq, hkv, d = shp.batch, shp.n_layers, shp.n_q_heads, shp.n_kv_heads, shp.head_dim
    rng = np.random.Generator(np.random.PCG64(shp.seed))
    pages_s = (shp.max_src_len + 15) // 16; pages_r = (shp.max_rsn_len + 15) // 16
    tab_s = torch.from_numpy(W.shuffled_page_table(rng, B, pages_s)).to(dev)
    tab_r = torch.from_numpy(W.shuffled_page_table(rng, B, pages_r)).to(dev)
    g = torch.Generator(device=dev); g.manual_seed(shp.seed)
    layers = []
    len_s_all = torch.zeros((L, B), dtype=torch.int32, device=dev); len_r_all = torch.zeros((L, B), dtype=torch.int32, device=dev)
    for li in range(L):
        cs = st.KVCache(B * pages_s, B, pages_s, hkv, d, tab_s, fp8=fp8); cr = st.KVCache(B * pages_r, B, pages_r, hkv, d, tab_r, fp8=fp8)
        cs.appended_len = len_s_all[li]; cr.appended_len = len_r_all[li]      # one tensor for all layers: one reset per step
        for c in (cs, cr):                                  # any bit pattern is valid cache content: fill in place
            if fp8:                                         # (any finite code: 0x7f / 0xff are the NaN codes)
                c.k_pool.random_(0, 0x7f, generator=g); c.v_pool.random_(0, 0x7f, generator=g)
                c.k_scale.fill_(2.0 ** -7); c.v_scale.fill_(2.0 ** -7)
            else:
                c.k_pool.normal_(generator=g); c.v_pool.normal_(generator=g)
        layers.append(st.DualCache(cs, cr))
    src_vis = torch.from_numpy(shp.src_visible_len).to(dev)
    rsn_len = torch.from_numpy(shp.rsn_len).to(dev)
    rsn_before = (rsn_len - 1).contiguous()
    q = torch.randn((B, 1, hq, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_tok = torch.randn((B, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_tok = torch.randn((B, 1, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_src = torch.randn((B, shp.src_append, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_src = torch.randn((B, shp.src_append, hkv, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    max_s, max_r = int(shp.src_visible_len.max()), int(shp.rsn_len.max())
    ws = torch.empty(st.st_decode_workspace_bytes(B, hq, hkv, d, 1, max_s, max_r), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()

    def step(i_timed, source_appends=True):
        main = torch.cuda.current_stream()                              # (under capture: the capturing stream)
        len_s_all.copy_(src_vis.expand(L, B)); len_r_all.copy_(rsn_before.expand(L, B))
        side.wait_stream(main)
        for li, dc in enumerate(layers):
            if source_appends:
                with torch.cuda.stream(side):
                    st.st_kv_append(dc, st.ST_SOURCE, k_src, v_src, host_len_upper_bound=shp.max_src_len, stream=side)
            if fp8:
                st.st_kv_append(dc, st.ST_REASONING, k_tok, v_tok, host_len_upper_bound=max_r)
                st.st_attn_decode_dual(q, dc, src_vis, rsn_len, max_s, max_r, out=out, workspace=ws)
            else:                                          # store the token and attend, one call
                st.st_attn_decode_dual_append(q, k_tok, v_tok, dc, src_vis, rsn_len, max_s, max_r, out=out, workspace=ws)
        main.wait_stream(side)

    for _ in range(warmup):
        step(None)
    torch.cuda.synchronize()
    # kernel-only duration of the split kernel (HIP events on the launch stream), from eager steps
    st.st_profile_enable(True)
    for i in range(min(steps, 3)):
        step(i)
    torch.cuda.synchronize()
    st.st_profile_enable(False)
    layer_ms, n_rec = st.st_profile_read(st.ST_PROF_DECODE_SPLIT)
    assert n_rec == min(steps, 3) * L
    timeline = None
    if not fp8:
        timeline = _wave_timeline(st, torch, lambda: st.st_attn_decode_dual_append(q, k_tok, v_tok, layers[L - 1], src_vis, rsn_len, max_s, max_r, out=out,
                                                                                  workspace=ws), lambda: len_r_all[L - 1].copy_(rsn_before))
    # the timed steps, two ways: the whole 28-layer step (both streams) as replays of one HIP graph (checked against the
    # eager step, second stream included) and as plain launches; the faster one is the step time, both are reported
    mode = "hip-graph"
    graph = None
    if use_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with _no_gc(), torch.cuda.graph(graph):
                step(None)
            step(None)                                     # eager result of the same step
            torch.cuda.synchronize()
            ref = out.clone()
            for _ in range(3):                             # every replay, with eager work in between, must reproduce it
                out.zero_()
                graph.replay()
                torch.cuda.synchronize()
                if not torch.equal(ref, out):
                    raise RuntimeError("graph replay differs from the eager step")
                if not torch.equal(len_s_all, (src_vis + shp.src_append).expand(L, B)):   # the second stream's appends ran in the replay
                    raise RuntimeError("graph replay did not run the source appends")
                step(None)
                torch.cuda.synchronize()
        except Exception as exc:                           # noqa: BLE001
            print(f"bench.py: HIP graph capture not used ({exc}); timing eager launches", file=sys.stderr)
            graph = None
    times, mode = _time_launch_modes(torch, steps, graph, lambda: step(None))
    dt = times[mode] * steps
    # the decode stream of the same step with nothing on the second stream (what the concurrent source appends cost)
    alone_ms = _event_ms(torch, lambda: step(None, source_appends=False), steps)
    tokens = float((shp.src_visible_len.astype(np.int64) + shp.rsn_len).sum())
    # bytes per cached token and KV head: K and V rows of D elements; 8-bit rows carry an fp32 scale each
    per_layer = tokens * hkv * ((2 * d + 8) if fp8 else 2 * d * 2)
    append_bytes = float(B * (shp.src_append + 1)) * hkv * (2 * d * 2 + ((2 * d + 8) if fp8 else 2 * d * 2)) * L
    return {"shape": shp, "wave_timeline": timeline, "bytes_per_step": per_layer * L, "append_bytes_per_step": append_bytes, "sec_per_step": dt / steps,
            "layer_decode_ms": layer_ms, "bytes_per_layer": per_layer, "mode": mode, "sec_per_step_by_launch": times,
            "sec_per_step_decode_stream_alone": alone_ms * 1e-3}


def bench_source_chunk(st, torch, W, steps, warmup):
    """Alg. 1's prefill loop on the Qwen3-8B-shaped streaming shape (configs[4]), one layer: a 32-token source chunk per
    sequence is appended and attends causally over source caches of 1-8K tokens."""
    dev = "cuda"
    shp = W.config5()
    B, hq, hkv, d, n_new = shp.batch, shp.n_q_heads, shp.n_kv_heads, shp.head_dim, shp.src_append
    rng = np.random.Generator(np.random.PCG64(shp.seed))
    pages = (shp.max_src_len + 15) // 16
    cs = st.KVCache(B * pages, B, pages, hkv, d, torch.from_numpy(W.shuffled_page_table(rng, B, pages)).to(dev))
    cr = st.KVCache(B, B, 1, hkv, d, torch.arange(B, dtype=torch.int32, device=dev).reshape(B, 1).contiguous())
    g = torch.Generator(device=dev); g.manual_seed(shp.seed)
    cs.k_pool.normal_(generator=g); cs.v_pool.normal_(generator=g)
    caches = st.DualCache(cs, cr)
    before = torch.from_numpy(shp.src_visible_len).to(dev)
    total = torch.from_numpy((shp.src_visible_len + n_new).astype(np.int32)).to(dev)
    k_new = torch.randn((B, n_new, hkv, d), generator=g, device=dev).to(torch.bfloat16)
    v_new = torch.randn((B, n_new, hkv, d), generator=g, device=dev).to(torch.bfloat16)
    q = torch.randn((B, n_new, hq, d), generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty_like(q)
    max_s = int(shp.src_visible_len.max()) + n_new
    ws = torch.empty(st.st_source_chunk_workspace_bytes(B, hq, hkv, d, n_new, max_s), dtype=torch.uint8, device=dev)

    def step():
        cs.appended_len.copy_(before)
        st.st_kv_append(caches, st.ST_SOURCE, k_new, v_new, host_len_upper_bound=shp.max_src_len)
        st.st_attn_source_chunk(q, caches, total, max_s, out=out, workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    st.st_profile_read(st.ST_PROF_SOURCE_CHUNK)
    st.st_profile_enable(True)
    for _ in range(min(steps, 10)):
        step()
    torch.cuda.synchronize()
    st.st_profile_enable(False)
    kern_ms, _ = st.st_profile_read(st.ST_PROF_SOURCE_CHUNK)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    tok = shp.src_visible_len.astype(np.float64) + n_new
    flops = 4.0 * d * hq * float((n_new * tok - n_new * (n_new - 1) / 2).sum())      # causal inside the chunk
    return {"ms_per_step": dt * 1e3, "cache_bytes": float(tok.sum()) * 2 * hkv * d * 2, "flops": flops, "batch": B, "n_new": n_new,
            "kernel_ms": kern_ms}


def cpu_baseline(W, O):
    """The fp64 oracle, as it stands, on a bounded sample of the headline workload (configs[3]): the two query heads of KV
    head 0, sequence by sequence and, within a sequence, one interleaved quarter of its query rows at a time, until 10 s
    are spent (RoPE of the slice included)."""
    cfg = W.config4a()
    d = cfg.head_dim
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    # rows 0, 4, 8, ... first, then 1, 5, 9, ... and so on: every pass has the sequence's mix of row lengths
    dt, vis, n_rows, passes = 0.0, 0, 0, 0
    for b in range(cfg.batch):
        s, e = int(cfg.cu_seqlens[b]), int(cfg.cu_seqlens[b + 1])
        n = e - s
        rng = np.random.Generator(np.random.PCG64(cfg.seed + 1000 + b))
        q = W.normal(rng, (n, 2, d), "bf16"); k = W.normal(rng, (n, 1, d), "bf16"); v = W.normal(rng, (n, 1, d), "bf16")
        stream, seg, pos = cfg.stream_ids[s:e], cfg.segment_ids[s:e], cfg.positions[s:e]
        for off in range(4):
            rows = np.arange(off, n, 4)
            t0 = time.perf_counter()
            qr = O.rope(q, pos, cfg.theta); kr = O.rope(k, pos, cfg.theta)
            O.attention_dense(qr, kr, v, stream, seg, pos, rows=rows)
            dt += time.perf_counter() - t0
            vis += int(O.mask_rows(stream, seg, pos, rows).sum())         # visible pairs of the sampled rows
            n_rows += len(rows); passes += 1
            if dt >= 10.0:
                break
        if dt >= 10.0:
            break
    fl = 4.0 * d * 2 * vis
    whole = cfg.closed_form_pairs()
    total_pairs = float(sum(whole)) * cfg.n_q_heads
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"configs[3], the 2 query heads of KV head 0, {passes} passes of a quarter of a sequence's query rows each (interleaved "
                      f"rows; {passes / 4.0:g} of the 8 sequences, {n_rows} rows, {vis} visible pairs per head): RoPE + dense-mask fp64 "
                      f"attention in {dt:.1f} s; extrapolated per visible pair, the whole batch (8 sequences x 32 heads, "
                      f"{total_pairs:.3g} pairs) would take {dt * total_pairs / (2.0 * vis) / 60:.0f} min on these cores"}


def _hbm_roofline(kernel, nbytes, ms, traffic_key=None, note=None):
    gbps = nbytes / (ms * 1e-3) / 1e9
    r = {"kernel": kernel, "bound": "hbm", "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
         "frac": round(gbps / PEAK_HBM_GBPS, 4), "traffic": measured_traffic(traffic_key) if traffic_key else None,
         "avg_kernel_ms": round(ms, 5), "algorithmic_bytes_per_launch": nbytes}
    if note:
        r["note"] = note
    return r


def _prefill_objects(pre, name, fused_rope):
    """(step TFLOP/s, roofline object of the attention kernel, stages object) of one prefill step result."""
    cfg = pre["cfg"]
    tflops_step = pre["flops"] / pre["sec_per_step"] / 1e12
    tflops_kernel = pre["flops"] / (pre["prefill_kernel_ms"] * 1e-3) / 1e12
    kern = f"prefill_attn_kernel<{cfg.head_dim}, {2 if pre['two_heads'] else 1}, {'true' if fused_rope else 'false'}>"
    roof = {"kernel": kern, "bound": "mfma", "achieved": round(tflops_kernel, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tflops_kernel / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(f"prefill_attn_kernel@{name}"),
            "avg_kernel_ms": round(pre["prefill_kernel_ms"], 4), "algorithmic_flops_per_launch": pre["flops"]}
    ms = pre["stage_ms"]
    stages = {"note": "every stage of the step alone, back-to-back launches timed with events on the launch stream; tile_pack and attention "
                      "from events around the kernel inside st_attn_prefill during whole steps",
              "ms": {k: round(v, 5) for k, v in ms.items()},
              "rope_qk": {"roofline": _hbm_roofline("rope_kernel<bf16, 128> (st_rope_apply_qk: q and k of all tokens in one launch, read + write)", pre["stage_bytes"]["rope_qk"],
                                                    ms["rope_qk"], f"rope_qk_kernel@{name}")},
              "tile_pack": {"roofline": _hbm_roofline("tile_pack_kernel (k, v rows gathered into K tiles and V^T tiles)", pre["stage_bytes"]["tile_pack"],
                                                      ms["tile_pack"], f"tile_pack_kernel@{name}")},
              "append_source_chunk": {"roofline": _hbm_roofline("kv_append_kernel (64-token source chunk per sequence, alone on the GPU)",
                                                                pre["stage_bytes"]["append_source_chunk"], ms["append_source_chunk"], None,
                                                                "a launch of a few MB: bound by its own latency, not by bandwidth")}}
    return tflops_step, roof, stages


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--decode-steps", type=int, default=None, help="steps of the 28-layer decode workload (default: min(steps, 10))")
    ap.add_argument("--stream-steps", type=int, default=3, help="steps of the configs[4] streaming step (8 decoded tokens x 36 layers each)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="leave out every decode leg (configs[4], configs[2], source chunk)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP graph replays of the steps")
    ap.add_argument("--fused-rope", action="store_true",
                    help="prefill steps: st_attn_prefill_rope on unrotated q, k instead of st_rope_apply_qk + st_attn_prefill")
    ap.add_argument("--decode-layers", type=int, default=None, help="override the 28 layers of the configs[2] decode workload (for profiling)")
    ap.add_argument("--only", default=None,
                    help="comma-separated legs to run besides the headline step, e.g. 'decode,decode_small' (for profiling); names: decode, "
                         "prefill_small, decode_small, source_chunk, decode_fp8, prefill_backward, stream_session, probes, power_check")
    ap.add_argument("--no-headline", action="store_true", help="skip the configs[3] step (for profiling single legs); prints what was asked for")
    ap.add_argument("--stream-step-layers", type=int, default=None,
                    help="distinct per-layer caches of the configs[4] step (default: all 36 if memory allows; fewer are cycled)")
    ap.add_argument("--stream-time-scale", type=float, default=0.01, help="compression of the arrival times of the stream session")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline step, the two decode workloads, the configs[1] step and the source chunk")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference point for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU; there is no multi-GPU mode (sequences and KV heads shard "
              "without communication; sharding one sequence's caches by token range needs one exchange of partial results). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2510_17238_amd as st
    import workloads as W
    st.load_library()
    st.st_profile_repeat(PROF_REPEAT)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    if args.copy_calibration:
        a = torch.full((1 << 29,), 1.0, dtype=torch.bfloat16, device="cuda"); b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": a.numel() * 2, "bytes_written_per_copy": a.numel() * 2, "copies": 5}))
        return
    legs = ["decode", "prefill_small", "decode_small", "source_chunk"]
    if not args.no_extras:
        legs += ["decode_fp8", "prefill_backward", "stream_session", "probes", "power_check"]
    if args.only is not None:
        legs = [x for x in args.only.split(",") if x]
    if args.no_decode:
        legs = [x for x in legs if x not in ("decode", "decode_small", "source_chunk", "decode_fp8")]
    use_graph = not args.no_graph
    rope_text = "inside st_attn_prefill_rope" if args.fused_rope else "st_rope_apply_qk on q and k"
    step_text = ("step = plan + RoPE (" + rope_text + ") + tile packing + streaming-mask prefill + paged append (64-token source chunk "
                 "per sequence on a second stream, 1 reasoning token) + dual-cache decode of one token over the batch's own caches")
    line = {"metric": "streaming-mask prefill TFLOP/s + dual-cache decode GB/s, % of MI355X peak"}
    if not args.no_headline:
        pre = bench_prefill_step(st, torch, W, W.config4a(), args.steps, args.warmup, use_graph, args.fused_rope)
        tflops_step, roof, stages = _prefill_objects(pre, "cfg4a", args.fused_rope)
        line.update({
            "value": round(tflops_step, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(pre["sec_per_step"] * 1e3, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "launch": pre["mode"],
            "ms_per_step_by_launch": {k: round(v * 1e3, 4) for k, v in pre["sec_per_step_by_launch"].items()},
            "config": {"workload": "configs[3] (the length-pinned reading, 4a): Qwen3-4B-shaped layer, batch 8 x 16,384 tokens, 32 q / 8 kv heads, "
                                   "head_dim 128, bf16, source segments of 64-192 tokens interleaved with reasoning segments of 64-256 tokens; " + step_text,
                       "n_tokens": pre["n_tokens"], "effective_flops_per_step": pre["flops"]},
            "prefill_pct_of_peak": round(100.0 * roof["frac"], 2), "roofline": roof, "stages": stages})
        del pre
        gc.collect(); torch.cuda.empty_cache()
    else:
        line.update({"value": None, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
                     "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": {"workload": "legs only: " + ",".join(legs)}})
    # the paper's own latency figures for context (Table 4, "Efficiency evaluation on Qwen3-4B": whole model, 100
    # GSM-Symbolic samples, input read at 150 words per minute); its text names no GPU
    line["paper_reference"] = {
        "source": "Table 4 (Qwen3-4B, whole model, another machine: context, not a target)", "hardware": "not stated in the paper",
        "prefill_s_per_sentence": {"streaming": 0.041, "batch": 0.052}, "decode_s_per_token": {"streaming": 0.037, "batch": 0.039},
        "decoded_tokens": {"streaming": 439, "batch": 436}, "first_token_latency_s": {"streaming": 6.231, "batch": 28.003}}

    if "decode" in legs:
        with _leg(line, "decode", torch):
            ss = bench_stream_step(st, torch, W, args.stream_steps, 1, args.stream_step_layers, use_graph)
            gbps = ss["read_bytes"] / ss["sec_per_step"] / 1e9
            line["decode"] = {
                "workload": "configs[4]: Qwen3-8B-shaped end-to-end streaming step, 36 layers, 64 streams, 32 q / 8 kv heads, head_dim 128, "
                            "bf16, source caches U[1024,8192] and reasoning caches U[2048,16384] tokens in 16-token pages (shuffled); per "
                            "step every layer appends a 32-token source chunk on a second stream while 8 reasoning tokens are decoded one "
                            "after the other through all layers (st_attn_decode_dual_append: store the token, attend over both caches)",
                "value": round(gbps, 1), "unit": "GB/s", "pct_of_peak": round(100.0 * gbps / PEAK_HBM_GBPS, 2), "steps": args.stream_steps,
                "ms_per_step": round(ss["sec_per_step"] * 1e3, 2), "ms_per_token": round(ss["sec_per_step"] * 1e3 / ss["n_tok"], 2),
                "algorithmic_read_bytes_per_step": ss["read_bytes"], "append_bytes_per_step": ss["append_bytes"], "launch": ss["mode"],
                "ms_per_step_by_launch": {k: round(v * 1e3, 4) for k, v in ss["sec_per_step_by_launch"].items()},
                "distinct_layer_caches": ss["distinct_layers"], "resident_cache_gb": round(ss["resident_gb"], 1),
                "tokens_per_s": round(ss["batch"] * ss["n_tok"] / ss["sec_per_step"], 1),
                "roofline": _hbm_roofline("decode_split16_kernel<128, false> (one layer, one token of all 64 streams)", ss["bytes_per_launch"],
                                          ss["split_kernel_ms"], "decode_split16_kernel@cfg5"),
                "append": {"roofline": _hbm_roofline("kv_append_kernel with rotation (32-token source chunk of 64 streams, one layer, alone on the GPU)",
                                                     ss["append_layer_bytes"], ss["append_layer_ms"], None,
                                                     "17 MB per launch: bound by its own latency, not by bandwidth")}}
            del ss
            gc.collect(); torch.cuda.empty_cache()
    if "prefill_small" in legs:
        with _leg(line, "prefill_small", torch):
            ps = bench_prefill_step(st, torch, W, W.config2(), args.steps, args.warmup, use_graph, args.fused_rope)
            tf, roof, stages = _prefill_objects(ps, "cfg2", args.fused_rope)
            line["prefill_small"] = {
                "workload": "configs[1]: Qwen3-0.6B-shaped layer, batch 4, 16 q / 8 kv heads, head_dim 128, bf16, 32 source (24-64 tok) + 32 "
                            "reasoning (32-128 tok) segments per sequence, interleaved; " + step_text,
                "value": round(tf, 3), "unit": "TFLOP/s", "ms_per_step": round(ps["sec_per_step"] * 1e3, 4), "launch": ps["mode"],
                "ms_per_step_by_launch": {k: round(v * 1e3, 4) for k, v in ps["sec_per_step_by_launch"].items()},
                "n_tokens": ps["n_tokens"], "effective_flops_per_step": ps["flops"], "roofline": roof, "stages": stages}
            del ps
    dec = None
    if "decode_small" in legs:
        with _leg(line, "decode_small", torch):
            dsteps = args.decode_steps if args.decode_steps is not None else min(args.steps, 10)
            dec = bench_decode(st, torch, W, dsteps, min(args.warmup, 3), args.decode_layers, use_graph)
            gbps_step = dec["bytes_per_step"] / dec["sec_per_step"] / 1e9
            line["decode_small"] = {
                "workload": "configs[2]: Qwen3-1.7B-shaped decode, 28 layers, batch 32, 16 q / 8 kv heads, head_dim 128, bf16, "
                            "source cache 2048 + reasoning cache U[1024,6144], 16-token pages (shuffled), one token per step, "
                            "concurrent 64-token source append per layer on a second stream",
                "value": round(gbps_step, 1), "unit": "GB/s", "steps": dsteps, "launch": dec["mode"],
                "ms_per_step_by_launch": {k: round(v * 1e3, 4) for k, v in dec["sec_per_step_by_launch"].items()},
                "ms_per_step": round(dec["sec_per_step"] * 1e3, 4),
                "algorithmic_bytes_per_step": dec["bytes_per_step"], "append_bytes_per_step": dec["append_bytes_per_step"],
                "pct_of_peak": round(100.0 * gbps_step / PEAK_HBM_GBPS, 2),
                "decode_stream_alone": {
                    "note": "the same 28-layer step with no source appends on the second stream, plain launches",
                    "ms_per_step": round(dec["sec_per_step_decode_stream_alone"] * 1e3, 4),
                    "pct_of_peak": round(100.0 * dec["bytes_per_step"] / dec["sec_per_step_decode_stream_alone"] / 1e9 / PEAK_HBM_GBPS, 2)},
                "roofline": _hbm_roofline("decode_split16_kernel<128, true> (one layer)", dec["bytes_per_layer"], dec["layer_decode_ms"],
                                          "decode_split16_kernel@cfg3"),
                "wave_timeline": dec["wave_timeline"]}
    if "source_chunk" in legs:
        with _leg(line, "source_chunk", torch):
            sc = bench_source_chunk(st, torch, W, min(args.steps, 20), min(args.warmup, 3))
            # 125 flop per cache byte: below the ridge (312 flop / byte), so the roof is the HBM one
            line["source_chunk"] = {
                "workload": "configs[4] source side, one layer: batch 64, 32 q / 8 kv heads, 32-token chunk appended to source caches "
                            "U[1024,8192] (16-token pages) and attended causally over them (Alg. 1 prefill loop)",
                "ms_per_step": round(sc["ms_per_step"], 4), "tflops": round(sc["flops"] / (sc["ms_per_step"] * 1e-3) / 1e12, 2),
                "cache_read_once_gbps": round(sc["cache_bytes"] / (sc["ms_per_step"] * 1e-3) / 1e9, 1),
                "roofline": _hbm_roofline("chunk_split_lds_kernel<128> (the cache read once)", sc["cache_bytes"], sc["kernel_ms"], "chunk_split_lds_kernel@cfg5",
                                          f"{sc['flops'] / sc['cache_bytes']:.0f} flop per cache byte, below the ridge of 312: HBM is the roof; the kernel's "
                                          f"matrix rate is {sc['flops'] / (sc['kernel_ms'] * 1e-3) / 1e12:.0f} TFLOP/s"),
                "note": "append + attention; the 128 (token, head) rows of a sequence and KV head are one workgroup (4 waves x 32 rows) "
                        "that shares the cache pages through LDS"}
    if "probes" in legs:
        with _leg(line, "probes", torch):
            line["probes"] = bench_probes(st, torch)
    if "decode_fp8" in legs:
        with _leg(line, "decode_fp8", torch):
            dsteps = args.decode_steps if args.decode_steps is not None else min(args.steps, 10)
            d8 = bench_decode(st, torch, W, dsteps, min(args.warmup, 3), args.decode_layers, use_graph, fp8=True)
            g8_step = d8["bytes_per_step"] / d8["sec_per_step"] / 1e9
            line["decode_fp8"] = {
                "workload": "configs[2] with both caches stored in 8 bits (E4M3 codes + one fp32 power-of-two scale per key row and per "
                            "value row: 264 B instead of 512 B per cached token and KV head); same step as 'decode_small'",
                "value": round(g8_step, 1), "unit": "GB/s", "steps": dsteps, "launch": d8["mode"],
                "ms_per_step_by_launch": {k: round(v * 1e3, 4) for k, v in d8["sec_per_step_by_launch"].items()},
                "ms_per_step": round(d8["sec_per_step"] * 1e3, 4), "algorithmic_bytes_per_step": d8["bytes_per_step"],
                "speedup_vs_bf16_step": round(dec["sec_per_step"] / d8["sec_per_step"], 3) if dec else None,
                "roofline": _hbm_roofline("decode_split16_fp8_kernel<128> (one layer)", d8["bytes_per_layer"], d8["layer_decode_ms"],
                                          "decode_split16_fp8_kernel@cfg3")}
    if "prefill_backward" in legs:
        with _leg(line, "prefill_backward", torch):
            bw = bench_prefill_backward(st, torch, W, 10)
            tf = bw["flops"] / (bw["ms"] * 1e-3) / 1e12
            tf_dq = 1.5 * bw["flops_fwd"] / (bw["dq_ms"] * 1e-3) / 1e12
            tf_dkv = 2.0 * bw["flops_fwd"] / (bw["dkv_ms"] * 1e-3) / 1e12
            line["prefill_backward"] = {
                "workload": "configs[1], gradients dq / dk / dv of the attention stage, bf16 (tile gathering, row statistics and "
                            "both matrix-core kernels)",
                "ms": round(bw["ms"], 3), "algorithmic_flops": bw["flops"], "tflops": round(tf, 1),
                "kernels": {"bwd_dq_mfma_kernel<128>": {"avg_ms": round(bw["dq_ms"], 4), "executed_tflops": round(tf_dq, 1)},
                            "bwd_dkv_mfma_kernel<128>": {"avg_ms": round(bw["dkv_ms"], 4), "executed_tflops": round(tf_dkv, 1)}},
                "roofline": {"kernel": "bwd_dq_mfma_kernel<128> + bwd_dkv_mfma_kernel<128>", "bound": "mfma",
                             "achieved": round(bw["flops"] / ((bw["dq_ms"] + bw["dkv_ms"]) * 1e-3) / 1e12, 1), "peak": PEAK_BF16_TFLOPS,
                             "unit": "TFLOP/s", "frac": round(bw["flops"] / ((bw["dq_ms"] + bw["dkv_ms"]) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                             "traffic": (lambda a, b: a + b if a is not None and b is not None else None)(
                                 measured_traffic("bwd_dq_mfma_kernel@cfg2"), measured_traffic("bwd_dkv_mfma_kernel@cfg2")),
                             "note": "algorithmic = 5 products of 2 D flop per visible (query, key, head) triple (2.5x the forward); the two "
                                     "kernels execute 7 (scores and dP are recomputed on the key side); executed_tflops counts those"}}
    if "stream_session" in legs:
        with _leg(line, "stream_session", torch):
            line["stream_session"] = bench_stream_session(st, torch, W, args.stream_time_scale)
    if "power_check" in legs:
        with _leg(line, "power_check", torch):
            pc = bench_prefill_zero_inputs(st, torch, W, 5)
            line["power_check"] = {
                "workload": "configs[3], attention kernel alone: the same launches on random and on all-zero inputs (the same instruction "
                            "stream, no operand bits toggling: the difference is the power limit, not the schedule)",
                "random_inputs": {"avg_kernel_ms": round(pc["kernel_ms"], 3), "tflops": round(pc["flops"] / (pc["kernel_ms"] * 1e-3) / 1e12, 1)},
                "all_zero_inputs": {"avg_kernel_ms": round(pc["zero_input_kernel_ms"], 3),
                                    "tflops": round(pc["flops"] / (pc["zero_input_kernel_ms"] * 1e-3) / 1e12, 1)}}
            br = bench_prefill_backward(st, torch, W, 5)
            bz = bench_prefill_backward(st, torch, W, 5, zero_inputs=True)
            line["power_check"]["backward_kernels_configs1"] = {
                "random_inputs": {"bwd_dq_mfma_kernel_ms": round(br["dq_ms"], 4), "bwd_dkv_mfma_kernel_ms": round(br["dkv_ms"], 4)},
                "all_zero_inputs": {"bwd_dq_mfma_kernel_ms": round(bz["dq_ms"], 4), "bwd_dkv_mfma_kernel_ms": round(bz["dkv_ms"], 4)}}
    if not args.no_cpu_baseline:
        from oracle import streaming_attention as O
        line["cpu_baseline"] = cpu_baseline(W, O)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
