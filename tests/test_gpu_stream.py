"""GPU: the Alg. 1 scheduler (st_stream_run).  A streaming session over the two paged caches must give, for
every token, the row of the dense streaming-mask attention (Eq. 2) over the equivalent interleaved sequence
[S_1 R_1 S_2 R_2 ...] with stream-local position ids -- inference reproduces the training mask -- whatever the
timing of the two loops; the reported event times must respect Alg. 1's ordering."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import streaming_attention as O

pytestmark = pytest.mark.gpu

from gpu_helpers import DEV, make_cache, to_dev, to_f64  # noqa: E402


@pytest.fixture(scope="module")
def st():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_17238_amd as st_
    st_.load_library()
    return st_


def _session(rng, batch, hq, hkv, d, s, r):
    """Per-sequence activations of one session and their sentence-major / step-major device layouts."""
    S, R = int(sum(s)), int(sum(r))
    act = {name: W.normal(rng, (batch, n, h, d), "bf16") for name, n, h in
           (("sq", S, hq), ("sk", S, hkv), ("sv", S, hkv), ("rq", R, hq), ("rk", R, hkv), ("rv", R, hkv))}
    cut = np.concatenate([[0], np.cumsum(s)])
    dev = {}
    for name in ("sq", "sk", "sv"):
        blocks = [act[name][:, cut[k]:cut[k + 1]].reshape(-1) for k in range(len(s))]
        dev[name] = to_dev(np.concatenate(blocks) if blocks else np.zeros(0, np.float32), "bf16")
    for name in ("rq", "rk", "rv"):
        dev[name] = to_dev(np.ascontiguousarray(act[name].transpose(1, 0, 2, 3)), "bf16")      # [steps, batch, heads, D]
    return act, dev


def _layers(st, rng, n_layers, batch, hkv, d, S, R):
    out = []
    for _ in range(n_layers):
        cs, _ = make_cache(batch, (S + 15) // 16 + 1, hkv, d, rng, fill=float("nan"))
        cr, _ = make_cache(batch, (R + 15) // 16 + 1, hkv, d, rng, fill=float("nan"))
        out.append(st.DualCache(cs, cr))
    return out


def _unpack_src(src_out, batch, s, hq, d):
    """sentence-major flat tensor -> [batch, S, hq, d]"""
    parts, off = [], 0
    for n in s:
        sz = batch * n * hq * d
        parts.append(src_out[off:off + sz].view(batch, n, hq, d)); off += sz
    return torch.cat(parts, dim=1) if parts else src_out.view(batch, 0, hq, d)


def _oracle_rows(act, b, s, r, theta, all_sources_visible=False):
    """Dense-mask attention over the interleaved sequence of sequence b; returns (source rows, reasoning rows)."""
    stream, seg, pos = W.tokens_from_segments(list(s), list(r), "interleaved")
    src = np.nonzero(stream == O.SRC)[0]; rsn = np.nonzero(stream == O.RSN)[0]
    n = len(stream)
    hq, hkv, d = act["sq"].shape[2], act["sk"].shape[2], act["sq"].shape[3]
    q = np.zeros((n, hq, d)); k = np.zeros((n, hkv, d)); v = np.zeros((n, hkv, d))
    q[src], k[src], v[src] = act["sq"][b], act["sk"][b], act["sv"][b]
    q[rsn], k[rsn], v[rsn] = act["rq"][b], act["rk"][b], act["rv"][b]
    if all_sources_visible:
        seg = seg.copy(); seg[stream == O.RSN] = seg.max()
    o, _ = O.attention_dense(O.rope(q, pos, theta), O.rope(k, pos, theta), v, stream, seg, pos)
    return o[src], o[rsn]


def _check_report(rep, s, r, arrival=None):
    K = len(s)
    for t in range(K):
        assert rep["first_token"][t] >= rep["prefill_done"][t] - 1e-6            # a unit needs its sentence in the cache
        assert rep["unit_done"][t] >= rep["first_token"][t] - 1e-6
        if t:
            assert rep["first_token"][t] >= rep["unit_done"][t - 1] - 1e-6       # units in order
            assert rep["prefill_done"][t] >= rep["prefill_done"][t - 1] - 1e-6   # sentences in arrival order
        if arrival is not None:
            assert rep["prefill_done"][t] >= arrival[t] - 2e-3                   # never before it arrived (host vs GPU clock)
    assert rep["total_s"] >= rep["unit_done"][-1] - 2e-3 if K else True


@pytest.mark.parametrize("d,hq,hkv,n_layers,graph", [(128, 4, 2, 2, True), (64, 8, 2, 1, True), (128, 4, 2, 2, False)])
def test_stream_session_equals_dense_streaming_mask(st, d, hq, hkv, n_layers, graph):
    """Every token of a session -- decoded by replays of one recorded graph (graph = True) or by plain launches --
    against the dense Eq. 2 mask over the equivalent interleaved sequence."""
    rng = np.random.Generator(np.random.PCG64(1300 + d))
    batch, theta = 2, 1.0e6
    s, r = [5, 20, 3, 17], [4, 1, 9, 3]
    act, dev = _session(rng, batch, hq, hkv, d, s, r)
    results = {}
    for mode in (st.ST_SCHED_STREAMING, st.ST_SCHED_SERIAL):
        layers = _layers(st, rng, n_layers, batch, hkv, d, sum(s), sum(r))
        src_out, rsn_out, rep = st.st_stream_run(mode, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"],
                                                 dev["rv"], theta, decode_graph=graph)
        _check_report(rep, s, r)
        for c in layers:
            assert c.source.appended_len.cpu().tolist() == [sum(s)] * batch
            assert c.reasoning.appended_len.cpu().tolist() == [sum(r)] * batch
        results[mode] = (src_out, rsn_out)
        so = _unpack_src(src_out, batch, s, hq, d)
        for b in range(batch):
            o_src, o_rsn = _oracle_rows(act, b, s, r, theta)
            assert np.abs(to_f64(so[b]) - o_src).max() <= 2e-2, (mode, b)
            assert np.abs(to_f64(rsn_out[:, b]) - o_rsn).max() <= 2e-2, (mode, b)
    # the two loops running side by side change nothing: same bits as the alternating schedule
    assert torch.equal(results[st.ST_SCHED_STREAMING][0], results[st.ST_SCHED_SERIAL][0])
    assert torch.equal(results[st.ST_SCHED_STREAMING][1], results[st.ST_SCHED_SERIAL][1])


@pytest.mark.parametrize("graph", [True, False])
def test_stream_session_growing_past_the_short_cache_path(st, graph):
    """A session whose caches grow from a few hundred to 1,400 tokens: with plain launches the decoding step changes
    over, mid-session, from the single-launch kernel for short caches to the split kernel that stores the token through
    an extra work unit; the recorded graph takes the split kernel from the first token.  Every row against the dense
    Eq. 2 mask."""
    rng = np.random.Generator(np.random.PCG64(1340))
    batch, hq, hkv, d, theta = 1, 4, 2, 64, 1.0e6
    s, r = [600, 300], [300, 200]
    act, dev = _session(rng, batch, hq, hkv, d, s, r)
    layers = _layers(st, rng, 1, batch, hkv, d, sum(s), sum(r))
    src_out, rsn_out, rep = st.st_stream_run(st.ST_SCHED_SERIAL, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"],
                                             dev["rv"], theta, decode_graph=graph)
    _check_report(rep, s, r)
    assert layers[0].reasoning.appended_len.cpu().tolist() == [sum(r)] and layers[0].source.appended_len.cpu().tolist() == [sum(s)]
    o_src, o_rsn = _oracle_rows(act, 0, s, r, theta)
    assert np.abs(to_f64(_unpack_src(src_out, batch, s, hq, d)[0]) - o_src).max() <= 2e-2
    assert np.abs(to_f64(rsn_out[:, 0]) - o_rsn).max() <= 2e-2


def test_stream_session_with_arrival_times(st):
    """Sentences arriving slower than they are reasoned about: every unit waits for its prefill (Alg. 1, second
    branch), nothing happens before its sentence has arrived, results unchanged."""
    rng = np.random.Generator(np.random.PCG64(1310))
    batch, hq, hkv, d, theta = 1, 4, 2, 128, 1.0e6
    s, r = [6, 9, 2], [3, 5, 2]
    arrival = [0.0, 0.15, 0.30]
    act, dev = _session(rng, batch, hq, hkv, d, s, r)
    layers = _layers(st, rng, 1, batch, hkv, d, sum(s), sum(r))
    src_out, rsn_out, rep = st.st_stream_run(st.ST_SCHED_STREAMING, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"],
                                             dev["rk"], dev["rv"], theta, arrival_s=arrival)
    _check_report(rep, s, r, arrival)
    # (unit 0's sentence is there at time 0: whether its decode finds the prefill already done is up to the threads)
    assert rep["waited"].tolist()[1:] == [True, True] and not rep["sliced"].any()
    assert rep["first_token"][2] >= arrival[2] - 2e-3 and rep["total_s"] >= arrival[2]
    o_src, o_rsn = _oracle_rows(act, 0, s, r, theta)
    assert np.abs(to_f64(rsn_out[:, 0]) - o_rsn).max() <= 2e-2
    # the batch paradigm on the same trace: nothing is decoded before the last sentence is there, and every
    # unit sees the whole input
    layers = _layers(st, rng, 1, batch, hkv, d, sum(s), sum(r))
    _, rsn_b, rep_b = st.st_stream_run(st.ST_SCHED_BATCH, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"],
                                       dev["rv"], theta, arrival_s=arrival)
    assert rep_b["first_token"][0] >= arrival[2] - 2e-3
    assert rep_b["first_token"][0] > rep["first_token"][0]                        # streaming answers first
    _, o_rsn_all = _oracle_rows(act, 0, s, r, theta, all_sources_visible=True)
    assert np.abs(to_f64(rsn_b[:, 0]) - o_rsn_all).max() <= 2e-2


def test_stream_session_slices_when_input_is_ahead(st):
    """Everything has arrived at the start and units are long: when unit t starts, sentence t + 1 is already cached
    and the decoding loop must select a slice of the source cache (Alg. 1, first branch) -- results still those of
    the streaming mask."""
    rng = np.random.Generator(np.random.PCG64(1320))
    batch, hq, hkv, d, theta = 2, 4, 2, 128, 1.0e6
    s, r = [4, 4, 4, 4], [40, 40, 40, 5]
    act, dev = _session(rng, batch, hq, hkv, d, s, r)
    layers = _layers(st, rng, 2, batch, hkv, d, sum(s), sum(r))
    _, rsn_out, rep = st.st_stream_run(st.ST_SCHED_STREAMING, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"],
                                       dev["rv"], theta)
    _check_report(rep, s, r)
    assert rep["sliced"][1] and rep["sliced"][2] and not rep["sliced"][3]
    for b in range(batch):
        _, o_rsn = _oracle_rows(act, b, s, r, theta)
        assert np.abs(to_f64(rsn_out[:, b]) - o_rsn).max() <= 2e-2


def test_stream_run_rejects_bad_jobs(st):
    rng = np.random.Generator(np.random.PCG64(1330))
    batch, hq, hkv, d = 1, 4, 2, 64
    s, r = [3], [2]
    act, dev = _session(rng, batch, hq, hkv, d, s, r)
    layers = _layers(st, rng, 1, batch, hkv, d, 3, 2)
    same = torch.cuda.Stream()
    with pytest.raises(st.StError) as e:
        st.st_stream_run(st.ST_SCHED_STREAMING, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"], dev["rv"],
                         prefill_stream=same, decode_stream=same)
    assert e.value.status == 1
    layers[0].source.appended_len.fill_(1)
    with pytest.raises(st.StError) as e:
        st.st_stream_run(st.ST_SCHED_SERIAL, layers, hq, s, r, dev["sq"], dev["sk"], dev["sv"], dev["rq"], dev["rk"], dev["rv"])
    assert e.value.status == 1 and "empty" in str(e.value)
    layers = _layers(st, rng, 1, batch, hkv, d, 3, 2)
    with pytest.raises(st.StError) as e:          # more tokens than the page table holds
        st.st_stream_run(st.ST_SCHED_SERIAL, layers, hq, [3], [200], dev["sq"], dev["sk"], dev["sv"],
                         torch.zeros(200 * hq * d, dtype=torch.bfloat16, device=DEV), torch.zeros(200 * hkv * d, dtype=torch.bfloat16, device=DEV),
                         torch.zeros(200 * hkv * d, dtype=torch.bfloat16, device=DEV))
    assert e.value.status == 4
