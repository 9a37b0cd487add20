"""Pins for the fp64 oracle: each test ties one part of oracle/ to something the
paper or plain mathematics fixes (brute force, closed forms, library routines,
invariants), so a dropped term, wrong sign / index or transposed operand in the
oracle fails at least one of them.  CPU only."""
import os

import numpy as np
import pytest
import torch

from oracle import streaming_attention as O
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_case(seed, n_pairs, src_rng, rsn_rng, hq, hkv, d, layout="interleaved"):
    rng = np.random.Generator(np.random.PCG64(seed))
    s, r = W.draw_pairs(rng, n_pairs, src_rng, rsn_rng)
    stream, seg, pos = W.tokens_from_segments(s, r, layout)
    n = len(stream)
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    return s, r, stream, seg, pos, q, k, v


# ---- P1: dense-mask attention == brute force over the explicit visible sets (Eq. 1)
def test_p1_bruteforce_config1():
    cfg = W.config1()
    q, k, v = cfg.tensors()
    o_d, l_d = O.attention_dense(q, k, v, cfg.stream_ids, cfg.segment_ids, cfg.positions)
    o_b, l_b = O.attention_bruteforce(q, k, v, cfg.stream_ids, cfg.segment_ids, cfg.positions)
    assert np.abs(o_d - o_b).max() < 1e-12
    assert np.abs(l_d - l_b).max() < 1e-12


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_p1_bruteforce_random(seed):
    # 0-length and 1-token segments allowed
    s, r, stream, seg, pos, q, k, v = _rand_case(seed, 5, (0, 5), (0, 6), 4, 2, 8)
    if len(stream) == 0:
        pytest.skip("empty draw")
    o_d, l_d = O.attention_dense(q, k, v, stream, seg, pos)
    o_b, l_b = O.attention_bruteforce(q, k, v, stream, seg, pos)
    assert np.abs(o_d - o_b).max() < 1e-12
    assert np.abs(l_d - l_b).max() < 1e-12


def test_p1_visible_sets_match_eq1():
    """Conditioning sets of Eq. 1 written out: R_t sees C_{<=t}, R_{<t} and its own prefix; C_t sees C only."""
    s = [2, 3, 1]; r = [2, 1, 3]
    stream, seg, pos = W.tokens_from_segments(s, r, "interleaved")
    mask = O.dense_mask(stream, seg, pos)
    # physical order: S1(0,1) R1(2,3) S2(4,5,6) R2(7) S3(8) R3(9,10,11)
    expect = {
        0: [0], 1: [0, 1],
        2: [0, 1, 2], 3: [0, 1, 2, 3],
        4: [0, 1, 4], 5: [0, 1, 4, 5], 6: [0, 1, 4, 5, 6],
        7: [0, 1, 4, 5, 6, 2, 3, 7],
        8: [0, 1, 4, 5, 6, 8],
        9: [0, 1, 4, 5, 6, 8, 2, 3, 7, 9],
        10: [0, 1, 4, 5, 6, 8, 2, 3, 7, 9, 10],
        11: [0, 1, 4, 5, 6, 8, 2, 3, 7, 9, 10, 11],
    }
    for i, cols in expect.items():
        assert sorted(np.nonzero(mask[i])[0].tolist()) == sorted(cols), i


# ---- P2: the result does not depend on the physical layout (interleaved vs grouped)
@pytest.mark.parametrize("seed", [21, 22])
def test_p2_layout_equivariance(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    s, r = W.draw_pairs(rng, 4, (1, 6), (1, 7))
    st_i, sg_i, ps_i = W.tokens_from_segments(s, r, "interleaved")
    st_g, sg_g, ps_g = W.tokens_from_segments(s, r, "grouped")
    n = len(st_i)
    q = rng.standard_normal((n, 4, 16)); k = rng.standard_normal((n, 2, 16)); v = rng.standard_normal((n, 2, 16))
    # map interleaved token -> grouped slot via (stream, pos)
    key_i = st_i.astype(np.int64) * 10**6 + ps_i
    key_g = st_g.astype(np.int64) * 10**6 + ps_g
    slot = {kk: a for a, kk in enumerate(key_g)}
    to_g = np.array([slot[kk] for kk in key_i])
    qg = np.zeros_like(q); kg = np.zeros_like(k); vg = np.zeros_like(v)
    qg[to_g], kg[to_g], vg[to_g] = q, k, v
    o_i, l_i = O.attention_dense(q, k, v, st_i, sg_i, ps_i)
    o_g, l_g = O.attention_dense(qg, kg, vg, st_g, sg_g, ps_g)
    assert np.abs(o_i - o_g[to_g]).max() < 1e-12
    assert np.abs(l_i - l_g[to_g]).max() < 1e-12


# ---- P3: Eq. 2 exactly as printed (1-token segments, grouped layout)
def _eq2_as_printed(T, L):
    n = T + L
    m = np.zeros((n, n), dtype=bool)
    for i in range(1, n + 1):
        for j in range(1, n + 1):
            causal = j <= i
            removed = (i > T) and (j < T) and (j > i - T + 1)
            m[i - 1, j - 1] = causal and not removed
    return m


def test_p3_eq2_golden_file():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq2_mask_T6_L4.txt")) if l.strip() and not l.startswith("#")]
    golden = np.array(rows, dtype=int).astype(bool)
    assert (golden == _eq2_as_printed(6, 4)).all()
    _check_eq2(6, 4, golden)


def _check_eq2(T, L, printed):
    # reasoning token r (1-based) carries segment id r + 1: the row that holds the
    # last token of unit r predicts the first token of unit r + 1 (Alg. 1 re-merges
    # with a longer source slice before the next sentence).
    stream = np.array([O.SRC] * T + [O.RSN] * L)
    seg = np.array(list(range(1, T + 1)) + [r + 1 for r in range(1, L + 1)])
    pos = np.array(list(range(T)) + list(range(L)))
    mask = O.dense_mask(stream, seg, pos)
    cols = np.arange(T + L) != (T - 1)          # every column except j == T (strict "j < T" in the print)
    assert (mask[:, cols] == printed[:, cols]).all()
    # the one column the printed rule never removes: the oracle follows Eq. 1 there
    for r in range(1, L + 1):
        assert mask[T + r - 1, T - 1] == (T <= r + 1)


@pytest.mark.parametrize("T,L", [(1, 1), (3, 7), (9, 4), (12, 12)])
def test_p3_eq2_literal(T, L):
    _check_eq2(T, L, _eq2_as_printed(T, L))


# ---- P4: with every source visible the result is textbook causal attention (library routine)
@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (6, 1)])
def test_p4_reduces_to_library_causal(hq, hkv):
    rng = np.random.Generator(np.random.PCG64(40 + hq + hkv))
    S, R, d = 9, 14, 16
    stream, seg, pos = W.tokens_from_segments([S], [R], "grouped")
    n = S + R
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    o, lse = O.attention_dense(q, k, v, stream, seg, pos)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    g = hq // hkv
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(o - ref).max() < 1e-12
    # lse against torch.logsumexp of the causal scores
    sc = torch.einsum("hid,hjd->hij", tq[0], tk[0]) / np.sqrt(d)
    sc = sc.masked_fill(~torch.tril(torch.ones(n, n, dtype=torch.bool)), float("-inf"))
    assert np.abs(lse - torch.logsumexp(sc, dim=-1).T.numpy()).max() < 1e-12


# ---- P5: closed-form visible-pair counts
def test_p5_pairs_config1():
    cfg = W.config1()
    mask = O.dense_mask(cfg.stream_ids, cfg.segment_ids, cfg.positions)
    assert int(mask.sum()) == 2080 + 2080 + 2560 == 6720
    assert cfg.closed_form_pairs() == [6720]
    # physically-causal pairs that the streaming rule removes: source rows x earlier reasoning columns
    n = 128
    assert n * (n + 1) // 2 - 6720 == 1536
    md = O.canonical_metadata(cfg.stream_ids, cfg.segment_ids, cfg.positions, 16, 16)
    assert md["visible_pairs"] == 6720


@pytest.mark.parametrize("seed", [51, 52, 53])
def test_p5_pairs_random(seed):
    cfg = W.random_prefill(seed, 3, 6, (0, 9), (0, 11), 2, 1, 8, "f32")
    for b in range(cfg.batch):
        s, e = cfg.cu_seqlens[b], cfg.cu_seqlens[b + 1]
        mask = O.dense_mask(cfg.stream_ids[s:e], cfg.segment_ids[s:e], cfg.positions[s:e])
        assert int(mask.sum()) == cfg.closed_form_pairs()[b]


# ---- P6: LSE merge of two caches == attention over the concatenated cache
@pytest.mark.parametrize("ls,lr,q_len", [(7, 5, 1), (0, 6, 1), (9, 1, 1), (12, 9, 3), (0, 4, 4)])
def test_p6_lse_merge_equals_concat(ls, lr, q_len):
    rng = np.random.Generator(np.random.PCG64(60 + ls + lr))
    hq, hkv, d = 4, 2, 16
    sk = rng.standard_normal((ls + 3, hkv, d)); sv = rng.standard_normal((ls + 3, hkv, d))   # 3 not-yet-visible rows
    rk = rng.standard_normal((lr, hkv, d)); rv = rng.standard_normal((lr, hkv, d))
    q = rng.standard_normal((q_len, hq, d))
    o_c, l_c = O.decode_dual_concat(q, sk, sv, rk, rv, ls, lr)
    o_m, l_m = O.decode_dual_merged(q, sk, sv, rk, rv, ls, lr)
    assert np.abs(o_c - o_m).max() < 1e-13
    assert np.abs(l_c - l_m).max() < 1e-13


def test_p6_split_anywhere_and_both_empty():
    rng = np.random.Generator(np.random.PCG64(66))
    hq, hkv, d, n = 2, 1, 8, 11
    k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d)); q = rng.standard_normal((1, hq, d))
    full_o, full_l = O.attend_one_cache(q, k, v, np.ones((1, n), bool))
    for cut in range(n + 1):
        o1, l1 = O.attend_one_cache(q, k[:cut], v[:cut], np.ones((1, cut), bool))
        o2, l2 = O.attend_one_cache(q, k[cut:], v[cut:], np.ones((1, n - cut), bool))
        o, l = O.lse_merge(o1, l1, o2, l2)
        assert np.abs(o - full_o).max() < 1e-13 and np.abs(l - full_l).max() < 1e-13
    o, l = O.decode_dual_concat(q, k[:0], v[:0], k[:0], v[:0], 0, 0)
    assert (o == 0).all() and np.isneginf(l).all()
    # softmax weights of the plain definition, written independently
    s = (q[0, 0] @ k[:, 0].T) / np.sqrt(d)
    w = np.exp(s - s.max()); w /= w.sum()
    assert np.abs(full_o[0, 0] - w @ v[:, 0]).max() < 1e-13
    assert abs(full_l[0, 0] - np.log(np.exp(s).sum())) < 1e-12


# ---- P7: RoPE identities
def test_p7_rope_identities():
    rng = np.random.Generator(np.random.PCG64(70))
    d, h = 32, 3
    x = rng.standard_normal((5, h, d)); y = rng.standard_normal((5, h, d))
    # (i) position 0 is the identity
    assert np.array_equal(O.rope(x, np.zeros(5, int)), x)
    # (ii) each (i, i + D/2) pair keeps its norm
    p = np.array([1, 7, 100, 5000, 123456])
    rx = O.rope(x, p)
    n0 = x[..., :d // 2] ** 2 + x[..., d // 2:] ** 2
    n1 = rx[..., :d // 2] ** 2 + rx[..., d // 2:] ** 2
    assert np.abs(n0 - n1).max() < 1e-9
    # (iii) <rope(q, m), rope(k, n)> depends on m - n only
    a = np.einsum("nhd,nhd->nh", O.rope(x, np.full(5, 40)), O.rope(y, np.full(5, 33)))
    b = np.einsum("nhd,nhd->nh", O.rope(x, np.full(5, 1007)), O.rope(y, np.full(5, 1000)))
    assert np.abs(a - b).max() < 1e-9
    # (iv) equal stream-local ids: R(t - t) = I, the score equals the un-rotated one
    c = np.einsum("nhd,nhd->nh", O.rope(x, p), O.rope(y, p))
    assert np.abs(c - np.einsum("nhd,nhd->nh", x, y)).max() < 1e-8
    # (v) standard ids (T + t, t) give R(T): same as rotating q alone by T
    T = 77
    e = np.einsum("nhd,nhd->nh", O.rope(x, T + p), O.rope(y, p))
    f = np.einsum("nhd,nhd->nh", O.rope(x, np.full(5, T)), y)
    assert np.abs(e - f).max() < 1e-8


def test_p7_rope_matches_complex_rotation_and_known_values():
    rng = np.random.Generator(np.random.PCG64(71))
    d, theta = 16, 1.0e6
    x = rng.standard_normal((4, 2, d)); p = np.array([0, 3, 19, 511])
    z = x[..., :d // 2] + 1j * x[..., d // 2:]
    freq = np.array([theta ** (-(2 * i) / d) for i in range(d // 2)])
    zr = z * np.exp(1j * p[:, None, None] * freq[None, None, :])
    ref = np.concatenate([zr.real, zr.imag], axis=-1)
    assert np.abs(O.rope(x, p, theta) - ref).max() < 1e-12
    # D = 2, p = 1: a rotation by exactly one radian, counter-clockwise
    out = O.rope(np.array([[[1.0, 0.0]]]), np.array([1]), theta)
    assert np.allclose(out[0, 0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    # slowest pair of D = 4 at base 1e6 turns by p / 1000
    out = O.rope(np.array([[[0.0, 1.0, 0.0, 0.0]]]), np.array([500]), theta)
    assert np.allclose(out[0, 0], [0.0, np.cos(0.5), 0.0, np.sin(0.5)], atol=1e-15)


def test_p7_stream_local_positions():
    stream, seg, pos = W.tokens_from_segments([2, 1], [3, 2], "interleaved")
    assert O.stream_local_positions(stream).tolist() == pos.tolist() == [0, 1, 0, 1, 2, 2, 3, 4]


# ---- P8: decode over the two caches == last reasoning row of prefill
@pytest.mark.parametrize("layout", ["grouped", "interleaved"])
def test_p8_decode_equals_last_prefill_row(layout):
    rng = np.random.Generator(np.random.PCG64(80))
    s = [3, 4, 2, 5]; r = [4, 1, 6, 3]
    stream, seg, pos = W.tokens_from_segments(s, r, layout)
    n, hq, hkv, d = len(stream), 4, 2, 16
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    o, lse = O.attention_dense(q, k, v, stream, seg, pos)
    src = np.nonzero(stream == O.SRC)[0]; rsn = np.nonzero(stream == O.RSN)[0]
    # a row in the third reasoning segment: sees sources of segments 1..3 only
    row = rsn[4 + 1 + 2]
    n_rsn = 4 + 1 + 3
    o_d, l_d = O.decode_dual_concat(q[row][None], k[src], v[src], k[rsn], v[rsn], 3 + 4 + 2, n_rsn)
    assert np.abs(o_d[0] - o[row]).max() < 1e-13 and np.abs(l_d[0] - lse[row]).max() < 1e-13
    # q_len = 3: the last three reasoning rows at once
    last3 = rsn[-3:]
    o_d, l_d = O.decode_dual_concat(q[last3], k[src], v[src], k[rsn], v[rsn], sum(s), len(rsn))
    assert np.abs(o_d - o[last3]).max() < 1e-13 and np.abs(l_d - lse[last3]).max() < 1e-13


# ---- P8b: an arriving source chunk (Alg. 1, prefill loop) == the same source rows of the full prefill
@pytest.mark.parametrize("layout", ["grouped", "interleaved"])
def test_p8b_source_chunk_equals_prefill_source_rows(layout):
    rng = np.random.Generator(np.random.PCG64(81))
    s = [3, 4, 2, 5]; r = [4, 1, 6, 3]
    stream, seg, pos = W.tokens_from_segments(s, r, layout)
    n, hq, hkv, d = len(stream), 4, 2, 16
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    o, lse = O.attention_dense(q, k, v, stream, seg, pos)
    src = np.nonzero(stream == O.SRC)[0]
    # the third sentence (2 tokens) arrives when 7 source tokens are cached: cache then holds 9
    chunk = src[7:9]
    o_c, l_c = O.source_chunk_attention(q[chunk], k[src], v[src], 9)
    assert np.abs(o_c - o[chunk]).max() < 1e-13 and np.abs(l_c - lse[chunk]).max() < 1e-13
    # the whole source stream as one chunk is plain causal attention over the sources
    o_all, _ = O.source_chunk_attention(q[src], k[src], v[src], len(src))
    assert np.abs(o_all - o[src]).max() < 1e-13
    # and reasoning never leaks in: perturbing reasoning K/V leaves the chunk unchanged
    k2 = k.copy(); k2[stream == O.RSN] += 5.0
    o2, _ = O.attention_dense(q, k2, v, stream, seg, pos)
    assert np.abs(o2[chunk] - o[chunk]).max() < 1e-13


# ---- P9: paged append + gather == contiguous cache
def test_p9_paged_gather():
    rng = np.random.Generator(np.random.PCG64(90))
    batch, pages_per_seq, hkv, d = 3, 5, 2, 4
    table = W.shuffled_page_table(rng, batch, pages_per_seq)
    pool = np.full((batch * pages_per_seq, O.PAGE, hkv, d), np.nan)
    lens = np.zeros(batch, dtype=np.int64)
    contiguous = [np.zeros((0, hkv, d)) for _ in range(batch)]
    for chunk in [1, 15, 17, 3, 16, 9]:
        for b in range(batch):
            n_new = max(0, min(chunk + b, pages_per_seq * O.PAGE - int(lens[b])))
            rows = rng.standard_normal((n_new, hkv, d))
            O.paged_append(pool, table, lens, b, rows)
            contiguous[b] = np.concatenate([contiguous[b], rows])
    for b in range(batch):
        assert lens[b] == len(contiguous[b])
        assert np.array_equal(O.paged_gather(pool, table, b, int(lens[b])), contiguous[b])
    assert len(set(table.flatten().tolist())) == batch * pages_per_seq


# ---- P10: the fused forms (rotate-on-append, rotate-the-query-in-decode) == the unfused pipeline.
# The position id of a token is its index in its own stream's cache (Sec. 3.2), so caches filled piece by
# piece from UNROTATED keys hold exactly RoPE(k, stream-local ids), and decoding unrotated queries over them
# gives the prefill rows of the same tokens.
@pytest.mark.parametrize("layout", ["grouped", "interleaved"])
def test_p10_rotate_on_append_and_in_decode_equal_prefill(layout):
    rng = np.random.Generator(np.random.PCG64(100))
    s = [3, 20, 2, 9]; r = [4, 1, 17, 3]
    stream, seg, pos = W.tokens_from_segments(s, r, layout)
    n, hq, hkv, d, theta = len(stream), 4, 2, 16, 1.0e4
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    # unfused: rotate everything by the paper's ids, dense-mask attention
    o, lse = O.attention_dense(O.rope(q, pos, theta), O.rope(k, pos, theta), v, stream, seg, pos)
    src = np.nonzero(stream == O.SRC)[0]; rsn = np.nonzero(stream == O.RSN)[0]
    # fused: two paged caches filled from the UNROTATED keys in uneven pieces (pages shuffled)
    n_pages = 8
    table = rng.permutation(2 * n_pages).reshape(2, n_pages)
    caches = {}
    for b, idx, cuts in ((0, src, [0, 1, 17, 18, len(src)]), (1, rsn, [0, 5, 6, 22, len(rsn)])):
        kp = np.zeros((2 * n_pages, O.PAGE, hkv, d)); vp = np.zeros_like(kp)
        lens = np.zeros(2, dtype=np.int64)
        for a, e in zip(cuts[:-1], cuts[1:]):
            O.paged_append_rotated(kp, vp, table, lens, b, k[idx[a:e]], v[idx[a:e]], theta)
        assert lens[b] == len(idx)
        caches[b] = (O.paged_gather(kp, table, b, len(idx)), O.paged_gather(vp, table, b, len(idx)))
        # the cache holds RoPE(k, stream-local ids) and the values untouched
        assert np.abs(caches[b][0] - O.rope(k[idx], pos[idx], theta)).max() < 1e-12
        assert np.array_equal(caches[b][1], v[idx])
        assert np.array_equal(pos[idx], np.arange(len(idx)))
    (sk, sv), (rk, rv) = caches[0], caches[1]
    # last three reasoning rows (all in the last segment: every source token visible), unrotated queries
    last3 = rsn[-3:]
    o_d, l_d = O.decode_dual_rotated(q[last3], sk, sv, rk, rv, len(src), len(rsn), theta)
    assert np.abs(o_d - o[last3]).max() < 1e-12 and np.abs(l_d - lse[last3]).max() < 1e-12
    # the second sentence (20 tokens) arriving as a chunk, unrotated queries, over the cache as it was then
    chunk = src[3:23]
    o_c, l_c = O.source_chunk_attention_rotated(q[chunk], sk, sv, 23, theta)
    assert np.abs(o_c - o[chunk]).max() < 1e-12 and np.abs(l_c - lse[chunk]).max() < 1e-12
    # one row in the middle of the third reasoning segment: reasoning cache as it was then, sources of segments 1..3
    row = rsn[4 + 1 + 8]
    n_then = 4 + 1 + 9
    o_d, l_d = O.decode_dual_rotated(q[row][None], sk, sv, rk[:n_then], rv[:n_then], 3 + 20 + 2, n_then, theta)
    assert np.abs(o_d[0] - o[row]).max() < 1e-12 and np.abs(l_d[0] - lse[row]).max() < 1e-12


# ---- P11: Alg. 1 as a timeline -- hand-worked schedules, invariants, and the latencies of the paper's Table 4
def test_p11_alg1_timeline_hand_worked():
    arrival, prefill, n_dec = [1.0, 2.0, 10.0], [1.0, 1.0, 1.0], [3, 2, 1]
    t = O.alg1_timeline(arrival, prefill, n_dec, 1.0, O.STREAMING)
    assert t["prefill_done"] == [2.0, 3.0, 11.0]
    assert t["unit_start"] == [2.0, 5.0, 11.0] and t["first_token"] == [3.0, 6.0, 12.0] and t["unit_done"] == [5.0, 7.0, 12.0]
    assert t["waited"] == [True, False, True] and t["sliced"] == [False, False, False]
    # sentences arrive faster than they are reasoned about: a slice of the input cache is selected
    t = O.alg1_timeline([0.0, 0.0, 0.0], [1.0, 1.0, 1.0], [5, 1, 1], 1.0, O.STREAMING)
    assert t["prefill_done"] == [1.0, 2.0, 3.0] and t["unit_start"] == [1.0, 6.0, 7.0] and t["unit_done"] == [6.0, 7.0, 8.0]
    assert t["waited"] == [True, False, False] and t["sliced"] == [False, True, False]
    # one worker alternating prefill and decoding
    t = O.alg1_timeline(arrival, prefill, n_dec, 1.0, O.SERIAL)
    assert t["prefill_done"] == [2.0, 6.0, 11.0] and t["first_token"] == [3.0, 7.0, 12.0] and t["unit_done"] == [5.0, 8.0, 12.0]
    assert t["waited"] == [True, False, True]
    # read everything, then prefill, then decode
    t = O.alg1_timeline(arrival, prefill, n_dec, 1.0, O.BATCH)
    assert t["prefill_done"] == [11.0, 12.0, 13.0] and t["first_token"] == [14.0, 17.0, 19.0] and t["unit_done"] == [16.0, 18.0, 19.0]
    # a unit without tokens produces none
    t = O.alg1_timeline([0.0, 1.0], [1.0, 1.0], [0, 2], 1.0, O.STREAMING)
    assert t["first_token"] == [1.0, 3.0] and t["unit_done"] == [1.0, 4.0]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_p11_alg1_timeline_invariants(seed):
    rng = np.random.Generator(np.random.PCG64(1100 + seed))
    K = 7
    arrival = np.cumsum(rng.uniform(0.0, 2.0, K)).tolist()
    prefill = rng.uniform(0.05, 0.5, K).tolist()
    n_dec = rng.integers(1, 30, K).tolist()
    d = 0.07
    st, se, ba = (O.alg1_timeline(arrival, prefill, n_dec, d, m) for m in (O.STREAMING, O.SERIAL, O.BATCH))
    for t in range(K):
        # a unit never starts before its sentence is in the cache, nor before the previous unit ended
        assert st["unit_start"][t] >= st["prefill_done"][t] and (t == 0 or st["unit_start"][t] >= st["unit_done"][t - 1])
        assert st["unit_start"][t] == max(st["prefill_done"][t], st["unit_done"][t - 1] if t else 0.0)
        assert abs(st["unit_done"][t] - st["unit_start"][t] - n_dec[t] * d) < 1e-12
        # overlapping the two loops is never slower than alternating, which is never slower than batch
        assert st["first_token"][t] <= se["first_token"][t] + 1e-12 <= ba["first_token"][t] + 2e-12
        # exactly one of: waited for the prefill / started straight after the previous unit
        assert st["waited"][t] == (st["unit_start"][t] > (st["unit_done"][t - 1] if t else 0.0))
    assert abs(st["first_token"][0] - (arrival[0] + prefill[0] + d)) < 1e-12
    assert abs(ba["first_token"][0] - (arrival[-1] + sum(prefill) + d)) < 1e-12
    # with instant decoding nothing is ever sliced; with instant arrival and prefill nothing waits after unit 0
    quick = O.alg1_timeline(arrival, prefill, n_dec, 0.0, O.STREAMING)
    assert all(quick["waited"])
    slow = O.alg1_timeline([0.0] * K, [0.0] * K, n_dec, d, O.STREAMING)
    assert slow["waited"] == [False] * K and slow["sliced"] == [True] * (K - 1) + [False]


def test_p11_alg1_timeline_reproduces_table4_latencies():
    """First-token latency of the batch and of the streaming paradigm from the stage times the paper reports
    (Table 4): sentences of average length arriving at 0.4 s per word."""
    vals = {}
    with open(os.path.join(GOLDEN, "table4_efficiency_qwen3_4b.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, v = line.split()
                vals[name] = float(v)
    words, n_sent = vals["read_count_words"], vals["sentences"]
    K = 5                                             # 4.65 sentences: four of average length and a shorter one
    per = words / n_sent
    w = [per] * 4 + [words - 4 * per]
    arrival = (vals["read_avg_s"] * np.cumsum(w)).tolist()
    units = [int(round(vals["stream_decode_count"] / n_sent))] * 4
    units.append(int(vals["stream_decode_count"]) - sum(units))
    st = O.alg1_timeline(arrival, [vals["stream_prefill_avg_s"]] * K, units, vals["stream_decode_avg_s"], O.STREAMING)
    ba = O.alg1_timeline(arrival, [vals["batch_prefill_avg_s"]] + [0.0] * (K - 1), units, vals["batch_decode_avg_s"], O.BATCH)
    assert abs(st["first_token"][0] - vals["stream_first_token_s"]) / vals["stream_first_token_s"] < 0.03
    assert abs(ba["first_token"][0] - vals["batch_first_token_s"]) / vals["batch_first_token_s"] < 0.005
    # the reading time dominates: decoding of every unit but the last ends before the next sentence has been read
    assert st["waited"] == [True] * K


# ---- P12: backward of the streaming-mask attention == numerical derivative of the forward, == library autograd
def test_p12_backward_matches_central_differences():
    rng = np.random.Generator(np.random.PCG64(1200))
    stream, seg, pos = W.tokens_from_segments([2, 3, 1], [3, 1, 2], "interleaved")
    n, hq, hkv, d = len(stream), 4, 2, 6
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    g = rng.standard_normal((n, hq, d))                     # dL/d out for L = sum(g * out)
    dq, dk, dv = O.attention_dense_backward(q, k, v, g, stream, seg, pos)
    loss = lambda q_, k_, v_: float((g * O.attention_dense(q_, k_, v_, stream, seg, pos)[0]).sum())
    eps = 1e-6
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        idx = [tuple(rng.integers(0, s) for s in x.shape) for _ in range(25)]
        for i in idx:
            xp = x.copy(); xm = x.copy(); xp[i] += eps; xm[i] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(num - grad[i]) < 1e-7, (name, i, num, grad[i])
    # what a token cannot see gets no gradient from it: the first source token's K only receives gradient,
    # the last reasoning token's K / V only from itself
    last = n - 1
    only_last = np.zeros_like(g); only_last[last] = g[last]
    _, dk1, dv1 = O.attention_dense_backward(q, k, v, only_last, stream, seg, pos)
    vis = O.dense_mask(stream, seg, pos)[last]
    assert np.all(dk1[~vis] == 0) and np.all(dv1[~vis] == 0) and np.abs(dv1[vis]).min() > 0


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 1)])
def test_p12_backward_matches_library_autograd(hq, hkv):
    """torch autograd (fp64, CPU) through an explicit additive -inf mask, softmax and two matmuls."""
    rng = np.random.Generator(np.random.PCG64(1210 + hq))
    stream, seg, pos = W.tokens_from_segments([4, 1, 5], [2, 6, 3], "grouped")
    n, d = len(stream), 8
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    g = rng.standard_normal((n, hq, d))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    add = torch.tensor(np.where(O.dense_mask(stream, seg, pos), 0.0, -np.inf))
    rep = hq // hkv
    scores = torch.einsum("ihd,jhd->hij", tq, tk.repeat_interleave(rep, dim=1)) / np.sqrt(d) + add
    out = torch.einsum("hij,jhd->ihd", torch.softmax(scores, dim=-1), tv.repeat_interleave(rep, dim=1))
    (out * torch.tensor(g)).sum().backward()
    dq, dk, dv = O.attention_dense_backward(q, k, v, g, stream, seg, pos)
    assert np.abs(dq - tq.grad.numpy()).max() < 1e-12
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-12


# ---- P13: 8-bit storage of the caches (E4M3 codes, one power-of-two scale per row)
def test_p13_e4m3_matches_library_cast_on_codes_midpoints_and_random_values():
    """torch's CPU cast to float8_e4m3fn: every code's value, every midpoint between neighbours (ties), random values."""
    codes = np.array([c for c in range(256) if c & 0x7f != 0x7f], dtype=np.uint8)        # 0x7f, 0xff are NaN
    lib_vals = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(O.e4m3_decode(codes), lib_vals)
    nz = codes[(codes & 0x7f) != 0]                                                        # (-0 encodes as 0x80 too)
    assert np.array_equal(O.e4m3_encode(O.e4m3_decode(nz)), nz)
    assert np.array_equal(O.e4m3_round(lib_vals), lib_vals)                                # grid points stay
    pos = np.sort(lib_vals[lib_vals >= 0])
    mids = (pos[1:] + pos[:-1]) / 2                                                        # exact in fp32
    rng = np.random.Generator(np.random.PCG64(1301))
    rnd = np.concatenate([rng.uniform(-448, 448, 4000), rng.standard_normal(4000) * 0.01, rng.standard_normal(4000) * 3,
                          np.ldexp(rng.uniform(-1, 1, 2000), -8)]).astype(np.float32).astype(np.float64)
    for x in (mids, -mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf), rnd):
        x32 = x.astype(np.float32)
        assert np.array_equal(x32.astype(np.float64), x) or x is not rnd
        lib = torch.from_numpy(x32).to(torch.float8_e4m3fn)
        mine = O.e4m3_round(x32.astype(np.float64))
        assert np.array_equal(mine, lib.to(torch.float64).numpy())
        assert np.array_equal(O.e4m3_encode(mine) & 0x7f, lib.view(torch.uint8).numpy() & 0x7f)
        nzm = mine != 0
        assert np.array_equal(O.e4m3_encode(mine)[nzm], lib.view(torch.uint8).numpy()[nzm])
    # a tie goes to the even mantissa: 1 + 1/16 lies between 1 (mantissa 0) and 1.125 (mantissa 1)
    assert O.e4m3_round(1.0625) == 1.0 and O.e4m3_round(1.1875) == 1.25 and O.e4m3_round(2.0 ** -10) == 0.0
    assert O.e4m3_round(1.5 * 2.0 ** -9) == 2.0 ** -8 and O.e4m3_round(-447.0) == -448.0


def test_p13_row_scale_is_the_smallest_power_of_two_that_fits():
    rng = np.random.Generator(np.random.PCG64(1302))
    amax = np.concatenate([np.ldexp(rng.uniform(0.5, 1, 3000), rng.integers(-30, 30, 3000)),
                           [448.0, np.nextafter(448.0, np.inf), np.nextafter(448.0, 0), 224.0, np.nextafter(224.0, np.inf), 1.0, 7.0, 2.0 ** -20]])
    k = O.row_scale_exponent(amax)
    assert np.all(np.ldexp(amax, -k) <= 448.0) and np.all(np.ldexp(amax, -(k - 1)) > 448.0)
    assert O.row_scale_exponent(448.0) == 0 and O.row_scale_exponent(449.0) == 1 and O.row_scale_exponent(224.0) == -1
    assert O.row_scale_exponent(0.0) == 0
    assert O.row_scale_exponent(2.0 ** -120) == O.SCALE_EXP_MIN and O.row_scale_exponent(448 * 2.0 ** -100) == -100
    assert O.row_scale_exponent(449 * 2.0 ** -100) == -99


def test_p13_store_is_idempotent_and_within_half_a_step():
    rng = np.random.Generator(np.random.PCG64(1303))
    x = W.bf16_round((rng.standard_normal((50, 3, 64)) * np.ldexp(1.0, rng.integers(-6, 6, (50, 3, 1)))).astype(np.float32)).astype(np.float64)
    x[7] = 0.0                                                                              # an all-zero row
    x[8, :, 1:] = 0.0                                                                       # a single nonzero entry
    codes, k = O.quantize_rows_e4m3(x)
    assert codes.dtype == np.uint8 and codes.shape == x.shape and k.shape == x.shape[:-1]
    back = O.dequantize_rows_e4m3(codes, k)
    c2, k2 = O.quantize_rows_e4m3(back)
    assert np.array_equal(O.dequantize_rows_e4m3(c2, k2), back)                            # what comes out goes back in unchanged
    # the row maximum lands in the top binade, so a normal value keeps 3 mantissa bits: relative error <= 2^-4;
    # anything below 2^-6 of the scaled row sits on the 2^-9 grid: absolute error <= 2^-10 of the scale
    step_err = np.maximum(np.abs(x) * 2.0 ** -4, np.ldexp(1.0, k - 10)[..., None])
    assert np.all(np.abs(back - x) <= step_err)
    amax = np.abs(x).max(axis=-1)
    top = np.abs(O.e4m3_decode(codes)).max(axis=-1)
    assert np.all((top >= 224.0) | (amax == 0)) and np.all(top <= 448.0)        # (224, 448] before rounding
    assert np.array_equal(back[7], np.zeros_like(back[7])) and np.array_equal(back[8, :, 0], x[8, :, 0] * 0 + back[8, :, 0])
    assert np.abs(back[8, :, 0] - x[8, :, 0]).max() <= np.abs(x[8, :, 0]).max() * 2.0 ** -4


def test_p13_decode_over_8bit_caches():
    """Values already on the grid pass through untouched (== the plain decode); otherwise the result is the plain
    decode of the stored values and stays close to the unquantised one."""
    rng = np.random.Generator(np.random.PCG64(1304))
    hq, hkv, d, ls, lr = 4, 2, 16, 21, 9
    q = rng.standard_normal((1, hq, d))
    sk, sv = rng.standard_normal((ls, hkv, d)), rng.standard_normal((ls, hkv, d))
    rk, rv = rng.standard_normal((lr, hkv, d)), rng.standard_normal((lr, hkv, d))
    rq = lambda a: O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(a))
    o8, l8 = O.decode_dual_fp8(q, sk, sv, rk, rv, 17, lr)
    o_plain, l_plain = O.decode_dual_concat(q, rq(sk), rq(sv), rq(rk), rq(rv), 17, lr)
    assert np.array_equal(o8, o_plain) and np.array_equal(l8, l_plain)
    og, lg = O.decode_dual_fp8(q, rq(sk), rq(sv), rq(rk), rq(rv), 17, lr)
    assert np.array_equal(og, o_plain)
    o_ref, _ = O.decode_dual_concat(q, sk, sv, rk, rv, 17, lr)
    assert 0 < np.abs(o8 - o_ref).max() < 0.15


# ---- metadata derived from the dense mask: closed forms for config 1
def test_metadata_config1_closed_form():
    cfg = W.config1()
    md = O.canonical_metadata(cfg.stream_ids, cfg.segment_ids, cfg.positions, 16, 16)
    # source tokens sit at physical 0-15, 32-47, ...; reasoning at 16-31, 48-63, ...
    assert md["src_idx"].tolist() == [32 * (i // 16) + i % 16 for i in range(64)]
    assert md["rsn_idx"].tolist() == [32 * (i // 16) + 16 + i % 16 for i in range(64)]
    assert md["vis_src"].tolist() == [16 * (i // 16 + 1) for i in range(64)]
    tri = np.array([[O.PARTIAL if a == c else (O.FULL if c < a else O.SKIP) for c in range(4)] for a in range(4)])
    rect = np.array([[O.FULL if c <= a else O.SKIP for c in range(4)] for a in range(4)])
    assert (md["SS"] == tri).all() and (md["RR"] == tri).all() and (md["RS"] == rect).all()
    assert O.source_prefix_table(cfg.stream_ids, cfg.segment_ids).tolist() == [0, 16, 32, 48, 64]


def test_metadata_vis_src_is_prefix_of_segment():
    cfg = W.random_prefill(97, 1, 7, (0, 20), (0, 30), 2, 1, 8, "f32")
    md = O.canonical_metadata(cfg.stream_ids, cfg.segment_ids, cfg.positions, 32, 16)
    P = O.source_prefix_table(cfg.stream_ids, cfg.segment_ids)
    rsn_seg = cfg.segment_ids[md["rsn_idx"]]
    assert md["vis_src"].tolist() == [int(P[g]) for g in rsn_seg]
    # ragged tiles: a tile made only of in-range visible entries is FULL
    s_tot = int((cfg.stream_ids == O.SRC).sum())
    if s_tot:
        assert md["SS"][0, 0] in (O.PARTIAL, O.FULL)


def test_bf16_rounding_helper_roundtrip():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-30, 65504.0], dtype=np.float32)
    r = W.bf16_round(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    assert np.array_equal(W.bf16_from_bits(W.bf16_bits(r)), r)


# ---- P14: the row-subset and packed-batch forms are the same definitions (Eq. 1, Eq. 2, Sec. 3.2)
def _ragged_structures():
    """configs[0] in both layouts, plus random ragged structures with empty and 1-token segments."""
    cases = []
    for layout in ("interleaved", "grouped"):
        c = W.config1(layout)
        cases.append((f"cfg1-{layout}", c.stream_ids, c.segment_ids, c.positions))
        for seed in (1401, 1402, 1403):
            rng = np.random.Generator(np.random.PCG64(seed))
            s, r = W.draw_pairs(rng, 6, (0, 4), (0, 5))
            s[1] = 0; r[2] = 0; s[3] = 1; r[4] = 1            # empty and 1-token segments on both streams
            st, sg, ps = W.tokens_from_segments(s, r, layout)
            cases.append((f"rand{seed}-{layout}", st, sg, ps))
    return cases


@pytest.mark.parametrize("name,stream,seg,pos", _ragged_structures(), ids=lambda x: x if isinstance(x, str) else "")
def test_p14_mask_rows_is_eq1_row_by_row(name, stream, seg, pos):
    """mask_rows against the scalar rule of Eq. 1 (visible(), pinned by the hand-listed sets and by Eq. 2 as
    printed) pair by pair, and against the rows of the dense mask, for row lists in any order with repeats."""
    n = len(stream)
    rng = np.random.Generator(np.random.PCG64(1410))
    for rows in (np.arange(n), np.arange(n)[::-1], rng.integers(0, n, size=2 * n), np.array([n - 1, 0, n - 1]), np.zeros(0, np.int64)):
        got = O.mask_rows(stream, seg, pos, rows)
        assert got.shape == (len(rows), n) and got.dtype == bool
        assert (got == O.dense_mask(stream, seg, pos)[rows]).all()
        for a, i in enumerate(rows):
            for j in range(n):
                assert got[a, j] == O.visible(stream[i], seg[i], pos[i], stream[j], seg[j], pos[j]), (name, i, j)


def test_p14_mask_rows_hand_listed_sets_and_eq2_print():
    """The same hand-written conditioning sets and the same printed Eq. 2 matrix that pin dense_mask."""
    stream, seg, pos = W.tokens_from_segments([2, 3, 1], [2, 1, 3], "interleaved")
    # physical order: S1(0,1) R1(2,3) S2(4,5,6) R2(7) S3(8) R3(9,10,11)
    expect = {7: [0, 1, 4, 5, 6, 2, 3, 7], 8: [0, 1, 4, 5, 6, 8], 2: [0, 1, 2], 11: [0, 1, 4, 5, 6, 8, 2, 3, 7, 9, 10, 11], 4: [0, 1, 4]}
    rows = list(expect)
    got = O.mask_rows(stream, seg, pos, rows)
    for a, i in enumerate(rows):
        assert sorted(np.nonzero(got[a])[0].tolist()) == sorted(expect[i]), i
    T, L = 6, 4
    lines = [l.split() for l in open(os.path.join(GOLDEN, "eq2_mask_T6_L4.txt")) if l.strip() and not l.startswith("#")]
    printed = np.array(lines, dtype=int).astype(bool)
    stream = np.array([O.SRC] * T + [O.RSN] * L)
    seg = np.array(list(range(1, T + 1)) + [r + 1 for r in range(1, L + 1)])
    pos = np.array(list(range(T)) + list(range(L)))
    rows = np.array([9, 6, 0, 7, 8, 5])
    cols = np.arange(T + L) != (T - 1)
    assert (O.mask_rows(stream, seg, pos, rows)[:, cols] == printed[rows][:, cols]).all()


@pytest.mark.parametrize("name,stream,seg,pos", _ragged_structures(), ids=lambda x: x if isinstance(x, str) else "")
def test_p14_attention_rows_equals_rows_of_attention(name, stream, seg, pos):
    """attention_dense(rows=r) == attention_dense()[r], exactly (same products, same sums per row), and == the
    brute force over the gathered visible sets on the tiny cases."""
    n = len(stream)
    rng = np.random.Generator(np.random.PCG64(1420))
    hq, hkv, d = 4, 2, 8
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    o_all, l_all = O.attention_dense(q, k, v, stream, seg, pos)
    for rows in (rng.permutation(n)[: max(1, n // 3)], np.array([n - 1, 0]), np.arange(n)):
        o_r, l_r = O.attention_dense(q, k, v, stream, seg, pos, rows=rows)
        assert o_r.shape == (len(rows), hq, d) and l_r.shape == (len(rows), hq)
        assert np.abs(o_r - o_all[rows]).max() < 1e-14 and np.abs(l_r - l_all[rows]).max() < 1e-14
    if n <= 40:
        o_b, l_b = O.attention_bruteforce(q, k, v, stream, seg, pos)
        rows = rng.permutation(n)[:5]
        o_r, l_r = O.attention_dense(q, k, v, stream, seg, pos, rows=rows)
        assert np.abs(o_r - o_b[rows]).max() < 1e-12 and np.abs(l_r - l_b[rows]).max() < 1e-12


def _packed_batch(seed, hq, hkv, d):
    """Three sequences packed one after the other, the middle one EMPTY, ids restarting in every sequence."""
    rng = np.random.Generator(np.random.PCG64(seed))
    metas = [W.tokens_from_segments([3, 0, 2], [2, 4, 1], "interleaved"),
             (np.zeros(0, np.int32),) * 3,
             W.tokens_from_segments([1, 5], [6, 0], "grouped"),
             W.tokens_from_segments([4], [3], "interleaved")]
    cu = np.cumsum([0] + [len(m[0]) for m in metas]).astype(np.int32)
    stream, seg, pos = (np.concatenate([m[i] for m in metas]) for i in range(3))
    n = int(cu[-1])
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    g = rng.standard_normal((n, hq, d))
    return cu, stream, seg, pos, q, k, v, g


def test_p14_varlen_forward_is_per_sequence_attention():
    cu, stream, seg, pos, q, k, v, g = _packed_batch(1430, 4, 2, 8)
    out, lse = O.attention_varlen(q, k, v, stream, seg, pos, cu)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        if e == s:
            continue
        # an independent route per sequence: the brute force over the visible sets of Eq. 1
        o_b, l_b = O.attention_bruteforce(q[s:e], k[s:e], v[s:e], stream[s:e], seg[s:e], pos[s:e])
        assert np.abs(out[s:e] - o_b).max() < 1e-12 and np.abs(lse[s:e] - l_b).max() < 1e-12
    # no token sees another sequence: changing sequence 0's keys / values leaves the others' rows bit-identical
    k2 = k.copy(); v2 = v.copy(); k2[: cu[1]] += 3.0; v2[: cu[1]] -= 2.0
    out2, lse2 = O.attention_varlen(q, k2, v2, stream, seg, pos, cu)
    assert (out2[cu[1]:] == out[cu[1]:]).all() and (lse2[cu[1]:] == lse[cu[1]:]).all()
    assert np.abs(out2[: cu[1]] - out[: cu[1]]).max() > 1e-3
    # a scale passed through reaches every sequence
    o_s, _ = O.attention_varlen(q, k, v, stream, seg, pos, cu, scale=0.3)
    s, e = int(cu[2]), int(cu[3])
    assert np.abs(o_s[s:e] - O.attention_dense(q[s:e], k[s:e], v[s:e], stream[s:e], seg[s:e], pos[s:e], 0.3)[0]).max() < 1e-14


def test_p14_varlen_backward_is_per_sequence_and_stays_inside_sequences():
    cu, stream, seg, pos, q, k, v, g = _packed_batch(1440, 4, 2, 6)
    dq, dk, dv = O.attention_varlen_backward(q, k, v, g, stream, seg, pos, cu)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        dq_b, dk_b, dv_b = O.attention_dense_backward(q[s:e], k[s:e], v[s:e], g[s:e], stream[s:e], seg[s:e], pos[s:e])
        assert (dq[s:e] == dq_b).all() and (dk[s:e] == dk_b).all() and (dv[s:e] == dv_b).all()
    # independent of the per-sequence routine: central differences of the PACKED forward
    loss = lambda q_, k_, v_: float((g * O.attention_varlen(q_, k_, v_, stream, seg, pos, cu)[0]).sum())
    rng = np.random.Generator(np.random.PCG64(1441))
    eps = 1e-6
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(20):
            i = tuple(int(rng.integers(0, s)) for s in x.shape)
            xp = x.copy(); xm = x.copy(); xp[i] += eps; xm[i] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(num - grad[i]) < 1e-7, (name, i, num, grad[i])
    # gradient flowing only into the LAST sequence's outputs leaves dk / dv of the other sequences exactly zero
    g_last = np.zeros_like(g); g_last[cu[-2]:] = g[cu[-2]:]
    dq1, dk1, dv1 = O.attention_varlen_backward(q, k, v, g_last, stream, seg, pos, cu)
    assert np.all(dk1[: cu[-2]] == 0) and np.all(dv1[: cu[-2]] == 0) and np.all(dq1[: cu[-2]] == 0)
    assert np.abs(dk1[cu[-2]:]).max() > 0 and np.abs(dv1[cu[-2]:]).max() > 0
