"""fp64 CPU oracle for streaming-constrained attention (StreamingThinker).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP
kernels are checked against.  It may be imported by tests/, by the smoke check
and by the bench's cpu_baseline leg -- never by the product package, and it
imports nothing from it.  Everything is numpy in float64, one definition per
function, no blocking / fusion / reordering.

What the paper fixes and where:
  * which token may attend to which      -- Eq. 1 (conditioning sets), Eq. 2
    (streaming mask on top of the causal mask), Sec. 3.2 "Streaming Attention
    Mask Matrix", Appendix E.1, Alg. 1 (N_EOS == N_EOT + 1)
  * stream-local position ids for RoPE    -- Sec. 3.2 "Streaming Position
    Encoding" (input and reasoning tokens are numbered independently from 0)
  * two KV caches read jointly at decode  -- Sec. 3.3 "Parallel KV caches",
    Alg. 1 (merge of the source slice and the reasoning cache before decoding)

Readings taken where the paper is silent (softmax scale 1/sqrt(D), grouped-query
head mapping, rotate-half RoPE pairing, base 1e6) are pinned to the textbook /
library convention by tests/test_oracle_pins.py.

Pins (all in tests/test_oracle_pins.py): brute-force gather, layout
equivariance, Eq. 2 as printed, reduction to library causal attention, source chunk == source rows of prefill,
closed-form visible-pair counts, LSE-merge == concatenation, RoPE identities,
decode == last prefill row, paged gather == contiguous, rotate-on-append / rotate-in-decode ==
the unfused pipeline, Alg. 1 timeline == hand-worked schedules and the paper's Table 4 latencies,
backward == central differences of the forward and == library autograd of a dense-mask softmax,
E4M3 rounding / bytes == a library's cast over all codes, midpoints and random values, row scales == their
defining inequality, 8-bit store idempotent and within half a grid step, the row-subset mask / attention ==
the scalar rule pair by pair, the hand-listed sets, Eq. 2 as printed and the rows of the full result, the
packed-batch forward / backward == brute force per sequence and central differences of the packed forward.
No function here is "parity unpinned".
"""
import numpy as np

SRC = 0  # token of the input ("source") stream
RSN = 1  # token of the reasoning stream

PAGE = 16  # tokens per KV-cache page


# --------------------------------------------------------------------------
# Visibility (Eq. 1 / Eq. 2 / Alg. 1)
# --------------------------------------------------------------------------
def visible(stream_i, seg_i, pos_i, stream_j, seg_j, pos_j):
    """May query token i attend to key token j (same sequence)?

    Eq. 1: reasoning unit R_t conditions on C_{<=t} and R_{<=t-1} (plus itself,
    causally); input sentences condition on earlier input only.  Eq. 2 states
    the same thing as a mask: causal everywhere, and in the reasoning-rows x
    input-columns block the inputs of later steps are removed.
    """
    if stream_i == SRC:
        # a source row never sees reasoning; among sources it is causal
        return stream_j == SRC and pos_j <= pos_i
    # reasoning row
    if stream_j == RSN:
        return pos_j <= pos_i           # causal over the whole reasoning stream
    return seg_j <= seg_i               # source segments up to the row's own step


def dense_mask(stream, seg, pos):
    """bool[n, n]: mask[i, j] = visible(i, j), for one sequence.

    Same rule as visible(), written with broadcasting.
    """
    stream = np.asarray(stream); seg = np.asarray(seg); pos = np.asarray(pos)
    si, sj = stream[:, None], stream[None, :]
    src_row = (si == SRC) & (sj == SRC) & (pos[None, :] <= pos[:, None])
    rsn_rsn = (si == RSN) & (sj == RSN) & (pos[None, :] <= pos[:, None])
    rsn_src = (si == RSN) & (sj == SRC) & (seg[None, :] <= seg[:, None])
    return src_row | rsn_rsn | rsn_src


def mask_rows(stream, seg, pos, rows):
    """bool[len(rows), n]: the rows `rows` of dense_mask, without building it all."""
    stream = np.asarray(stream); seg = np.asarray(seg); pos = np.asarray(pos)
    rows = np.asarray(rows)
    si, sj = stream[rows][:, None], stream[None, :]
    pi, gi = pos[rows][:, None], seg[rows][:, None]
    return (((si == SRC) & (sj == SRC) & (pos[None, :] <= pi))
            | ((si == RSN) & (sj == RSN) & (pos[None, :] <= pi))
            | ((si == RSN) & (sj == SRC) & (seg[None, :] <= gi)))


# --------------------------------------------------------------------------
# Masked softmax attention (plain definition)
# --------------------------------------------------------------------------
def _softmax_attend(scores, mask, v):
    """scores[m, n] (already scaled), mask[m, n] bool, v[n, D] -> out[m, D], lse[m].

    Max-subtracted softmax over the visible columns.  A row with no visible
    column gives out = 0 and lse = -inf.
    """
    s = np.where(mask, scores, -np.inf)
    mx = s.max(axis=1, keepdims=True, initial=-np.inf)
    mx_safe = np.where(np.isfinite(mx), mx, 0.0)
    e = np.where(mask, np.exp(s - mx_safe), 0.0)
    den = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        out = np.where(den > 0, (e @ v) / np.where(den > 0, den, 1.0), 0.0)
        lse = np.where(den[:, 0] > 0, mx_safe[:, 0] + np.log(np.where(den[:, 0] > 0, den[:, 0], 1.0)), -np.inf)
    return out, lse


def attention_dense(q, k, v, stream, seg, pos, scale=None, rows=None):
    """Streaming-mask attention for ONE sequence.

    q[n, Hq, D], k[n, Hkv, D], v[n, Hkv, D] (any float dtype; promoted to fp64).
    Query head h reads KV head h // (Hq // Hkv).  Returns out[m, Hq, D] and
    lse[m, Hq] (natural log of the softmax denominator), m = n or len(rows).
    """
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, hq, d = q.shape
    hkv = k.shape[1]
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    if rows is None:
        rows = np.arange(n)
        mask = dense_mask(stream, seg, pos)
    else:
        rows = np.asarray(rows)
        mask = mask_rows(stream, seg, pos, rows)
    out = np.zeros((len(rows), hq, d)); lse = np.zeros((len(rows), hq))
    for h in range(hq):
        hk = h // group
        scores = scale * (q[rows, h, :] @ k[:, hk, :].T)
        out[:, h, :], lse[:, h] = _softmax_attend(scores, mask, v[:, hk, :])
    return out, lse


def attention_varlen(q, k, v, stream, seg, pos, cu_seqlens, scale=None):
    """attention_dense over a packed batch; cu_seqlens has B + 1 entries."""
    q = np.asarray(q); out = np.zeros(q.shape, dtype=np.float64)
    lse = np.zeros(q.shape[:2], dtype=np.float64)
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        out[s:e], lse[s:e] = attention_dense(q[s:e], k[s:e], v[s:e], stream[s:e], seg[s:e], pos[s:e], scale)
    return out, lse


def attention_bruteforce(q, k, v, stream, seg, pos, scale=None):
    """Same result as attention_dense, from the conditioning SETS of Eq. 1.

    No mask matrix: for each row the list of visible token indices is gathered
    by walking the segments (source steps <= the row's step; reasoning tokens
    up to and including the row), then a softmax over that list.  Pure-Python
    loops; tiny inputs only.
    """
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, hq, d = q.shape
    group = hq // k.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((n, hq, d)); lse = np.zeros((n, hq))
    for i in range(n):
        vis = [j for j in range(n)
               if visible(stream[i], seg[i], pos[i], stream[j], seg[j], pos[j])]
        for h in range(hq):
            hk = h // group
            sc = [scale * sum(q[i, h, t] * k[j, hk, t] for t in range(d)) for j in vis]
            mx = max(sc)
            w = [np.exp(x - mx) for x in sc]
            den = sum(w)
            for t in range(d):
                out[i, h, t] = sum(w[a] * v[vis[a], hk, t] for a in range(len(vis))) / den
            lse[i, h] = mx + np.log(den)
    return out, lse


def attention_dense_backward(q, k, v, d_out, stream, seg, pos, scale=None):
    """Gradients of attention_dense for ONE sequence (streaming-constrained training, Sec. 3.2: the
    mask of Eq. 2 is applied in the forward pass, so masked pairs carry no gradient).

    Given d_out = dL/d out [n, Hq, D], returns dq [n, Hq, D], dk, dv [n, Hkv, D] (summed over the
    query heads of a KV group).  With P = softmax over the visible keys and delta_i = sum_d d_out_i * out_i:
        dV_j = sum_i P_ij d_out_i        dP_ij = d_out_i . V_j        dS_ij = P_ij (dP_ij - delta_i)
        dQ_i = scale sum_j dS_ij K_j     dK_j = scale sum_i dS_ij Q_i
    which is the chain rule through out = P V, P = softmax(scale Q K^T) written out.
    """
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64); d_out = np.asarray(d_out, dtype=np.float64)
    n, hq, d = q.shape
    hkv = k.shape[1]
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    mask = dense_mask(stream, seg, pos)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for h in range(hq):
        hk = h // group
        s = np.where(mask, scale * (q[:, h, :] @ k[:, hk, :].T), -np.inf)
        mx = s.max(axis=1, keepdims=True, initial=-np.inf)
        mx = np.where(np.isfinite(mx), mx, 0.0)
        e = np.where(mask, np.exp(s - mx), 0.0)
        den = e.sum(axis=1, keepdims=True)
        p = e / np.where(den > 0, den, 1.0)
        out = p @ v[:, hk, :]
        delta = (d_out[:, h, :] * out).sum(axis=1, keepdims=True)
        d_p = d_out[:, h, :] @ v[:, hk, :].T
        d_s = p * (d_p - delta)
        dv[:, hk, :] += p.T @ d_out[:, h, :]
        dq[:, h, :] = scale * (d_s @ k[:, hk, :])
        dk[:, hk, :] += scale * (d_s.T @ q[:, h, :])
    return dq, dk, dv


def attention_varlen_backward(q, k, v, d_out, stream, seg, pos, cu_seqlens, scale=None):
    """attention_dense_backward over a packed batch."""
    dq = np.zeros(np.asarray(q).shape); dk = np.zeros(np.asarray(k).shape); dv = np.zeros(np.asarray(v).shape)
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        dq[s:e], dk[s:e], dv[s:e] = attention_dense_backward(q[s:e], k[s:e], v[s:e], d_out[s:e], stream[s:e], seg[s:e], pos[s:e], scale)
    return dq, dk, dv


# --------------------------------------------------------------------------
# RoPE with stream-local positions (Sec. 3.2 "Streaming Position Encoding")
# --------------------------------------------------------------------------
def rope(x, positions, theta=1.0e6):
    """Rotate x[n, H, D] by positions[n]; rotate-half pairing (i, i + D/2).

    f_i = theta ** (-2 i / D); a = p * f_i;
    y_i       = x_i cos a - x_{i+D/2} sin a
    y_{i+D/2} = x_{i+D/2} cos a + x_i sin a
    The positions are whatever the caller assigns; the paper's assignment is
    one counter per stream, both starting at 0 (see stream_local_positions).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    freq = theta ** (-2.0 * i / d)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def stream_local_positions(stream):
    """The paper's position ids: the n-th token of each stream gets id n (0-based)."""
    stream = np.asarray(stream)
    pos = np.zeros(len(stream), dtype=np.int64)
    for kind in (SRC, RSN):
        idx = np.nonzero(stream == kind)[0]
        pos[idx] = np.arange(len(idx))
    return pos


# --------------------------------------------------------------------------
# Dual-cache decode (Sec. 3.3 "Parallel KV caches"; Alg. 1 merge + decode)
# --------------------------------------------------------------------------
def decode_dual_concat(q, src_k, src_v, rsn_k, rsn_v, src_visible_len, rsn_len, scale=None):
    """One sequence.  q[q_len, Hq, D]; caches [len, Hkv, D] (logical order).

    The merged cache of Alg. 1 written out: keys = visible source slice
    followed by the reasoning cache.  Query row t (of q_len, the LAST q_len
    reasoning tokens, already appended) sees the whole source slice and
    reasoning tokens [0, rsn_len - q_len + t].  Returns out[q_len, Hq, D],
    lse[q_len, Hq].
    """
    q = np.asarray(q, dtype=np.float64)
    q_len, hq, d = q.shape
    sk = np.asarray(src_k, dtype=np.float64)[:src_visible_len]
    sv = np.asarray(src_v, dtype=np.float64)[:src_visible_len]
    rk = np.asarray(rsn_k, dtype=np.float64)[:rsn_len]
    rv = np.asarray(rsn_v, dtype=np.float64)[:rsn_len]
    kk = np.concatenate([sk, rk], axis=0); vv = np.concatenate([sv, rv], axis=0)
    hkv = kk.shape[1]
    group = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    n = kk.shape[0]
    col = np.arange(n)[None, :]
    limit = src_visible_len + rsn_len - q_len + np.arange(q_len)[:, None]   # last visible column
    mask = col <= limit
    out = np.zeros((q_len, hq, d)); lse = np.zeros((q_len, hq))
    for h in range(hq):
        hk = h // group
        scores = scale * (q[:, h, :] @ kk[:, hk, :].T)
        out[:, h, :], lse[:, h] = _softmax_attend(scores, mask, vv[:, hk, :])
    return out, lse


def attend_one_cache(q, k, v, mask, scale=None):
    """Softmax attention of q[m, Hq, D] over ONE cache k, v[n, Hkv, D] -> (out, lse)."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    m, hq, d = q.shape
    group = hq // k.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((m, hq, d)); lse = np.zeros((m, hq))
    for h in range(hq):
        hk = h // group
        scores = scale * (q[:, h, :] @ k[:, hk, :].T)
        out[:, h, :], lse[:, h] = _softmax_attend(scores, mask, v[:, hk, :])
    return out, lse


def lse_merge(o1, lse1, o2, lse2):
    """Combine two partial attentions over disjoint key sets.

    m = max(lse1, lse2); w_c = exp(lse_c - m); o = (w1 o1 + w2 o2) / (w1 + w2);
    lse = m + log(w1 + w2).  An empty set has lse = -inf, weight 0.
    """
    m = np.maximum(lse1, lse2)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w1 = np.where(np.isfinite(lse1), np.exp(lse1 - m_safe), 0.0)
    w2 = np.where(np.isfinite(lse2), np.exp(lse2 - m_safe), 0.0)
    den = w1 + w2
    den_safe = np.where(den > 0, den, 1.0)
    o = np.where(den[..., None] > 0, (w1[..., None] * o1 + w2[..., None] * o2) / den_safe[..., None], 0.0)
    with np.errstate(divide="ignore"):
        lse = np.where(den > 0, m_safe + np.log(den_safe), -np.inf)
    return o, lse


def decode_dual_merged(q, src_k, src_v, rsn_k, rsn_v, src_visible_len, rsn_len, scale=None):
    """decode_dual_concat computed as two separate softmaxes + lse_merge."""
    q = np.asarray(q, dtype=np.float64)
    q_len = q.shape[0]
    m_src = np.ones((q_len, src_visible_len), dtype=bool)
    col = np.arange(rsn_len)[None, :]
    m_rsn = col <= (rsn_len - q_len + np.arange(q_len)[:, None])
    o1, l1 = attend_one_cache(q, np.asarray(src_k)[:src_visible_len], np.asarray(src_v)[:src_visible_len], m_src, scale)
    o2, l2 = attend_one_cache(q, np.asarray(rsn_k)[:rsn_len], np.asarray(rsn_v)[:rsn_len], m_rsn, scale)
    return lse_merge(o1, l1, o2, l2)


def source_chunk_attention(q, src_k, src_v, src_len, scale=None):
    """Attention of an arriving source chunk (Alg. 1, prefill loop), one sequence.

    q[n_new, Hq, D] are the queries of the n_new NEWEST source tokens, whose keys / values are
    already rows src_len - n_new .. src_len - 1 of the source cache [src_len, Hkv, D].  Source
    tokens see source tokens at positions <= their own and nothing else (Eq. 1: C_t conditions
    on earlier input only), so row t sees cache rows [0, src_len - n_new + t].
    """
    q = np.asarray(q, dtype=np.float64)
    n_new = q.shape[0]
    col = np.arange(src_len)[None, :]
    mask = col <= (src_len - n_new + np.arange(n_new)[:, None])
    return attend_one_cache(q, np.asarray(src_k)[:src_len], np.asarray(src_v)[:src_len], mask, scale)


def source_chunk_attention_rotated(q, src_k, src_v, src_len, theta=1.0e6, scale=None):
    """source_chunk_attention for UNROTATED queries: query row t is the source token at index
    src_len - n_new + t of the source stream, and that index is its position id (Sec. 3.2)."""
    n_new = np.asarray(q).shape[0]
    return source_chunk_attention(rope(q, src_len - n_new + np.arange(n_new), theta), src_k, src_v, src_len, scale)


# --------------------------------------------------------------------------
# Paged cache model (append / gather)
# --------------------------------------------------------------------------
def paged_append(pool, page_table, lens, b, new_rows):
    """Write new_rows[n_new, Hkv, D] at logical positions lens[b].. of sequence b.

    pool[n_pages, PAGE, Hkv, D] is the LOGICAL pool (page, slot); logical
    position p of sequence b lives in page page_table[b][p // PAGE], slot
    p % PAGE.  lens[b] is advanced.
    """
    for t in range(new_rows.shape[0]):
        p = int(lens[b]) + t
        pool[page_table[b][p // PAGE], p % PAGE] = new_rows[t]
    lens[b] += new_rows.shape[0]


def paged_gather(pool, page_table, b, length):
    """Logical rows [0, length) of sequence b as a contiguous [length, Hkv, D] array."""
    out = np.zeros((length,) + pool.shape[2:], dtype=pool.dtype)
    for p in range(length):
        out[p] = pool[page_table[b][p // PAGE], p % PAGE]
    return out


def paged_append_rotated(k_pool, v_pool, page_table, lens, b, k_rows, v_rows, theta=1.0e6):
    """Append UNROTATED keys: key t of the call gets the position id of its stream, which is
    its index in that stream's cache, lens[b] + t (Sec. 3.2: the ids of a stream count its own
    tokens from 0, so they never change when caches are merged or split), is rotated by it and
    stored; values are stored as they are.  lens[b] is advanced once.
    """
    n = k_rows.shape[0]
    positions = int(lens[b]) + np.arange(n)
    start = lens.copy()
    paged_append(k_pool, page_table, lens, b, rope(k_rows, positions, theta))
    paged_append(v_pool, page_table, start, b, v_rows)


def decode_dual_rotated(q, src_k, src_v, rsn_k, rsn_v, src_visible_len, rsn_len, theta=1.0e6, scale=None):
    """decode_dual_concat for UNROTATED queries: query row t of the q_len rows is the reasoning
    token at index rsn_len - q_len + t of its stream (it is already in the reasoning cache, Alg. 1),
    and that index is its position id.
    """
    q_len = q.shape[0]
    positions = rsn_len - q_len + np.arange(q_len)
    return decode_dual_concat(rope(q, positions, theta), src_k, src_v, rsn_k, rsn_v, src_visible_len, rsn_len, scale)


# --------------------------------------------------------------------------
# 8-bit storage of the two caches (Sec. 3.3's caches in the OCP FP8 E4M3 format; the paper stores
# them in the model's precision -- this is a storage variant of the same operator, defined here)
# --------------------------------------------------------------------------
E4M3_MAX = 448.0          # largest finite E4M3 value: 1.75 * 2^8
_E4M3_MIN_EXP = -6        # exponent of the smallest normal value; below it the grid step stays 2^-9


def e4m3_round(x):
    """Nearest value of the E4M3 grid, ties to the even mantissa, for |x| <= 448 (the quantiser below
    never asks for more).  E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; the grid step in the binade
    [2^e, 2^(e+1)) is 2^(e-3), and 2^-9 everywhere below 2^-6 (subnormals)."""
    x = np.asarray(x, dtype=np.float64)
    assert np.all(np.abs(x) <= E4M3_MAX)
    _, ex = np.frexp(np.abs(x))                     # |x| = m 2^ex with m in [0.5, 1)
    e = np.maximum(ex - 1, _E4M3_MIN_EXP)
    step = np.ldexp(1.0, e - 3)
    return np.sign(x) * np.rint(np.abs(x) / step) * step      # rint rounds halves to even


def e4m3_encode(v):
    """Byte of a value that lies on the E4M3 grid: sign << 7 | exponent field << 3 | mantissa."""
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    _, ex = np.frexp(a)
    e = ex - 1
    normal = a >= np.ldexp(1.0, _E4M3_MIN_EXP)
    mant = np.where(normal, (a / np.ldexp(1.0, np.where(normal, e, 0)) - 1.0) * 8.0, a / np.ldexp(1.0, -9))
    field = np.where(normal, e + 7, 0)
    assert np.all(mant == np.rint(mant)) and np.all(mant < 8) and np.all(field <= 15)
    sign = np.signbit(v).astype(np.int64)
    return (sign << 7 | field.astype(np.int64) << 3 | mant.astype(np.int64)).astype(np.uint8)


def e4m3_decode(code):
    """Value of an E4M3 byte (0x7f / 0xff, the NaN codes, never occur here)."""
    c = np.asarray(code).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    field, mant = (c >> 3) & 15, c & 7
    mag = np.where(field == 0, mant * np.ldexp(1.0, -9), (1.0 + mant / 8.0) * np.ldexp(1.0, field - 7))
    return sign * mag


SCALE_EXP_MIN = -100      # the scale 2^k is stored as an fp32 number and has to stay a normal one


def row_scale_exponent(amax):
    """Power-of-two scale of a row: the smallest integer k with amax * 2^-k <= 448, but not below SCALE_EXP_MIN
    (rows that small -- below 2^-91 -- lose their last bits); 0 for an all-zero row."""
    amax = np.asarray(amax, dtype=np.float64)
    m, ex = np.frexp(amax)                           # amax = m 2^ex, m in [0.5, 1);  448 = 0.875 * 2^9
    k = np.maximum(np.where(m <= 0.875, ex - 9, ex - 8), SCALE_EXP_MIN)
    return np.where(amax == 0, 0, k).astype(np.int64)


def quantize_rows_e4m3(x):
    """x[..., D] -> (codes uint8 [..., D], k int [...]): every row (one token, one head) is divided by its own
    power of two 2^k -- exact -- and rounded to E4M3; the row's largest magnitude lands in (224, 448]."""
    x = np.asarray(x, dtype=np.float64)
    k = row_scale_exponent(np.abs(x).max(axis=-1)) if x.shape[-1] else np.zeros(x.shape[:-1], np.int64)
    return e4m3_encode(e4m3_round(np.ldexp(x, -k[..., None]))), k


def dequantize_rows_e4m3(codes, k):
    return np.ldexp(e4m3_decode(codes), np.asarray(k)[..., None])


def decode_dual_fp8(q, src_k, src_v, rsn_k, rsn_v, src_visible_len, rsn_len, scale=None):
    """The decode step over caches stored in 8 bits: keys and values are what comes back out of the store,
    everything after that is decode_dual_concat unchanged (queries, probabilities and sums are not quantised)."""
    rq = lambda a: dequantize_rows_e4m3(*quantize_rows_e4m3(a))
    return decode_dual_concat(q, rq(src_k), rq(src_v), rq(rsn_k), rq(rsn_v), src_visible_len, rsn_len, scale)


# --------------------------------------------------------------------------
# Alg. 1 as a timeline: when does each reasoning unit start, given when sentences arrive
# --------------------------------------------------------------------------
STREAMING, SERIAL, BATCH = 0, 1, 2


def alg1_timeline(arrival, prefill_s, n_decode, decode_s, mode=STREAMING):
    """Event times of Alg. 1 for one stream, with the two loops on resources of their own.

    arrival[k]   time sentence k has been read completely (non-decreasing)
    prefill_s[k] time to prefill sentence k into the input cache
    n_decode[k]  decoding steps of reasoning unit k, each taking decode_s

    STREAMING (Alg. 1): the prefill loop takes sentences in arrival order, one at a time; the
    decoding loop starts unit t when unit t-1 is finished AND sentence t is prefilled
    (N_EOS >= N_EOT + 1).  `waited[t]`: the loop had to wait for the prefill (N_EOS < N_EOT + 1
    when it got there); `sliced[t]`: later sentences were already cached when unit t started, so
    a slice of the input cache had to be selected (N_EOS > N_EOT + 1).
    SERIAL: one worker alternates -- prefill sentence k, decode unit k -- and sentences that
    arrive meanwhile wait.  BATCH: everything is read first, then prefilled, then decoded.
    Returns a dict of lists: prefill_done, unit_start, first_token, unit_done, waited, sliced.
    """
    K = len(arrival)
    pf_done, start, first, done, waited, sliced = [], [], [], [], [], []
    if mode == STREAMING:
        t_free = 0.0
        for k in range(K):
            t_free = max(arrival[k], t_free) + prefill_s[k]
            pf_done.append(t_free)
        ready = 0.0
        for t in range(K):
            waited.append(pf_done[t] > ready)
            st = max(ready, pf_done[t])
            sliced.append(t + 1 < K and pf_done[t + 1] <= st)
            start.append(st)
            first.append(st + decode_s if n_decode[t] > 0 else st)
            ready = st + n_decode[t] * decode_s
            done.append(ready)
    elif mode == SERIAL:
        t_free = 0.0
        for k in range(K):
            pf = max(arrival[k], t_free) + prefill_s[k]
            pf_done.append(pf)
            waited.append(arrival[k] > t_free)
            sliced.append(False)
            start.append(pf)
            first.append(pf + decode_s if n_decode[k] > 0 else pf)
            t_free = pf + n_decode[k] * decode_s
            done.append(t_free)
    elif mode == BATCH:
        t_free = arrival[K - 1] if K else 0.0
        for k in range(K):
            t_free += prefill_s[k]
            pf_done.append(t_free)
        for t in range(K):
            waited.append(t == 0)
            sliced.append(False)
            start.append(t_free)
            first.append(t_free + decode_s if n_decode[t] > 0 else t_free)
            t_free += n_decode[t] * decode_s
            done.append(t_free)
    else:
        raise ValueError(mode)
    return dict(prefill_done=pf_done, unit_start=start, first_token=first, unit_done=done, waited=waited, sliced=sliced)


# --------------------------------------------------------------------------
# Canonical skip metadata, derived by REDUCING the dense mask
# --------------------------------------------------------------------------
SKIP, FULL, PARTIAL = 0, 1, 2


def _tile_classes(block, bm, bn):
    """block[m, n] bool -> uint8[ceil(m/bm), ceil(n/bn)] of SKIP / FULL / PARTIAL.

    Ragged edge tiles are judged on their in-range elements only.
    """
    m, n = block.shape
    tq, tk = -(-m // bm), -(-n // bn)
    cls = np.zeros((tq, tk), dtype=np.uint8)
    for a in range(tq):
        for c in range(tk):
            t = block[a * bm:(a + 1) * bm, c * bn:(c + 1) * bn]
            cls[a, c] = FULL if t.all() else (PARTIAL if t.any() else SKIP)
    return cls


def canonical_metadata(stream, seg, pos, bm, bn):
    """Segment-skip metadata of ONE sequence in grouped stream-compact order.

    The sequence is permuted to [all source tokens by position | all reasoning
    tokens by position] (the paper's grouped training layout, Appendix E.1),
    the dense mask is built there, and everything is read off that matrix:
      src_idx, rsn_idx : physical index of each compact row
      vis_src[r]       : number of source columns row r (reasoning) can see
      classes of the three blocks SS (source rows x source cols),
      RS (reasoning rows x source cols), RR (reasoning x reasoning)
      visible_pairs    : number of True entries of the mask
    """
    stream = np.asarray(stream); seg = np.asarray(seg); pos = np.asarray(pos)
    src_idx = np.nonzero(stream == SRC)[0]
    rsn_idx = np.nonzero(stream == RSN)[0]
    src_idx = src_idx[np.argsort(pos[src_idx], kind="stable")]
    rsn_idx = rsn_idx[np.argsort(pos[rsn_idx], kind="stable")]
    perm = np.concatenate([src_idx, rsn_idx])
    mask = dense_mask(stream[perm], seg[perm], pos[perm])
    s = len(src_idx)
    ss, rs, rr = mask[:s, :s], mask[s:, :s], mask[s:, s:]
    assert not mask[:s, s:].any()
    return {
        "src_idx": src_idx.astype(np.int32),
        "rsn_idx": rsn_idx.astype(np.int32),
        "vis_src": rs.sum(axis=1).astype(np.int32),
        "SS": _tile_classes(ss, bm, bn),
        "RS": _tile_classes(rs, bm, bn),
        "RR": _tile_classes(rr, bm, bn),
        "visible_pairs": int(mask.sum()),
    }


def source_prefix_table(stream, seg):
    """P[g] = number of source tokens with segment id <= g, g = 0 .. max id."""
    stream = np.asarray(stream); seg = np.asarray(seg)
    gmax = int(seg.max()) if len(seg) else -1
    return np.array([int(((stream == SRC) & (seg <= g)).sum()) for g in range(gmax + 1)], dtype=np.int32)
