"""Seeded synthetic inputs for the streaming-constrained attention path.

This module only MAKES INPUTS: token metadata (stream / segment / position
ids), segment-length draws, Gaussian tensors and their bf16 rounding, page
tables.  It holds none of the method's arithmetic (no mask, no softmax, no
rotation) and is shared by the CPU oracle's tests and the GPU path's tests and
bench, so that both sides receive the same bits.

The shapes follow the five benchmark configurations: sentence-sized source
segments interleaved with longer reasoning segments, one reasoning segment per
source segment, Qwen3-like head geometry.  They stand in for the paper's
tokenised prompts and model activations, which need datasets and weights.
"""
from dataclasses import dataclass, field
import numpy as np

SRC = 0
RSN = 1
PAGE = 16


# ---------------------------------------------------------------- tensors --
def bf16_round(x):
    """float32 array -> float32 array whose values are exactly bf16-representable (RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """float32 array of bf16-representable values -> uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).reshape(bits.shape)


def normal(rng, shape, dtype):
    """i.i.d. N(0, 1) as float32; rounded to bf16 values when dtype == 'bf16'."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    return bf16_round(x) if dtype == "bf16" else x


# --------------------------------------------------------- token metadata --
def tokens_from_segments(src_lens, rsn_lens, layout="interleaved", first_seg=1):
    """stream_ids, segment_ids, positions (int32) of one sequence.

    Segment pair t (t = 0, 1, ..) gets id first_seg + t on both streams.
    layout 'interleaved' = [S1 R1 S2 R2 ...]; 'grouped' = [S1 S2 .. | R1 R2 ..].
    Positions count tokens per stream, from 0.
    """
    assert len(src_lens) == len(rsn_lens)
    pieces = []
    for t, (s, r) in enumerate(zip(src_lens, rsn_lens)):
        pieces.append((SRC, first_seg + t, int(s)))
        pieces.append((RSN, first_seg + t, int(r)))
    if layout == "grouped":
        pieces = [p for p in pieces if p[0] == SRC] + [p for p in pieces if p[0] == RSN]
    stream = np.concatenate([np.full(n, k, np.int32) for k, _, n in pieces]) if pieces else np.zeros(0, np.int32)
    seg = np.concatenate([np.full(n, g, np.int32) for _, g, n in pieces]) if pieces else np.zeros(0, np.int32)
    pos = np.zeros(len(stream), np.int32)
    for kind in (SRC, RSN):
        idx = np.nonzero(stream == kind)[0]
        pos[idx] = np.arange(len(idx), dtype=np.int32)
    return stream, seg, pos


def draw_pairs(rng, n_pairs, src_range, rsn_range):
    s = rng.integers(src_range[0], src_range[1], size=n_pairs, endpoint=True)
    r = rng.integers(rsn_range[0], rsn_range[1], size=n_pairs, endpoint=True)
    return s.astype(np.int64), r.astype(np.int64)


def draw_until(rng, total, src_range, rsn_range):
    """Alternate source / reasoning draws until `total` tokens; the last segment is truncated."""
    s_list, r_list, n = [], [], 0
    while n < total:
        s = int(rng.integers(src_range[0], src_range[1], endpoint=True)); s = min(s, total - n); n += s
        r = int(rng.integers(rsn_range[0], rsn_range[1], endpoint=True)); r = min(r, total - n); n += r
        s_list.append(s); r_list.append(r)
    return np.array(s_list, np.int64), np.array(r_list, np.int64)


@dataclass
class PrefillBatch:
    name: str
    dtype: str               # 'f32' | 'bf16'
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    cu_seqlens: np.ndarray   # int32 [B + 1]
    stream_ids: np.ndarray   # int32 [N]
    segment_ids: np.ndarray  # int32 [N]
    positions: np.ndarray    # int32 [N]
    src_lens: list = field(default_factory=list)   # per sequence: source segment lengths
    rsn_lens: list = field(default_factory=list)
    theta: float = 1.0e6
    seed: int = 0

    @property
    def batch(self):
        return len(self.cu_seqlens) - 1

    @property
    def n_tokens(self):
        return int(self.cu_seqlens[-1])

    def tensors(self):
        """q[N, Hq, D], k[N, Hkv, D], v[N, Hkv, D] as float32 (bf16-exact when dtype is bf16)."""
        rng = np.random.Generator(np.random.PCG64(self.seed + 1000))
        n = self.n_tokens
        q = normal(rng, (n, self.n_q_heads, self.head_dim), self.dtype)
        k = normal(rng, (n, self.n_kv_heads, self.head_dim), self.dtype)
        v = normal(rng, (n, self.n_kv_heads, self.head_dim), self.dtype)
        return q, k, v

    def closed_form_pairs(self):
        """Per sequence: S(S+1)/2 + R(R+1)/2 + sum_k r_k * P_k (P_k = source tokens in segments <= k)."""
        res = []
        for s, r in zip(self.src_lens, self.rsn_lens):
            S, R = int(s.sum()), int(r.sum())
            P = np.cumsum(s)
            res.append(S * (S + 1) // 2 + R * (R + 1) // 2 + int((r * P).sum()))
        return res


def _assemble(name, dtype, hq, hkv, d, seg_lists, layout, seed):
    streams, segs, poss, cu = [], [], [], [0]
    for s, r in seg_lists:
        st, sg, ps = tokens_from_segments(s, r, layout)
        streams.append(st); segs.append(sg); poss.append(ps); cu.append(cu[-1] + len(st))
    return PrefillBatch(name, dtype, hq, hkv, d, np.array(cu, np.int32),
                        np.concatenate(streams), np.concatenate(segs), np.concatenate(poss),
                        [s for s, _ in seg_lists], [r for _, r in seg_lists], 1.0e6, seed)


def config1(layout="interleaved"):
    """Tiny case: 4 source x 16 tokens interleaved with 4 reasoning x 16; 2 q heads / 1 kv head, D = 64, fp32, seed 0."""
    s = np.full(4, 16, np.int64); r = np.full(4, 16, np.int64)
    return _assemble("cfg1-tiny", "f32", 2, 1, 64, [(s, r)], layout, 0)


def config2(layout="interleaved", batch=4):
    """Qwen3-0.6B-shaped layer: batch 4, 16/8 heads, D = 128, bf16, 32 pairs, s~U[24,64], r~U[32,128]; seed 1 + b."""
    lists = []
    for b in range(batch):
        rng = np.random.Generator(np.random.PCG64(1 + b))
        lists.append(draw_pairs(rng, 32, (24, 64), (32, 128)))
    return _assemble("cfg2-qwen3-0.6b-prefill", "bf16", 16, 8, 128, lists, layout, 1)


def config4a(layout="interleaved", batch=8):
    """Qwen3-4B-shaped layer, length-pinned: 16,384 tokens per sequence, s~U[64,192], r~U[64,256]; seed 3 + b."""
    lists = []
    for b in range(batch):
        rng = np.random.Generator(np.random.PCG64(3 + b))
        lists.append(draw_until(rng, 16384, (64, 192), (64, 256)))
    return _assemble("cfg4a-qwen3-4b-prefill-16k", "bf16", 32, 8, 128, lists, layout, 3)


def config4b(layout="interleaved", batch=8):
    """Qwen3-4B-shaped layer, count-pinned: 128 pairs per sequence (about 37K tokens); seed 3 + b."""
    lists = []
    for b in range(batch):
        rng = np.random.Generator(np.random.PCG64(3 + b))
        lists.append(draw_pairs(rng, 128, (64, 192), (64, 256)))
    return _assemble("cfg4b-qwen3-4b-prefill-128pairs", "bf16", 32, 8, 128, lists, layout, 3)


def random_prefill(seed, batch, max_pairs, src_range, rsn_range, hq, hkv, d, dtype, layout="interleaved"):
    """Small random structures for property-style tests (1-token and empty segments allowed by the ranges)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lists = []
    for _ in range(batch):
        n_pairs = int(rng.integers(1, max_pairs, endpoint=True))
        lists.append(draw_pairs(rng, n_pairs, src_range, rsn_range))
    return _assemble(f"random-{seed}", dtype, hq, hkv, d, lists, layout, seed)


# ----------------------------------------------------------------- decode --
@dataclass
class DecodeShape:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    src_visible_len: np.ndarray   # int32 [B]
    rsn_len: np.ndarray           # int32 [B] (includes the token being decoded)
    src_append: int               # tokens appended to the source cache per step
    max_src_len: int              # capacity to provision per sequence
    max_rsn_len: int
    seed: int = 0


def config3(batch=32, n_layers=28):
    """Qwen3-1.7B-shaped decode: source cache 2K, reasoning cache U[1024, 6144], 64-token source append per step; seed 2."""
    rng = np.random.Generator(np.random.PCG64(2))
    rsn = rng.integers(1024, 6144, size=batch, endpoint=True).astype(np.int32)
    src = np.full(batch, 2048, np.int32)
    return DecodeShape("cfg3-qwen3-1.7b-decode", n_layers, batch, 16, 8, 128, src, rsn, 64, 2048 + 64, 6144, 2)


def config5(batch=64, n_layers=36):
    """Qwen3-8B-shaped streaming step: src U[1024, 8192] (multiple of 32), rsn U[2048, 16384], 32-token appends; seed 4."""
    rng = np.random.Generator(np.random.PCG64(4))
    src = (rng.integers(1024 // 32, 8192 // 32, size=batch, endpoint=True) * 32).astype(np.int32)
    rsn = rng.integers(2048, 16384, size=batch, endpoint=True).astype(np.int32)
    return DecodeShape("cfg5-qwen3-8b-stream", n_layers, batch, 32, 8, 128, src, rsn, 32, 8192 + 32, 16384 + 8, 4)


def shuffled_page_table(rng, batch, pages_per_seq):
    """int32 [batch, pages_per_seq]: a random permutation of distinct page ids (no page shared)."""
    ids = rng.permutation(batch * pages_per_seq).astype(np.int32)
    return ids.reshape(batch, pages_per_seq)
