"""Shared helpers of the GPU parity tests (argument plumbing only)."""
import numpy as np
import torch

import paper_2510_17238_amd as st
import workloads as W

DEV = "cuda"


def to_dev(x, dtype):
    """float32 numpy (bf16-exact when dtype == 'bf16') -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def ids_to_dev(cfg):
    return (torch.from_numpy(cfg.segment_ids).to(DEV), torch.from_numpy(cfg.stream_ids).to(DEV),
            torch.from_numpy(cfg.positions).to(DEV))


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def make_cache(batch, max_pages_per_seq, n_kv_heads, head_dim, rng, fill=None, fp8=False):
    """A cache with a shuffled page table and pools of exactly batch * max_pages pages."""
    table = W.shuffled_page_table(rng, batch, max_pages_per_seq)
    return st.KVCache(batch * max_pages_per_seq, batch, max_pages_per_seq, n_kv_heads, head_dim,
                      torch.from_numpy(table).to(DEV), fill=fill, fp8=fp8), table
