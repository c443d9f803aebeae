"""Byte and FLOP accounting of decode attention (host arithmetic only).

Follows the paper's KV-bytes formula and arithmetic-intensity model
(Section 3.1, Table 1), extended with the decoupled-RoPE key, which the paper's
table leaves out but its kernels read.
"""
from __future__ import annotations

import math


def cache_bytes_per_token(h_c: int, d_v: int, d_r: int, tp: int = 1, elem_bytes: int = 2) -> int:
    """Bytes of cache per token per device: the state heads are sharded over
    `tp` ranks (replicated once tp exceeds h_c), the single RoPE key is
    replicated on every rank."""
    heads_per_rank = max(1, math.ceil(h_c / tp))
    return elem_bytes * (heads_per_rank * d_v + d_r)


def kv_bytes_per_token_heads(h_kv: int, d_h: int, m_kv: int, tp: int = 1, elem_bytes: int = 2) -> int:
    """Section 3.1's KV-bytes formula for one token on one device:
    m_kv * (h_q / g_q) * d_h * sizeof(dtype) with the h_kv heads split over tp."""
    return m_kv * max(1, math.ceil(h_kv / tp)) * d_h * elem_bytes


def duplication_factor(n_shards: int, g_q: int, h_q: int) -> int:
    """D = ceil(N * g_q / h_q) (Section 3.2)."""
    return max(1, math.ceil(n_shards * g_q / h_q))


def visible_keys(seq_len: int, q_len: int, t: int, causal: bool = True) -> int:
    n = seq_len - q_len + 1 + t if causal else seq_len
    return max(0, n)


def flops(seq_lens, q_len: int, h_q: int, d_n: int, d_r: int, d_v: int, causal: bool = True) -> int:
    """2 (d_n + d_r) for the score and 2 d_v for the weighted sum, per query
    row, head and visible key."""
    per = 2 * (d_n + d_r) + 2 * d_v
    tot = 0
    for L in seq_lens:
        for t in range(q_len):
            tot += visible_keys(int(L), q_len, t, causal) * h_q * per
    return tot


def cache_bytes(seq_lens, h_c: int, d_v: int, d_r: int) -> int:
    """Unique cache bytes a call must read: every cached token once."""
    return sum(max(0, int(L)) for L in seq_lens) * cache_bytes_per_token(h_c, d_v, d_r)


def io_bytes(seq_lens, q_len: int, h_q: int, d_n: int, d_r: int, d_v: int, out_bytes: int = 2) -> int:
    """Query + output + lse bytes of a call."""
    B = len(seq_lens)
    return B * q_len * h_q * ((d_n + d_r) * 2 + d_v * out_bytes + 4)


def paper_arithmetic_intensity(L: float, h_q: int, g_q: int, m_kv: int) -> float:
    """Table 1's general formulation: 2 L h_q / (2 h_q + m_kv (h_q / g_q) L),
    in FLOPs per ELEMENT-pair as the paper counts it (no RoPE dims)."""
    return 2.0 * L * h_q / (2.0 * h_q + m_kv * (h_q / g_q) * L)
