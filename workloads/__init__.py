"""Seeded synthetic decode workloads (inputs only).

This module builds the INPUTS of a decode-attention call over a paged cache:
absorbed queries, paged latent / tied states, the shared RoPE-key pages, a page
table and per-sequence lengths.  It holds none of the attention arithmetic and
is imported by both the CPU oracle's tests and the GPU path's tests/bench, which
otherwise share nothing.

Shapes follow the paper's kernel benchmarks (GLA: 2 latent heads of 256 plus a
RoPE key of 64, MLA: one latent head of 512 plus 64, page size 64; Section 5.3
and Appendix B.5) and its tied-state definition for GTA (Section 3.3.1).  All
values are bf16 draws from N(0, 1) from a seeded CPU generator.

Storage is "compact": only the pages a batch really uses are materialised
(`state_pages[i]`, `rope_pages[i]`), together with `page_ids[i]`, the physical
slot that page occupies in a much larger pool.  The CPU side consumes the
compact arrays through `table_compact`; the GPU side scatters them into a pool
of `num_pages` slots and uses `table_pool`.  Both describe the same logical
cache.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Sequence

import numpy as np
import torch

BASE_SEED = 250521487


@dataclasses.dataclass
class DecodeProblem:
    name: str
    kind: str            # "gla" (d_n == d_v), "gta" (d_n == d_v // 2) or "gqa" (separate key cache, d_r == 0)
    B: int
    T: int               # query length, 1..4
    h_q: int
    h_c: int             # latent heads (GLA) / tied KV heads (GTA)
    d_v: int
    d_n: int
    d_r: int
    page_size: int
    max_pages: int       # row length of the page tables
    num_pages: int       # physical pool size
    scale: float
    causal: int
    seq_lens: np.ndarray          # int32 [B]
    q_nope: torch.Tensor          # bf16 [B, T, h_q, d_n]
    q_rope: torch.Tensor          # bf16 [B, T, h_q, d_r]
    state_pages: torch.Tensor     # bf16 [n_used, h_c, page_size, d_v]
    rope_pages: torch.Tensor      # bf16 [n_used, page_size, d_r]
    page_ids: np.ndarray          # int64 [n_used] physical slot of compact page i
    table_compact: np.ndarray     # int32 [B, max_pages] -> compact index, -1 unused
    table_pool: np.ndarray        # int32 [B, max_pages] -> physical slot, -1 unused
    key_pages: Optional[torch.Tensor] = None   # kind "gqa" only: bf16 [n_used, h_c, page_size, d_n] (keys of their own)

    @property
    def g_q(self) -> int:
        return self.h_q // self.h_c

    @property
    def total_tokens(self) -> int:
        return int(np.maximum(self.seq_lens, 0).astype(np.int64).sum())

    @property
    def cache_bytes_per_token(self) -> int:
        if self.kind == "gqa":
            return 2 * self.h_c * (self.d_n + self.d_v)
        return 2 * (self.h_c * self.d_v + self.d_r)


def _bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns (numpy has no bf16)."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return _bits(t)


def make_problem(
    name: str,
    *,
    kind: str = "gla",
    seq_lens: Sequence[int],
    T: int = 1,
    h_q: int,
    h_c: int,
    d_v: int,
    d_r: int = 64,
    page_size: int = 64,
    num_pages: Optional[int] = None,
    identity_table: bool = False,
    scale: Optional[float] = None,
    causal: int = 1,
    seed: int = BASE_SEED,
    q_gain: float = 1.0,
    poison_tail: bool = False,
    extra_table_cols: int = 0,
    table_seed: Optional[int] = None,
    page_offset: int = 0,
) -> DecodeProblem:
    """Draw one decode problem.

    q_gain > 1 makes the softmax peaky (large outputs, heavy rescaling).
    poison_tail writes NaN into every cached slot at or beyond a sequence's
    length inside its last page: no correct implementation may read them into
    a result.  Page ids are the slice [page_offset, page_offset + n_used) of a
    random permutation of the pool drawn from `table_seed` (default: the value
    seed), so problems sharing a table_seed can occupy disjoint pages of one pool.
    """
    assert kind in ("gla", "gta", "gqa")
    d_n = d_v // 2 if kind == "gta" else d_v
    if kind == "gqa":
        d_r = 0          # the rotated dims are part of the cached key
    if scale is None:
        scale = 1.0 / math.sqrt(d_n + d_r)
    seq = np.asarray(seq_lens, dtype=np.int32)
    B = int(seq.shape[0])
    pages_per_seq = (np.maximum(seq, 0).astype(np.int64) + page_size - 1) // page_size
    n_used = int(pages_per_seq.sum())
    max_pages = int(max(1, pages_per_seq.max() if B else 1)) + int(extra_table_cols)
    if num_pages is None:
        num_pages = max(n_used, 1)
    assert num_pages >= n_used

    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    q_nope = (torch.randn(B, T, h_q, d_n, generator=g) * q_gain).to(torch.bfloat16)
    q_rope = (torch.randn(B, T, h_q, d_r, generator=g) * q_gain).to(torch.bfloat16)
    state_pages = torch.randn(max(n_used, 1), h_c, page_size, d_v, generator=g).to(torch.bfloat16)
    rope_pages = torch.randn(max(n_used, 1), page_size, d_r, generator=g).to(torch.bfloat16)
    key_pages = torch.randn(max(n_used, 1), h_c, page_size, d_n, generator=g).to(torch.bfloat16) if kind == "gqa" else None

    if identity_table:
        page_ids = np.arange(n_used, dtype=np.int64)
    else:
        gt = g
        if table_seed is not None:
            gt = torch.Generator(device="cpu")
            gt.manual_seed(int(table_seed))
        perm = torch.randperm(int(num_pages), generator=gt).numpy().astype(np.int64)
        assert page_offset + n_used <= num_pages
        page_ids = perm[page_offset:page_offset + n_used].copy()

    table_compact = np.full((B, max_pages), -1, dtype=np.int32)
    table_pool = np.full((B, max_pages), -1, dtype=np.int32)
    cur = 0
    for b in range(B):
        n = int(pages_per_seq[b])
        table_compact[b, :n] = np.arange(cur, cur + n, dtype=np.int32)
        table_pool[b, :n] = page_ids[cur:cur + n].astype(np.int32)
        if poison_tail and n > 0:
            used = int(seq[b]) - (n - 1) * page_size
            if used < page_size:
                state_pages[cur + n - 1, :, used:, :] = float("nan")
                rope_pages[cur + n - 1, used:, :] = float("nan")
                if key_pages is not None:
                    key_pages[cur + n - 1, :, used:, :] = float("nan")
        cur += n

    return DecodeProblem(
        name=name, kind=kind, B=B, T=T, h_q=h_q, h_c=h_c, d_v=d_v, d_n=d_n, d_r=d_r,
        page_size=page_size, max_pages=max_pages, num_pages=int(num_pages),
        scale=float(scale), causal=int(causal), seq_lens=seq,
        q_nope=q_nope, q_rope=q_rope, state_pages=state_pages[:max(n_used, 1)],
        rope_pages=rope_pages[:max(n_used, 1)], page_ids=page_ids,
        table_compact=table_compact, table_pool=table_pool, key_pages=key_pages,
    )


# --------------------------------------------------------------------------
# The five benchmark configurations (index = position in the config list).
# --------------------------------------------------------------------------

POOL_PAGES = 600_000


def log_uniform_lengths(n: int, lo: int, hi: int, seed: int) -> np.ndarray:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    u = torch.rand(n, generator=g, dtype=torch.float64).numpy()
    return np.floor(np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))).astype(np.int32)


def uniform_lengths(n: int, lo: int, hi: int, seed: int) -> np.ndarray:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return torch.randint(lo, hi + 1, (n,), generator=g).numpy().astype(np.int32)


def config(index: int, *, T: Optional[int] = None, draw: int = 0, batch: Optional[int] = None,
           max_len: Optional[int] = None, page_offset: int = 0, page_size: int = 64) -> DecodeProblem:
    """BASELINE configuration `index` (0-based).  `draw` re-draws the values
    (seed offset) while the pool permutation stays that of draw 0, so draws
    placed at disjoint `page_offset`s share one pool; `batch` / `max_len` shrink
    the problem for quick tests while keeping its head and cache shape; `page_size`
    other than the stated 64 keeps the pool's byte size (more, smaller pages)."""
    seed = BASE_SEED + index + 1000 * draw
    tbl = dict(table_seed=BASE_SEED + index + 500, page_offset=page_offset)
    if page_size != 64:
        tbl["page_size"] = page_size
    pool = POOL_PAGES * 64 // page_size
    if index == 0:
        return make_problem("tiny_gla2", seq_lens=[256] * (batch or 1), T=T or 1, h_q=16, h_c=2,
                            d_v=256, identity_table=True, seed=seed)
    if index == 1:
        L = min(8192, max_len or 8192)
        return make_problem("gla2_b64_l8192", seq_lens=[L] * (batch or 64), T=T or 1, h_q=128,
                            h_c=2, d_v=256, num_pages=pool, seed=seed, **tbl)
    if index == 2:
        L = min(16384, max_len or 16384)
        return make_problem("gla2_spec_b32_l16384", seq_lens=[L] * (batch or 32), T=T or 2,
                            h_q=128, h_c=2, d_v=256, num_pages=pool, seed=seed, **tbl)
    if index == 3:
        lens = log_uniform_lengths(batch or 128, 512, max_len or 32768, seed + 7)
        return make_problem("mla_ragged_b128", seq_lens=lens, T=T or 1, h_q=128, h_c=1,
                            d_v=512, num_pages=pool, seed=seed, **tbl)
    if index == 4:
        hi = max_len or 32768
        lens = uniform_lengths(batch or 128, min(4096, hi), hi, seed + 7)
        return make_problem("gta4_b128", kind="gta", seq_lens=lens, T=T or 1, h_q=32, h_c=4,
                            d_v=128, num_pages=pool, seed=seed, **tbl)
    if index == 5:
        # not one of the five stated configurations: the GLA-2 head shape on a ragged
        # batch of contexts up to 32K, for the q_len sweep (MFMA utilisation vs q_len)
        hi = max_len or 32768
        lens = uniform_lengths(batch or 64, min(4096, hi), hi, seed + 7)
        return make_problem("gla2_ragged_b64", seq_lens=lens, T=T or 1, h_q=128, h_c=2, d_v=256,
                            num_pages=pool, seed=seed, **tbl)
    if index in (6, 7, 8):
        # not among the five stated configurations: the lengths of configuration 4 (GTA-4, d_h 128) on the
        # head shapes of the smaller models and on the grouped-query baseline GTA is compared with
        hi = max_len or 32768
        lens = uniform_lengths(batch or 128, min(4096, hi), hi, BASE_SEED + 4 + 1000 * draw + 7)
        if index == 6:   # GTA-4 with d_h 64 (RoPE key 32)
            return make_problem("gta4_dh64_b128", kind="gta", seq_lens=lens, T=T or 1, h_q=32, h_c=4, d_v=64, d_r=32,
                                num_pages=pool, seed=seed, **tbl)
        if index == 7:   # GQA-4 with d_h 128: separate key and value caches
            return make_problem("gqa4_dh128_b128", kind="gqa", seq_lens=lens, T=T or 1, h_q=32, h_c=4, d_v=128,
                                num_pages=pool, seed=seed, **tbl)
        return make_problem("gta4_dh96_b128", kind="gta", seq_lens=lens, T=T or 1, h_q=24, h_c=4, d_v=96, d_r=48,
                            num_pages=pool, seed=seed, **tbl)
    if index == 9:
        # configuration 1 with a RoPE key of 32 dims
        L = min(8192, max_len or 8192)
        return make_problem("gla2_b64_l8192_rope32", seq_lens=[L] * (batch or 64), T=T or 1, h_q=128, h_c=2, d_v=256,
                            d_r=32, num_pages=pool, seed=seed, **tbl)
    raise ValueError(f"no config {index}")


def projection_weights(groups: int, n: int, k: int, *, seed: int, gain: float = 1.0) -> torch.Tensor:
    """Seeded random weights [groups][n][k] (output-major) for the projections
    around the attention: bf16 draws from N(0, gain^2 / (groups * k)), so that a
    sum over all groups and input features of unit-variance inputs has variance
    gain^2.  Inputs only: no arithmetic of the method."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    w = torch.empty(groups, n, k, dtype=torch.bfloat16)
    std = gain / math.sqrt(groups * k)
    for i in range(groups):                      # one group at a time: bounded fp32 staging
        w[i] = (torch.randn(n, k, generator=g) * std).to(torch.bfloat16)
    return w


def parse_lens(spec: str):
    """'1024x15,65536' -> [1024] * 15 + [65536]."""
    out = []
    for part in spec.split(","):
        if "x" in part:
            v, n = part.split("x")
            out += [int(v)] * int(n)
        else:
            out.append(int(part))
    return out


def latency_workload(spec: str, *, shape: str = "gla2", T: int = 1, draw: int = 0,
                     page_offset: int = 0, page_size: int = 64) -> DecodeProblem:
    """Kernel-latency workloads in the style of the paper's appendix on kernel
    execution time: batch 1 at one context length, or a few short sequences plus
    one long one (imbalanced batch).  shape: 'gla2' (2 x 256 + 64, 128 heads) or
    'mla' (1 x 512 + 64, 128 heads)."""
    lens = parse_lens(spec)
    seed = BASE_SEED + 77 + 1000 * draw
    tbl = dict(table_seed=BASE_SEED + 577, page_offset=page_offset)
    if page_size != 64:
        tbl["page_size"] = page_size
    pool = POOL_PAGES * 64 // page_size
    if shape == "gla2":
        return make_problem(f"latency_gla2[{spec}]", seq_lens=lens, T=T, h_q=128, h_c=2, d_v=256,
                            num_pages=pool, seed=seed, **tbl)
    if shape == "mla":
        return make_problem(f"latency_mla[{spec}]", seq_lens=lens, T=T, h_q=128, h_c=1, d_v=512,
                            num_pages=pool, seed=seed, **tbl)
    raise ValueError(shape)
