"""CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader around `gla_oracle.c`, the plain fp64 definition of GLA /
GTA decode attention over a paged cache.  Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; the GPU library never
does, and nothing here imports the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gla_oracle.c")
_LIB = os.path.join(_HERE, "libgla_oracle.so")
_lib = None

INT64_MAX = np.iinfo(np.int64).max


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP for the row loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.gla_oracle_threads.restype = ctypes.c_int
        lib.gla_oracle_decode.restype = ctypes.c_int
        lib.gla_oracle_decode.argtypes = (
            [ctypes.c_void_p] * 6 + [ctypes.c_int] * 9 + [ctypes.c_double, ctypes.c_int,
                                                         ctypes.c_int64, ctypes.c_int64,
                                                         ctypes.c_void_p, ctypes.c_int64,
                                                         ctypes.c_void_p, ctypes.c_void_p,
                                                         ctypes.c_void_p, ctypes.c_int64])
        lib.gla_oracle_merge.restype = ctypes.c_int
        lib.gla_oracle_merge.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                         ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p]
        lib.gla_oracle_gqa_decode.restype = ctypes.c_int
        lib.gla_oracle_gqa_decode.argtypes = ([ctypes.c_void_p] * 5 + [ctypes.c_int] * 8 +
                                              [ctypes.c_double, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64,
                                               ctypes.c_void_p, ctypes.c_void_p])
        lib.gla_oracle_project.restype = ctypes.c_int
        lib.gla_oracle_project.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_void_p]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().gla_oracle_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def decode(q_nope: np.ndarray, q_rope: Optional[np.ndarray], state: np.ndarray,
           rope: Optional[np.ndarray], page_table: np.ndarray, seq_lens: np.ndarray, *,
           h_c: int, scale: float, causal: int = 1, key_range: Tuple[int, int] = (0, INT64_MAX),
           sel: Optional[Sequence[Tuple[int, int, int]]] = None,
           return_weights: bool = False):
    """Run the oracle.

    q_nope [B,T,h_q,d_n], q_rope [B,T,h_q,d_r], state [n_pages,h_c,P,d_v],
    rope [n_pages,P,d_r]: uint16 arrays of bf16 bit patterns.  Returns
    (out fp64 [B,T,h_q,d_v] or [n_sel,d_v], lse fp64 [B,T,h_q] or [n_sel]) and,
    if asked, the softmax weights [rows, max(seq_lens)].
    """
    lib = _load()
    q_nope = np.ascontiguousarray(q_nope, dtype=np.uint16)
    B, T, h_q, d_n = q_nope.shape
    state = np.ascontiguousarray(state, dtype=np.uint16)
    _, hc2, P, d_v = state.shape
    assert hc2 == h_c
    d_r = 0
    if q_rope is not None and q_rope.shape[-1] > 0:
        q_rope = np.ascontiguousarray(q_rope, dtype=np.uint16)
        rope = np.ascontiguousarray(rope, dtype=np.uint16)
        d_r = q_rope.shape[-1]
        assert rope.shape[1] == P and rope.shape[2] == d_r
    else:
        q_rope, rope = None, None
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    assert page_table.shape[0] == B and seq_lens.shape == (B,)
    sel_arr = None
    if sel is not None:
        sel_arr = np.ascontiguousarray(np.asarray(sel, dtype=np.int32).reshape(-1, 3))
        rows = sel_arr.shape[0]
        out = np.empty((rows, d_v), dtype=np.float64)
        lse = np.empty((rows,), dtype=np.float64)
    else:
        rows = B * T * h_q
        out = np.empty((B, T, h_q, d_v), dtype=np.float64)
        lse = np.empty((B, T, h_q), dtype=np.float64)
    w = None
    w_stride = 0
    if return_weights:
        w_stride = int(max(1, seq_lens.max() if B else 1))
        w = np.empty((rows, w_stride), dtype=np.float64)
    rc = lib.gla_oracle_decode(_ptr(q_nope), _ptr(q_rope), _ptr(state), _ptr(rope),
                               _ptr(page_table), _ptr(seq_lens), B, T, h_q, h_c, d_v, d_n, d_r,
                               P, page_table.shape[1], float(scale), int(causal),
                               int(key_range[0]), int(key_range[1]), _ptr(sel_arr),
                               0 if sel_arr is None else sel_arr.shape[0], _ptr(out), _ptr(lse),
                               _ptr(w), w_stride)
    if rc != 0:
        raise ValueError("gla_oracle_decode: bad argument")
    return (out, lse, w) if return_weights else (out, lse)


def merge(part_out: np.ndarray, part_lse: np.ndarray):
    """Merge partial results over disjoint key ranges: part_out [S, ..., d_v],
    part_lse [S, ...] -> (out [..., d_v], lse [...])."""
    lib = _load()
    part_out = np.ascontiguousarray(part_out, dtype=np.float64)
    part_lse = np.ascontiguousarray(part_lse, dtype=np.float64)
    S = part_out.shape[0]
    d_v = part_out.shape[-1]
    rows = int(np.prod(part_lse.shape[1:], dtype=np.int64))
    out = np.empty(part_out.shape[1:], dtype=np.float64)
    lse = np.empty(part_lse.shape[1:], dtype=np.float64)
    rc = lib.gla_oracle_merge(_ptr(part_out), _ptr(part_lse), S, rows, d_v, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError("gla_oracle_merge: bad argument")
    return out, lse


def project(a: np.ndarray, w: np.ndarray, *, sum_groups: bool) -> np.ndarray:
    """Projection by per-group weights: a [M, G, K] and w [G, N, K] are uint16
    arrays of bf16 bit patterns; returns fp64 [M, G, N] (sum_groups False: the
    absorbed queries, one weight matrix per head) or [M, N] summed over the
    groups (the grouped output projection)."""
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.uint16)
    w = np.ascontiguousarray(w, dtype=np.uint16)
    M, G, K = a.shape
    G2, N, K2 = w.shape
    assert G2 == G and K2 == K
    c = np.empty((M, N) if sum_groups else (M, G, N), dtype=np.float64)
    rc = lib.gla_oracle_project(_ptr(a), G * K, K, _ptr(w), M, G, N, K, int(bool(sum_groups)), _ptr(c))
    if rc != 0:
        raise ValueError("gla_oracle_project: bad argument")
    return c


def gqa_decode(q: np.ndarray, kcache: np.ndarray, vcache: np.ndarray, page_table: np.ndarray,
               seq_lens: np.ndarray, *, scale: float, causal: int = 1,
               sel: Optional[Sequence[Tuple[int, int, int]]] = None):
    """Grouped-query decode with separate key / value caches: q [B,T,h_q,d_k],
    kcache [n_pages,h_kv,P,d_k], vcache [n_pages,h_kv,P,d_v] (uint16 bf16 bits).
    Returns (out fp64 [B,T,h_q,d_v] or [n_sel,d_v], lse)."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.uint16)
    kcache = np.ascontiguousarray(kcache, dtype=np.uint16)
    vcache = np.ascontiguousarray(vcache, dtype=np.uint16)
    B, T, h_q, d_k = q.shape
    _, h_kv, P, d_k2 = kcache.shape
    d_v = vcache.shape[-1]
    assert d_k2 == d_k and vcache.shape[:3] == kcache.shape[:3]
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    sel_arr = None
    if sel is not None:
        sel_arr = np.ascontiguousarray(np.asarray(sel, dtype=np.int32).reshape(-1, 3))
        out = np.empty((sel_arr.shape[0], d_v), dtype=np.float64)
        lse = np.empty((sel_arr.shape[0],), dtype=np.float64)
    else:
        out = np.empty((B, T, h_q, d_v), dtype=np.float64)
        lse = np.empty((B, T, h_q), dtype=np.float64)
    rc = lib.gla_oracle_gqa_decode(_ptr(q), _ptr(kcache), _ptr(vcache), _ptr(page_table), _ptr(seq_lens),
                                   B, T, h_q, h_kv, d_k, d_v, P, page_table.shape[1], float(scale), int(causal),
                                   _ptr(sel_arr), 0 if sel_arr is None else sel_arr.shape[0], _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError("gla_oracle_gqa_decode: bad argument")
    return out, lse


def decode_problem(p, **kw):
    """Oracle on a `workloads.DecodeProblem` (compact pages + compact table)."""
    from workloads import bf16_bits
    if p.kind == "gqa":
        return gqa_decode(bf16_bits(p.q_nope), bf16_bits(p.key_pages), bf16_bits(p.state_pages), p.table_compact,
                          p.seq_lens, scale=p.scale, causal=p.causal, **kw)
    return decode(bf16_bits(p.q_nope), bf16_bits(p.q_rope), bf16_bits(p.state_pages),
                  bf16_bits(p.rope_pages), p.table_compact, p.seq_lens, h_c=p.h_c,
                  scale=p.scale, causal=p.causal, **kw)
