"""ctypes binding of libgla_decode.so (declared in include/gla_decode.h).

Argument marshalling only: tensors are PyTorch device tensors used as plain
device memory, the stream is PyTorch's current HIP stream, every step of the
computation runs in the library's kernels.  There is no fallback: if the shared
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgla_decode.so")

GLA_OK = 0
GLA_ERR_INVALID_ARG = -1
GLA_ERR_UNSUPPORTED_SHAPE = -2
GLA_ERR_WORKSPACE_TOO_SMALL = -3
GLA_ERR_LAUNCH = -4
GLA_IMPL_AUTO, GLA_IMPL_GENERIC, GLA_IMPL_TUNED = 0, 1, 2
GLA_OUT_BF16, GLA_OUT_FP32 = 0, 1
GLA_DECODE_NOALLOC_SCRATCH_BYTES = 72 << 20

EXPORTS = ("gla_decode", "gta_decode", "gqa_decode", "gla_decode_noalloc", "gla_absorb_query", "gla_output_proj",
           "gla_proj_workspace_size", "gla_decode_workspace_size", "gla_decode_select_impl",
           "gla_decode_profile", "gla_decode_check_contents", "gla_status_string", "gla_decode_version")


class GlaDecodeParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("q_len", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32), ("num_groups", ctypes.c_int32),
        ("d_v", ctypes.c_int32), ("d_nope", ctypes.c_int32), ("d_rope", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("causal", ctypes.c_int32), ("num_pages", ctypes.c_int64),
        ("q_nope", ctypes.c_void_p), ("q_nope_stride", ctypes.c_int64 * 3),
        ("q_rope", ctypes.c_void_p), ("q_rope_stride", ctypes.c_int64 * 3),
        ("state_cache", ctypes.c_void_p), ("state_stride", ctypes.c_int64 * 3),
        ("rope_cache", ctypes.c_void_p), ("rope_stride", ctypes.c_int64 * 2),
        ("page_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("softmax_scale", ctypes.c_float), ("out_dtype", ctypes.c_int32),
        ("out", ctypes.c_void_p), ("out_stride", ctypes.c_int64 * 3),
        ("lse", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("num_splits", ctypes.c_int32), ("impl", ctypes.c_int32),
        ("stream", ctypes.c_void_p),
    ]


class GlaProjParams(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int32), ("groups", ctypes.c_int32), ("n", ctypes.c_int32), ("k", ctypes.c_int32),
        ("a", ctypes.c_void_p), ("a_row_stride", ctypes.c_int64), ("a_group_stride", ctypes.c_int64),
        ("w", ctypes.c_void_p),
        ("c", ctypes.c_void_p), ("c_row_stride", ctypes.c_int64), ("c_group_stride", ctypes.c_int64),
        ("c_dtype", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
    ]


class GlaError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"gla_decode: {gla_status_string(status)} ({status})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2505_21487_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(GlaDecodeParams)
        lib.gla_decode.argtypes = [P]
        lib.gla_decode.restype = ctypes.c_int
        lib.gta_decode.argtypes = [P]
        lib.gta_decode.restype = ctypes.c_int
        lib.gqa_decode.argtypes = [P, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)]
        lib.gqa_decode.restype = ctypes.c_int
        lib.gla_decode_noalloc.argtypes = [P, ctypes.c_int]
        lib.gla_decode_noalloc.restype = ctypes.c_int
        PP = ctypes.POINTER(GlaProjParams)
        lib.gla_absorb_query.argtypes = [PP]
        lib.gla_absorb_query.restype = ctypes.c_int
        lib.gla_output_proj.argtypes = [PP]
        lib.gla_output_proj.restype = ctypes.c_int
        lib.gla_proj_workspace_size.argtypes = [PP, ctypes.c_int]
        lib.gla_proj_workspace_size.restype = ctypes.c_size_t
        lib.gla_decode_workspace_size.argtypes = [P, ctypes.c_int]
        lib.gla_decode_workspace_size.restype = ctypes.c_size_t
        lib.gla_decode_select_impl.argtypes = [P, ctypes.c_int]
        lib.gla_decode_select_impl.restype = ctypes.c_int
        lib.gla_decode_profile.argtypes = [P, ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_float),
                                           ctypes.POINTER(ctypes.c_float)]
        lib.gla_decode_profile.restype = ctypes.c_int
        lib.gla_decode_check_contents.argtypes = [P, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        lib.gla_decode_check_contents.restype = ctypes.c_int
        lib.gla_status_string.argtypes = [ctypes.c_int]
        lib.gla_status_string.restype = ctypes.c_char_p
        lib.gla_decode_version.argtypes = []
        lib.gla_decode_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def gla_status_string(status: int) -> str:
    return load_library().gla_status_string(int(status)).decode()


def gla_decode_version() -> int:
    return int(load_library().gla_decode_version())


def shape_params(*, batch, q_len, num_q_heads, num_groups, d_v, d_nope, d_rope, page_size,
                 max_pages_per_seq, num_pages=0, causal=1, num_splits=0, impl=GLA_IMPL_AUTO,
                 out_dtype=GLA_OUT_BF16) -> GlaDecodeParams:
    """A parameter block with only the host-visible shape fields set."""
    p = GlaDecodeParams()
    p.batch, p.q_len, p.num_q_heads, p.num_groups = batch, q_len, num_q_heads, num_groups
    p.d_v, p.d_nope, p.d_rope = d_v, d_nope, d_rope
    p.page_size, p.max_pages_per_seq, p.num_pages = page_size, max_pages_per_seq, num_pages
    p.causal, p.num_splits, p.impl, p.out_dtype = int(causal), num_splits, impl, out_dtype
    return p


def gla_decode_workspace_size(p: GlaDecodeParams, is_gta: bool = False) -> int:
    return int(load_library().gla_decode_workspace_size(ctypes.byref(p), int(is_gta)))


def gla_decode_select_impl(p: GlaDecodeParams, is_gta: bool = False) -> int:
    return int(load_library().gla_decode_select_impl(ctypes.byref(p), int(is_gta)))


def _strides(t: torch.Tensor, n: int):
    assert t.stride(-1) == 1 or t.shape[-1] <= 1, "last dimension must be contiguous"
    return tuple(int(s) for s in t.stride()[:n])


def make_params(q_nope: torch.Tensor, q_rope: Optional[torch.Tensor], state_cache: torch.Tensor,
                rope_cache: Optional[torch.Tensor], page_table: torch.Tensor,
                seq_lens: torch.Tensor, softmax_scale: float, *, out: torch.Tensor,
                lse: torch.Tensor, workspace: Optional[torch.Tensor], causal: bool = True,
                num_splits: int = 0, impl: int = GLA_IMPL_AUTO) -> GlaDecodeParams:
    B, T, h_q, d_n = q_nope.shape
    n_pages, h_c, P, d_v = state_cache.shape
    d_r = 0 if q_rope is None else q_rope.shape[-1]
    assert q_nope.dtype == torch.bfloat16 and state_cache.dtype == torch.bfloat16
    assert page_table.dtype == torch.int32 and page_table.is_contiguous()
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous()
    assert lse.dtype == torch.float32 and lse.is_contiguous() and tuple(lse.shape) == (B, T, h_q)
    assert tuple(out.shape) == (B, T, h_q, d_v)
    out_dtype = {torch.bfloat16: GLA_OUT_BF16, torch.float32: GLA_OUT_FP32}[out.dtype]
    p = shape_params(batch=B, q_len=T, num_q_heads=h_q, num_groups=h_c, d_v=d_v, d_nope=d_n,
                     d_rope=d_r, page_size=P, max_pages_per_seq=page_table.shape[1],
                     num_pages=n_pages, causal=causal, num_splits=num_splits, impl=impl,
                     out_dtype=out_dtype)
    p.q_nope = q_nope.data_ptr()
    p.q_nope_stride = _strides(q_nope, 3)
    if d_r > 0:
        assert q_rope.dtype == torch.bfloat16 and rope_cache.dtype == torch.bfloat16
        assert tuple(q_rope.shape) == (B, T, h_q, d_r)
        assert tuple(rope_cache.shape) == (n_pages, P, d_r)
        p.q_rope = q_rope.data_ptr()
        p.q_rope_stride = _strides(q_rope, 3)
        p.rope_cache = rope_cache.data_ptr()
        p.rope_stride = _strides(rope_cache, 2)
    p.state_cache = state_cache.data_ptr()
    p.state_stride = _strides(state_cache, 3)
    p.page_table = page_table.data_ptr()
    p.seq_lens = seq_lens.data_ptr()
    p.softmax_scale = float(softmax_scale)
    p.out = out.data_ptr()
    p.out_stride = _strides(out, 3)
    p.lse = lse.data_ptr()
    if workspace is not None:
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel() * workspace.element_size()
    p.stream = torch.cuda.current_stream(q_nope.device).cuda_stream
    return p


def _decode(is_gta, q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens,
            softmax_scale, *, causal=True, out=None, lse=None, workspace=None, num_splits=0,
            impl=GLA_IMPL_AUTO, out_dtype=torch.bfloat16, key_cache=None) -> Tuple[torch.Tensor, torch.Tensor]:
    lib = load_library()
    B, T, h_q, _ = q_nope.shape
    d_v = state_cache.shape[-1]
    dev = q_nope.device
    if out is None:
        out = torch.empty(B, T, h_q, d_v, dtype=out_dtype, device=dev)
    if lse is None:
        lse = torch.empty(B, T, h_q, dtype=torch.float32, device=dev)
    p = make_params(q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens, softmax_scale,
                    out=out, lse=lse, workspace=workspace, causal=causal, num_splits=num_splits,
                    impl=impl)
    if workspace is None:
        need = int(lib.gla_decode_workspace_size(ctypes.byref(p), int(is_gta)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel()
    with torch.cuda.device(dev):
        if key_cache is not None:
            assert key_cache.dtype == torch.bfloat16 and key_cache.stride(-1) == 1
            ks = (ctypes.c_int64 * 3)(*_strides(key_cache, 3))
            rc = lib.gqa_decode(ctypes.byref(p), key_cache.data_ptr(), ks)
        else:
            rc = (lib.gta_decode if is_gta else lib.gla_decode)(ctypes.byref(p))
    if rc != GLA_OK:
        raise GlaError(rc)
    return out, lse


def gla_decode(q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens, softmax_scale, **kw):
    """GLA / MLA-shape absorbed decode attention (Section 3.3.2).  Returns
    (out [B,T,h_q,d_c], lse [B,T,h_q]); enqueued on the current stream."""
    return _decode(False, q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens,
                   softmax_scale, **kw)


def gta_decode(q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens, softmax_scale, **kw):
    """GTA decode attention (Section 3.3.1): V = tied state, K = [its first
    half, shared RoPE key]."""
    return _decode(True, q_nope, q_rope, state_cache, rope_cache, page_table, seq_lens,
                   softmax_scale, **kw)


def gqa_decode(q, key_cache, value_cache, page_table, seq_lens, softmax_scale, **kw):
    """Grouped-query decode baseline (separate key / value caches, Section 3.3.1's
    comparison).  q [B,T,h_q,d_k]; returns (out [B,T,h_q,d_v], lse)."""
    return _decode(2, q, None, value_cache, None, page_table, seq_lens, softmax_scale, key_cache=key_cache, **kw)


def decode_prepared(p: GlaDecodeParams, is_gta: bool = False) -> None:
    """Enqueue one decode call from an already filled parameter block (see
    make_params): the per-call path of a serving loop, with no tensor
    inspection and no allocation on the Python side."""
    lib = load_library()
    rc = (lib.gta_decode if is_gta else lib.gla_decode)(ctypes.byref(p))
    if rc != GLA_OK:
        raise GlaError(rc)


def gla_decode_noalloc(p: GlaDecodeParams, is_gta: bool = False) -> None:
    """Enqueue one decode call from a filled parameter block through the entry
    point that allocates nothing: partial results go to the library's own fixed
    buffer, p.workspace is ignored."""
    rc = load_library().gla_decode_noalloc(ctypes.byref(p), int(is_gta))
    if rc != GLA_OK:
        raise GlaError(rc)


def _proj(sum_groups: bool, a: torch.Tensor, w: torch.Tensor, *, out=None, out_dtype=torch.bfloat16,
          workspace=None) -> torch.Tensor:
    """a [rows, G, K] (strided rows / groups, K contiguous), w [G, N, K] contiguous."""
    lib = load_library()
    M, G, K = a.shape
    G2, N, K2 = w.shape
    assert (G2, K2) == (G, K) and a.dtype == torch.bfloat16 and w.dtype == torch.bfloat16
    assert a.stride(-1) == 1 and w.is_contiguous()
    if out is None:
        out = torch.empty((M, N) if sum_groups else (M, G, N), dtype=out_dtype, device=a.device)
    assert out.stride(-1) == 1
    p = GlaProjParams()
    p.rows, p.groups, p.n, p.k = M, G, N, K
    p.a, p.a_row_stride, p.a_group_stride = a.data_ptr(), a.stride(0), a.stride(1)
    p.w = w.data_ptr()
    p.c, p.c_row_stride = out.data_ptr(), out.stride(0)
    p.c_group_stride = 0 if sum_groups else out.stride(1)
    p.c_dtype = {torch.bfloat16: GLA_OUT_BF16, torch.float32: GLA_OUT_FP32}[out.dtype]
    need = int(lib.gla_proj_workspace_size(ctypes.byref(p), int(sum_groups)))
    if need == 0:
        raise GlaError(GLA_ERR_UNSUPPORTED_SHAPE)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    p.stream = torch.cuda.current_stream(a.device).cuda_stream
    with torch.cuda.device(a.device):
        rc = (lib.gla_output_proj if sum_groups else lib.gla_absorb_query)(ctypes.byref(p))
    if rc != GLA_OK:
        raise GlaError(rc)
    return out


def gla_absorb_query(q: torch.Tensor, w_uk: torch.Tensor, **kw) -> torch.Tensor:
    """Absorbed queries (Section 2.1): q [rows, h_q, d_h] raw non-RoPE queries,
    w_uk [h_q, d_c, d_h] -> [rows, h_q, d_c]."""
    return _proj(False, q, w_uk, **kw)


def gla_output_proj(o: torch.Tensor, w_vo: torch.Tensor, **kw) -> torch.Tensor:
    """Grouped output projection (Section 3.3.2): o [rows, h_c, g_q * d_c] latent
    outputs grouped by latent head, w_vo [h_c, D, g_q * d_c] -> [rows, D]."""
    return _proj(True, o, w_vo, **kw)


def gqa_decode_prepared(p: GlaDecodeParams, key_cache: torch.Tensor) -> None:
    """decode_prepared for the grouped-query entry point."""
    ks = (ctypes.c_int64 * 3)(*_strides(key_cache, 3))
    rc = load_library().gqa_decode(ctypes.byref(p), key_cache.data_ptr(), ks)
    if rc != GLA_OK:
        raise GlaError(rc)


def gla_decode_check_contents(p: GlaDecodeParams, is_gta: bool = False) -> int:
    """Number of out-of-range lengths and held page-table entries in the device
    buffers of `p` (0 = what the decode calls trust holds).  Synchronises p.stream."""
    n = ctypes.c_int(0)
    rc = load_library().gla_decode_check_contents(ctypes.byref(p), int(is_gta), ctypes.byref(n))
    if rc != GLA_OK:
        raise GlaError(rc)
    return int(n.value)


def gla_decode_profile(p: GlaDecodeParams, is_gta: bool, iters: int) -> Tuple[float, float]:
    """Mean (main kernel, combine kernel) durations in microseconds over
    `iters` calls, measured with HIP events on p.stream."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    rc = load_library().gla_decode_profile(ctypes.byref(p), int(is_gta), int(iters),
                                           ctypes.byref(a), ctypes.byref(b))
    if rc != GLA_OK:
        raise GlaError(rc)
    return float(a.value), float(b.value)
