"""Thin ctypes binding over libspecprefill.so (argument marshalling only).

Every function here has the name of the C entry point it forwards to.  Tensors are
torch device tensors used purely as device memory; the stream is torch's current
HIP stream unless one is given.  There is no fallback: if the shared library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

SP_OK = 0
SP_EINVAL, SP_ENULL, SP_EALIGN, SP_EWORKSPACE, SP_EUNSUPPORTED, SP_ELAUNCH, SP_ETIMEOUT = -1, -2, -3, -4, -5, -6, -7
SP_LAYER_MAX, SP_LAYER_MEAN = 0, 1
SP_MAX_LAYERS, SP_MAX_QUERIES = 128, 16
SP_SCORE_EXCLUSIVE_DEVICE = 1
SP_SCORE_WORKSPACE_KEPT = 2
SP_K_BF16, SP_K_FP8_E4M3 = 0, 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspecprefill.so")

EXPORTS = (
    "sp_score_workspace_bytes", "sp_score", "sp_score_general", "sp_score_check", "sp_set_wait_budget",
    "sp_keep_upper_bound", "sp_pool_select_workspace_bytes", "sp_pool_select", "sp_pool_select_static", "sp_score_pool_select",
    "sp_gather", "sp_strerror", "sp_version",
)


class SpError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed with status {status}: {strerror(status)}")


class ScoreArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("N", C.c_int32), ("L", C.c_int32), ("H", C.c_int32), ("H_kv", C.c_int32),
        ("d", C.c_int32), ("T", C.c_int64), ("d_q", C.c_void_p), ("k_layers", C.POINTER(C.c_void_p)),
        ("k_token_stride", C.c_int64), ("k_head_stride", C.c_int64), ("d_cu_seqlens", C.c_void_p),
        ("d_n_valid", C.c_void_p), ("scale", C.c_float), ("layer_reduce", C.c_int32),
        ("rope_theta", C.c_float), ("d_q_pos", C.c_void_p), ("d_scores", C.c_void_p), ("d_lse", C.c_void_p),
        ("d_workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("d_block_table", C.c_void_p), ("page_size", C.c_int32), ("blocks_per_seq", C.c_int32),
        ("k_page_stride", C.c_int64), ("flags", C.c_uint32), ("max_seqlen", C.c_int32),
        ("k_dtype", C.c_int32), ("d_k_scale", C.c_void_p),
    ]


class PoolSelectArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("T", C.c_int64), ("d_cu_seqlens", C.c_void_p), ("d_scores", C.c_void_p),
        ("chunk", C.c_int32), ("pool_window", C.c_int32), ("keep_rate", C.c_double),
        ("d_kept_idx", C.c_void_p), ("kept_capacity", C.c_int64), ("d_cu_keep", C.c_void_p),
        ("d_chunk_scores", C.c_void_p), ("d_workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class GatherArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("d_cu_seqlens", C.c_void_p), ("d_cu_keep", C.c_void_p), ("d_kept_idx", C.c_void_p),
        ("d_token_ids", C.c_void_p), ("d_embed", C.c_void_p), ("V", C.c_int32), ("D", C.c_int32),
        ("d_kept_ids", C.c_void_p), ("d_kept_pos", C.c_void_p), ("d_decode_pos", C.c_void_p),
        ("d_out_embed", C.c_void_p), ("kept_capacity", C.c_int64),
    ]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2502_02789_amd.build)")
    lib = C.CDLL(LIB_PATH)
    lib.sp_score_workspace_bytes.restype = C.c_size_t
    lib.sp_score_workspace_bytes.argtypes = [C.POINTER(ScoreArgs)]
    lib.sp_score.restype = C.c_int
    lib.sp_score.argtypes = [C.POINTER(ScoreArgs), C.c_void_p]
    lib.sp_score_general.restype = C.c_int
    lib.sp_score_general.argtypes = [C.POINTER(ScoreArgs), C.c_void_p]
    lib.sp_score_check.restype = C.c_int
    lib.sp_score_check.argtypes = [C.POINTER(ScoreArgs), C.c_void_p]
    lib.sp_set_wait_budget.restype = C.c_int32
    lib.sp_set_wait_budget.argtypes = [C.c_int32]
    lib.sp_keep_upper_bound.restype = C.c_int64
    lib.sp_keep_upper_bound.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_double]
    lib.sp_pool_select_workspace_bytes.restype = C.c_size_t
    lib.sp_pool_select_workspace_bytes.argtypes = [C.POINTER(PoolSelectArgs)]
    lib.sp_pool_select.restype = C.c_int
    lib.sp_pool_select.argtypes = [C.POINTER(PoolSelectArgs), C.c_void_p]
    lib.sp_pool_select_static.restype = C.c_int
    lib.sp_pool_select_static.argtypes = [C.POINTER(PoolSelectArgs), C.c_void_p]
    lib.sp_score_pool_select.restype = C.c_int
    lib.sp_score_pool_select.argtypes = [C.POINTER(ScoreArgs), C.POINTER(PoolSelectArgs), C.c_void_p]
    lib.sp_gather.restype = C.c_int
    lib.sp_gather.argtypes = [C.POINTER(GatherArgs), C.c_void_p]
    lib.sp_strerror.restype = C.c_char_p
    lib.sp_strerror.argtypes = [C.c_int]
    lib.sp_version.restype = C.c_int32
    lib.sp_version.argtypes = []
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().sp_strerror(int(status)).decode()


def sp_version() -> int:
    return int(load_library().sp_version())


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream) or None


def _check(fn: str, status: int) -> None:
    if status != SP_OK:
        raise SpError(fn, status)


# ----------------------------------------------------------------------------
# sp_score
# ----------------------------------------------------------------------------
def make_score_args(q, k_layers: Sequence, cu_seqlens, scores, *, H_kv: int, scale: float,
                    layer_reduce: int = SP_LAYER_MAX, n_valid=None, lse=None, workspace=None,
                    k_token_stride: Optional[int] = None, k_head_stride: Optional[int] = None,
                    T: Optional[int] = None, rope_theta: float = 0.0, q_pos=None,
                    block_table=None, page_size: int = 0, flags: int = 0, max_seqlen: int = 0, k_scale=None) -> ScoreArgs:
    """q: bf16 [L,B,N,H,d]; k_layers: L bf16 tensors [T,H_kv,d] (any token/head strides), or, with
    block_table (int32 [B, blocks_per_seq]), L page pools [pages, page_size, H_kv, d] (then T must be given).
    uint8 layers are taken as an 8-bit float cache (SP_K_FP8_E4M3) with k_scale fp32 [L, H_kv] (None: all 1)."""
    L, B, N, H, d = q.shape
    a = ScoreArgs()
    a.B, a.N, a.L, a.H, a.H_kv, a.d = B, N, L, H, H_kv, d
    a.T = int(k_layers[0].shape[0]) if T is None else int(T)
    a.d_q = _ptr(q)
    arr = (C.c_void_p * len(k_layers))(*[_ptr(k) for k in k_layers])
    a._keepalive = arr                    # the struct only holds a pointer to this host array
    a.k_layers = C.cast(arr, C.POINTER(C.c_void_p))
    if block_table is not None:
        if T is None:
            raise ValueError("T (total tokens) must be given with a paged cache")
        a.d_block_table = _ptr(block_table)
        a.page_size = int(page_size)
        a.blocks_per_seq = int(block_table.shape[1])
        a.k_page_stride = int(k_layers[0].stride(0))
        a._keepalive_table = block_table
        a.k_token_stride = int(k_layers[0].stride(1)) if k_token_stride is None else int(k_token_stride)
        a.k_head_stride = int(k_layers[0].stride(2)) if k_head_stride is None else int(k_head_stride)
    else:
        a.k_token_stride = int(k_layers[0].stride(0)) if k_token_stride is None else int(k_token_stride)
        a.k_head_stride = int(k_layers[0].stride(1)) if k_head_stride is None else int(k_head_stride)
    a.d_cu_seqlens = _ptr(cu_seqlens)
    a.d_n_valid = _ptr(n_valid)
    a.scale = float(scale)
    a.layer_reduce = int(layer_reduce)
    a.rope_theta = float(rope_theta)
    a.d_q_pos = _ptr(q_pos)
    a.d_scores = _ptr(scores)
    a.d_lse = _ptr(lse)
    a.d_workspace = _ptr(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.flags = int(flags)
    a.max_seqlen = int(max_seqlen)
    a.k_dtype = SP_K_FP8_E4M3 if k_layers[0].element_size() == 1 else SP_K_BF16
    a.d_k_scale = _ptr(k_scale)
    a._keepalive_scale = k_scale
    return a


def sp_score_workspace_bytes(args: ScoreArgs) -> int:
    return int(load_library().sp_score_workspace_bytes(C.byref(args)))


def sp_score(args: ScoreArgs, stream=None) -> None:
    _check("sp_score", load_library().sp_score(C.byref(args), _stream_handle(stream)))


def sp_score_check(args: ScoreArgs, stream=None) -> None:
    """Synchronises the stream; raises SpError(SP_ETIMEOUT) if a device-side wait expired."""
    _check("sp_score_check", load_library().sp_score_check(C.byref(args), _stream_handle(stream)))


def sp_set_wait_budget(polls: int) -> int:
    """Sets the bound on polls per wave of the single-pass kernels' waits; returns the previous one."""
    return int(load_library().sp_set_wait_budget(int(polls)))


def sp_score_general(args: ScoreArgs, stream=None) -> None:
    _check("sp_score_general", load_library().sp_score_general(C.byref(args), _stream_handle(stream)))


# ----------------------------------------------------------------------------
# sp_pool_select
# ----------------------------------------------------------------------------
def make_pool_select_args(scores, cu_seqlens, kept_idx, cu_keep, *, chunk: int, pool_window: int,
                          keep_rate: float, chunk_scores=None, workspace=None,
                          kept_capacity: Optional[int] = None) -> PoolSelectArgs:
    a = PoolSelectArgs()
    a.B = int(cu_seqlens.numel()) - 1
    a.T = int(scores.numel())
    a.d_cu_seqlens = _ptr(cu_seqlens)
    a.d_scores = _ptr(scores)
    a.chunk, a.pool_window, a.keep_rate = int(chunk), int(pool_window), float(keep_rate)
    a.d_kept_idx = _ptr(kept_idx)
    a.kept_capacity = int(kept_idx.numel()) if kept_capacity is None else int(kept_capacity)
    a.d_cu_keep = _ptr(cu_keep)
    a.d_chunk_scores = _ptr(chunk_scores)
    a.d_workspace = _ptr(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return a


def sp_keep_upper_bound(seqlens: Sequence[int], chunk: int, keep_rate: float) -> int:
    arr = (C.c_int32 * max(1, len(seqlens)))(*[int(x) for x in seqlens])
    return int(load_library().sp_keep_upper_bound(len(seqlens), arr, int(chunk), float(keep_rate)))


def sp_pool_select_workspace_bytes(args: PoolSelectArgs) -> int:
    return int(load_library().sp_pool_select_workspace_bytes(C.byref(args)))


def sp_pool_select(args: PoolSelectArgs, stream=None) -> None:
    _check("sp_pool_select", load_library().sp_pool_select(C.byref(args), _stream_handle(stream)))


def sp_score_pool_select(score: ScoreArgs, select: PoolSelectArgs, stream=None) -> None:
    """One short prompt scored and selected in a single launch (raises SpError(SP_EUNSUPPORTED) if it does not fit)."""
    _check("sp_score_pool_select",
           load_library().sp_score_pool_select(C.byref(score), C.byref(select), _stream_handle(stream)))


SP_STATIC_MAX_SEQS, SP_STATIC_MAX_CHUNKS = 4096, 131072


def sp_pool_select_static(args: PoolSelectArgs, stream=None) -> None:
    """sp_pool_select on the library's built-in scratch space (no workspace, nothing allocated)."""
    _check("sp_pool_select_static", load_library().sp_pool_select_static(C.byref(args), _stream_handle(stream)))


# ----------------------------------------------------------------------------
# sp_gather
# ----------------------------------------------------------------------------
def make_gather_args(cu_seqlens, cu_keep, kept_idx, kept_pos, decode_pos, *, token_ids=None, kept_ids=None,
                     embed=None, out_embed=None, kept_capacity: Optional[int] = None) -> GatherArgs:
    a = GatherArgs()
    a.B = int(cu_seqlens.numel()) - 1
    a.d_cu_seqlens, a.d_cu_keep, a.d_kept_idx = _ptr(cu_seqlens), _ptr(cu_keep), _ptr(kept_idx)
    a.d_token_ids = _ptr(token_ids)
    a.d_embed = _ptr(embed)
    a.V = 0 if embed is None else int(embed.shape[0])
    a.D = 0 if embed is None else int(embed.shape[1])
    a.d_kept_ids, a.d_kept_pos, a.d_decode_pos = _ptr(kept_ids), _ptr(kept_pos), _ptr(decode_pos)
    a.d_out_embed = _ptr(out_embed)
    a.kept_capacity = int(kept_pos.numel()) if kept_capacity is None else int(kept_capacity)
    return a


def sp_gather(args: GatherArgs, stream=None) -> None:
    _check("sp_gather", load_library().sp_gather(C.byref(args), _stream_handle(stream)))
