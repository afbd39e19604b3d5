"""ctypes binding of libpa.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks their
dtype, shape and contiguity, and passes raw device pointers plus the current
HIP stream to the C ABI declared in include/pa.h.  There is no fallback: if
the shared library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

from .build import LIB

PA_F32, PA_F16, PA_BF16 = 0, 1, 2
PA_PARTITION_AUTO = -1

EXPORTS = ("pa_decode", "pa_decode_workspace_bytes", "pa_decode_static", "pa_decode_shared", "pa_decode_shared_workspace_bytes", "pa_shared_plan", "pa_decode_shared_planned", "pa_decode_multi", "pa_reshape_and_cache", "pa_copy_blocks", "pa_swap_blocks",
           "pa_debug_validate", "pa_stream_read", "pa_status_string", "pa_version")

_DT = {torch.float32: PA_F32, torch.float16: PA_F16, torch.bfloat16: PA_BF16}

_lib = None


class PAError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("libpa: %s (status %d)" % (what, code))
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the in-tree libpa.so (build it first with paper_2309_06180_amd.build.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB):
        raise FileNotFoundError(
            "%s not found: run `python -c 'import __graft_entry__ as g; g.build()'` first" % LIB)
    lib = ctypes.CDLL(LIB)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.pa_decode.restype = ctypes.c_int
    lib.pa_decode.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i64, ctypes.c_int,
                              ctypes.c_float, i32, i32, vp, sz, vp]
    lib.pa_decode_static.restype = ctypes.c_int
    lib.pa_decode_static.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i64, ctypes.c_int,
                                     ctypes.c_float, i32, i32, vp]
    lib.pa_decode_workspace_bytes.restype = sz
    lib.pa_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.pa_decode_shared.restype = ctypes.c_int
    lib.pa_decode_shared.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i64, ctypes.c_int,
                                     ctypes.c_float, i32, vp, sz, vp]
    lib.pa_shared_plan.restype = ctypes.c_int
    lib.pa_shared_plan.argtypes = [vp, i32, vp, i32, i32, i32, i32, i64, ctypes.c_int, i32, vp, sz, vp]
    lib.pa_decode_shared_planned.restype = ctypes.c_int
    lib.pa_decode_shared_planned.argtypes = lib.pa_decode_shared.argtypes
    lib.pa_decode_shared_workspace_bytes.restype = sz
    lib.pa_decode_shared_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.pa_decode_multi.restype = ctypes.c_int
    lib.pa_decode_multi.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i64, ctypes.c_int,
                                    ctypes.c_float, i32, vp]
    lib.pa_reshape_and_cache.restype = ctypes.c_int
    lib.pa_reshape_and_cache.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, ctypes.c_int, vp]
    lib.pa_copy_blocks.restype = ctypes.c_int
    lib.pa_copy_blocks.argtypes = [vp, vp, i32, vp, i32, i32, i32, i32, i64, ctypes.c_int, vp]
    lib.pa_swap_blocks.restype = ctypes.c_int
    lib.pa_swap_blocks.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i64, i64, ctypes.c_int, vp]
    lib.pa_debug_validate.restype = ctypes.c_int
    lib.pa_debug_validate.argtypes = [vp, i32, vp, i32, i32, vp, i32, vp, i32, i32, i64, vp]
    lib.pa_stream_read.restype = ctypes.c_int
    lib.pa_stream_read.argtypes = [vp, sz, vp, vp]
    lib.pa_status_string.restype = ctypes.c_char_p
    lib.pa_status_string.argtypes = [ctypes.c_int]
    lib.pa_version.restype = ctypes.c_int
    lib.pa_version.argtypes = []
    _lib = lib
    return lib


def _check(code: int) -> None:
    if code != 0:
        raise PAError(code, load_library().pa_status_string(code).decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, name: str, dtype=None) -> int:
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def pa_version() -> int:
    return int(load_library().pa_version())


def pa_decode_workspace_bytes(num_seqs: int, num_heads: int, head_dim: int, block_size: int,
                              max_context_len: int, partition_size: int) -> int:
    return int(load_library().pa_decode_workspace_bytes(num_seqs, num_heads, head_dim, block_size,
                                                        max_context_len, partition_size))


def pa_decode(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
              block_tables: torch.Tensor, context_lens: torch.Tensor, block_size: int, scale: float,
              max_context_len: int, partition_size: int = 0,
              workspace: Optional[torch.Tensor] = None) -> None:
    """out[S][H][D] = paged attention of q[S][H][D] over k_cache/v_cache [NB][H][B][D]."""
    S, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    if (H2, B, D2) != (H, block_size, D) or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent shapes")
    if block_tables.dim() != 2 or block_tables.shape[0] != S or context_lens.shape != (S,):
        raise ValueError("block_tables must be [S][MB], context_lens [S]")
    dt = _DT[q.dtype]
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(load_library().pa_decode(
        _dev(out, "out", q.dtype), _dev(q, "q"), _dev(k_cache, "k_cache", q.dtype),
        _dev(v_cache, "v_cache", q.dtype), _dev(block_tables, "block_tables", torch.int32),
        block_tables.shape[1], _dev(context_lens, "context_lens", torch.int32), S, H, D, B, NB, dt,
        float(scale), int(max_context_len), int(partition_size), ws_ptr, ws_bytes, _stream()))


PA_STATIC_SCRATCH_BYTES = 16 << 20


def pa_decode_static(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                     block_tables: torch.Tensor, context_lens: torch.Tensor, block_size: int, scale: float,
                     max_context_len: int, partition_size: int = 0) -> None:
    """pa_decode whose split-context partials live in the library's own static device array."""
    S, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    if (H2, B, D2) != (H, block_size, D) or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent shapes")
    if block_tables.dim() != 2 or block_tables.shape[0] != S or context_lens.shape != (S,):
        raise ValueError("block_tables must be [S][MB], context_lens [S]")
    _check(load_library().pa_decode_static(
        _dev(out, "out", q.dtype), _dev(q, "q"), _dev(k_cache, "k_cache", q.dtype),
        _dev(v_cache, "v_cache", q.dtype), _dev(block_tables, "block_tables", torch.int32),
        block_tables.shape[1], _dev(context_lens, "context_lens", torch.int32), S, H, D, B, NB, _DT[q.dtype],
        float(scale), int(max_context_len), int(partition_size), _stream()))


def pa_decode_shared_workspace_bytes(num_seqs: int, num_heads: int, head_dim: int,
                                     max_blocks_per_seq: int) -> int:
    return int(load_library().pa_decode_shared_workspace_bytes(num_seqs, num_heads, head_dim,
                                                               max_blocks_per_seq))


def pa_decode_shared(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                     block_tables: torch.Tensor, context_lens: torch.Tensor, block_size: int, scale: float,
                     max_context_len: int, workspace: torch.Tensor) -> None:
    """pa_decode that reads blocks shared by neighbouring sequences once per group."""
    S, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    if (H2, B, D2) != (H, block_size, D) or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent shapes")
    if block_tables.dim() != 2 or block_tables.shape[0] != S or context_lens.shape != (S,):
        raise ValueError("block_tables must be [S][MB], context_lens [S]")
    _check(load_library().pa_decode_shared(
        _dev(out, "out", q.dtype), _dev(q, "q"), _dev(k_cache, "k_cache", q.dtype),
        _dev(v_cache, "v_cache", q.dtype), _dev(block_tables, "block_tables", torch.int32),
        block_tables.shape[1], _dev(context_lens, "context_lens", torch.int32), S, H, D, B, NB,
        _DT[q.dtype], float(scale), int(max_context_len), _dev(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), _stream()))


def pa_shared_plan(block_tables: torch.Tensor, context_lens: torch.Tensor, num_heads: int, head_dim: int,
                   block_size: int, num_blocks: int, dtype: torch.dtype, max_context_len: int,
                   workspace: torch.Tensor) -> None:
    """Build pa_decode_shared's plan (groups and tile lists) for these tables in `workspace`."""
    S = context_lens.shape[0]
    if block_tables.dim() != 2 or block_tables.shape[0] != S:
        raise ValueError("block_tables must be [S][MB], context_lens [S]")
    _check(load_library().pa_shared_plan(
        _dev(block_tables, "block_tables", torch.int32), block_tables.shape[1],
        _dev(context_lens, "context_lens", torch.int32), S, int(num_heads), int(head_dim), int(block_size),
        int(num_blocks), _DT[dtype], int(max_context_len), _dev(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), _stream()))


def pa_decode_shared_planned(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                             block_tables: torch.Tensor, context_lens: torch.Tensor, block_size: int,
                             scale: float, max_context_len: int, plan: torch.Tensor) -> None:
    """pa_decode_shared's decode launch alone, reading a plan that pa_shared_plan built for the same tables."""
    S, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    if (H2, B, D2) != (H, block_size, D) or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent shapes")
    if block_tables.dim() != 2 or block_tables.shape[0] != S or context_lens.shape != (S,):
        raise ValueError("block_tables must be [S][MB], context_lens [S]")
    _check(load_library().pa_decode_shared_planned(
        _dev(out, "out", q.dtype), _dev(q, "q"), _dev(k_cache, "k_cache", q.dtype),
        _dev(v_cache, "v_cache", q.dtype), _dev(block_tables, "block_tables", torch.int32),
        block_tables.shape[1], _dev(context_lens, "context_lens", torch.int32), S, H, D, B, NB,
        _DT[q.dtype], float(scale), int(max_context_len), _dev(plan, "plan"),
        plan.numel() * plan.element_size(), _stream()))


def pa_decode_multi(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                    block_tables: torch.Tensor, context_lens: torch.Tensor, q_start: torch.Tensor,
                    max_q_len: int, block_size: int, scale: float, max_context_len: int) -> None:
    """out[T][H][D]: causal attention of each sequence's last q_len tokens (rows q_start[s]..q_start[s+1])."""
    T, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    S = context_lens.shape[0]
    if (H2, B, D2) != (H, block_size, D) or v_cache.shape != k_cache.shape or out.shape != q.shape:
        raise ValueError("inconsistent shapes")
    if block_tables.dim() != 2 or block_tables.shape[0] != S or q_start.shape != (S + 1,):
        raise ValueError("block_tables must be [S][MB], q_start [S+1]")
    _check(load_library().pa_decode_multi(
        _dev(out, "out", q.dtype) if T else None, _dev(q, "q") if T else None,
        _dev(k_cache, "k_cache", q.dtype), _dev(v_cache, "v_cache", q.dtype),
        _dev(block_tables, "block_tables", torch.int32), block_tables.shape[1],
        _dev(context_lens, "context_lens", torch.int32), _dev(q_start, "q_start", torch.int32), S,
        int(max_q_len), H, D, B, NB, _DT[q.dtype], float(scale), int(max_context_len), _stream()))


def pa_reshape_and_cache(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor,
                         v_cache: torch.Tensor, slot_mapping: torch.Tensor) -> None:
    """Store k[t], v[t] ([T][H][D]) at slot_mapping[t] of the caches [NB][H][B][D]."""
    T, H, D = k.shape
    NB, H2, B, D2 = k_cache.shape
    if (H2, D2) != (H, D) or v.shape != k.shape or v_cache.shape != k_cache.shape or slot_mapping.shape != (T,):
        raise ValueError("inconsistent shapes")
    _check(load_library().pa_reshape_and_cache(
        _dev(k, "k"), _dev(v, "v", k.dtype), _dev(k_cache, "k_cache", k.dtype),
        _dev(v_cache, "v_cache", k.dtype), _dev(slot_mapping, "slot_mapping", torch.int64),
        T, H, D, B, NB, _DT[k.dtype], _stream()))


def pa_copy_blocks(k_caches: Sequence[torch.Tensor], v_caches: Sequence[torch.Tensor],
                   src_dst_pairs: torch.Tensor) -> None:
    """For every layer: cache[dst] = cache[src] for each (src, dst) row of src_dst_pairs [N][2]."""
    L = len(k_caches)
    if L == 0 or len(v_caches) != L:
        raise ValueError("need as many V caches as K caches, at least one")
    NB, H, B, D = k_caches[0].shape
    dtype = k_caches[0].dtype
    for c in list(k_caches) + list(v_caches):
        if c.shape != (NB, H, B, D):
            raise ValueError("all caches must share one shape")
        _dev(c, "cache", dtype)
    if src_dst_pairs.dim() != 2 or src_dst_pairs.shape[1] != 2:
        raise ValueError("src_dst_pairs must be [N][2]")
    kp = (ctypes.c_void_p * L)(*[c.data_ptr() for c in k_caches])
    vp = (ctypes.c_void_p * L)(*[c.data_ptr() for c in v_caches])
    n = src_dst_pairs.shape[0]
    _check(load_library().pa_copy_blocks(
        kp, vp, L, _dev(src_dst_pairs, "src_dst_pairs", torch.int64) if n else None, n, H, D, B, NB,
        _DT[dtype], _stream()))


def pa_swap_blocks(src_k: Sequence[torch.Tensor], src_v: Sequence[torch.Tensor],
                   dst_k: Sequence[torch.Tensor], dst_v: Sequence[torch.Tensor],
                   src_dst_pairs: torch.Tensor) -> None:
    """For every layer: dst[dst_block] = src[src_block] per (src_block, dst_block) row of src_dst_pairs.
    Caches on either side may be GPU tensors or pinned CPU tensors."""
    L = len(src_k)
    if L == 0 or len(src_v) != L or len(dst_k) != L or len(dst_v) != L:
        raise ValueError("need the same number of layers on every side")
    NBS, H, B, D = src_k[0].shape
    NBD = dst_k[0].shape[0]
    dtype = src_k[0].dtype
    for c, nb in [(x, NBS) for x in list(src_k) + list(src_v)] + [(x, NBD) for x in list(dst_k) + list(dst_v)]:
        if c.shape != (nb, H, B, D) or c.dtype != dtype or not c.is_contiguous():
            raise ValueError("caches of one side must share shape and dtype and be contiguous")
        if not (c.is_cuda or c.is_pinned()):
            raise ValueError("a cache must live on the GPU or in pinned host memory")
    if src_dst_pairs.dim() != 2 or src_dst_pairs.shape[1] != 2:
        raise ValueError("src_dst_pairs must be [N][2]")
    arr = lambda ts: (ctypes.c_void_p * L)(*[t.data_ptr() for t in ts])
    n = src_dst_pairs.shape[0]
    _check(load_library().pa_swap_blocks(
        arr(src_k), arr(src_v), arr(dst_k), arr(dst_v), L,
        _dev(src_dst_pairs, "src_dst_pairs", torch.int64) if n else None, n, H, D, B, NBS, NBD,
        _DT[dtype], _stream()))


def pa_debug_validate(block_tables: Optional[torch.Tensor], context_lens: Optional[torch.Tensor],
                      max_context_len: int, slot_mapping: Optional[torch.Tensor],
                      src_dst_pairs: Optional[torch.Tensor], block_size: int, num_blocks: int) -> int:
    """Returns the status code (0 = all index arrays are within the contract)."""
    bt = _dev(block_tables, "block_tables", torch.int32) if block_tables is not None else None
    cl = _dev(context_lens, "context_lens", torch.int32) if context_lens is not None else None
    sm = _dev(slot_mapping, "slot_mapping", torch.int64) if slot_mapping is not None else None
    pr = _dev(src_dst_pairs, "src_dst_pairs", torch.int64) if src_dst_pairs is not None and src_dst_pairs.numel() else None
    return int(load_library().pa_debug_validate(
        bt, block_tables.shape[1] if block_tables is not None else 0, cl,
        context_lens.shape[0] if context_lens is not None else 0, int(max_context_len), sm,
        slot_mapping.shape[0] if slot_mapping is not None else 0, pr,
        src_dst_pairs.shape[0] if pr is not None else 0, int(block_size), int(num_blocks), _stream()))


def pa_stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Bandwidth probe: read all of `src` once with 16-byte loads."""
    nbytes = src.numel() * src.element_size()
    if sink.numel() * sink.element_size() < 4 * 65536:
        raise ValueError("sink must hold at least 256 KiB")
    _check(load_library().pa_stream_read(_dev(src, "src"), nbytes, _dev(sink, "sink"), _stream()))
