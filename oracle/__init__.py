"""Python face of the fp64 CPU oracle (oracle/pa_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg; the GPU library and its binding never import
this package, and this package imports nothing from them.

Arrays are numpy, in the cache's storage representation: float32, float16, or
uint16 bit patterns for bfloat16.  Cache arrays are [NB][H][B][D].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pa_oracle.c")
_LIB = os.path.join(_HERE, "libpa_oracle.so")

DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
_NP_OF = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP only for the outer loop over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        lib.pa_oracle_decode.restype = ctypes.c_int
        lib.pa_oracle_decode.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32,
                                         ctypes.c_float, i32, vp, i64, i32]
        lib.pa_oracle_decode_multi.restype = ctypes.c_int
        lib.pa_oracle_decode_multi.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32,
                                               ctypes.c_float, i32]
        lib.pa_oracle_reshape_and_cache.restype = None
        lib.pa_oracle_reshape_and_cache.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32]
        lib.pa_oracle_copy_blocks.restype = None
        lib.pa_oracle_copy_blocks.argtypes = [vp, vp, i32, vp, i32, i32, i32, i32, i32]
        lib.pa_oracle_swap_blocks.restype = None
        lib.pa_oracle_swap_blocks.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32]
        lib.pa_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _chk(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != np.dtype(dtype) or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous numpy array of %s" % (name, np.dtype(dtype)))
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().pa_oracle_max_threads())


def decode(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_tables: np.ndarray,
           context_lens: np.ndarray, scale, dtype: str, partition_size: int = 0,
           rows: Optional[np.ndarray] = None, threads: int = 0, return_threads: bool = False):
    """fp64 attention output [S][H][D] (or [R][D] for the listed (seq, head) rows)."""
    st = _NP_OF[dtype]
    _chk(q, st, "q"); _chk(k_cache, st, "k_cache"); _chk(v_cache, st, "v_cache")
    _chk(block_tables, np.int32, "block_tables"); _chk(context_lens, np.int32, "context_lens")
    S, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    assert (H2, D2) == (H, D) and v_cache.shape == k_cache.shape
    assert block_tables.ndim == 2 and block_tables.shape[0] == S and context_lens.shape == (S,)
    if rows is None:
        out = np.empty((S, H, D), dtype=np.float64)
        nrows, rp = S * H, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
        out = np.empty((rows.shape[0], D), dtype=np.float64)
        nrows, rp = rows.shape[0], _ptr(rows)
    used = _load().pa_oracle_decode(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                    _ptr(block_tables), block_tables.shape[1], _ptr(context_lens),
                                    S, H, D, B, DTYPE_CODE[dtype], float(np.float32(scale)),
                                    int(partition_size), rp, nrows, int(threads))
    return (out, used) if return_threads else out


def decode_multi(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_tables: np.ndarray,
                 context_lens: np.ndarray, q_start: np.ndarray, scale, dtype: str, threads: int = 0):
    """fp64 causal attention [T][H][D] of each sequence's last q_len tokens (rows q_start[s]..q_start[s+1])."""
    st = _NP_OF[dtype]
    _chk(q, st, "q"); _chk(k_cache, st, "k_cache"); _chk(v_cache, st, "v_cache")
    _chk(block_tables, np.int32, "block_tables"); _chk(context_lens, np.int32, "context_lens")
    _chk(q_start, np.int32, "q_start")
    T, H, D = q.shape
    NB, H2, B, D2 = k_cache.shape
    S = context_lens.shape[0]
    assert (H2, D2) == (H, D) and v_cache.shape == k_cache.shape
    assert q_start.shape == (S + 1,) and q_start[0] == 0 and q_start[-1] == T
    q_len = np.diff(q_start)
    assert (q_len >= 0).all() and (q_len <= context_lens).all()
    out = np.empty((T, H, D), dtype=np.float64)
    _load().pa_oracle_decode_multi(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                   block_tables.shape[1], _ptr(context_lens), _ptr(q_start), S, H, D, B,
                                   DTYPE_CODE[dtype], float(np.float32(scale)), int(threads))
    return out


def reshape_and_cache(k: np.ndarray, v: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                      slot_mapping: np.ndarray, dtype: str) -> None:
    """In place: store k[t], v[t] at slot_mapping[t] (negative = skip)."""
    st = _NP_OF[dtype]
    _chk(k, st, "k"); _chk(v, st, "v"); _chk(k_cache, st, "k_cache"); _chk(v_cache, st, "v_cache")
    _chk(slot_mapping, np.int64, "slot_mapping")
    T, H, D = k.shape
    NB, H2, B, D2 = k_cache.shape
    assert (H2, D2) == (H, D) and v.shape == k.shape and slot_mapping.shape == (T,)
    assert slot_mapping.max(initial=-1) < NB * B
    _load().pa_oracle_reshape_and_cache(_ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache),
                                        _ptr(slot_mapping), T, H, D, B, DTYPE_CODE[dtype])


def copy_blocks(k_caches: Sequence[np.ndarray], v_caches: Sequence[np.ndarray],
                src_dst_pairs: np.ndarray, dtype: str) -> None:
    """In place, for every layer: cache[dst] = cache[src] for each (src, dst) pair."""
    st = _NP_OF[dtype]
    L = len(k_caches)
    assert len(v_caches) == L and L >= 1
    pairs = _chk(np.asarray(src_dst_pairs), np.int64, "src_dst_pairs").reshape(-1, 2)
    NB, H, B, D = k_caches[0].shape
    for c in list(k_caches) + list(v_caches):
        _chk(c, st, "cache"); assert c.shape == (NB, H, B, D)
    assert pairs.size == 0 or (pairs.min() >= 0 and pairs.max() < NB)
    kp = (ctypes.c_void_p * L)(*[c.ctypes.data for c in k_caches])
    vp = (ctypes.c_void_p * L)(*[c.ctypes.data for c in v_caches])
    _load().pa_oracle_copy_blocks(kp, vp, L, _ptr(pairs), pairs.shape[0], H, D, B,
                                  DTYPE_CODE[dtype])


def swap_blocks(src_k: Sequence[np.ndarray], src_v: Sequence[np.ndarray], dst_k: Sequence[np.ndarray],
                dst_v: Sequence[np.ndarray], src_dst_pairs: np.ndarray, dtype: str) -> None:
    """In place on the destination pools, for every layer: dst[dst_block] = src[src_block]."""
    st = _NP_OF[dtype]
    L = len(src_k)
    assert L >= 1 and len(src_v) == L and len(dst_k) == L and len(dst_v) == L
    pairs = _chk(np.asarray(src_dst_pairs), np.int64, "src_dst_pairs").reshape(-1, 2)
    NBS, H, B, D = src_k[0].shape
    NBD = dst_k[0].shape[0]
    for c in list(src_k) + list(src_v):
        _chk(c, st, "cache"); assert c.shape == (NBS, H, B, D)
    for c in list(dst_k) + list(dst_v):
        _chk(c, st, "cache"); assert c.shape == (NBD, H, B, D)
    if pairs.size:
        assert pairs.min() >= 0 and pairs[:, 0].max() < NBS and pairs[:, 1].max() < NBD
    arr = lambda cs: (ctypes.c_void_p * L)(*[c.ctypes.data for c in cs])
    _load().pa_oracle_swap_blocks(arr(src_k), arr(src_v), arr(dst_k), arr(dst_v), L, _ptr(pairs),
                                  pairs.shape[0], H, D, B, DTYPE_CODE[dtype])
