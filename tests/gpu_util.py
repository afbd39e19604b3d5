"""Plumbing shared by the GPU parity tests: move a workload to the device, run the
library's three calls in timeline order, and run the oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from harness import workloads as W

TOL = {"f16": 2e-3, "bf16": 1.6e-2, "f32": 1e-5}   # max-abs error against the fp64 oracle


def to_dev(a: np.ndarray, dtype: str | None = None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_np(t: torch.Tensor, dtype: str) -> np.ndarray:
    t = t.detach().cpu()
    if dtype == "bf16":
        return t.view(torch.uint16).numpy() if hasattr(torch, "uint16") else t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def out_to_f64(t: torch.Tensor, dtype: str) -> np.ndarray:
    return W.storage_to_f64(to_np(t, dtype), dtype)


class DeviceWorkload:
    def __init__(self, w: W.Workload, v: W.Values):
        self.w = w
        d = w.dtype
        self.q = to_dev(v.q, d)
        self.k_cache = to_dev(v.k_cache, d)
        self.v_cache = to_dev(v.v_cache, d)
        self.k_new = to_dev(v.k_new, d)
        self.v_new = to_dev(v.v_new, d)
        self.block_tables = to_dev(w.block_tables)
        self.context_lens = to_dev(w.context_lens)
        self.write_slots = to_dev(w.write_slots)
        self.copy_pairs = to_dev(w.copy_pairs)


def gpu_cache_ops(pa, dw: DeviceWorkload) -> None:
    """copy-on-write copies, then the new tokens' K/V, as a decode step orders them."""
    pa.pa_copy_blocks([dw.k_cache], [dw.v_cache], dw.copy_pairs)
    pa.pa_reshape_and_cache(dw.k_new, dw.v_new, dw.k_cache, dw.v_cache, dw.write_slots)


def gpu_decode(pa, dw: DeviceWorkload, partition_size: int = 0, max_context_len: int | None = None) -> torch.Tensor:
    w = dw.w
    mcl = w.max_context_len if max_context_len is None else max_context_len
    out = torch.full_like(dw.q, float("nan"))
    ws = None
    nbytes = pa.pa_decode_workspace_bytes(w.num_seqs, w.num_heads, w.head_dim, w.block_size, mcl, partition_size)
    if nbytes:
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    pa.pa_decode(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                 float(w.scale), mcl, partition_size, ws)
    torch.cuda.synchronize()
    return out


def oracle_cache_ops(w: W.Workload, v: W.Values):
    kc, vc = v.k_cache.copy(), v.v_cache.copy()
    oracle.copy_blocks([kc], [vc], w.copy_pairs, w.dtype)
    oracle.reshape_and_cache(v.k_new, v.v_new, kc, vc, w.write_slots, w.dtype)
    return kc, vc


def same_bits(t: torch.Tensor, a: np.ndarray, dtype: str) -> bool:
    return np.array_equal(to_np(t, dtype).view(np.uint8), a.view(np.uint8))


def gpu_decode_shared(pa, dw: DeviceWorkload) -> torch.Tensor:
    w = dw.w
    out = torch.full_like(dw.q, float("nan"))
    ws = torch.empty(pa.pa_decode_shared_workspace_bytes(w.num_seqs, w.num_heads, w.head_dim, w.max_blocks_per_seq),
                     dtype=torch.uint8, device="cuda")
    pa.pa_decode_shared(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                        float(w.scale), w.max_context_len, ws)
    torch.cuda.synchronize()
    return out
