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


def mixed_sharing_workload(dtype: str) -> W.Workload:
    """Sharing patterns side by side: three forks that have not diverged (every block shared, the partial
    last one included), a loner, a parent and four children that grew by different amounts, a pair with
    exactly one full block in common, ten forks of one prompt, forty forks of another."""
    from harness.blocks import BlockManager
    rng = np.random.default_rng(33)
    B, NB, H, D = 16, 1400, 2, 128
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    seqs = []
    a = mgr.allocate(70)
    seqs += [a, mgr.fork(a), mgr.fork(a)]                     # identical: 4 full blocks + 6 tokens
    seqs.append(mgr.allocate(33))                             # loner
    b = mgr.allocate(200)
    kids = [mgr.fork(b) for _ in range(4)]
    grow = [0, 5, 40, 90, 17]
    for sq, gsteps in zip([b] + kids, grow):
        for _ in range(gsteps):
            mgr.append(sq)
    seqs += [b] + kids
    c = mgr.allocate(16)
    seqs += [c, mgr.fork(c)]                                  # exactly one shared full block, nothing else
    d = mgr.allocate(150)
    many = [d] + [mgr.fork(d) for _ in range(9)]
    for i, sq in enumerate(many):
        for _ in range(3 * i):
            mgr.append(sq)
    seqs += many
    e = mgr.allocate(260)
    crowd = [e] + [mgr.fork(e) for _ in range(39)]
    for i, sq in enumerate(crowd):
        for _ in range((7 * i) % 45):
            mgr.append(sq)
    seqs += crowd
    mgr.take_copies()
    filled = np.zeros((NB, B), dtype=bool)
    for sq in seqs:
        for j, pb in enumerate(sq.blocks):
            filled[pb, : min(B, sq.length - j * B)] = True
    mb = max(len(sq.blocks) for sq in seqs) + 1
    bt = np.full((len(seqs), mb), -1, dtype=np.int32)
    for i, sq in enumerate(seqs):
        bt[i, : len(sq.blocks)] = sq.blocks
    return W.Workload("mixed", dtype, H, D, B, NB, np.float32(1 / np.sqrt(D)), bt,
                      np.array([sq.length for sq in seqs], dtype=np.int32), filled,
                      np.zeros((0, 2), dtype=np.int64), np.zeros(0, dtype=np.int64),
                      np.zeros(len(seqs), dtype=np.int64), seed=34)
