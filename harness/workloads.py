"""Seeded synthetic workloads shaped like the paper's serving traces.

The paper evaluates on ShareGPT / Alpaca derived traces with OPT-13B/66B/175B
and LLaMA-13B (Sec. 6.1, Table 1); those datasets are not available here, so
every workload below is synthetic: lengths are drawn from stated
distributions, physical block ids come from a seeded permutation of the pool
(so logically adjacent blocks are scattered in memory, Sec. 4.1/4.3), and
q/K/V values are i.i.d. N(0,1) rounded to the storage type.

A workload is a short timeline on one layer's cache:

  1. the cache initially holds the tokens flagged in ``init_filled``
     (everything else is poison: NaN for float types),
  2. ``copy_pairs``  - copy-on-write block copies queued by the block manager
     (Sec. 4.4), executed first,
  3. ``write_slots`` - slots that receive new K/V vectors (Sec. 4.3: new KV is
     saved into the physical blocks before attention reads it),
  4. decode: one query token per sequence attends to ``context_lens[s]``
     tokens reached through ``block_tables[s]`` (Sec. 4.1, Eq. 4).

This module holds none of the method's arithmetic; it is the only code the
oracle tests and the HIP tests have in common.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

from .blocks import BlockManager, Sequence

ELEM_BYTES = {"f32": 4, "f16": 2, "bf16": 2}


# --------------------------------------------------------------------------
# storage-type helpers (input quantisation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = np.isnan(x)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 samples -> array in the cache's storage representation."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def storage_np_dtype(dtype: str):
    return {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]


def poison_value(dtype: str):
    """Bit pattern written to every slot that holds no token (a quiet NaN)."""
    return {"f32": np.float32(np.nan), "f16": np.float16(np.nan), "bf16": np.uint16(0x7FC0)}[dtype]


# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    dtype: str
    num_heads: int
    head_dim: int
    block_size: int
    num_blocks: int
    scale: np.float32
    block_tables: np.ndarray            # int32 [S][MB]
    context_lens: np.ndarray            # int32 [S]
    init_filled: np.ndarray             # bool  [NB][B]
    copy_pairs: np.ndarray              # int64 [N][2]
    write_slots: np.ndarray             # int64 [T]
    step_slots: np.ndarray              # int64 [S] slot of each sequence's newest token
    seed: int = 0
    meta: Dict = field(default_factory=dict)

    @property
    def num_seqs(self) -> int:
        return int(self.context_lens.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def elem_bytes(self) -> int:
        return ELEM_BYTES[self.dtype]

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if self.num_seqs else 0

    def cache_shape(self) -> Tuple[int, int, int, int]:
        return (self.num_blocks, self.num_heads, self.block_size, self.head_dim)

    def final_filled(self) -> np.ndarray:
        """bool [NB][B]: slots that hold a token when decode runs."""
        f = np.zeros((self.num_blocks, self.block_size), dtype=bool)
        B = self.block_size
        for s in range(self.num_seqs):
            n = int(self.context_lens[s])
            nb = (n + B - 1) // B
            for j in range(nb):
                cnt = min(B, n - j * B)
                f[self.block_tables[s, j], :cnt] = True
        return f

    def kv_bytes_logical(self) -> int:
        """K+V bytes one decode call must read, counting shared blocks once per reader."""
        return int(self.context_lens.astype(np.int64).sum()) * self.num_heads * self.head_dim * self.elem_bytes * 2

    def kv_bytes_unique(self) -> int:
        """K+V bytes of distinct filled slots referenced by the block tables."""
        return int(self.final_filled().sum()) * self.num_heads * self.head_dim * self.elem_bytes * 2


# --------------------------------------------------------------------------
def _tables_from(seqs: List[Sequence], pad_blocks: int, rng: np.random.Generator,
                 num_blocks: int) -> np.ndarray:
    """int32 [S][MB]; entries past a sequence's last block are garbage on
    purpose (negative or far out of range) since they must never be read."""
    mb = max([len(s.blocks) for s in seqs] + [1]) + pad_blocks
    t = np.empty((len(seqs), mb), dtype=np.int32)
    junk = np.array([-1, -7, 2**31 - 1, num_blocks, num_blocks + 12345], dtype=np.int64)
    t[:] = rng.choice(junk, size=t.shape).astype(np.int32)
    for i, s in enumerate(seqs):
        t[i, : len(s.blocks)] = s.blocks
    return t


def _finish(name, dtype, H, D, B, mgr: BlockManager, seqs, init_filled, copy_pairs, write_slots,
            rng, seed, meta, pad_blocks=2) -> Workload:
    NB = mgr.alloc.num_blocks
    step_slots = np.array([mgr.slot_of(s, s.length - 1) if s.length > 0 else -1 for s in seqs], dtype=np.int64)
    w = Workload(
        name=name, dtype=dtype, num_heads=H, head_dim=D, block_size=B, num_blocks=NB,
        scale=np.float32(1.0 / math.sqrt(D)),
        block_tables=_tables_from(seqs, pad_blocks, rng, NB),
        context_lens=np.array([s.length for s in seqs], dtype=np.int32),
        init_filled=init_filled,
        copy_pairs=np.array(copy_pairs, dtype=np.int64).reshape(-1, 2),
        write_slots=np.array(write_slots, dtype=np.int64),
        step_slots=step_slots, seed=seed, meta=meta)
    return w


def _mark(filled: np.ndarray, mgr: BlockManager, seq: Sequence, upto: int) -> None:
    B = mgr.block_size
    for j in range((upto + B - 1) // B):
        filled[seq.blocks[j], : min(B, upto - j * B)] = True


def independent_sequences(name: str, dtype: str, H: int, D: int, B: int, lens: np.ndarray,
                          seed: int, pool_factor: float = 1.2, num_blocks: Optional[int] = None) -> Workload:
    """Sequences with private blocks; the step writes each one's newest token.

    Pool = ceil(pool_factor * blocks needed) unless ``num_blocks`` is given;
    ids are handed out in the order of a seeded permutation of the pool.
    """
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int64)
    need = int(((lens + B - 1) // B).sum())
    NB = int(num_blocks) if num_blocks is not None else max(1, math.ceil(pool_factor * need))
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    seqs, filled, slots = [], np.zeros((NB, B), dtype=bool), []
    # interleave allocation across sequences block by block, as a server
    # growing many requests at once would, so one sequence's blocks are not a
    # contiguous run of the permutation
    for n in lens:
        seqs.append(Sequence())
    # every sequence first gets context_len-1 tokens (state before the step)
    target = np.maximum(lens - 1, 0)
    grown = np.zeros_like(lens)
    while (grown < target).any():
        for i in np.nonzero(grown < target)[0]:
            take = int(min(B - (grown[i] % B), target[i] - grown[i]))
            for _ in range(take):
                mgr.append(seqs[i])
            grown[i] += take
    for i, s in enumerate(seqs):
        _mark(filled, mgr, s, s.length)
    for i, s in enumerate(seqs):
        if lens[i] > 0:
            slots.append(mgr.append(s))
    assert not mgr.pending_copies
    return _finish(name, dtype, H, D, B, mgr, seqs, filled, [], slots, rng, seed,
                   {"kind": "independent", "pool_factor": pool_factor, "blocks_needed": need})


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
def config1(seed: int = 1000) -> Workload:
    """Tiny paged decode: H=4, D=64, B=16, fp32, 8 sequences, ctx ~ U{1..128}, pool of 128 blocks."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, 129, size=8)
    return independent_sequences("cfg1_tiny", "f32", 4, 64, 16, lens, seed + 1, num_blocks=128)


def config2(seed: int = 2000, num_seqs: int = 64, max_len: int = 2048, H: int = 40) -> Workload:
    """OPT-13B-shaped layer (Table 1: 40 heads x 128): fp16, B=16, 64 sequences, ctx ~ U{1..2048}, pool 1.2x."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, size=num_seqs)
    return independent_sequences("cfg2_opt13b", "f16", H, 128, 16, lens, seed + 1)


def config4(seed: int = 4000, num_seqs: int = 128, H: int = 18, median: float = 900.0,
            sigma: float = 0.5, cap: int = 2048) -> Workload:
    """One GPU's share of a 4-way tensor-parallel OPT-66B layer (72 heads / 4, Sec. 4.6): bf16, B=16,
    ctx ~ clip(round(LogNormal(ln 900, 0.5)), 1, 2048)."""
    rng = np.random.default_rng(seed)
    lens = np.clip(np.rint(rng.lognormal(math.log(median), sigma, size=num_seqs)), 1, cap).astype(np.int64)
    return independent_sequences("cfg4_opt66b_tp4", "bf16", H, 128, 16, lens, seed + 1)


def config3(seed: int = 3000, num_groups: int = 64, group: int = 4, H: int = 40,
            prompt_median: float = 160.0, prompt_sigma: float = 1.0, prompt_cap: int = 1024,
            max_out: int = 512, dtype: str = "f16", D: int = 128, B: int = 16) -> Workload:
    """Parallel sampling (Sec. 4.4): each prompt's blocks are shared by `group` samples through
    reference counts; the first generated token copies the last, partial prompt block for all
    but the last writer; every sample then appends 1..max_out private tokens."""
    rng = np.random.default_rng(seed)
    prompts = np.clip(np.rint(rng.lognormal(math.log(prompt_median), prompt_sigma, size=num_groups)),
                      1, prompt_cap).astype(np.int64)
    outs = rng.integers(1, max_out + 1, size=(num_groups, group))
    need_shared = int(((prompts + B - 1) // B).sum())
    need_private = int(((outs + B - 1) // B + 1).sum())
    NB = math.ceil(1.2 * (need_shared + need_private))
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    filled = np.zeros((NB, B), dtype=bool)
    seqs: List[Sequence] = []
    groups = []
    for g in range(num_groups):
        parent = mgr.allocate(int(prompts[g]))
        _mark(filled, mgr, parent, parent.length)
        kids = [parent] + [mgr.fork(parent) for _ in range(group - 1)]
        groups.append(list(range(len(seqs), len(seqs) + group)))
        seqs.extend(kids)
    # generation: round-robin over all samples, one token per iteration, so
    # private blocks of different samples interleave in the pool
    slots: List[int] = []
    left = outs.reshape(-1).copy()
    while (left > 0).any():
        for i in np.nonzero(left > 0)[0]:
            slots.append(mgr.append(seqs[i]))
            left[i] -= 1
    pairs = mgr.take_copies()
    w = _finish("cfg3_parallel_sampling", dtype, H, D, B, mgr, seqs, filled, pairs, slots, rng, seed,
                {"kind": "parallel_sampling", "groups": groups, "prompts": prompts.tolist(),
                 "group": group})
    return w


def config5(seed: int = 5000, num_seqs: int = 128, width: int = 6, H: int = 40, D: int = 128,
            B: int = 32, min_len: int = 512, max_len: int = 4096, shared_frac: float = 0.55,
            pool_factor: float = 1.05, dtype: str = "bf16") -> Workload:
    """Beam search with copy-on-write (Sec. 4.4) at LLaMA-13B shape.  Beams of a group have equal
    length L_g ~ U{min_len..max_len}; the first floor(shared_frac * blocks) blocks are shared by the
    whole group, the rest are private.  One search step is then played: every group draws `width`
    parents with replacement from its beams, children fork them, the old beams are freed and every
    child appends one token, which copies the last block wherever it is partial and still shared."""
    rng = np.random.default_rng(seed)
    sizes = [width] * (num_seqs // width)
    if num_seqs % width:
        sizes.append(num_seqs % width)
    L = rng.integers(min_len, max_len + 1, size=len(sizes))
    # state before the step holds L-1 tokens per beam
    need = 0
    for sz, n in zip(sizes, L):
        nb = (int(n) - 1 + B - 1) // B
        sh = int(shared_frac * nb)
        need += sh + sz * (nb - sh) + sz  # + room for the step's new/copied blocks
    NB = math.ceil(pool_factor * need)
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    filled = np.zeros((NB, B), dtype=bool)
    old_groups: List[List[Sequence]] = []
    for sz, n in zip(sizes, L):
        n0 = int(n) - 1
        nb = (n0 + B - 1) // B
        sh = int(shared_frac * nb)
        root = mgr.allocate(sh * B) if sh > 0 else Sequence()
        beams = []
        for b in range(sz):
            s = mgr.fork(root) if sh > 0 else Sequence()
            while s.length < n0:
                mgr.append(s)
            beams.append(s)
        if sh > 0:
            mgr.free(root)
        assert not mgr.pending_copies
        for s in beams:
            _mark(filled, mgr, s, s.length)
        old_groups.append(beams)
    seqs: List[Sequence] = []
    slots: List[int] = []
    groups = []
    for beams in old_groups:
        sz = len(beams)
        parents = rng.integers(0, sz, size=sz)
        kids = [mgr.fork(beams[p]) for p in parents]
        for s in beams:
            mgr.free(s)
        groups.append(list(range(len(seqs), len(seqs) + sz)))
        for s in kids:
            slots.append(mgr.append(s))
        seqs.extend(kids)
    pairs = mgr.take_copies()
    return _finish("cfg5_beam_search", dtype, H, D, B, mgr, seqs, filled, pairs, slots, rng, seed,
                   {"kind": "beam_search", "groups": groups, "width": width,
                    "shared_frac": shared_frac})


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------
@dataclass
class Values:
    q: np.ndarray          # [S][H][D] storage type
    k_cache: np.ndarray    # [NB][H][B][D] initial contents (poison where init_filled is False)
    v_cache: np.ndarray
    k_new: np.ndarray      # [T][H][D] vectors written to write_slots
    v_new: np.ndarray


def _randn(rng: np.random.Generator, shape, dtype: str, mult: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if mult != 1.0:
        x *= np.float32(mult)
    return to_storage(x, dtype)


def make_values(w: Workload, seed: Optional[int] = None, poison: bool = True,
                q_mult: float = 1.0) -> Values:
    """Seeded N(0,1) values in the storage type.  Slots that hold no token get NaN when
    `poison` is set (the result must not depend on them)."""
    rng = np.random.default_rng((w.seed if seed is None else seed) + 77)
    S, H, D, B, NB = w.num_seqs, w.num_heads, w.head_dim, w.block_size, w.num_blocks
    T = int(w.write_slots.shape[0])
    q = _randn(rng, (S, H, D), w.dtype, q_mult)
    k_cache = _randn(rng, (NB, H, B, D), w.dtype)
    v_cache = _randn(rng, (NB, H, B, D), w.dtype)
    k_new = _randn(rng, (T, H, D), w.dtype)
    v_new = _randn(rng, (T, H, D), w.dtype)
    if poison:
        hole = ~w.init_filled                      # [NB][B]
        pv = poison_value(w.dtype)
        for c in (k_cache, v_cache):
            c.transpose(0, 2, 1, 3)[hole] = pv
    return Values(q, k_cache, v_cache, k_new, v_new)
