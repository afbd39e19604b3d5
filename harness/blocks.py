"""Host-side KV block manager (paper Sec. 4.2-4.4, 5.2).

A sequence owns a list of logical blocks, each mapped to a physical block id;
blocks are filled left to right, so at most the last one is partial
(Sec. 4.3).  Physical blocks carry a reference count so that several sequences
may map the same physical block (Sec. 4.4, parallel sampling); a write into a
block whose count is above one triggers copy-on-write: a fresh block is
allocated, a (src, dst) copy is queued for the block engine and the old
block's count drops by one, so the last writer writes in place.

The three sequence operations are the ones every decoding algorithm in the
paper reduces to (Sec. 5.2): fork, append, free.

This is test and benchmark scaffolding: it produces the index arrays the
kernels consume.  It is not part of the C-ABI library.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from typing import Iterable, List, Optional, Sequence as Seq, Tuple


class OutOfBlocks(RuntimeError):
    pass


class BlockAllocator:
    """Free list + reference counts over `num_blocks` physical block ids.

    `order` fixes the order in which free ids are handed out (the workload
    generators pass a seeded permutation so physical placement is scattered,
    as it is in a long-running server).
    """

    def __init__(self, num_blocks: int, order: Optional[Iterable[int]] = None):
        self.num_blocks = int(num_blocks)
        ids = list(range(self.num_blocks)) if order is None else [int(i) for i in order]
        if sorted(ids) != list(range(self.num_blocks)):
            raise ValueError("order must be a permutation of range(num_blocks)")
        # FIFO: `order[0]` is handed out first and freed ids queue at the back,
        # which is the behaviour the paper's beam-search example shows (blocks
        # freed in an iteration are not the ones allocated next)
        self._free = deque(ids)
        self.ref: List[int] = [0] * self.num_blocks

    @property
    def num_free(self) -> int:
        return len(self._free)

    def alloc(self) -> int:
        if not self._free:
            raise OutOfBlocks("no free physical block")
        pb = self._free.popleft()
        assert self.ref[pb] == 0
        self.ref[pb] = 1
        return pb

    def incref(self, pb: int) -> None:
        assert self.ref[pb] > 0
        self.ref[pb] += 1

    def decref(self, pb: int) -> None:
        assert self.ref[pb] > 0
        self.ref[pb] -= 1
        if self.ref[pb] == 0:
            self._free.append(pb)


@dataclass
class Sequence:
    blocks: List[int] = field(default_factory=list)   # logical -> physical
    length: int = 0                                   # tokens stored


class BlockManager:
    """Block tables for a set of sequences over one allocator."""

    def __init__(self, num_blocks: int, block_size: int, order: Optional[Iterable[int]] = None):
        self.block_size = int(block_size)
        self.alloc = BlockAllocator(num_blocks, order)
        self.pending_copies: List[Tuple[int, int]] = []

    # -- sequence operations -------------------------------------------------
    def allocate(self, num_tokens: int) -> Sequence:
        """New sequence holding `num_tokens` tokens (the prompt phase)."""
        B = self.block_size
        seq = Sequence()
        for _ in range((num_tokens + B - 1) // B):
            seq.blocks.append(self.alloc.alloc())
        seq.length = int(num_tokens)
        return seq

    def fork(self, parent: Sequence) -> Sequence:
        """Child maps every logical block of `parent` to the same physical block."""
        for pb in parent.blocks:
            self.alloc.incref(pb)
        return Sequence(list(parent.blocks), parent.length)

    def append(self, seq: Sequence) -> int:
        """Reserve the slot for one more token and return it (slot = pb*B + off).

        Opens a new physical block when the last one is full; copies the last
        block first when it is shared (the copy lands in `pending_copies`).
        """
        B = self.block_size
        off = seq.length % B
        if off == 0:
            seq.blocks.append(self.alloc.alloc())
        else:
            last = seq.blocks[-1]
            if self.alloc.ref[last] > 1:
                fresh = self.alloc.alloc()
                self.pending_copies.append((last, fresh))
                self.alloc.decref(last)
                seq.blocks[-1] = fresh
        seq.length += 1
        return seq.blocks[-1] * B + off

    def free(self, seq: Sequence) -> None:
        for pb in seq.blocks:
            self.alloc.decref(pb)
        seq.blocks = []
        seq.length = 0

    # -- block engine hand-off -------------------------------------------------
    def take_copies(self) -> List[Tuple[int, int]]:
        out, self.pending_copies = self.pending_copies, []
        return out

    # -- helpers -----------------------------------------------------------
    def slot_of(self, seq: Sequence, pos: int) -> int:
        B = self.block_size
        return seq.blocks[pos // B] * B + pos % B


def unique_blocks(seqs: Seq[Sequence]) -> int:
    s = set()
    for q in seqs:
        s.update(q.blocks)
    return len(s)
