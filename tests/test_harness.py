"""Host block manager and workload generators against the paper's worked examples.

Fixtures under tests/golden/ carry the citation of the passage they restate.
"""
import os

import numpy as np
import pytest

from harness import workloads as W
from harness.blocks import BlockManager, Sequence

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _order(first, total=16):
    first = [int(x) for x in first]
    return first + [i for i in range(total) if i not in first]


def test_block_table_walkthrough():
    rows = _read("block_table_example.txt")
    kv = {r[0]: r[1:] for r in rows if not r[0].isdigit()}
    B, prompt = int(kv["block_size"][0]), int(kv["prompt_len"][0])
    mgr = BlockManager(16, B, order=_order(kv["alloc_order"]))
    seq = mgr.allocate(prompt)
    assert seq.blocks == [7, 1]
    expect = [[int(x) for x in r] for r in rows if r[0].isdigit()]
    for pos, lb, pb, off, slot in expect:
        if pos >= prompt:
            got = mgr.append(seq)
            assert got == slot
        assert pos // B == lb and pos % B == off
        assert seq.blocks[lb] == pb
        assert mgr.slot_of(seq, pos) == slot == pb * B + off
    assert seq.blocks == [7, 1, 3] and seq.length == 9
    assert mgr.take_copies() == []


def test_parallel_sampling_copy_on_write():
    kv = {r[0]: r[1:] for r in _read("parallel_sampling_cow_example.txt")}
    B = int(kv["block_size"][0])
    mgr = BlockManager(16, B, order=_order(kv["alloc_order"]))
    a1 = mgr.allocate(int(kv["prompt_len"][0]))
    a2 = mgr.fork(a1)
    for item in kv["refcount_after_fork"]:
        pb, c = item.split(":")
        assert mgr.alloc.ref[int(pb)] == int(c)
    s1 = mgr.append(a1)
    s2 = mgr.append(a2)
    pairs = mgr.take_copies()
    assert pairs == [tuple(int(x) for x in p.split(">")) for p in kv["copy_pairs"]]
    assert a1.blocks == [int(x) for x in kv["a1_table"]]
    assert a2.blocks == [int(x) for x in kv["a2_table"]]
    assert (s1, s2) == (int(kv["a1_slot"][0]), int(kv["a2_slot"][0]))
    for item in kv["refcount_after_step"]:
        pb, c = item.split(":")
        assert mgr.alloc.ref[int(pb)] == int(c)


def test_beam_search_example():
    rows = _read("beam_search_example.txt")
    before = {int(r[1][:-1]): [int(x) for x in r[2:]] for r in rows if r[0] == "before"}
    after = {int(r[1][:-1]): [int(x) for x in r[2:]] for r in rows if r[0] == "after"}
    kv = {r[0]: [int(x) for x in r[1:]] for r in rows if r[0] not in ("before", "after")}
    B = kv["block_size"][0]
    # allocation order that reproduces the figure's physical ids
    mgr = BlockManager(13, B, order=[0, 1, 3, 4, 5, 8, 2, 6, 7, 9, 10, 11, 12])
    root = mgr.allocate(B)                       # block 0, shared by all
    c012 = mgr.fork(root)
    for _ in range(2 * B):
        mgr.append(c012)                         # blocks 1, 3
    c3 = mgr.fork(root)
    for _ in range(3 * B):
        mgr.append(c3)                           # blocks 4, 5, 8
    cands = []
    for _ in range(3):
        c = mgr.fork(c012)
        for _ in range(B):
            mgr.append(c)                        # blocks 2, 6, 7
        cands.append(c)
    cands.append(c3)
    mgr.free(root)
    mgr.free(c012)
    assert mgr.take_copies() == []
    for i, c in enumerate(cands):
        assert c.blocks == before[i] and c.length == 4 * B
    kids = [mgr.fork(cands[p]) for p in kv["parents"]]
    for c in cands:
        mgr.free(c)
    assert sorted(pb for pb in range(13) if mgr.alloc.ref[pb] == 0 and pb < 9) == kv["freed"]
    for k in kids:
        mgr.append(k)
    assert mgr.take_copies() == []               # full last blocks: nothing to copy
    assert sorted(k.blocks[-1] for k in kids) == kv["new_blocks"]
    for i, k in enumerate(kids):
        assert k.blocks == after[i]
    for pb in kv["shared_by_all"]:
        assert mgr.alloc.ref[pb] == 4
    assert mgr.alloc.ref[6] == 2 and mgr.alloc.ref[7] == 2


def test_kv_bytes_per_token_opt13b():
    kv = {r[0]: int(r[1]) for r in _read("kv_bytes_opt13b.txt")}
    assert kv["heads"] * kv["head_dim"] == kv["hidden"]
    lens = np.array([1], dtype=np.int64)
    w = W.independent_sequences("one_token", "f16", kv["heads"], kv["head_dim"], 16, lens, 1)
    assert w.kv_bytes_logical() * kv["layers"] == kv["bytes_per_token"]
    assert w.kv_bytes_unique() == w.kv_bytes_logical()


def test_refcounts_and_free():
    mgr = BlockManager(8, 4)
    a = mgr.allocate(6)
    b = mgr.fork(a)
    assert mgr.alloc.num_free == 6
    mgr.free(a)
    assert mgr.alloc.num_free == 6 and all(mgr.alloc.ref[pb] == 1 for pb in b.blocks)
    mgr.append(b)                                # sole owner: in place
    assert mgr.take_copies() == []
    mgr.free(b)
    assert mgr.alloc.num_free == 8 and sum(mgr.alloc.ref) == 0


@pytest.mark.parametrize("make", [W.config1, W.config2, W.config3, W.config4,
                                  lambda: W.config5(num_seqs=14, min_len=40, max_len=300)])
def test_workload_invariants(make):
    w = make()
    B, NB = w.block_size, w.num_blocks
    S = w.num_seqs
    assert w.block_tables.dtype == np.int32 and w.context_lens.dtype == np.int32
    assert w.write_slots.dtype == np.int64 and w.copy_pairs.dtype == np.int64
    # every block a sequence can reach is a valid id
    for s in range(S):
        nb = (int(w.context_lens[s]) + B - 1) // B
        ids = w.block_tables[s, :nb]
        assert ids.min(initial=0) >= 0 and ids.max(initial=0) < NB
    # slots written in one call are distinct, and copies never alias
    assert len(set(w.write_slots.tolist())) == len(w.write_slots)
    if len(w.copy_pairs):
        src, dst = w.copy_pairs[:, 0], w.copy_pairs[:, 1]
        assert len(set(dst.tolist())) == len(dst) and not set(dst.tolist()) & set(src.tolist())
    # after copies and writes, exactly the slots decode will read are filled
    filled = w.init_filled.copy()
    for src, dst in w.copy_pairs:
        filled[dst] = filled[src]
    filled.reshape(-1)[w.write_slots] = True
    need = w.final_filled()
    assert (filled | ~need).all(), "decode would read a slot nobody wrote"
    # the newest token of each sequence is among the written slots
    assert set(w.step_slots.tolist()) <= set(w.write_slots.tolist())
    assert w.kv_bytes_unique() <= w.kv_bytes_logical()


def test_config_shapes_match_spec():
    w1, w2, w4 = W.config1(), W.config2(), W.config4()
    assert (w1.num_seqs, w1.num_heads, w1.head_dim, w1.block_size, w1.dtype, w1.num_blocks) == (8, 4, 64, 16, "f32", 128)
    assert 1 <= w1.context_lens.min() and w1.context_lens.max() <= 128
    assert (w2.num_seqs, w2.num_heads, w2.head_dim, w2.block_size, w2.dtype) == (64, 40, 128, 16, "f16")
    assert w2.context_lens.max() <= 2048 and abs(w2.num_blocks / w2.meta["blocks_needed"] - 1.2) < 0.01
    assert (w4.num_seqs, w4.num_heads, w4.head_dim, w4.dtype) == (128, 18, 128, "bf16")
    assert w4.context_lens.max() <= 2048
    w3 = W.config3()
    assert w3.num_seqs == 256 and len(w3.meta["groups"]) == 64
    # one copy per sample except the last writer, only where the prompt ends mid-block
    partial = sum(1 for p in w3.meta["prompts"] if p % 16)
    assert len(w3.copy_pairs) == 3 * partial
    assert w3.kv_bytes_unique() < w3.kv_bytes_logical()


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40, 0.0], dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(b)
    # ties to even on the 8-bit significand: 1+2^-8 -> 1, 1+3*2^-8 -> 1+2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert back[3] == -2.5
    assert np.all(np.abs(back[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -8)


@pytest.mark.parametrize("seed", range(6))
def test_block_manager_random_walk_keeps_its_books(seed):
    """A seeded random mix of allocate / fork / append / free (Sec. 5.2: every decoding algorithm
    reduces to these) against a shadow model that stores every sequence's tokens explicitly.
    After every operation: reference counts equal the number of tables that map each block, free
    plus mapped blocks are the whole pool, and replaying the queued copies and the writes on a
    shadow pool gives every sequence exactly its own tokens back (copy-on-write never lets one
    sequence see another's writes)."""
    from collections import Counter
    from harness.blocks import BlockManager
    rng = np.random.default_rng(100 + seed)
    B = int(rng.choice([2, 4, 16]))
    NB = 96
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    pool = np.full((NB, B), -1, dtype=np.int64)          # shadow K/V: one integer per slot
    live, truth = [], []                                  # sequences and the token ids each should hold
    next_token = [0]

    def write(seq, toks, slot):
        pool.reshape(-1)[slot] = next_token[0]
        toks.append(next_token[0])
        next_token[0] += 1

    def flush_copies():
        for src, dst in mgr.take_copies():
            pool[dst] = pool[src]

    for step in range(400):
        op = rng.choice(["allocate", "fork", "append", "append", "append", "free"])
        try:
            if op == "allocate" or not live:
                n = int(rng.integers(1, 3 * B))
                if mgr.alloc.num_free * B < n:
                    continue
                s = mgr.allocate(n)
                toks = []
                for t in range(n):
                    write(s, toks, mgr.slot_of(s, t))
                live.append(s); truth.append(toks)
            elif op == "fork":
                i = int(rng.integers(0, len(live)))
                live.append(mgr.fork(live[i])); truth.append(list(truth[i]))
            elif op == "append":
                i = int(rng.integers(0, len(live)))
                if mgr.alloc.num_free == 0:
                    continue
                slot = mgr.append(live[i])
                flush_copies()                            # the copy is executed before the write (Sec. 4.4)
                write(live[i], truth[i], slot)
            else:
                i = int(rng.integers(0, len(live)))
                mgr.free(live.pop(i)); truth.pop(i)
        finally:
            flush_copies()
        mapped = Counter(pb for s in live for pb in s.blocks)
        assert all(mgr.alloc.ref[pb] == mapped.get(pb, 0) for pb in range(NB))
        assert mgr.alloc.num_free + len(mapped) == NB
        for s, toks in zip(live, truth):
            assert s.length == len(toks) and len(s.blocks) == (s.length + B - 1) // B
            got = [int(pool.reshape(-1)[mgr.slot_of(s, t)]) for t in range(s.length)]
            assert got == toks
