"""CPU pins of the host reference of the sharing plan (tests/plan_reference.py): hand-written cases."""
import numpy as np

import plan_reference as ref


def tables(rows, width):
    bt = np.full((len(rows), width), -7, dtype=np.int32)
    for i, r in enumerate(rows):
        bt[i, : len(r)] = r
    return bt


def test_parallel_sampling_example_of_the_paper():
    # Sec. 4.4's figure scaled up: two samples share the prompt's blocks 7 and 1 (full) and hold
    # private copies of the third; B = 16
    bt = tables([[7, 1, 3], [7, 1, 5], [9, 2]], 4)
    lens = np.array([40, 41, 20], dtype=np.int32)
    p = ref.plan(bt, lens, 16)
    assert p["adj"] == [0, 2, 0]
    assert p["groups"] == [(0, 2)] and p["singles"] == [2]
    assert p["tiles"][0] == [(7, 0b11, 0, 0, 16), (1, 0b11, 0, 1, 16), (3, 0b01, 1, 2, 8), (5, 0b10, 1, 2, 9)]


def test_short_common_run_is_not_worth_a_group():
    # one shared block of 16 tokens: below the 32-token floor; two shared blocks against contexts of 600: below 1/8
    bt = tables([[1, 2, 3], [1, 5, 6]], 40)
    assert ref.plan(bt, np.array([40, 40], dtype=np.int32), 16)["groups"] == []
    long0, long1 = [1, 2] + list(range(10, 46)), [1, 2] + list(range(50, 86))
    assert ref.plan(tables([long0, long1], 40), np.array([600, 600], dtype=np.int32), 16)["groups"] == []
    assert ref.plan(tables([long0, long1], 40), np.array([256, 600], dtype=np.int32), 16)["groups"] == [(0, 2)]


def test_only_full_blocks_of_the_shorter_context_count():
    bt = tables([[4, 5, 6], [4, 5, 6]], 3)
    assert ref.plan(bt, np.array([48, 47], dtype=np.int32), 16)["adj"] == [0, 2]
    assert ref.plan(bt, np.array([48, 48], dtype=np.int32), 16)["adj"] == [0, 3]


def test_chain_longer_than_sixteen_is_cut_in_order():
    rows = [[1, 2, 3, 100 + i] for i in range(35)]
    p = ref.plan(tables(rows, 4), np.full(35, 60, dtype=np.int32), 16)
    assert p["groups"] == [(0, 16), (16, 16), (32, 3)]
    assert p["tiles"][32] == [(1, 0b111, 0, 0, 16), (2, 0b111, 0, 1, 16), (3, 0b111, 0, 2, 16),
                              (132, 0b001, 1, 3, 12), (133, 0b010, 1, 3, 12), (134, 0b100, 1, 3, 12)]


def test_subsets_sharing_beyond_the_common_prefix():
    # a beam tree: all three share blocks 1 and 2; the last two also share block 8
    bt = tables([[1, 2, 7, 20], [1, 2, 8, 21], [1, 2, 8, 22]], 4)
    p = ref.plan(bt, np.array([64, 64, 56], dtype=np.int32), 16)
    assert p["adj"] == [0, 2, 3]
    assert p["groups"] == [(0, 3)]
    assert p["tiles"][0] == [(1, 0b111, 0, 0, 16), (2, 0b111, 0, 1, 16), (7, 0b001, 0, 2, 16), (8, 0b110, 0, 2, 16),
                             (20, 0b001, 0, 3, 16), (21, 0b010, 0, 3, 16), (22, 0b100, 1, 3, 8)]


def test_work_items_are_groups_then_singles_then_nothing():
    rows = [[1, 2, 10], [1, 2, 11], [9], [3, 4, 5, 6, 12], [3, 4, 5, 6, 13], [7, 8, 14]]
    p = ref.plan(tables(rows, 5), np.array([40, 40, 9, 70, 70, 40], dtype=np.int32), 16)
    assert p["groups"] == [(0, 2), (3, 2)] and p["singles"] == [2, 5]
    assert ref.items_of(p, 6) == [(2, 0, 2, 4), (2, 3, 2, 6), (1, 2, 1, 0), (1, 5, 1, 0), (0, 0, 0, 0), (0, 0, 0, 0)]


def test_decode_device_plan_layout():
    S, MB = 3, 2
    nwords = ref.plan_words(S)
    assert nwords == 24 + 12                      # 6S + 4 = 22 -> items start at word 24
    words = np.zeros(nwords, dtype=np.int32)
    words[0:3] = [1, 1, 0]; words[3:6] = [2, 0, 1]; words[6:9] = [1, 0, 0]; words[9:12] = [0, 2, 0]
    words[12] = 2; words[15] = 0; words[18] = 1; words[19] = 1
    words[24:28] = [2, 0, 2, 1]; words[28:32] = [1, 2, 1, 0]
    off = (nwords * 4 + 15) // 16 * 16
    raw = np.zeros(off + S * MB * 16, dtype=np.uint8)
    raw[: words.nbytes] = words.view(np.uint8)
    ent = np.array([5, 0b11 | (1 << 16), 0, 9], dtype=np.int32)
    raw[off: off + 16] = ent.view(np.uint8)
    got = ref.decode_device_plan(raw, S, MB)
    assert got["group_firsts"] == [0] and got["singles"] == [2] and got["tiles"][0] == [(5, 0b11, 1, 0, 9)]
    assert got["items"] == [(2, 0, 2, 1), (1, 2, 1, 0), (0, 0, 0, 0)]
