"""Pure-index host reference of pa_decode_shared's sharing plan (no attention arithmetic).

Restates, from the layout documented in include/pa.h, what the plan must contain for given
block tables and context lengths: which consecutive sequences form groups, and for every
group the list of (physical block, member set, logical position, tokens) entries.  The GPU
tests compare the plan the device built with this, entry by entry.

Rules (Sec. 4.4 workloads: forked sequences map their common logical blocks to the same
physical blocks):
  * adj[s] = number of leading FULL blocks (of the shorter of the two contexts) at which
    sequences s-1 and s map the same physical block;
  * s is tied to s-1 if adj[s]*B >= 32 tokens and adj[s]*B*8 >= min(n[s-1], n[s]);
  * a maximal chain of tied sequences is cut into groups of at most 16, in order; groups of
    one are "singles";
  * a group's tile list holds, position by position, each distinct physical block that some
    member maps at that position, with the set of members mapping it there;
  * work item i is group i (ascending), then the singles ascending, then nothing.
"""
from __future__ import annotations

import numpy as np

GROUP_MAX = 16
SHARE_MIN_TOKENS = 32
SHARE_MIN_FRACTION = 8


def leading_common_blocks(row0, row1, n0, n1, B):
    lim = min(int(n0), int(n1)) // B
    a = 0
    while a < lim and row0[a] == row1[a]:
        a += 1
    return a


def plan(block_tables: np.ndarray, context_lens: np.ndarray, B: int, tie_rule=None):
    """Returns dict(adj, in_group, group_size, groups=[(first, size)], singles=[s...], tiles={first: [(blk, mask, ragged, pos, tokens)...]})."""
    S = len(context_lens)
    n = [int(x) for x in context_lens]
    if tie_rule is None:
        def tie_rule(common, n0, n1):
            t = common * B
            return t >= SHARE_MIN_TOKENS and t * SHARE_MIN_FRACTION >= min(n0, n1)
    adj = [0] * S
    tie = [False] * S
    for s in range(1, S):
        adj[s] = leading_common_blocks(block_tables[s - 1], block_tables[s], n[s - 1], n[s], B)
        tie[s] = bool(tie_rule(adj[s], n[s - 1], n[s]))
    groups, singles = [], []
    in_group = [0] * S
    group_size = [0] * S
    s = 0
    while s < S:
        e = s + 1
        while e < S and tie[e]:
            e += 1
        for first in range(s, e, GROUP_MAX):          # the chain s .. e-1 in pieces of at most 16
            size = min(GROUP_MAX, e - first)
            group_size[first] = size
            if size >= 2:
                groups.append((first, size))
                for j in range(size):
                    in_group[first + j] = 1
            else:
                singles.append(first)
        s = e
    tiles = {}
    for first, size in groups:
        nb = [(n[first + j] + B - 1) // B for j in range(size)]
        entries = []
        for pos in range(max(nb)):
            seen = {}
            for j in range(size):
                if pos < nb[j]:
                    seen.setdefault(int(block_tables[first + j][pos]), []).append(j)
            # in the order of each set's first member
            for blk, members in sorted(seen.items(), key=lambda kv: kv[1][0]):
                nmax = max(n[first + j] for j in members)
                nmin = min(n[first + j] for j in members)
                tokens = min(B, nmax - pos * B)
                ragged = 1 if nmin < (pos + 1) * B else 0
                mask = sum(1 << j for j in members)
                entries.append((blk, mask, ragged, pos, tokens))
        tiles[first] = entries
    return dict(adj=adj, in_group=in_group, group_size=group_size, groups=groups, singles=singles, tiles=tiles)


def items_of(p, S):
    """The S work items (kind, first, members, entries) that a plan implies."""
    items = [(2, first, size, len(p["tiles"][first])) for first, size in p["groups"]]
    items += [(1, s, 1, 0) for s in p["singles"]]
    items += [(0, 0, 0, 0)] * (S - len(items))
    return items


def plan_words(S: int) -> int:
    return (6 * S + 4 + 3) // 4 * 4 + 4 * S


def decode_device_plan(raw: np.ndarray, S: int, max_blocks: int):
    """Splits the bytes of a device plan (the workspace pa_shared_plan filled) by the documented layout."""
    words = raw.view(np.int32)
    g = words[: plan_words(S)]
    ginfo_bytes = (plan_words(S) * 4 + 15) // 16 * 16
    tiles = raw[ginfo_bytes: ginfo_bytes + S * max_blocks * 16].view(np.int32).reshape(S * max_blocks, 4)
    group_count, single_count = int(g[6 * S]), int(g[6 * S + 1])
    item0 = (6 * S + 4 + 3) // 4 * 4
    out = dict(in_group=g[0:S].tolist(), group_size=g[S:2 * S].tolist(), tile_count=g[2 * S:3 * S].tolist(),
               adj=g[3 * S:4 * S].tolist(), singles=g[4 * S:4 * S + single_count].tolist(),
               group_firsts=g[5 * S:5 * S + group_count].tolist(),
               items=[tuple(int(x) for x in g[item0 + 4 * i: item0 + 4 * i + 4]) for i in range(S)], tiles={})
    for first in out["group_firsts"]:
        cnt = out["tile_count"][first]
        ent = tiles[first * max_blocks: first * max_blocks + cnt]
        out["tiles"][first] = [(int(e[0]), int(e[1]) & 0xffff, (int(e[1]) >> 16) & 1, int(e[2]), int(e[3])) for e in ent]
    return out
