"""The sharing plan pa_shared_plan leaves in its workspace, compared entry by entry with a pure-index
host reference (tests/plan_reference.py), so that a decode which silently fell through to the
one-pass path, or a tile list that misses or repeats a block, fails here and not only in timing."""
import numpy as np
import pytest
import torch

from harness import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import mixed_sharing_workload, to_dev  # noqa: E402
import plan_reference as ref  # noqa: E402


@pytest.fixture(scope="module")
def pa():
    import paper_2309_06180_amd as pa
    pa.load_library()
    return pa


def device_plan(pa, w):
    S, H, D, B = w.num_seqs, w.num_heads, w.head_dim, w.block_size
    ws = torch.zeros(pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq), dtype=torch.uint8, device="cuda")
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[w.dtype]
    pa.pa_shared_plan(to_dev(w.block_tables), to_dev(w.context_lens), H, D, B, w.num_blocks, tdt, w.max_context_len, ws)
    torch.cuda.synchronize()
    return ref.decode_device_plan(ws.cpu().numpy(), S, w.max_blocks_per_seq)


def unique_tokens_of(w, first, size):
    """tokens a group's members see, counted once per physical block (from the tables alone)."""
    B = w.block_size
    best = {}
    for s in range(first, first + size):
        n = int(w.context_lens[s])
        for pos in range((n + B - 1) // B):
            blk = int(w.block_tables[s, pos])
            best[(pos, blk)] = max(best.get((pos, blk), 0), min(B, n - pos * B))
    return sum(best.values())


def check(pa, w, min_groups=1, expect_sizes=None):
    want = ref.plan(w.block_tables, w.context_lens, w.block_size)
    got = device_plan(pa, w)
    assert got["adj"] == want["adj"]
    assert got["in_group"] == want["in_group"]
    assert got["group_size"] == want["group_size"]
    assert got["group_firsts"] == [f for f, _ in want["groups"]]
    assert got["singles"] == want["singles"]
    assert got["items"] == ref.items_of(want, w.num_seqs)
    assert len(got["group_firsts"]) >= min_groups, "no sharing found: the decode would run the one-pass path only"
    for first, size in want["groups"]:
        assert got["tiles"][first] == want["tiles"][first], "tile list of the group at %d differs" % first
        listed = sum(e[4] for e in got["tiles"][first])
        assert listed == unique_tokens_of(w, first, size)
        logical = int(w.context_lens[first:first + size].sum())
        assert listed <= logical
    if expect_sizes is not None:
        assert sorted(s for _, s in want["groups"]) == sorted(expect_sizes)
    return want


def test_plan_parallel_sampling(pa):
    w = W.config3(num_groups=9, H=2, prompt_median=120, prompt_cap=400, max_out=90)
    want = check(pa, w)
    # a sample group of 4 either forms one group or (short prompt against long outputs) none
    assert all(size <= 4 for _, size in want["groups"])
    saved = sum(int(w.context_lens[f:f + s].sum()) - unique_tokens_of(w, f, s) for f, s in want["groups"])
    assert saved > 0


def test_plan_beam_search(pa):
    w = W.config5(num_seqs=20, H=2, min_len=100, max_len=900)
    check(pa, w, min_groups=3)
    w = W.config5(seed=5031, num_seqs=36, width=12, H=2, min_len=200, max_len=700)
    check(pa, w, expect_sizes=[12, 12, 12])


def test_plan_mixed_patterns(pa):
    w = mixed_sharing_workload("f16")
    want = check(pa, w)
    sizes = sorted(s for _, s in want["groups"])
    # the three un-diverged forks, the family of five, the ten, the forty (16 + 16 + 8); the loner and the
    # pair with a single 16-token block in common (too little to be worth a group) stay on their own
    assert sizes == sorted([3, 5, 10, 16, 16, 8]), sizes
    assert want["singles"] == [3, 9, 10]
    first = 0
    assert (0, 3) in want["groups"]
    # un-diverged forks: every block, the partial last one included, is listed once for all three
    assert all(e[1] == 0b111 for e in want["tiles"][first]) and len(want["tiles"][first]) == 5
    assert want["tiles"][first][-1][2] == 1 and want["tiles"][first][-1][4] == 70 - 64


def test_plan_batch_wide_prefix_and_large_batch(pa):
    w = W.config3(seed=3022, num_groups=1, group=96, H=2, prompt_median=341, prompt_sigma=1e-9, prompt_cap=341, max_out=128)
    check(pa, w, expect_sizes=[16] * 6)
    w = W.config3(seed=3011, num_groups=640, H=1, prompt_median=30, prompt_cap=70, max_out=24)
    assert w.num_seqs == 2560                     # more than the discovery kernel keeps in LDS
    check(pa, w, min_groups=100)


def test_plan_without_sharing_is_empty(pa):
    lens = np.random.default_rng(31).integers(1, 500, size=40)
    w = W.independent_sequences("private", "f16", 2, 128, 16, lens, seed=32)
    got = device_plan(pa, w)
    assert got["group_firsts"] == [] and got["singles"] == list(range(40)) and not any(got["in_group"])
    assert got["items"] == [(1, s, 1, 0) for s in range(40)]
