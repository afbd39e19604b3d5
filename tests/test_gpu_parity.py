"""GPU parity: the HIP library against the fp64 CPU oracle, element by element, on
the same seeded inputs.  Cache writes and block copies must match bit for bit;
decode must stay within the stated max-abs tolerance (fp16 2e-3, bf16 1.6e-2,
fp32 1e-5) of the oracle."""
import numpy as np
import pytest
import torch

import oracle
from harness import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pa():
    import paper_2309_06180_amd as pa
    pa.load_library()
    return pa


from gpu_util import (TOL, DeviceWorkload, gpu_cache_ops, gpu_decode, gpu_decode_shared,  # noqa: E402
                      mixed_sharing_workload, oracle_cache_ops, out_to_f64, same_bits, to_dev, to_np)


SHARED = "shared"     # pseudo partition value: run pa_decode_shared


def run_and_compare(pa, w, partitions=(0,), q_mult=1.0, seed=None, rows=None):
    v = W.make_values(w, seed=seed, q_mult=q_mult)
    dw = DeviceWorkload(w, v)
    assert pa.pa_debug_validate(dw.block_tables, dw.context_lens, w.max_context_len, dw.write_slots,
                                dw.copy_pairs, w.block_size, w.num_blocks) == 0
    gpu_cache_ops(pa, dw)
    torch.cuda.synchronize()
    kc, vc = oracle_cache_ops(w, v)
    assert same_bits(dw.k_cache, kc, w.dtype), "%s: K cache differs after copy/write" % w.name
    assert same_bits(dw.v_cache, vc, w.dtype), "%s: V cache differs after copy/write" % w.name
    ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype, rows=rows)
    errs = {}
    for ps in partitions:
        out = out_to_f64(gpu_decode_shared(pa, dw) if ps == SHARED else gpu_decode(pa, dw, ps), w.dtype)
        if rows is not None:
            out = out[rows[:, 0], rows[:, 1]]
        assert np.isfinite(out).all(), "%s ps=%s: non-finite output" % (w.name, ps)
        errs[ps] = float(np.abs(out - ref).max())
        assert errs[ps] <= TOL[w.dtype], "%s ps=%s: max abs err %g" % (w.name, ps, errs[ps])
    return errs


# ---------------------------------------------------------------------------
def test_config1_tiny_fp32(pa):
    print(run_and_compare(pa, W.config1(), partitions=(0, 16, 32, 64, pa.PA_PARTITION_AUTO)))


@pytest.mark.parametrize("seed", [1, 2])
def test_config2_reduced_fp16(pa, seed):
    # several blocks per wave, ragged tails, 1..700 tokens
    w = W.config2(seed=seed, num_seqs=24, max_len=700, H=5)
    print(run_and_compare(pa, w, partitions=(0, 64, 256, 512, pa.PA_PARTITION_AUTO)))


def test_config4_reduced_bf16(pa):
    w = W.config4(num_seqs=20, H=3, median=400, cap=1100)
    print(run_and_compare(pa, w, partitions=(0, 128, 512)))


def test_config3_reduced_sharing(pa):
    w = W.config3(num_groups=6, H=4, prompt_median=60, prompt_cap=300, max_out=90)
    assert len(w.copy_pairs) > 0
    print(run_and_compare(pa, w, partitions=(0, 64)))


def test_config5_reduced_beam_one_layer(pa):
    w = W.config5(num_seqs=14, H=4, min_len=100, max_len=700)
    print(run_and_compare(pa, w, partitions=(0, 256)))


@pytest.mark.parametrize("dtype,D,B", [("f16", 128, 16), ("f16", 128, 32), ("f16", 64, 16), ("f16", 64, 8),
                                       ("bf16", 128, 16), ("bf16", 128, 32), ("bf16", 64, 32),
                                       ("f32", 64, 16), ("f32", 128, 16), ("f32", 64, 32),
                                       ("f16", 128, 8), ("f16", 128, 64), ("bf16", 128, 128)])
def test_shape_matrix(pa, dtype, D, B):
    rng = np.random.default_rng(D * 1000 + B)
    lens = rng.integers(1, 6 * B + 40, size=9)
    w = W.independent_sequences("matrix", dtype, 3, D, B, lens, seed=D + B)
    ps = 2 * B if 2 * B >= 32 else 32
    print(run_and_compare(pa, w, partitions=(0, ps)))


@pytest.mark.parametrize("max_len", [40, 64, 200, 256, 400, 512, 1500])
def test_every_workgroup_width(pa, max_len):
    # the launch planner picks 2, 4, 8 or 16 waves per workgroup from max_context_len
    rng = np.random.default_rng(max_len)
    lens = np.concatenate([rng.integers(1, max_len + 1, size=10), [max_len, 1]])
    for dtype in ("f16", "bf16"):
        w = W.independent_sequences("widths", dtype, 3, 128, 16, lens, seed=max_len)
        print(dtype, run_and_compare(pa, w, partitions=(0, 64, 512, 1024)))


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_cases(pa, seed):
    # a seeded walk through the supported set: workload kind, type, head size, block size, heads,
    # lengths and partition sizes all drawn at random; every case through one-pass, split, auto and
    # the sharing-aware call
    rng = np.random.default_rng(9000 + seed)
    dtype = ["f16", "bf16", "f32"][rng.integers(0, 3)]
    D = [64, 128][rng.integers(0, 2)]
    B = [8, 16, 32, 64, 128][rng.integers(0, 5)]
    H = int(rng.integers(1, 6))
    kind = ["independent", "sampling", "beam"][rng.integers(0, 3)]
    top = int(rng.integers(1, 900))
    if kind == "independent":
        lens = rng.integers(0, top + 1, size=int(rng.integers(1, 20)))
        w = W.independent_sequences("rand", dtype, H, D, B, lens, seed=seed)
    elif kind == "sampling":
        w = W.config3(seed=seed, num_groups=int(rng.integers(1, 6)), group=int(rng.integers(2, 6)), H=H, D=D, B=B,
                      dtype=dtype, prompt_median=max(2, top // 4), prompt_cap=top + 2, max_out=int(rng.integers(1, 120)))
    else:
        w = W.config5(seed=seed, num_seqs=int(rng.integers(2, 20)), width=int(rng.integers(2, 10)), H=H, D=D, B=B,
                      dtype=dtype, min_len=max(2, top // 3), max_len=top + 2)
    ps = int(rng.integers(1, 9)) * max(B, 32)
    print(kind, dtype, D, B, H, w.num_seqs, w.max_context_len, ps,
          run_and_compare(pa, w, partitions=(0, ps, pa.PA_PARTITION_AUTO, SHARED)))


# ---------------------------------------------------------------------------
# shared-prefix decode: same oracle, same tolerance
# ---------------------------------------------------------------------------
def test_shared_decode_parallel_sampling(pa):
    w = W.config3(num_groups=7, H=4, prompt_median=80, prompt_cap=300, max_out=90)
    print(run_and_compare(pa, w, partitions=(SHARED, 0)))


def test_shared_decode_beam_groups_of_six(pa):
    # beams share 55% of their blocks
    w = W.config5(num_seqs=20, H=3, min_len=100, max_len=900)
    print(run_and_compare(pa, w, partitions=(SHARED, 0)))
    # contexts past 2048 tokens
    w = W.config5(seed=5007, num_seqs=8, H=2, min_len=1800, max_len=2400)
    assert w.max_context_len > 2048
    print(run_and_compare(pa, w, partitions=(SHARED,)))


def test_shared_decode_large_batch(pa):
    # more sequences than the group discovery keeps in LDS (2048) and than it has threads (1024)
    w = W.config3(seed=3011, num_groups=640, H=1, prompt_median=30, prompt_cap=70, max_out=24)
    assert w.num_seqs == 2560
    print(run_and_compare(pa, w, partitions=(SHARED, 0)))


def test_shared_decode_without_sharing(pa):
    # nothing in common: no group forms, every sequence goes through the one-pass items
    for dtype, D in (("f16", 128), ("bf16", 128), ("f32", 64)):
        rng = np.random.default_rng(31)
        lens = np.concatenate([rng.integers(1, 500, size=9), [0, 1, 16]])
        w = W.independent_sequences("private", dtype, 3, D, 16, lens, seed=32)
        print(dtype, run_and_compare(pa, w, partitions=(SHARED,)))


def test_shared_decode_fully_shared_and_mixed(pa):
    # forks that have not diverged (every block shared, the partial last one included), a group
    # whose members share different numbers of blocks, a loner in between, a group of 5, a pair
    # with exactly one full block in common, ten forks, forty forks (three groups)
    for dtype in ("f16", "bf16"):
        print(dtype, run_and_compare(pa, mixed_sharing_workload(dtype), partitions=(SHARED, 0)))


def test_shared_decode_group_of_forty_and_batch_wide_prefix(pa):
    # one prompt forked 40 times (16 + 16 + 8), and one prefix mapped by every sequence of the batch
    w = W.config3(seed=3021, num_groups=1, group=40, H=3, prompt_median=200, prompt_sigma=1e-9, prompt_cap=200, max_out=70)
    assert w.num_seqs == 40
    print(run_and_compare(pa, w, partitions=(SHARED, 0)))
    for dtype_seed in (3022, 3023):
        w = W.config3(seed=dtype_seed, num_groups=1, group=96, H=2, prompt_median=341, prompt_sigma=1e-9, prompt_cap=341,
                      max_out=128)
        print(run_and_compare(pa, w, partitions=(SHARED,)))
    w = W.config5(seed=5031, num_seqs=36, width=12, H=2, min_len=200, max_len=700)     # beams of twelve, bf16, B = 32
    print(run_and_compare(pa, w, partitions=(SHARED, 0)))


def test_shared_plan_reused_across_layers(pa):
    # one plan per decoding step: three "layers" (different cache contents and queries, same
    # tables) decoded from one plan give the bits of the one-call path and match the oracle;
    # also a shape that has no several-query kernel (the plan is empty, the decode still right)
    for w in (W.config5(num_seqs=14, H=2, min_len=60, max_len=500),
              W.config3(num_groups=3, H=2, prompt_median=40, prompt_cap=100, max_out=30)):
        S, H, D, B = w.num_seqs, w.num_heads, w.head_dim, w.block_size
        plan = torch.empty(pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq),
                           dtype=torch.uint8, device="cuda")
        layers = []
        for layer in range(3):
            v = W.make_values(w, seed=w.seed + 100 * layer)
            dw = DeviceWorkload(w, v)
            gpu_cache_ops(pa, dw)
            layers.append((v, dw))
        dw0 = layers[0][1]
        tdt = dw0.q.dtype
        pa.pa_shared_plan(dw0.block_tables, dw0.context_lens, H, D, B, w.num_blocks, tdt, w.max_context_len, plan)
        for v, dw in layers:
            out = torch.full_like(dw.q, float("nan"))
            pa.pa_decode_shared_planned(out, dw.q, dw.k_cache, dw.v_cache, dw0.block_tables, dw0.context_lens, B,
                                        float(w.scale), w.max_context_len, plan)
            torch.cuda.synchronize()
            assert same_bits(out, to_np(gpu_decode_shared(pa, dw), w.dtype), w.dtype)
            kc, vc = oracle_cache_ops(w, v)
            ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
            err = float(np.abs(out_to_f64(out, w.dtype) - ref).max())
            assert err <= TOL[w.dtype], err
    w = W.config1()
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    plan = torch.empty(max(16, pa.pa_decode_shared_workspace_bytes(w.num_seqs, w.num_heads, w.head_dim,
                                                                    w.max_blocks_per_seq)), dtype=torch.uint8, device="cuda")
    pa.pa_shared_plan(dw.block_tables, dw.context_lens, w.num_heads, w.head_dim, w.block_size, w.num_blocks,
                      dw.q.dtype, w.max_context_len, plan)
    out = torch.full_like(dw.q, float("nan"))
    pa.pa_decode_shared_planned(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                                float(w.scale), w.max_context_len, plan)
    torch.cuda.synchronize()
    assert same_bits(out, to_np(gpu_decode(pa, dw, 0), w.dtype), w.dtype)


# ---------------------------------------------------------------------------
# several query tokens per sequence (causal), on the matrix cores
# ---------------------------------------------------------------------------
def multi_case(pa, dtype, lens, q_lens, H=3, B=16, seed=41, scale=None):
    lens, q_lens = np.asarray(lens, dtype=np.int64), np.asarray(q_lens, dtype=np.int64)
    w = W.independent_sequences("multi", dtype, H, 128, B, lens, seed=seed)
    scale = w.scale if scale is None else np.float32(scale)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    kc, vc = oracle_cache_ops(w, v)
    q_start = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    T = int(q_start[-1])
    rng = np.random.default_rng(seed + 1)
    q = W.to_storage(rng.standard_normal((T, H, 128)).astype(np.float32), dtype)
    dq = to_dev(q, dtype)
    out = torch.full_like(dq, float("nan"))
    pa.pa_decode_multi(out, dq, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, to_dev(q_start),
                       int(q_lens.max()), B, float(scale), w.max_context_len)
    torch.cuda.synchronize()
    ref = oracle.decode_multi(q, kc, vc, w.block_tables, w.context_lens, q_start, scale, dtype)
    got = out_to_f64(out, dtype)
    assert np.isfinite(got).all()
    err = float(np.abs(got - ref).max())
    assert err <= TOL[dtype], "multi %s: max abs err %g" % (dtype, err)
    return err


def test_multi_query_other_scales(pa):
    # the scale is an argument (Sec. 4.1 fixes 1/sqrt(d); the interface does not): negative (the smallest
    # products win), zero (uniform weights) and large, through all three several-query kernels
    lens = [300, 77, 1200, 16, 130]
    for q_lens in ([16, 16, 9, 16, 1], [64, 33, 40, 16, 17], [200, 77, 256, 16, 130]):
        for dtype in ("f16", "bf16"):
            for scale in (-0.0883883, 0.0, 0.7):
                print(dtype, max(q_lens), scale, multi_case(pa, dtype, lens, q_lens, H=2, seed=61, scale=scale))


def test_multi_query_decode(pa):
    # q_len 1 (= decode), a few, exactly 16, 17 (two query blocks), the whole context, none
    lens = [1, 2, 15, 16, 17, 33, 64, 100, 257, 700, 700, 1025, 40, 300]
    q_lens = [1, 2, 15, 16, 17, 5, 64, 1, 16, 40, 3, 31, 0, 300]
    for dtype in ("f16", "bf16"):
        print(dtype, multi_case(pa, dtype, lens, q_lens))
    print("B=32", multi_case(pa, "bf16", lens, q_lens, H=2, B=32))
    # a few queries per sequence (draft tokens): the eight-wave variant
    few = [min(n, k) for n, k in zip(lens, [1, 2, 8, 4, 8, 5, 7, 1, 8, 3, 0, 6, 2, 8])]
    for dtype in ("f16", "bf16"):
        print(dtype, "q_len <= 8", multi_case(pa, dtype, lens, few, seed=43))
    print("B=64", multi_case(pa, "f16", [500, 130, 64], [20, 130, 1], H=2, B=64))


def test_multi_query_every_width(pa):
    # q_len across the switch from the token-splitting kernel (<= 16 queries) to the 64-query
    # workgroups, with partly filled last query blocks and contexts shorter than a block of queries
    lens = [70, 200, 129, 64, 513, 48, 1000, 333]
    for qmax in (16, 17, 31, 48, 63, 64, 65, 130, 200):
        q_lens = [min(n, qmax - (i % 3)) for i, n in enumerate(lens)]
        for dtype in ("f16", "bf16"):
            print(dtype, qmax, multi_case(pa, dtype, lens, q_lens, H=2, seed=50 + qmax))
    print("B=128", multi_case(pa, "f16", [700, 130, 128, 129, 5], [100, 130, 16, 1, 5], H=2, B=128, seed=77))
    print("B=128", multi_case(pa, "bf16", [700, 130, 128, 129, 5], [9, 16, 16, 1, 5], H=2, B=128, seed=78))


def test_multi_query_sharp_softmax(pa):
    # queries scaled by 8: one token dominates, the weights' two 16-bit pieces must carry it; at more than 64
    # queries per sequence the exponents' reference point moves lazily (only past 2^8), which scores that keep
    # rising along the context (K rows scaled by their position) exercise step after step
    for dtype in ("f16", "bf16"):
        lens = np.array([300, 77, 1200, 16], dtype=np.int64)
        for q_lens, rising in (([64, 16, 40, 16], False), ([200, 77, 130, 16], False), ([256, 16, 100, 5], True)):
            q_lens = np.array(q_lens, dtype=np.int64)
            w = W.independent_sequences("multi_sharp", dtype, 2, 128, 16, lens, seed=91)
            v = W.make_values(w)
            dw = DeviceWorkload(w, v)
            gpu_cache_ops(pa, dw)
            kc, vc = oracle_cache_ops(w, v)
            kdev = dw.k_cache
            if rising:
                # token at position t of every sequence gets its K row scaled by (1 + t / 64)
                kf = W.storage_to_f64(kc, dtype)
                for sq, n in enumerate(lens):
                    for t in range(int(n)):
                        b, o = w.block_tables[sq, t // 16], t % 16
                        kf[b, :, o, :] *= 1.0 + t / 64.0
                kc = W.to_storage(kf.astype(np.float32), dtype)
                kdev = to_dev(kc, dtype)
            q_start = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
            rng = np.random.default_rng(92)
            q = W.to_storage(8.0 * rng.standard_normal((int(q_start[-1]), 2, 128)).astype(np.float32), dtype)
            dq = to_dev(q, dtype)
            out = torch.full_like(dq, float("nan"))
            pa.pa_decode_multi(out, dq, kdev, dw.v_cache, dw.block_tables, dw.context_lens, to_dev(q_start),
                               int(q_lens.max()), 16, float(w.scale), w.max_context_len)
            torch.cuda.synchronize()
            ref = oracle.decode_multi(q, kc, vc, w.block_tables, w.context_lens, q_start, w.scale, dtype)
            err = float(np.abs(out_to_f64(out, dtype) - ref).max())
            assert err <= TOL[dtype], "sharp multi %s q_len %s rising=%s: %g" % (dtype, q_lens, rising, err)


def test_multi_query_deterministic_and_placement_invariant(pa):
    # same bits run to run, and when the physical blocks are relabelled by a permutation with their data
    # moved along (Sec. 4.1: placement is free; the summation order follows logical positions only)
    lens = np.array([300, 77, 1200, 16, 130], dtype=np.int64)
    w = W.independent_sequences("multi_place", "bf16", 2, 128, 16, lens, seed=73)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    perm = np.random.default_rng(4).permutation(w.num_blocks)
    inv = np.argsort(perm)
    kc2 = dw.k_cache[to_dev(inv)].contiguous()           # new block perm[i] holds old block i
    vc2 = dw.v_cache[to_dev(inv)].contiguous()
    bt = w.block_tables.copy()
    for s in range(w.num_seqs):
        nb = (int(w.context_lens[s]) + 15) // 16
        bt[s, :nb] = perm[bt[s, :nb]]
    bt2 = to_dev(bt)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(8)
    for q_lens in ([16, 16, 9, 16, 1], [64, 33, 40, 16, 17], [200, 77, 256, 16, 130]):
        q_start = to_dev(np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32))
        q = torch.randn((int(sum(q_lens)), 2, 128), device="cuda", generator=gen).to(torch.bfloat16)
        outs = []
        for kc, vc, tables in ((dw.k_cache, dw.v_cache, dw.block_tables), (dw.k_cache, dw.v_cache, dw.block_tables),
                               (kc2, vc2, bt2)):
            out = torch.full_like(q, float("nan"))
            pa.pa_decode_multi(out, q, kc, vc, tables, dw.context_lens, q_start, max(q_lens), 16, float(w.scale),
                               w.max_context_len)
            torch.cuda.synchronize()
            outs.append(out)
        assert torch.equal(outs[0], outs[1]), "q_len %d: run-to-run difference" % max(q_lens)
        assert torch.equal(outs[0], outs[2]), "q_len %d: result depends on block placement" % max(q_lens)


def test_multi_query_graph_replay(pa):
    # the several-query kernels hold no state between launches: a captured call replays with new queries
    # written in place and matches the eager result bit for bit, for each of the three kernels
    lens = np.array([300, 77, 1200, 16, 130], dtype=np.int64)
    w = W.independent_sequences("multi_graph", "f16", 2, 128, 16, lens, seed=71)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(6)
    for q_lens in ([16, 16, 9, 16, 1], [64, 33, 40, 16, 17], [200, 77, 256, 16, 130]):
        q_start = to_dev(np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32))
        T = int(sum(q_lens))
        q = torch.randn((T, 2, 128), device="cuda", generator=gen).to(torch.float16)
        out = torch.empty_like(q)

        def call():
            pa.pa_decode_multi(out, q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, q_start,
                               max(q_lens), 16, float(w.scale), w.max_context_len)

        call()
        torch.cuda.synchronize()
        first = out.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        for it in range(3):
            q.copy_(torch.randn(q.shape, device="cuda", generator=gen).to(q.dtype))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            replayed = out.clone()
            call()                                        # eager work between replays
            torch.cuda.synchronize()
            assert torch.equal(replayed, out), "q_len %d: replay %d differs from eager" % (max(q_lens), it)
            assert not torch.equal(replayed, first)


def test_multi_query_one_hot_operands_fail_by_position(pa):
    # K, V and Q made of single ones: every logit is 0 or 1 and every output element is a
    # small rational that names the (query, token, dimension) it came from, so a slip in an
    # MFMA operand or LDS layout shows up at the position it happens
    for dtype in ("f16", "bf16"):
        for q_len in (16, 64):
            n, H, D, B = 96, 2, 128, 16
            w = W.independent_sequences("onehot", dtype, H, D, B, np.array([n]), seed=3)
            kc = np.zeros(w.cache_shape(), dtype=np.float32)
            vc = np.zeros(w.cache_shape(), dtype=np.float32)
            q = np.zeros((q_len, H, D), dtype=np.float32)
            for t in range(n):
                pb, off = int(w.block_tables[0, t // B]), t % B
                for h in range(H):
                    kc[pb, h, off, (5 * t + 3 * h) % D] = 1.0          # token t's key: one dimension
                    vc[pb, h, off, (7 * t + h) % D] = 1.0 + (t % 5)    # its value: another one
            for i in range(q_len):
                for h in range(H):
                    q[i, h, (5 * (n - q_len + i - 2 * (i % 7)) + 3 * h) % D] = 4.0   # picks one earlier token
                    q[i, h, (11 * i + 1) % D] += 2.0
            kcs, vcs, qs_ = W.to_storage(kc, dtype), W.to_storage(vc, dtype), W.to_storage(q, dtype)
            q_start = np.array([0, q_len], dtype=np.int32)
            out = torch.full((q_len, H, D), float("nan"), dtype=torch.float16 if dtype == "f16" else torch.bfloat16,
                             device="cuda")
            pa.pa_decode_multi(out, to_dev(qs_, dtype), to_dev(kcs, dtype), to_dev(vcs, dtype), to_dev(w.block_tables),
                               to_dev(w.context_lens), to_dev(q_start), q_len, B, 1.0, n)
            torch.cuda.synchronize()
            ref = oracle.decode_multi(qs_, kcs, vcs, w.block_tables, w.context_lens, q_start, 1.0, dtype)
            got = out_to_f64(out, dtype)
            bad = np.argwhere(np.abs(got - ref) > TOL[dtype])
            assert len(bad) == 0, "%s q_len %d: first mismatches at (query, head, dim) %s" % (dtype, q_len, bad[:8].tolist())


def test_multi_query_of_one_equals_decode(pa):
    w = W.config2(seed=13, num_seqs=12, max_len=600, H=4)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    a = out_to_f64(gpu_decode(pa, dw, 0), w.dtype)
    out = torch.empty_like(dw.q)
    pa.pa_decode_multi(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens,
                       to_dev(np.arange(w.num_seqs + 1, dtype=np.int32)), 1, w.block_size, float(w.scale),
                       w.max_context_len)
    torch.cuda.synchronize()
    b = out_to_f64(out, w.dtype)
    # two kernels, two summation orders: equal within one rounding of the output type
    assert np.abs(a - b).max() <= 2 * TOL[w.dtype]


def test_edge_context_lengths(pa):
    # one below / at / one above every boundary the kernels have: block, chunk, partition
    B, PS = 16, 64
    lens = np.array([1, 2, 3, 4, 5, B - 1, B, B + 1, 2 * B - 1, 2 * B, 2 * B + 1, PS - 1, PS, PS + 1,
                     2 * PS - 1, 2 * PS, 2 * PS + 1, 8 * PS, 8 * PS + 1, 1023, 1024, 1025], dtype=np.int64)
    for dtype in ("f16", "bf16"):
        w = W.independent_sequences("edges", dtype, 2, 128, B, lens, seed=5)
        print(dtype, run_and_compare(pa, w, partitions=(0, PS, 256)))


@pytest.mark.parametrize("dtype,D,B", [("f16", 128, 16), ("bf16", 128, 32), ("f32", 64, 16)])
def test_one_long_sequence_among_short_ones(pa, dtype, D, B):
    # the launch is planned from the 2048-token sequence; the short items leave most of their workgroup's
    # waves without a chunk (those exit before the merge, which then covers the busy waves only)
    rng = np.random.default_rng(77)
    lens = np.concatenate([[2048], rng.integers(1, 65, size=40), [0, 1, 16, 17, 255, 256, 257]])
    w = W.independent_sequences("skewed", dtype, 3, D, B, lens, seed=78)
    print(dtype, run_and_compare(pa, w, partitions=(0, 512)))


@pytest.mark.parametrize("scale", [-0.0883883, 0.0, 0.7])
def test_other_scales(pa, scale):
    # the scale is an argument of the interface: negative (the smallest products win), zero (uniform weights)
    # and large, through the one-pass, split-context and sharing-aware calls
    for dtype in ("f16", "bf16"):
        w = mixed_sharing_workload(dtype)
        w.scale = np.float32(scale)
        print(dtype, scale, run_and_compare(pa, w, partitions=(0, 64, SHARED)))
    w = W.independent_sequences("scales_f32", "f32", 2, 64, 16, np.array([1, 40, 300, 17]), seed=15)
    w.scale = np.float32(scale)
    print("f32", scale, run_and_compare(pa, w, partitions=(0, 64)))


def test_empty_context_gives_zero_row(pa):
    w = W.independent_sequences("zeros", "f16", 2, 128, 16, np.array([0, 40, 0, 300]), seed=6)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    kc, vc = oracle_cache_ops(w, v)
    ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    for ps in (0, 64):
        out = out_to_f64(gpu_decode(pa, dw, ps), w.dtype)
        assert not out[0].any() and not out[2].any()
        assert np.abs(out - ref).max() <= TOL["f16"]


def test_sharp_softmax(pa):
    # queries scaled by 8: logits spread over tens of units, the running maximum moves a lot
    w = W.config2(seed=9, num_seqs=12, max_len=600, H=4)
    print(run_and_compare(pa, w, partitions=(0, 128), q_mult=8.0))


def test_context_len_one_is_bit_exact(pa):
    for dtype in ("f16", "bf16", "f32"):
        D = 64 if dtype == "f32" else 128
        w = W.independent_sequences("ones", dtype, 4, D, 16, np.ones(7, dtype=np.int64), seed=7)
        v = W.make_values(w)
        dw = DeviceWorkload(w, v)
        gpu_cache_ops(pa, dw)
        out = to_np(gpu_decode(pa, dw, 0), dtype)
        want = v.v_new                                   # the only token of each sequence
        assert np.array_equal(out.view(np.uint8), want.view(np.uint8))


def test_deterministic_and_placement_invariant(pa):
    w = W.config2(seed=11, num_seqs=10, max_len=500, H=4)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    for ps in (0, 128):
        a = to_np(gpu_decode(pa, dw, ps), w.dtype)
        b = to_np(gpu_decode(pa, dw, ps), w.dtype)
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), "run-to-run difference"
        # relabel physical blocks by a permutation, moving the data along (Sec. 4.1: placement is free)
        perm = np.random.default_rng(3).permutation(w.num_blocks)
        inv = np.argsort(perm)
        kc2 = dw.k_cache[to_dev(inv)].contiguous()       # new block perm[i] holds old block i
        vc2 = dw.v_cache[to_dev(inv)].contiguous()
        bt = w.block_tables.copy()
        B = w.block_size
        for s in range(w.num_seqs):
            nb = (int(w.context_lens[s]) + B - 1) // B
            bt[s, :nb] = perm[bt[s, :nb]]
        out = torch.empty_like(dw.q)
        ws = torch.empty(max(1, pa.pa_decode_workspace_bytes(w.num_seqs, w.num_heads, w.head_dim, B,
                                                            w.max_context_len, ps)), dtype=torch.uint8, device="cuda")
        pa.pa_decode(out, dw.q, kc2, vc2, to_dev(bt), dw.context_lens, B, float(w.scale),
                     w.max_context_len, ps, ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(out, w.dtype).view(np.uint8), a.view(np.uint8)), "placement changed the bits"


def test_shared_decode_deterministic_and_placement_invariant(pa):
    # the sharing-aware path: grouping looks at which table entries are equal, never at their values
    for w in (W.config5(seed=71, num_seqs=14, H=3, min_len=100, max_len=600),
              W.config3(seed=72, num_groups=5, H=3, prompt_median=50, prompt_cap=200, max_out=60)):
        v = W.make_values(w)
        dw = DeviceWorkload(w, v)
        gpu_cache_ops(pa, dw)
        a = to_np(gpu_decode_shared(pa, dw), w.dtype)
        b = to_np(gpu_decode_shared(pa, dw), w.dtype)
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), "run-to-run difference"
        perm = np.random.default_rng(5).permutation(w.num_blocks)
        inv = np.argsort(perm)
        B = w.block_size
        bt = w.block_tables.copy()
        for s in range(w.num_seqs):
            nb = (int(w.context_lens[s]) + B - 1) // B
            bt[s, :nb] = perm[bt[s, :nb]]
        moved = DeviceWorkload(w, v)
        moved.k_cache = dw.k_cache[to_dev(inv)].contiguous()
        moved.v_cache = dw.v_cache[to_dev(inv)].contiguous()
        moved.block_tables = to_dev(bt)
        c = to_np(gpu_decode_shared(pa, moved), w.dtype)
        assert np.array_equal(c.view(np.uint8), a.view(np.uint8)), "placement changed the bits"


def test_reshape_and_cache_prefill_sized(pa):
    # thousands of tokens in one call (a prompt phase storing its KV), with skipped padding tokens
    rng = np.random.default_rng(21)
    T, H, D, B, NB = 3000, 5, 128, 16, 400
    for dtype in ("f16", "bf16", "f32"):
        k = W.to_storage(rng.standard_normal((T, H, D)).astype(np.float32), dtype)
        v = W.to_storage(rng.standard_normal((T, H, D)).astype(np.float32), dtype)
        kc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), dtype)
        vc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), dtype)
        slots = rng.permutation(NB * B)[:T].astype(np.int64)
        slots[rng.integers(0, T, size=40)] = -1
        dk, dv = to_dev(kc, dtype), to_dev(vc, dtype)
        pa.pa_reshape_and_cache(to_dev(k, dtype), to_dev(v, dtype), dk, dv, to_dev(slots))
        torch.cuda.synchronize()
        oracle.reshape_and_cache(k, v, kc, vc, slots, dtype)
        assert same_bits(dk, kc, dtype) and same_bits(dv, vc, dtype)


def test_copy_blocks_multi_layer_fan_out(pa):
    rng = np.random.default_rng(22)
    L, NB, H, B, D = 5, 40, 3, 16, 128
    ks = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "bf16") for _ in range(L)]
    vs = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "bf16") for _ in range(L)]
    pairs = np.array([[1, 3], [7, 0], [7, 5], [7, 9], [39, 20], [2, 38]], dtype=np.int64)
    dks, dvs = [to_dev(k, "bf16") for k in ks], [to_dev(v, "bf16") for v in vs]
    pa.pa_copy_blocks(dks, dvs, to_dev(pairs))
    pa.pa_copy_blocks(dks, dvs, to_dev(np.zeros((0, 2), dtype=np.int64)))    # empty list: no launch
    torch.cuda.synchronize()
    oracle.copy_blocks(ks, vs, pairs, "bf16")
    for l in range(L):
        assert same_bits(dks[l], ks[l], "bf16") and same_bits(dvs[l], vs[l], "bf16")


def test_copy_blocks_many_layers_two_launches(pa):
    # more layers than one launch carries pointers for
    rng = np.random.default_rng(23)
    L, NB, H, B, D = 70, 6, 1, 8, 64
    ks = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f16") for _ in range(L)]
    vs = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f16") for _ in range(L)]
    pairs = np.array([[0, 4], [1, 5]], dtype=np.int64)
    dks, dvs = [to_dev(k) for k in ks], [to_dev(v) for v in vs]
    pa.pa_copy_blocks(dks, dvs, to_dev(pairs))
    torch.cuda.synchronize()
    oracle.copy_blocks(ks, vs, pairs, "f16")
    for l in range(L):
        assert same_bits(dks[l], ks[l], "f16") and same_bits(dvs[l], vs[l], "f16")


def test_copy_and_swap_blocks_longer_pair_lists_than_one_launch(pa):
    # a launch carries at most 65 535 pairs in its grid: longer lists take several launches
    rng = np.random.default_rng(29)
    N, H, B, D = 70000, 1, 8, 16                              # 256-byte blocks
    NB = 2 * N + 7
    k = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f16")
    v = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f16")
    perm = rng.permutation(NB)
    pairs = np.stack([perm[:N], perm[N:2 * N]], axis=1).astype(np.int64)
    dk, dv = to_dev(k), to_dev(v)
    pa.pa_copy_blocks([dk], [dv], to_dev(pairs))
    torch.cuda.synchronize()
    oracle.copy_blocks([k], [v], pairs, "f16")
    assert same_bits(dk, k, "f16") and same_bits(dv, v, "f16")
    # the same list as a swap into a second pool on the device
    k2, v2 = np.zeros_like(k), np.zeros_like(v)
    dk2, dv2 = to_dev(k2), to_dev(v2)
    pa.pa_swap_blocks([dk], [dv], [dk2], [dv2], to_dev(pairs))
    torch.cuda.synchronize()
    oracle.swap_blocks([k], [v], [k2], [v2], pairs, "f16")
    assert same_bits(dk2, k2, "f16") and same_bits(dv2, v2, "f16")


def test_an_earlier_hip_error_of_the_caller_is_not_reported_as_ours(pa):
    # the caller provokes a HIP error of its own (a copy with an invalid direction); the next library calls
    # must still report their own launches' status.  Everything is allocated beforehand: torch checks the
    # last error after its own launches.
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    buf = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    src = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(65536, dtype=torch.int32, device="cuda")
    w = W.config1()
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    out = torch.zeros_like(dw.q)
    torch.cuda.synchronize()
    try:
        assert hip.hipMemcpy(buf.data_ptr(), buf.data_ptr() + 512, 16, 99) != 0
        pa.pa_stream_read(src, sink)                          # raises on a non-zero status
        pa.pa_decode(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size, float(w.scale),
                     w.max_context_len)
    finally:
        hip.hipGetLastError()                                 # leave no error behind for the tests that follow
    torch.cuda.synchronize()
    kc, vc = oracle_cache_ops(w, v)
    ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    assert np.abs(out_to_f64(out, w.dtype) - ref).max() <= TOL[w.dtype]


def test_infinity_in_unused_slots_is_ignored(pa):
    # every slot that holds no token carries +Inf or -Inf instead of NaN: 0 * Inf would be NaN just the same
    for w in (W.config2(seed=17, num_seqs=9, max_len=300, H=3), W.config4(seed=18, num_seqs=7, H=2),
              W.config3(seed=19, num_groups=3, H=2, prompt_median=60, prompt_cap=200, max_out=50)):
        v = W.make_values(w)
        bits = {"f16": (0x7C00, 0xFC00), "bf16": (0x7F80, 0xFF80)}[w.dtype]
        for cache in (v.k_cache, v.v_cache):
            raw = cache.view(np.uint16)
            hole = np.broadcast_to((~w.init_filled)[:, None, :, None], raw.shape)
            alt = (np.arange(raw.size, dtype=np.uint32).reshape(raw.shape) & 1).astype(bool)
            raw[hole & alt] = bits[0]
            raw[hole & ~alt] = bits[1]
        dw = DeviceWorkload(w, v)
        gpu_cache_ops(pa, dw)
        kc, vc = oracle_cache_ops(w, v)
        ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
        assert np.isfinite(ref).all()
        for ps in (0, 64, SHARED):
            out = out_to_f64(gpu_decode_shared(pa, dw) if ps == SHARED else gpu_decode(pa, dw, ps), w.dtype)
            assert np.isfinite(out).all(), "%s ps=%s: Inf leaked" % (w.name, ps)
            assert np.abs(out - ref).max() <= TOL[w.dtype]


def test_swap_blocks_to_pinned_host_and_back(pa):
    # Sec. 4.5: evicted blocks go to a CPU pool (pinned, device-addressable) and return to other blocks
    rng = np.random.default_rng(24)
    L, NBG, NBC, H, B, D = 3, 60, 40, 5, 16, 128
    for dtype in ("f16", "bf16"):
        gk = [W.to_storage(rng.standard_normal((NBG, H, B, D)).astype(np.float32), dtype) for _ in range(L)]
        gv = [W.to_storage(rng.standard_normal((NBG, H, B, D)).astype(np.float32), dtype) for _ in range(L)]
        ck = [W.to_storage(rng.standard_normal((NBC, H, B, D)).astype(np.float32), dtype) for _ in range(L)]
        cv = [W.to_storage(rng.standard_normal((NBC, H, B, D)).astype(np.float32), dtype) for _ in range(L)]
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float16

        def pinned(a):
            t = torch.empty(a.shape, dtype=tdt, pin_memory=True)
            src = torch.from_numpy(a)
            t.copy_(src.view(torch.bfloat16) if dtype == "bf16" else src)
            return t

        dgk, dgv = [to_dev(x, dtype) for x in gk], [to_dev(x, dtype) for x in gv]
        hck, hcv = [pinned(x) for x in ck], [pinned(x) for x in cv]
        perm_g, perm_c = rng.permutation(NBG), rng.permutation(NBC)
        out_pairs = np.stack([perm_g[:25], perm_c[:25]], axis=1).astype(np.int64)
        pa.pa_swap_blocks(dgk, dgv, hck, hcv, to_dev(out_pairs))
        torch.cuda.synchronize()
        oracle.swap_blocks(gk, gv, ck, cv, out_pairs, dtype)
        for l in range(L):
            assert same_bits(hck[l], ck[l], dtype) and same_bits(hcv[l], cv[l], dtype)
        # the freed GPU blocks get overwritten, then the swapped-out blocks come back into other blocks
        for l in range(L):
            dgk[l][to_dev(perm_g[:25])] = 0
            gk[l][perm_g[:25]] = 0
        in_pairs = np.stack([perm_c[:25], rng.permutation(NBG)[:25]], axis=1).astype(np.int64)
        pa.pa_swap_blocks(hck, hcv, dgk, dgv, to_dev(in_pairs))
        torch.cuda.synchronize()
        oracle.swap_blocks(ck, cv, gk, gv, in_pairs, dtype)
        for l in range(L):
            assert same_bits(dgk[l], gk[l], dtype) and same_bits(dgv[l], gv[l], dtype)


def test_debug_validate_flags_bad_indices(pa):
    w = W.config1()
    bt, cl = to_dev(w.block_tables), to_dev(w.context_lens)
    ok = pa.pa_debug_validate(bt, cl, w.max_context_len, to_dev(w.write_slots), None, w.block_size, w.num_blocks)
    assert ok == 0
    bad = w.block_tables.copy()
    bad[0, 0] = w.num_blocks
    assert pa.pa_debug_validate(to_dev(bad), cl, w.max_context_len, None, None, w.block_size, w.num_blocks) == 7
    assert pa.pa_debug_validate(bt, cl, int(w.context_lens.max()) - 1, None, None, w.block_size, w.num_blocks) == 7
    dup = w.write_slots.copy()
    dup[1] = dup[0]
    assert pa.pa_debug_validate(None, None, 0, to_dev(dup), None, w.block_size, w.num_blocks) == 7
    pairs = np.array([[1, 2], [2, 3]], dtype=np.int64)          # a destination used as a source
    assert pa.pa_debug_validate(None, None, 0, None, to_dev(pairs), w.block_size, w.num_blocks) == 7


def test_workspace_and_argument_errors_on_device(pa):
    w = W.config2(seed=1, num_seqs=4, max_len=300, H=2)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    out = torch.empty_like(dw.q)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(pa.PAError) as e:
        pa.pa_decode(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                     float(w.scale), w.max_context_len, 64, small)
    assert e.value.code == 5
    with pytest.raises(pa.PAError) as e:
        pa.pa_decode(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                     float(w.scale), w.max_context_len, 24, small)       # not a multiple of the block size
    assert e.value.code == 2


def test_side_stream_and_graph_replay(pa):
    # the calls enqueue on torch's current stream; a captured step (cache write + decode) replays
    # with new inputs written in place, and every replay matches the eager result
    w = W.config2(seed=17, num_seqs=16, max_len=500, H=4)
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    out = torch.empty_like(dw.q)
    k_new, v_new = dw.k_new.clone(), dw.v_new.clone()

    def step():
        pa.pa_reshape_and_cache(k_new, v_new, dw.k_cache, dw.v_cache, dw.write_slots)
        pa.pa_decode(out, dw.q, dw.k_cache, dw.v_cache, dw.block_tables, dw.context_lens, w.block_size,
                     float(w.scale), w.max_context_len, 0, None)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    side.synchronize()
    eager0 = out.clone()
    kc, vc = oracle_cache_ops(w, v)
    ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    assert np.abs(out_to_f64(eager0, w.dtype) - ref).max() <= TOL[w.dtype]

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    for it in range(3):
        k_new.copy_(torch.randn(k_new.shape, device="cuda", generator=gen).to(k_new.dtype))
        v_new.copy_(torch.randn(v_new.shape, device="cuda", generator=gen).to(v_new.dtype))
        dw.q.copy_(torch.randn(dw.q.shape, device="cuda", generator=gen).to(dw.q.dtype))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        replayed = out.clone()
        step()                                        # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(replayed, out), "replay %d differs from eager" % it
        assert not torch.equal(replayed, eager0)
