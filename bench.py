#!/usr/bin/env python3
"""Benchmark of the paged-decode hot path on one MI355X.

A step is one decode iteration of one layer on a synthetic batch: copy-on-write block
copies queued for the step (none in the OPT-13B workload), the store of every
sequence's newest K/V vectors (pa_reshape_and_cache), then paged attention of one
query token per sequence (pa_decode).  Inputs are resident in HBM before timing.

Prints ONE JSON line.  `value` is the K+V bytes the step's attention reads, per
second of whole-step time; `roofline` is for the dominant kernel (the decode kernel)
from HIP events around back-to-back pa_decode calls on the launch stream;
`cpu_baseline` is the fp64 oracle timed on the host cores on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
MFMA_F16_PEAK = 2.5e15          # MI355X published dense f16/bf16 matrix peak, flop/s


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg5 runs one of its 40 layers")
    ap.add_argument("--decode", default="plain", choices=["plain", "shared"],
                    help="shared: pa_decode_shared (blocks common to neighbouring sequences read once)")
    ap.add_argument("--partition", type=int, default=None,
                    help="partition_size for pa_decode (0 = one pass, -1 = library's choice); "
                         "default: the library's choice")
    ap.add_argument("--cache-allocation", default="one", choices=["one", "two"],
                    help="one: K and V of the layer carved from one device allocation; two: an allocation each")
    ap.add_argument("--launch", default="eager", choices=["eager", "graph"],
                    help="eager: three library calls per step (default; measured 179 us per step); "
                         "graph: the step is captured once in a HIP graph and replayed (186 us: the replay "
                         "costs more than the launches it saves, the GPU is never waiting for the host here)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one pa_copy_blocks of known size (a plain copy kernel that "
                         "hardware-counter runs use to scale FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--others", dest="others", action="store_true", default=None,
                    help="also time configs 3, 4 and 5 (one layer) each way and add them to the line as \"others\" "
                         "(default for the default workload)")
    ap.add_argument("--no-others", dest="others", action="store_false")
    ap.add_argument("--block-size-sweep", action="store_true",
                    help="instead of the step benchmark: pa_decode at the OPT-13B shape for B = 8..128")
    ap.add_argument("--cfg5-full-step", action="store_true",
                    help="instead of the step benchmark: the whole 40-layer beam-search step of config 5 "
                         "(~142 GB of cache filled on the device): copy-on-write for all layers, then per "
                         "layer cache write + decode")
    ap.add_argument("--multi-query", action="store_true",
                    help="instead of the step benchmark: pa_decode_multi at the OPT-13B shape for several q_len")
    ap.add_argument("--q-lens", default="1,4,16,64,128,256",
                    help="--multi-query: the q_len values to run, comma separated")
    ap.add_argument("--paging-overhead", action="store_true",
                    help="instead of the step benchmark: pa_decode over randomly placed blocks against the same "
                         "sequences stored contiguously (the axis of the paper's kernel microbenchmark, Sec. 7.1)")
    ap.add_argument("--short-batches", action="store_true",
                    help="instead of the step benchmark: pa_decode on large batches of short sequences (the regime "
                         "of the paper's second trace, whose sequences are a few dozen tokens long)")
    ap.add_argument("--shared-prefix", action="store_true",
                    help="instead of the step benchmark: one prefix shared by every sequence of the batch "
                         "(Sec. 4.4 / 6.4), pa_decode against pa_decode_shared")
    ap.add_argument("--cache-ops", action="store_true",
                    help="instead of the step benchmark: pa_reshape_and_cache and pa_copy_blocks at several sizes")
    return ap.parse_args()


def source_hash():
    """Hash of the library's sources: ties a figure measured elsewhere (a counter pass) to the code it was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2309_06180_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload_name):
    """(HBM bytes per pa_decode launch, source) from the committed hardware-counter summary (FETCH_SIZE and
    WRITE_SIZE passes of rocprofv3, scaled by a plain copy of known size).  The summary names the hash of
    pa_decode's kernel file it was measured on: if that file has changed since, the figure is withheld."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "pa_decode_opt13b_hbm_traffic.md")
    try:
        kv = {}
        for line in open(path):
            if ":" in line and not line.startswith(("#", "|", " ")):
                k, _, val = line.partition(":")
                kv[k.strip()] = val.strip()
        kernel_file = os.path.join(ROOT, "paper_2309_06180_amd", "csrc", "pa_decode.hpp")
        now = hashlib.sha256(open(kernel_file, "rb").read()).hexdigest()[:16]
        if kv.get("workload") != workload_name:
            return None, "no counter summary for this workload"
        if kv.get("pa_decode_hpp_sha16") != now:
            return None, "profiles/pa_decode_opt13b_hbm_traffic.md was measured on another version of pa_decode.hpp"
        return int(kv["traffic_bytes_per_launch"]), ("profiles/pa_decode_opt13b_hbm_traffic.md (two rocprofv3 --pmc passes, "
                                                       "pa_decode.hpp sha16 %s; not measured by this run)" % now)
    except (OSError, KeyError, ValueError):
        return None, "no counter summary"


def _time_calls_us(fn, iters, torch, warmup=3, warm_ms=0.0):
    """Per-call GPU time of `fn` in us: an event pair around every call, on torch's current stream, which
    is the stream the library launches on.  Returns the list of the `iters` durations.  `warm_ms`: keep
    launching untimed for at least that long first (after seconds of host-only work the device's clocks
    take tens of milliseconds of load to come back up)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        starts[i].record()
        fn()
        ends[i].record()
    torch.cuda.synchronize()
    return [starts[i].elapsed_time(ends[i]) * 1e3 for i in range(iters)]


def _stats(us):
    srt = sorted(us)
    return {"mean_us": sum(us) / len(us), "median_us": srt[len(srt) // 2], "min_us": srt[0]}


def _time_us(fn, iters, torch):
    """Median per-call time in us (after 20 ms of untimed launches: see _time_calls_us)."""
    return _stats(_time_calls_us(fn, iters, torch, warm_ms=20.0))["median_us"]


def block_size_sweep(pa, W, np, torch, dev):
    """The paper's block-size ablation axis (Sec. 7.2) as a kernel microbenchmark: same sequences,
    same bytes, different B.  Caches are filled on the device (timing only)."""
    rng = np.random.default_rng(2000)
    lens = rng.integers(1, 2049, size=64)
    rows = []
    for B in (8, 16, 32, 64, 128):
        w = W.independent_sequences("opt13b_B%d" % B, "f16", 40, 128, B, lens, 2001)
        shape = (w.num_blocks, 40, B, 128)
        kc = torch.randn(shape, dtype=torch.float16, device=dev)
        vc = torch.randn(shape, dtype=torch.float16, device=dev)
        q = torch.randn((64, 40, 128), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        bt = torch.from_numpy(w.block_tables).to(dev)
        cl = torch.from_numpy(w.context_lens).to(dev)
        us = _time_us(lambda: pa.pa_decode(out, q, kc, vc, bt, cl, B, float(w.scale), w.max_context_len, 0, None),
                      100, torch)
        rows.append({"block_size": B, "us": us, "kv_GBps": w.kv_bytes_logical() / us / 1e3,
                     "frac_of_peak": w.kv_bytes_logical() / us / 1e3 / HBM_PEAK_GBPS,
                     "pool_blocks": w.num_blocks})
        del kc, vc
    print(json.dumps({"metric": "pa_decode_block_size_sweep", "workload": "OPT-13B shape, 64 seq, ctx U{1..2048}, fp16",
                      "rows": rows}))


def paging_overhead(pa, W, np, torch, dev):
    """The paper's kernel microbenchmark (Sec. 7.1) compares its kernel over scattered blocks with an
    attention kernel over contiguous K/V.  Here: the same kernel, the same 64 sequences and bytes, with
    (a) blocks placed at random in a pool 1.2x the need, (b) every sequence's blocks consecutive in the
    pool (what a contiguous per-sequence cache looks like through a block table), for B = 16 and 128.
    The table walk itself is part of both; the difference is what non-contiguity costs on this device."""
    rng = np.random.default_rng(2000)
    lens = rng.integers(1, 2049, size=64)
    H, D = 40, 128
    rows = []
    for B in (16, 128):
        w = W.independent_sequences("opt13b_B%d" % B, "f16", H, D, B, lens, 2001)
        nblk = (lens + B - 1) // B
        contiguous = np.full_like(w.block_tables, -1)
        start = 0
        for s_, nb in enumerate(nblk):
            contiguous[s_, :nb] = np.arange(start, start + nb)
            start += int(nb)
        kc = torch.randn((w.num_blocks, H, B, D), dtype=torch.float16, device=dev)
        vc = torch.randn_like(kc)
        q = torch.randn((64, H, D), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        cl = torch.from_numpy(w.context_lens).to(dev)
        row = {"block_size": B}
        for name, table in (("scattered", w.block_tables), ("contiguous", contiguous)):
            bt = torch.from_numpy(np.ascontiguousarray(table)).to(dev)
            us = min(_time_us(lambda: pa.pa_decode(out, q, kc, vc, bt, cl, B, float(w.scale), w.max_context_len,
                                                   0, None), 100, torch) for _ in range(3))
            row[name + "_us"] = us
            row[name + "_GBps"] = w.kv_bytes_logical() / us / 1e3
        row["scattered_over_contiguous"] = row["scattered_us"] / row["contiguous_us"]
        rows.append(row)
        del kc, vc
    print(json.dumps({"metric": "pa_decode_paging_overhead",
                      "workload": "OPT-13B shape, 64 seq, ctx U{1..2048}, fp16, best of 3 x 100 launches",
                      "rows": rows}))


def short_batches(pa, W, np, torch, dev):
    """Many short sequences per batch (Sec. 6.1: the second trace has prompts and outputs several times
    shorter than the first, and is served at batch sizes in the hundreds): per (sequence, head) only a
    few blocks, so launch planning and per-item overhead show.  OPT-13B shape, fp16, B = 16."""
    H, D, B = 40, 128, 16
    rows = []
    for S, top in ((128, 128), (256, 64), (256, 128), (256, 256), (512, 128), (1024, 128)):
        rng = np.random.default_rng(S + top)
        lens = rng.integers(1, top + 1, size=S)
        w = W.independent_sequences("short", "f16", H, D, B, lens, 1)
        kc = torch.randn((w.num_blocks, H, B, D), dtype=torch.float16, device=dev)
        vc = torch.randn_like(kc)
        q = torch.randn((S, H, D), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        bt = torch.from_numpy(w.block_tables).to(dev)
        cl = torch.from_numpy(w.context_lens).to(dev)
        us = _time_us(lambda: pa.pa_decode(out, q, kc, vc, bt, cl, B, float(w.scale), w.max_context_len, 0, None),
                      100, torch)
        kv = w.kv_bytes_logical()
        rows.append({"num_seqs": S, "max_len": top, "us": us, "kv_MB": kv / 1e6, "kv_GBps": kv / us / 1e3,
                     "frac_of_peak": kv / us / 1e3 / HBM_PEAK_GBPS, "query_tokens_per_s": S / us * 1e6,
                     "fits_infinity_cache": bool(kv < 256e6)})
        del kc, vc
    # one long sequence among short ones: the launch is planned from the longest context, so the short
    # items run in workgroups sized for the long one; compare with the two parts run on their own
    rng = np.random.default_rng(77)
    short = rng.integers(1, 65, size=255)
    mixed = {}
    for name, lens in (("mixed_1x2048_255xU64", np.concatenate([[2048], short])), ("long_only", np.array([2048])),
                       ("short_only", short)):
        S = len(lens)
        w = W.independent_sequences(name, "f16", H, D, B, lens, 2)
        kc = torch.randn((w.num_blocks, H, B, D), dtype=torch.float16, device=dev)
        vc = torch.randn_like(kc)
        q = torch.randn((S, H, D), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        bt = torch.from_numpy(w.block_tables).to(dev)
        cl = torch.from_numpy(w.context_lens).to(dev)
        ws = torch.empty(max(16, pa.pa_decode_workspace_bytes(S, H, D, B, w.max_context_len, pa.PA_PARTITION_AUTO)),
                         dtype=torch.uint8, device=dev)
        mixed[name] = {"us": _time_us(lambda: pa.pa_decode(out, q, kc, vc, bt, cl, B, float(w.scale), w.max_context_len,
                                                           pa.PA_PARTITION_AUTO, ws), 100, torch),
                       "kv_MB": w.kv_bytes_logical() / 1e6}
    mixed["mixed_over_sum_of_parts"] = mixed["mixed_1x2048_255xU64"]["us"] / (mixed["long_only"]["us"] + mixed["short_only"]["us"])
    print(json.dumps({"metric": "pa_decode_short_batches", "workload": "OPT-13B shape, fp16, B=16, ctx U{1..max_len}",
                      "rows": rows, "mixed_batch": mixed}))


def shared_prefix(pa, W, np, torch, dev):
    """Sec. 4.4 "Shared prefix" / Sec. 6.4: every request starts with the same prefix (the paper uses
    one example of 80 tokens and five examples of 341 tokens), stored once and mapped by all; each
    request adds its own tokens (here U{1..128}).  256 sequences, OPT-13B-like shape, fp16, B = 16."""
    S, H, D, B = 256, 40, 128, 16
    rows = []
    for prefix in (80, 341, 1024):
        w = W.config3(seed=6000 + prefix, num_groups=1, group=S, H=H, D=D, B=B, prompt_median=prefix,
                      prompt_sigma=1e-9, prompt_cap=prefix, max_out=128)
        kc = torch.randn((w.num_blocks, H, B, D), dtype=torch.float16, device=dev)
        vc = torch.randn_like(kc)
        q = torch.randn((S, H, D), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        bt = torch.from_numpy(w.block_tables).to(dev)
        cl = torch.from_numpy(w.context_lens).to(dev)
        ws = torch.empty(pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq), dtype=torch.uint8,
                         device=dev)
        mcl = w.max_context_len
        plain = _time_us(lambda: pa.pa_decode(out, q, kc, vc, bt, cl, B, float(w.scale), mcl, 0, None), 100, torch)
        sh = _time_us(lambda: pa.pa_decode_shared(out, q, kc, vc, bt, cl, B, float(w.scale), mcl, ws), 100, torch)
        rows.append({"prefix_tokens": prefix, "kv_MB_logical": w.kv_bytes_logical() / 1e6,
                     "kv_MB_unique": w.kv_bytes_unique() / 1e6, "pa_decode_us": plain, "pa_decode_shared_us": sh,
                     "query_tokens_per_s_plain": S / plain * 1e6, "query_tokens_per_s_shared": S / sh * 1e6})
        del kc, vc
    print(json.dumps({"metric": "pa_decode_shared_prefix", "workload": "256 seq share one prefix, + U{1..128} own "
                      "tokens each, 40 heads x 128, fp16, B=16", "rows": rows}))


def cfg5_full_step(pa, W, np, torch, dev, steps):
    """Config 5 at full size: 40 layers x 40 heads x 128, B = 32, bf16, 128 sequences in beam groups of 6,
    one beam-search step per iteration: pa_copy_blocks over all layers, then per layer
    pa_reshape_and_cache (T = 128) and decode.  Caches are filled on the device (timing only)."""
    L = 40
    w = W.config5()
    S, H, D, B, NB = w.num_seqs, w.num_heads, w.head_dim, w.block_size, w.num_blocks
    ks = [torch.randn((NB, H, B, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    vs = [torch.randn((NB, H, B, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    q = torch.randn((S, H, D), dtype=torch.bfloat16, device=dev)
    out = torch.empty_like(q)
    k_new = torch.randn((S, H, D), dtype=torch.bfloat16, device=dev)
    v_new = torch.randn((S, H, D), dtype=torch.bfloat16, device=dev)
    bt, cl = torch.from_numpy(w.block_tables).to(dev), torch.from_numpy(w.context_lens).to(dev)
    slots, pairs = torch.from_numpy(w.write_slots).to(dev), torch.from_numpy(w.copy_pairs).to(dev)
    mcl = w.max_context_len
    ws = torch.empty(max(pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq),
                         pa.pa_decode_workspace_bytes(S, H, D, B, mcl, pa.PA_PARTITION_AUTO), 16),
                     dtype=torch.uint8, device=dev)
    res = {"metric": "cfg5_full_step", "layers": L, "num_seqs": S, "pool_blocks": NB,
           "cache_GB": 2 * L * NB * H * B * D * 2 / 1e9, "copy_pairs": int(len(w.copy_pairs)),
           "kv_GB_logical_per_step": L * w.kv_bytes_logical() / 1e9,
           "kv_GB_unique_per_step": L * w.kv_bytes_unique() / 1e9}
    for name in ("plain", "shared", "shared_one_plan"):
        def step():
            pa.pa_copy_blocks(ks, vs, pairs)
            if name == "shared_one_plan":    # the tables are the same for every layer of the step
                pa.pa_shared_plan(bt, cl, H, D, B, NB, torch.bfloat16, mcl, ws)
            for l in range(L):
                pa.pa_reshape_and_cache(k_new, v_new, ks[l], vs[l], slots)
                if name == "shared":
                    pa.pa_decode_shared(out, q, ks[l], vs[l], bt, cl, B, float(w.scale), mcl, ws)
                elif name == "shared_one_plan":
                    pa.pa_decode_shared_planned(out, q, ks[l], vs[l], bt, cl, B, float(w.scale), mcl, ws)
                else:
                    pa.pa_decode(out, q, ks[l], vs[l], bt, cl, B, float(w.scale), mcl, pa.PA_PARTITION_AUTO, ws)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        res[name] = {"ms_per_step": ms, "query_tokens_per_s": S / ms * 1e3,
                     "logical_kv_GBps": L * w.kv_bytes_logical() / ms / 1e6,
                     "unique_kv_frac_of_peak": L * w.kv_bytes_unique() / ms / 1e6 / HBM_PEAK_GBPS}
    print(json.dumps(res))


def calibration_copy(pa, torch, dev, H=40, B=16, D=128, dtype=None):
    """A plain copy of known size (2048 whole blocks of K and of V, disjoint sources and destinations) for
    hardware-counter runs to scale FETCH_SIZE / WRITE_SIZE by."""
    dtype = dtype or torch.float16
    ck = torch.zeros((4096, H, B, D), dtype=dtype, device=dev)
    cv = torch.zeros((4096, H, B, D), dtype=dtype, device=dev)
    pr = torch.stack([torch.arange(0, 2048), torch.arange(2048, 4096)], dim=1).to(torch.int64).to(dev)
    pa.pa_copy_blocks([ck], [cv], pr)
    torch.cuda.synchronize()
    nbytes = 2 * 2048 * H * B * D * ck.element_size()
    return {"kernel": "copy_blocks_kernel", "bytes_read": nbytes, "bytes_written": nbytes}


def multi_query(pa, W, np, torch, dev, q_lens=(1, 4, 16, 64, 128, 256), calibrate=False):
    """pa_decode_multi at the OPT-13B layer shape: every sequence brings its last min(ctx, q_len) tokens as
    queries.  Per row a roofline: algorithmic bytes = K and V of every cached token once + q in + out;
    algorithmic flops = 4*D per (query, visible token) pair (both products, causal).  The bound is the one
    that takes longer at the published peaks (HBM 8 TB/s, dense f16 MFMA 2.5 PFLOP/s)."""
    rng = np.random.default_rng(2000)
    lens = rng.integers(1, 2049, size=64)
    w = W.independent_sequences("opt13b_multi", "f16", 40, 128, 16, lens, 2001)
    H, D, B = 40, 128, 16
    kc = torch.randn((w.num_blocks, H, B, D), dtype=torch.float16, device=dev)
    vc = torch.randn_like(kc)
    bt = torch.from_numpy(w.block_tables).to(dev)
    cl = torch.from_numpy(w.context_lens).to(dev)
    rows = []
    for qmax in q_lens:
        ql = np.minimum(lens, qmax)
        qs = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
        T = int(qs[-1])
        q = torch.randn((T, H, D), dtype=torch.float16, device=dev)
        out = torch.empty_like(q)
        dqs = torch.from_numpy(qs).to(dev)
        us = _time_us(lambda: pa.pa_decode_multi(out, q, kc, vc, bt, cl, dqs, qmax, B, float(w.scale),
                                                 w.max_context_len), 50, torch)
        algo_bytes = w.kv_bytes_logical() + 2 * T * H * D * 2
        pairs = int((ql * lens - ql * (ql - 1) // 2).sum())          # query i of q_len sees ctx - q_len + i + 1 tokens
        flops = 4 * D * pairs * H
        t_hbm, t_mfma = algo_bytes / (HBM_PEAK_GBPS * 1e9), flops / MFMA_F16_PEAK
        if t_hbm >= t_mfma:
            roof = {"bound": "hbm", "achieved": algo_bytes / us / 1e3, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
        else:
            roof = {"bound": "mfma", "achieved": flops / us / 1e6, "peak": MFMA_F16_PEAK / 1e12, "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        rows.append({"max_q_len": qmax, "query_tokens": T, "us": us, "query_tokens_per_s": T / us * 1e6,
                     "algorithmic_bytes": algo_bytes, "algorithmic_flops": flops,
                     "hbm_frac": algo_bytes / us / 1e3 / HBM_PEAK_GBPS, "mfma_frac": flops / us / 1e6 / (MFMA_F16_PEAK / 1e12),
                     "roofline": roof})
    q1 = torch.randn((64, H, D), dtype=torch.float16, device=dev)
    o1 = torch.empty_like(q1)
    us = _time_us(lambda: pa.pa_decode(o1, q1, kc, vc, bt, cl, B, float(w.scale), w.max_context_len, 0, None),
                  50, torch)
    res = {"metric": "pa_decode_multi", "workload": "OPT-13B shape, 64 seq, ctx U{1..2048}, fp16, "
           "q_len = min(ctx, max_q_len)", "rows": rows,
           "pa_decode_one_query": {"us": us, "kv_GBps": w.kv_bytes_logical() / us / 1e3}}
    if calibrate:
        res["calibration_copy"] = calibration_copy(pa, torch, dev)
    print(json.dumps(res))


def cache_ops(pa, np, torch, dev):
    """pa_reshape_and_cache from decode-step to prefill-sized token counts, pa_copy_blocks from a few
    pairs to thousands, at the OPT-13B layer shape; GB/s counts bytes read plus bytes written."""
    H, D, B, NB = 40, 128, 16, 8192
    kc = torch.zeros((NB, H, B, D), dtype=torch.float16, device=dev)
    vc = torch.zeros_like(kc)
    rng = np.random.default_rng(5)
    res = {"reshape_and_cache": [], "copy_blocks": []}
    for T in (64, 256, 1024, 4096, 16384, 65536):
        k = torch.randn((T, H, D), dtype=torch.float16, device=dev)
        v = torch.randn((T, H, D), dtype=torch.float16, device=dev)
        moved = 2 * 2 * T * H * D * 2
        # "scattered": every token in a slot of its own block, as the new tokens of T decoding sequences are;
        # "prompt": consecutive tokens fill consecutive slots of randomly placed blocks, as a prompt does (Sec. 4.3)
        scattered = rng.permutation(NB * B)[:T].astype(np.int64)
        blocks = rng.permutation(NB)[: (T + B - 1) // B].astype(np.int64)
        prompt = (blocks[:, None] * B + np.arange(B)[None, :]).reshape(-1)[:T]
        row = {"tokens": T}
        for name, sl in (("scattered", scattered), ("prompt", prompt)):
            slots = torch.from_numpy(np.ascontiguousarray(sl)).to(dev)
            us = _time_us(lambda: pa.pa_reshape_and_cache(k, v, kc, vc, slots), 50, torch)
            row[name + "_us"] = us
            row[name + "_GBps"] = moved / us / 1e3
        res["reshape_and_cache"].append(row)
    for N in (4, 41, 183, 1024, 4096):
        perm = rng.permutation(NB)
        pairs = torch.from_numpy(np.stack([perm[:N], perm[N:2 * N]], axis=1).astype(np.int64)).to(dev)
        us = _time_us(lambda: pa.pa_copy_blocks([kc], [vc], pairs), 50, torch)
        moved = 2 * 2 * N * H * B * D * 2
        res["copy_blocks"].append({"pairs": N, "us": us, "GBps": moved / us / 1e3})
    # swap to pinned host memory and back (one direction per call); GB/s counts bytes moved once
    res["swap_blocks"] = []
    NBH = 1024
    hk = torch.empty((NBH, H, B, D), dtype=torch.float16, pin_memory=True)
    hv = torch.empty((NBH, H, B, D), dtype=torch.float16, pin_memory=True)
    for N in (16, 128, 1024):
        gpu_ids, cpu_ids = rng.permutation(NB)[:N], rng.permutation(NBH)[:N]
        out_pairs = torch.from_numpy(np.stack([gpu_ids, cpu_ids], axis=1).astype(np.int64)).to(dev)
        in_pairs = torch.from_numpy(np.stack([cpu_ids, gpu_ids], axis=1).astype(np.int64)).to(dev)
        moved = 2 * N * H * B * D * 2
        us_out = _time_us(lambda: pa.pa_swap_blocks([kc], [vc], [hk], [hv], out_pairs), 10, torch)
        us_in = _time_us(lambda: pa.pa_swap_blocks([hk], [hv], [kc], [vc], in_pairs), 10, torch)
        res["swap_blocks"].append({"blocks": N, "out_us": us_out, "out_GBps": moved / us_out / 1e3,
                                   "in_us": us_in, "in_GBps": moved / us_in / 1e3})
    # for scale: the runtime's own device-to-device copy of one contiguous buffer of the size of 4096 block
    # pairs (K and V), same accounting (bytes read plus bytes written)
    n_elems = 2 * 4096 * H * B * D
    a = torch.empty(n_elems, dtype=torch.float16, device=dev)
    b = torch.empty_like(a)
    us = _time_us(lambda: b.copy_(a), 50, torch)
    res["reference_contiguous_device_copy"] = {"bytes_each_way": n_elems * 2, "us": us, "GBps": 2 * n_elems * 2 / us / 1e3}
    res["metric"] = "cache_ops_read_plus_write_GBps"
    res["shape"] = "H=40, D=128, B=16, fp16, pool of 8192 blocks"
    print(json.dumps(res))


def _to_host_storage(t, dtype, np, torch):
    t = t.cpu()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def others(pa, W, np, torch, dev, iters=30):
    """The other configurations of the benchmark spec, one decode launch each way, so that one run of the benchmark
    backs their figures too: config 3 (parallel sampling) and config 5 (beam search, one of its 40 layers)
    through pa_decode, pa_decode_shared (sharing plan built per call) and pa_decode_shared_planned (plan
    built once, as once per decoding step for all layers); config 4 in one pass and split at 512 tokens.
    Caches are filled on the device with seeded N(0,1) values (every slot, so the unused ones hold finite
    junk here; NaN in unused slots is what the tests cover).  Per entry: median / min / mean us over `iters`
    launches, algorithmic bytes (distinct K/V bytes once + q in + out), the fraction of the 8 TB/s HBM peak
    on those bytes, and the max abs error against the fp64 oracle on 32 sampled (sequence, head) rows."""
    import oracle
    from harness.workloads import storage_to_f64
    out = {}
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}
    for name, w, ways in (("cfg3_parallel_sampling", W.config3(), ("plain", "shared", "shared_planned")),
                          ("cfg4_opt66b_tp4", W.config4(), ("one_pass", "split_512")),
                          ("cfg5_beam_search_one_layer", W.config5(), ("plain", "shared", "shared_planned"))):
        S, H, D, B, NB = w.num_seqs, w.num_heads, w.head_dim, w.block_size, w.num_blocks
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed + 9)
        kc = torch.randn((NB, H, B, D), device=dev, dtype=tdt[w.dtype], generator=gen)
        vc = torch.randn((NB, H, B, D), device=dev, dtype=tdt[w.dtype], generator=gen)
        q = torch.randn((S, H, D), device=dev, dtype=tdt[w.dtype], generator=gen)
        bt, cl = torch.from_numpy(w.block_tables).to(dev), torch.from_numpy(w.context_lens).to(dev)
        mcl = w.max_context_len
        ws = torch.empty(max(pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq),
                             pa.pa_decode_workspace_bytes(S, H, D, B, mcl, 512), 16), dtype=torch.uint8, device=dev)
        rng = np.random.default_rng(w.seed + 1)
        rows = np.stack([rng.integers(0, S, size=32), rng.integers(0, H, size=32)], axis=1).astype(np.int32)
        hk, hv = _to_host_storage(kc, w.dtype, np, torch), _to_host_storage(vc, w.dtype, np, torch)
        ref = oracle.decode(_to_host_storage(q, w.dtype, np, torch), hk, hv, w.block_tables, w.context_lens, w.scale,
                            w.dtype, rows=rows)
        del hk, hv
        unique = w.kv_bytes_unique()
        algo = unique + 2 * S * H * D * w.elem_bytes
        entry = {"num_seqs": S, "context_tokens": int(w.context_lens.sum()), "kv_bytes_logical": w.kv_bytes_logical(),
                 "kv_bytes_unique": unique, "algorithmic_bytes": algo, "dtype": w.dtype, "calls": {}}
        for way in ways:
            o = torch.full_like(q, float("nan"))
            if way in ("plain", "one_pass"):
                fn = lambda: pa.pa_decode(o, q, kc, vc, bt, cl, B, float(w.scale), mcl, 0, None)
            elif way == "split_512":
                fn = lambda: pa.pa_decode(o, q, kc, vc, bt, cl, B, float(w.scale), mcl, 512, ws)
            elif way == "shared":
                fn = lambda: pa.pa_decode_shared(o, q, kc, vc, bt, cl, B, float(w.scale), mcl, ws)
            else:
                pa.pa_shared_plan(bt, cl, H, D, B, NB, tdt[w.dtype], mcl, ws)
                fn = lambda: pa.pa_decode_shared_planned(o, q, kc, vc, bt, cl, B, float(w.scale), mcl, ws)
            st = _stats(_time_calls_us(fn, iters, torch, warm_ms=50.0))
            torch.cuda.synchronize()
            got = storage_to_f64(_to_host_storage(o, w.dtype, np, torch), w.dtype)[rows[:, 0], rows[:, 1]]
            st["frac_of_hbm_peak"] = algo / st["median_us"] / 1e3 / HBM_PEAK_GBPS
            st["max_abs_err_sampled"] = float(np.abs(got - ref).max())
            entry["calls"][way] = st
        out[name] = entry
        del kc, vc
        torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2309_06180_amd as pa
    from harness import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    pa.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.block_size_sweep:
        return block_size_sweep(pa, W, np, torch, dev)
    if args.cache_ops:
        return cache_ops(pa, np, torch, dev)
    if args.paging_overhead:
        return paging_overhead(pa, W, np, torch, dev)
    if args.short_batches:
        return short_batches(pa, W, np, torch, dev)
    if args.shared_prefix:
        return shared_prefix(pa, W, np, torch, dev)
    if args.multi_query:
        return multi_query(pa, W, np, torch, dev, tuple(int(x) for x in args.q_lens.split(",")), args.calibrate_copy)
    if args.cfg5_full_step:
        return cfg5_full_step(pa, W, np, torch, dev, min(args.steps, 10))

    if args.others is None:
        args.others = args.workload == "cfg2" and args.decode == "plain" and args.partition is None
    make = {"cfg1": W.config1, "cfg2": W.config2, "cfg3": W.config3, "cfg4": W.config4,
            "cfg5": W.config5}[args.workload]
    w = make()
    v = W.make_values(w)
    # bring the cache to the state just before the step: everything but each
    # sequence's newest token is in place (host-side scatter of the inputs)
    kc, vc = v.k_cache, v.v_cache
    B = w.block_size
    if len(w.copy_pairs):
        kc[w.copy_pairs[:, 1]] = kc[w.copy_pairs[:, 0]]
        vc[w.copy_pairs[:, 1]] = vc[w.copy_pairs[:, 0]]
    step_set = set(w.step_slots.tolist())
    pre = np.array([i for i, s in enumerate(w.write_slots) if int(s) not in step_set], dtype=np.int64)
    if len(pre):
        sl = w.write_slots[pre]
        kc[sl // B, :, sl % B, :] = v.k_new[pre]
        vc[sl // B, :, sl % B, :] = v.v_new[pre]
    idx_of = {int(s): i for i, s in enumerate(w.write_slots)}
    step_idx = np.array([idx_of[int(s)] for s in w.step_slots], dtype=np.int64)

    def dev_t(a):
        t = torch.from_numpy(np.ascontiguousarray(a))
        if w.dtype == "bf16" and a.dtype == np.uint16:
            t = t.view(torch.bfloat16)
        return t.to(dev)

    # K and V of the layer are carved from one device allocation (K first, V at the next
    # 2 MiB boundary), as a serving engine lays out a layer's cache; --cache-allocation two
    # gives each its own (measured within 0.3% of each other at the OPT-13B shape).
    hk, hv = torch.from_numpy(np.ascontiguousarray(kc)), torch.from_numpy(np.ascontiguousarray(vc))
    if w.dtype == "bf16":
        hk, hv = hk.view(torch.bfloat16), hv.view(torch.bfloat16)
    nbytes = hk.numel() * hk.element_size()
    v_off = (nbytes + (1 << 21) - 1) >> 21 << 21
    if args.cache_allocation == "one":
        arena = torch.empty(v_off + nbytes, dtype=torch.uint8, device=dev)
        d_kc = arena[:nbytes].view(hk.dtype).view(hk.shape)
        d_vc = arena[v_off:v_off + nbytes].view(hk.dtype).view(hk.shape)
    else:
        d_kc = torch.empty(hk.shape, dtype=hk.dtype, device=dev)
        d_vc = torch.empty(hk.shape, dtype=hk.dtype, device=dev)
    d_kc.copy_(hk)
    d_vc.copy_(hv)
    del hk, hv
    d_q = dev_t(v.q)
    d_knew, d_vnew = dev_t(v.k_new[step_idx]), dev_t(v.v_new[step_idx])
    d_slots = dev_t(w.step_slots)
    d_bt, d_cl = dev_t(w.block_tables), dev_t(w.context_lens)
    d_pairs = torch.zeros((0, 2), dtype=torch.int64, device=dev)   # this step's copy-on-write list
    d_out = torch.empty_like(d_q)
    S, H, D = w.num_seqs, w.num_heads, w.head_dim
    mcl = w.max_context_len
    ps = pa.PA_PARTITION_AUTO if args.partition is None else args.partition
    shared = args.decode == "shared"
    ws_bytes = pa.pa_decode_shared_workspace_bytes(S, H, D, w.max_blocks_per_seq) if shared else \
        pa.pa_decode_workspace_bytes(S, H, D, B, mcl, ps)
    d_ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def decode():
        if shared:
            pa.pa_decode_shared(d_out, d_q, d_kc, d_vc, d_bt, d_cl, B, float(w.scale), mcl, d_ws)
        else:
            pa.pa_decode(d_out, d_q, d_kc, d_vc, d_bt, d_cl, B, float(w.scale), mcl, ps, d_ws)

    def step():
        pa.pa_copy_blocks([d_kc], [d_vc], d_pairs)
        pa.pa_reshape_and_cache(d_knew, d_vnew, d_kc, d_vc, d_slots)
        decode()

    kv_bytes = w.kv_bytes_logical()
    kv_unique = w.kv_bytes_unique()
    # algorithmic bytes of one decode launch: K and V of every cached token once,
    # plus q in and out once
    algo_bytes = kv_unique + 2 * S * H * D * w.elem_bytes

    calib = calibration_copy(pa, torch, dev, H, B, D, d_kc.dtype) if args.calibrate_copy else None

    run_step = step
    if args.launch == "graph":
        # launch-bound pieces (the cache write is a 5 us kernel) are replayed from a HIP graph
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # the same steps once more with an event pair around each: median and minimum next to the mean
    step_stats = _stats(_time_calls_us(run_step, args.steps, torch, warmup=2))

    # dominant kernel alone: one event pair on the launch stream around `steps` back-to-back decodes (the
    # mean that the roofline uses; it agrees with the profiler's kernel durations), then an event pair
    # around every call for the median and the minimum (each of those includes the pair's own ~2 us)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        decode()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        decode()
    e1.record()
    torch.cuda.synchronize()
    decode_ms = e0.elapsed_time(e1) / args.steps
    decode_stats = _stats(_time_calls_us(decode, args.steps, torch, warmup=2))

    # streaming-read ceiling of this device, for context
    probe = torch.empty(2 * 1024 ** 3, dtype=torch.uint8, device=dev)
    probe.random_(0, 255)
    sink = torch.zeros(65536, dtype=torch.int32, device=dev)
    for _ in range(3):
        pa.pa_stream_read(probe, sink)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(20):
        pa.pa_stream_read(probe, sink)
    e1.record()
    torch.cuda.synchronize()
    stream_gbps = probe.numel() / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e9
    del probe

    traffic, traffic_source = (profiled_traffic(w.name) if ps in (0, pa.PA_PARTITION_AUTO) and not shared
                               else (None, "no counter summary for this call"))
    result = {
        "metric": "pa_decode_kv_read_GBps",
        "value": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "accumulate": "f32", "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": S, "num_heads": H, "head_dim": D, "block_size": B,
                   "num_blocks": w.num_blocks, "context_tokens": int(w.context_lens.sum()),
                   "max_context_len": mcl, "partition_size": ps, "seed": w.seed, "decode": args.decode, "launch": args.launch, "cache_allocation": ("K and V of the layer in one device allocation" if args.cache_allocation == "one" else "K and V in separate device allocations"),
                   "kv_bytes_logical": kv_bytes, "kv_bytes_unique": kv_unique,
                   "step": "copy_blocks(0 pairs)+reshape_and_cache(T=S)+pa_decode"},
        "query_tokens_per_s": S / (ms_per_step * 1e-3),
        "pct_of_hbm_peak": 100.0 * kv_unique / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_us_per_call_events": step_stats,
        "decode_only_ms": decode_ms,
        "decode_only_us_per_call_events": decode_stats,
        "stream_read_GBps": stream_gbps,
        "roofline": {"bound": "hbm", "achieved": algo_bytes / (decode_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": algo_bytes / (decode_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "pa_shared_fused_kernel" if shared else "pa_decode_kernel",
                     "algorithmic_bytes_per_launch": algo_bytes},
        "library_source_sha16": source_hash(),
    }

    if calib:
        result["calibration_copy"] = calib

    if not args.no_check:
        # sampled parity at full size, in the configuration that was timed
        import oracle
        from harness.workloads import storage_to_f64
        rng = np.random.default_rng(1)
        rows = np.stack([rng.integers(0, S, size=48), rng.integers(0, H, size=48)], axis=1).astype(np.int32)
        torch.cuda.synchronize()
        hk = d_kc.cpu()
        hv = d_vc.cpu()
        if w.dtype == "bf16":
            hk, hv = hk.view(torch.int16), hv.view(torch.int16)
        hk, hv = hk.numpy(), hv.numpy()
        if w.dtype == "bf16":
            hk, hv = hk.view(np.uint16), hv.view(np.uint16)
        ref = oracle.decode(v.q, hk, hv, w.block_tables, w.context_lens, w.scale, w.dtype, rows=rows)
        ho = d_out.cpu()
        ho = ho.view(torch.int16).numpy().view(np.uint16) if w.dtype == "bf16" else ho.numpy()
        got = storage_to_f64(ho, w.dtype)[rows[:, 0], rows[:, 1]]
        result["max_abs_err_sampled"] = float(np.abs(got - ref).max())

        if not args.no_cpu_baseline:
            # the oracle as it stands on the host cores: one full pass over the same batch
            # full passes over the same batch until about 3 s of wall time (tens of core-seconds)
            passes, t0 = 0, time.perf_counter()
            while passes < 1 or time.perf_counter() - t0 < 3.0:
                _, used = oracle.decode(v.q, hk, hv, w.block_tables, w.context_lens, w.scale, w.dtype,
                                        threads=0, return_threads=True)
                passes += 1
            cdt = (time.perf_counter() - t0) / passes
            # one thread: every 16th (sequence, head) row of the same batch, scaled to the whole
            all_rows = np.stack(np.meshgrid(np.arange(S), np.arange(H), indexing="ij"), axis=-1).reshape(-1, 2)
            sub = np.ascontiguousarray(all_rows[::16]).astype(np.int32)
            t0 = time.perf_counter()
            oracle.decode(v.q, hk, hv, w.block_tables, w.context_lens, w.scale, w.dtype, rows=sub, threads=1)
            one = time.perf_counter() - t0
            sub_bytes = int(w.context_lens[sub[:, 0]].astype(np.int64).sum()) * D * w.elem_bytes * 2
            result["cpu_baseline"] = {"value": kv_bytes / cdt / 1e9, "unit": "GB/s", "cores": int(used),
                                      "kind": "oracle",
                                      "sample": "%d full pa_decode passes over the same batch (%d sequences x %d "
                                                "heads, %d cached tokens), %.2f s each"
                                                % (passes, S, H, int(w.context_lens.sum()), cdt),
                                      "query_tokens_per_s": S / cdt,
                                      "one_thread": {"value": sub_bytes / one / 1e9, "unit": "GB/s", "cores": 1,
                                                     "sample": "every 16th (sequence, head) row of the same batch, "
                                                               "%.2f s" % one}}
    if args.others:
        del d_kc, d_vc
        if args.cache_allocation == "one":
            del arena
        torch.cuda.empty_cache()
        result["others"] = others(pa, W, np, torch, dev)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
