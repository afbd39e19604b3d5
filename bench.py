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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one pa_copy_blocks of known size (a plain copy kernel that "
                         "hardware-counter runs use to scale FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-check", action="store_true")
    return ap.parse_args()


def profiled_traffic(workload_name):
    """HBM bytes per pa_decode launch from the committed hardware-counter summary (FETCH_SIZE and
    WRITE_SIZE passes of rocprofv3, scaled by a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", "pa_decode_opt13b_hbm_traffic.md")
    try:
        kv = {}
        for line in open(path):
            if ":" in line and not line.startswith(("#", "|", " ")):
                k, _, val = line.partition(":")
                kv[k.strip()] = val.strip()
        if kv.get("workload") == workload_name:
            return int(kv["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


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

    d_kc, d_vc, d_q = dev_t(kc), dev_t(vc), dev_t(v.q)
    d_knew, d_vnew = dev_t(v.k_new[step_idx]), dev_t(v.v_new[step_idx])
    d_slots = dev_t(w.step_slots)
    d_bt, d_cl = dev_t(w.block_tables), dev_t(w.context_lens)
    d_pairs = torch.zeros((0, 2), dtype=torch.int64, device=dev)   # this step's copy-on-write list
    d_out = torch.empty_like(d_q)
    S, H, D = w.num_seqs, w.num_heads, w.head_dim
    mcl = w.max_context_len
    ps = pa.PA_PARTITION_AUTO if args.partition is None else args.partition
    shared = args.decode == "shared"
    ws_bytes = pa.pa_decode_shared_workspace_bytes(S, H, D) if shared else \
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

    calib = None
    if args.calibrate_copy:
        # plain copy of known size: 2048 whole blocks of K and of V, disjoint sources and destinations
        ck = torch.zeros((4096, H, B, D), dtype=d_kc.dtype, device=dev)
        cv = torch.zeros((4096, H, B, D), dtype=d_kc.dtype, device=dev)
        pr = torch.stack([torch.arange(0, 2048), torch.arange(2048, 4096)], dim=1).to(torch.int64).to(dev)
        pa.pa_copy_blocks([ck], [cv], pr)
        torch.cuda.synchronize()
        calib = {"kernel": "copy_blocks_kernel", "bytes_read": 2 * 2048 * H * B * D * w.elem_bytes,
                 "bytes_written": 2 * 2048 * H * B * D * w.elem_bytes}
        del ck, cv

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # dominant kernel alone: events on the launch stream around back-to-back decodes
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

    result = {
        "metric": "pa_decode_kv_read_GBps",
        "value": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": S, "num_heads": H, "head_dim": D, "block_size": B,
                   "num_blocks": w.num_blocks, "context_tokens": int(w.context_lens.sum()),
                   "max_context_len": mcl, "partition_size": ps, "seed": w.seed, "decode": args.decode,
                   "kv_bytes_logical": kv_bytes, "kv_bytes_unique": kv_unique,
                   "step": "copy_blocks(0 pairs)+reshape_and_cache(T=S)+pa_decode"},
        "query_tokens_per_s": S / (ms_per_step * 1e-3),
        "pct_of_hbm_peak": 100.0 * kv_unique / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "decode_only_ms": decode_ms,
        "stream_read_GBps": stream_gbps,
        "roofline": {"bound": "hbm", "achieved": algo_bytes / (decode_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": algo_bytes / (decode_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": profiled_traffic(w.name) if ps in (0, pa.PA_PARTITION_AUTO) and not shared else None,
                     "kernel": "pa_decode_kernel",
                     "algorithmic_bytes_per_launch": algo_bytes},
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
            result["cpu_baseline"] = {"value": kv_bytes / cdt / 1e9, "unit": "GB/s", "cores": int(used),
                                      "kind": "oracle",
                                      "sample": "%d full pa_decode passes over the same batch (%d sequences x %d "
                                                "heads, %d cached tokens), %.2f s each"
                                                % (passes, S, H, int(w.context_lens.sum()), cdt),
                                      "query_tokens_per_s": S / cdt}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
