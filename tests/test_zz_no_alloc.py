"""pa_decode_static (split-context partials in the library's static device array) against
pa_decode with a caller workspace and against the fp64 oracle, straight through the C ABI.
Two calls in a row on the same GPU, the second on a smaller batch, so that what the first
call left in the array must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from harness import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import TOL, DeviceWorkload, gpu_cache_ops, oracle_cache_ops, out_to_f64, to_np  # noqa: E402

DT = {"f32": 0, "f16": 1, "bf16": 2}


@pytest.fixture(scope="module")
def lib():
    import paper_2309_06180_amd as pa
    return pa.load_library()


def prepared(pa, w):
    v = W.make_values(w)
    dw = DeviceWorkload(w, v)
    gpu_cache_ops(pa, dw)
    kc, vc = oracle_cache_ops(w, v)
    ref = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    return dw, ref


def call_both(lib, dw, ps):
    """(static, with workspace): outputs of the two entry points for one partition size."""
    w = dw.w
    S, H, D, B = w.num_seqs, w.num_heads, w.head_dim, w.block_size
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    common = (ctypes.c_void_p(dw.q.data_ptr()), ctypes.c_void_p(dw.k_cache.data_ptr()),
              ctypes.c_void_p(dw.v_cache.data_ptr()), ctypes.c_void_p(dw.block_tables.data_ptr()),
              w.max_blocks_per_seq, ctypes.c_void_p(dw.context_lens.data_ptr()), S, H, D, B, w.num_blocks,
              DT[w.dtype], ctypes.c_float(w.scale), w.max_context_len, ps)
    need = lib.pa_decode_workspace_bytes(S, H, D, B, w.max_context_len, ps)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    a = torch.full_like(dw.q, float("nan"))
    b = torch.full_like(dw.q, float("nan"))
    assert lib.pa_decode_static(ctypes.c_void_p(a.data_ptr()), *common, stream) == 0
    assert lib.pa_decode(ctypes.c_void_p(b.data_ptr()), *common, ctypes.c_void_p(ws.data_ptr()),
                         ctypes.c_size_t(need), stream) == 0
    torch.cuda.synchronize()
    return a, b


def test_static_scratch_matches_workspace_call_twice_in_a_row(lib):
    import paper_2309_06180_amd as pa
    big = W.config4(seed=71, num_seqs=40, H=6)                    # bf16, contexts up to 2048
    small = W.independent_sequences("small", "bf16", 3, 128, 16, np.array([700, 5, 0, 130, 64, 1]), seed=72)
    for w, sizes in ((big, (512, 256)), (small, (64, 512, -1, 0))):
        dw, ref = prepared(pa, w)
        for ps in sizes:
            a, b = call_both(lib, dw, ps)
            assert np.array_equal(to_np(a, w.dtype), to_np(b, w.dtype)), "%s ps=%d: entry points differ" % (w.name, ps)
            err = float(np.abs(out_to_f64(a, w.dtype) - ref).max())
            assert err <= TOL[w.dtype], "%s ps=%d: max abs err %g" % (w.name, ps, err)


def test_static_scratch_limit_is_refused(lib):
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    p = ctypes.c_void_p(buf.data_ptr())
    # 4096 x 64 x 128-token partitions of 16K tokens: 4096*64*128*(128+2)*4 B, far over 16 MiB
    st = lib.pa_decode_static(p, p, p, p, p, 1024, p, 4096, 64, 128, 16, 8, 1, ctypes.c_float(1.0), 16384, 128, None)
    assert st == 8 and b"static" in lib.pa_status_string(st)
