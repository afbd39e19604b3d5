"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU.  No kernel runs here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2309_06180_amd import binding, build
    if not os.path.exists(build.LIB):
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pa_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2309_06180_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.pa_version() >= 1
    seen = {lib.pa_status_string(c) for c in range(9)}
    assert len(seen) == 9 and all(s for s in seen)


def test_workspace_size_formula(lib):
    # S*H*ceil(max_ctx/PS)*(D+2) floats; zero for one pass
    assert lib.pa_decode_workspace_bytes(128, 18, 128, 16, 2048, 512) == 128 * 18 * 4 * 130 * 4
    assert lib.pa_decode_workspace_bytes(128, 18, 128, 16, 2048, 0) == 0
    assert lib.pa_decode_workspace_bytes(3, 2, 64, 16, 100, 64) == 3 * 2 * 2 * 66 * 4


def test_argument_errors_need_no_gpu(lib):
    buf = ctypes.create_string_buffer(64 + 16)
    p = (ctypes.addressof(buf) + 15) & ~15       # a 16-byte aligned non-null address, never dereferenced
    f32, f16 = 0, 1

    def decode(**kw):
        a = dict(out=p, q=p, k=p, v=p, bt=p, mb=8, cl=p, S=2, H=2, D=128, B=16, NB=4, dt=f16, scale=1.0,
                 mcl=100, ps=0, ws=None, wsb=0)
        a.update(kw)
        return lib.pa_decode(a["out"], a["q"], a["k"], a["v"], a["bt"], a["mb"], a["cl"], a["S"], a["H"],
                             a["D"], a["B"], a["NB"], a["dt"], a["scale"], a["mcl"], a["ps"], a["ws"],
                             a["wsb"], None)

    assert decode(S=0) == 0                       # empty batch: ok, nothing launched
    assert decode(q=None) == 1
    assert decode(H=0) == 2
    assert decode(mcl=8 * 16 + 1) == 2            # longer than the table can address
    assert decode(ps=24) == 2                     # not a multiple of the block size
    assert decode(D=96) == 3
    assert decode(B=12) == 3
    assert decode(dt=9) == 3
    assert decode(dt=f32, D=32) == 3
    assert decode(out=p + 4) == 4
    assert decode(ps=32, ws=None) == 5
    assert decode(ps=32, ws=p, wsb=8) == 5

    assert lib.pa_reshape_and_cache(p, p, p, p, p, 0, 2, 128, 16, 4, f16, None) == 0
    assert lib.pa_reshape_and_cache(None, p, p, p, p, 3, 2, 128, 16, 4, f16, None) == 1
    assert lib.pa_reshape_and_cache(p, p, p, p, p, 3, 2, 128, 0, 4, f16, None) == 2
    assert lib.pa_reshape_and_cache(p, p + 2, p, p, p, 3, 2, 128, 16, 4, f16, None) == 4

    arr = (ctypes.c_void_p * 1)(p)
    assert lib.pa_copy_blocks(arr, arr, 1, p, 0, 2, 128, 16, 4, f16, None) == 0
    assert lib.pa_copy_blocks(None, arr, 1, p, 2, 2, 128, 16, 4, f16, None) == 1
    assert lib.pa_copy_blocks(arr, arr, 0, p, 2, 2, 128, 16, 4, f16, None) == 2
    bad = (ctypes.c_void_p * 1)(p + 8)
    assert lib.pa_copy_blocks(bad, arr, 1, p, 2, 2, 128, 16, 4, f16, None) == 4

    assert lib.pa_stream_read(None, 1024, p, None) == 1
    assert lib.pa_stream_read(p, 1000, p, None) == 2


def test_argument_errors_of_the_wider_entry_points(lib):
    buf = ctypes.create_string_buffer(64 + 16)
    p = (ctypes.addressof(buf) + 15) & ~15       # aligned, non-null, never dereferenced
    f32, f16 = 0, 1

    def shared(fn=None, **kw):
        a = dict(out=p, q=p, k=p, v=p, bt=p, mb=8, cl=p, S=2, H=2, D=128, B=16, NB=4, dt=f16, scale=1.0,
                 mcl=100, ws=p, wsb=1 << 20)
        a.update(kw)
        return (fn or lib.pa_decode_shared)(a["out"], a["q"], a["k"], a["v"], a["bt"], a["mb"], a["cl"], a["S"],
                                            a["H"], a["D"], a["B"], a["NB"], a["dt"], a["scale"], a["mcl"],
                                            a["ws"], a["wsb"], None)

    need = lib.pa_decode_shared_workspace_bytes(2, 2, 128, 8)
    # group table (6S + 2 words, rounded up to four, + S items of four words) + one 16-byte tile entry per table entry
    assert need == (16 + 4 * 2) * 4 + 2 * 8 * 16
    assert lib.pa_decode_shared_workspace_bytes(5, 2, 128, 3) == (36 + 4 * 5) * 4 + 5 * 3 * 16
    for fn in (lib.pa_decode_shared, lib.pa_decode_shared_planned):
        assert shared(fn, S=0) == 0
        assert shared(fn, k=None) == 1
        assert shared(fn, mb=0) == 2
        assert shared(fn, mcl=8 * 16 + 1) == 2
        assert shared(fn, D=96) == 3
        assert shared(fn, v=p + 8) == 4
        assert shared(fn, ws=None) == 5
        assert shared(fn, wsb=need - 1) == 5
        assert shared(fn, ws=p + 4) == 4

    def plan(**kw):
        a = dict(bt=p, mb=8, cl=p, S=2, H=2, D=128, B=16, NB=4, dt=f16, mcl=100, ws=p, wsb=1 << 20)
        a.update(kw)
        return lib.pa_shared_plan(a["bt"], a["mb"], a["cl"], a["S"], a["H"], a["D"], a["B"], a["NB"], a["dt"],
                                  a["mcl"], a["ws"], a["wsb"], None)

    assert plan(S=0) == 0
    assert plan(bt=None) == 1
    assert plan(B=0) == 2
    assert plan(dt=7) == 3
    assert plan(wsb=need - 1) == 5
    assert plan(dt=f32, D=64) == 0               # no several-query kernel for this shape: nothing to plan

    def multi(**kw):
        a = dict(out=p, q=p, k=p, v=p, bt=p, mb=8, cl=p, qs=p, S=2, mq=4, H=2, D=128, B=16, NB=4, dt=f16,
                 scale=1.0, mcl=100)
        a.update(kw)
        return lib.pa_decode_multi(a["out"], a["q"], a["k"], a["v"], a["bt"], a["mb"], a["cl"], a["qs"], a["S"],
                                   a["mq"], a["H"], a["D"], a["B"], a["NB"], a["dt"], a["scale"], a["mcl"], None)

    assert multi(S=0) == 0
    assert multi(mq=0) == 0                      # no query rows: nothing to do
    assert multi(qs=None) == 1
    assert multi(mq=-1) == 2
    assert multi(dt=f32) == 3                    # two-byte types only
    assert multi(D=64) == 3
    assert multi(B=8) == 3
    assert multi(q=p + 2) == 4

    arr = (ctypes.c_void_p * 1)(p)
    swap = lambda sk=arr, L=1, n=2, nbs=4, nbd=4, pairs=p: lib.pa_swap_blocks(sk, arr, arr, arr, L, pairs, n, 2, 128,
                                                                               16, nbs, nbd, f16, None)
    assert swap(n=0) == 0
    assert swap(sk=None) == 1
    assert swap(pairs=None) == 1
    assert swap(L=0) == 2
    assert swap(nbd=0) == 2
