"""Pins for the CPU oracle: closed forms, invariants, brute force and library
cross-checks that hold whatever the implementation, so that a dropped term, a
wrong sign or index, or a transposed operand in oracle/pa_oracle.c fails here.

None of these tests touches the GPU library.
"""
import math
import os

import numpy as np
import pytest

import oracle
from harness import workloads as W
from harness.blocks import BlockManager

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# helpers: tiny paged caches built by hand (independent of harness.workloads)
# ---------------------------------------------------------------------------
def paged_from_contiguous(K, V, B, NB, rng, dtype="f32", fill=np.nan):
    """K, V: lists (per sequence) of [n][H][D] float32 -> caches [NB][H][B][D], tables, lens."""
    H, D = K[0].shape[1:]
    st = W.storage_np_dtype(dtype)
    kc = np.full((NB, H, B, D), fill, dtype=np.float32)
    vc = np.full((NB, H, B, D), fill, dtype=np.float32)
    ids = list(rng.permutation(NB))
    mb = max((k.shape[0] + B - 1) // B for k in K) + 1
    tables = np.full((len(K), mb), -1, dtype=np.int32)
    lens = np.array([k.shape[0] for k in K], dtype=np.int32)
    for s, (k, v) in enumerate(zip(K, V)):
        for t in range(k.shape[0]):
            if t % B == 0:
                tables[s, t // B] = ids.pop()
            pb = tables[s, t // B]
            kc[pb, :, t % B, :] = k[t]
            vc[pb, :, t % B, :] = v[t]
    return W.to_storage(kc, dtype), W.to_storage(vc, dtype), tables, lens


def python_attention(q, K, V, scale):
    """Eq. (attention-layer) of Sec. 2.1 with math.fsum / math.exp on Python floats."""
    n, D = len(K), len(q)
    x = [scale * math.fsum(q[d] * K[t][d] for d in range(D)) for t in range(n)]
    m = max(x)
    e = [math.exp(v - m) for v in x]
    Z = math.fsum(e)
    return [math.fsum(e[t] * V[t][d] for t in range(n)) / Z for d in range(D)]


def rand_seqs(rng, lens, H, D):
    K = [rng.standard_normal((n, H, D)).astype(np.float32) for n in lens]
    V = [rng.standard_normal((n, H, D)).astype(np.float32) for n in lens]
    q = rng.standard_normal((len(lens), H, D)).astype(np.float32)
    return q, K, V


# ---------------------------------------------------------------------------
def test_brute_force_tiny():
    rng = np.random.default_rng(1)
    lens, H, D, B = [5, 1, 3], 2, 3, 2          # H != B != D on purpose
    q, K, V = rand_seqs(rng, lens, H, D)
    kc, vc, tables, cl = paged_from_contiguous(K, V, B, 9, rng)
    scale = np.float32(0.37)
    out = oracle.decode(q, kc, vc, tables, cl, scale, "f32")
    for s in range(len(lens)):
        for h in range(H):
            ref = python_attention([float(x) for x in q[s, h]],
                                   [[float(x) for x in K[s][t, h]] for t in range(lens[s])],
                                   [[float(x) for x in V[s][t, h]] for t in range(lens[s])],
                                   float(scale))
            assert np.allclose(out[s, h], ref, rtol=0, atol=1e-14)


def test_against_torch_float64_softmax():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    lens, H, D, B = [37, 64, 1, 17], 3, 8, 16
    q, K, V = rand_seqs(rng, lens, H, D)
    kc, vc, tables, cl = paged_from_contiguous(K, V, B, 12, rng)
    scale = np.float32(1 / math.sqrt(D))
    out = oracle.decode(q, kc, vc, tables, cl, scale, "f32")
    for s, n in enumerate(lens):
        qt = torch.from_numpy(q[s]).double()                  # [H][D]
        Kt = torch.from_numpy(K[s]).double().permute(1, 0, 2)  # [H][n][D]
        Vt = torch.from_numpy(V[s]).double().permute(1, 0, 2)
        a = torch.softmax(torch.einsum("hd,hnd->hn", qt, Kt) * float(scale), dim=-1)
        ref = torch.einsum("hn,hnd->hd", a, Vt).numpy()
        assert np.abs(out[s] - ref).max() < 1e-13


def test_paged_equals_unpaged_and_permutation_invariant():
    # Sec. 4.1: blocks may sit anywhere in physical memory without changing the result
    rng = np.random.default_rng(3)
    lens, H, D, B = [50, 7, 33], 2, 16, 8
    q, K, V = rand_seqs(rng, lens, H, D)
    kc, vc, tables, cl = paged_from_contiguous(K, V, B, 20, rng)
    out = oracle.decode(q, kc, vc, tables, cl, 0.25, "f32")
    # unpaged: one block as large as the longest sequence, identity table
    big = 64
    kc1, vc1, t1, cl1 = paged_from_contiguous(K, V, big, 3, np.random.default_rng(0))
    out1 = oracle.decode(q, kc1, vc1, t1, cl1, 0.25, "f32")
    assert np.array_equal(out, out1)
    # relabel physical blocks with a permutation, moving the data along
    perm = rng.permutation(20)
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    t2 = tables.copy()
    valid = tables >= 0
    t2[valid] = perm[tables[valid]]
    out2 = oracle.decode(q, kc2, vc2, t2, cl, 0.25, "f32")
    assert np.array_equal(out, out2)


def test_context_len_one_returns_value():
    rng = np.random.default_rng(4)
    for dtype in ("f32", "f16", "bf16"):
        q, K, V = rand_seqs(rng, [1, 1], 3, 8)
        kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 5, rng, dtype)
        qs = W.to_storage(q, dtype)
        out = oracle.decode(qs, kc, vc, tables, cl, 0.5, dtype)
        for s in range(2):
            want = W.storage_to_f64(W.to_storage(V[s][0], dtype), dtype)
            assert np.array_equal(out[s], want)


def test_identical_keys_give_mean_of_values():
    rng = np.random.default_rng(5)
    n, H, D = 23, 2, 8
    q, K, V = rand_seqs(rng, [n], H, D)
    K[0][:] = K[0][0]
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 8, rng)
    out = oracle.decode(q, kc, vc, tables, cl, 0.3, "f32")
    assert np.abs(out[0] - V[0].astype(np.float64).mean(axis=0)).max() < 1e-14


def test_zero_scale_gives_mean_of_values():
    rng = np.random.default_rng(6)
    q, K, V = rand_seqs(rng, [11], 2, 4)
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 4, rng)
    out = oracle.decode(q, kc, vc, tables, cl, 0.0, "f32")
    assert np.abs(out[0] - V[0].astype(np.float64).mean(axis=0)).max() < 1e-14


def test_dominant_key_selects_its_value():
    rng = np.random.default_rng(7)
    n, H, D = 19, 2, 8
    q, K, V = rand_seqs(rng, [n], H, D)
    star = 13
    for h in range(H):
        K[0][:, h] *= 0.01
        K[0][star, h] = q[0, h] * 200.0 / float(q[0, h] @ q[0, h])   # logit 200*scale above the rest
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 8, rng)
    out = oracle.decode(q, kc, vc, tables, cl, 1.0, "f32")
    assert np.abs(out[0] - V[0][star].astype(np.float64)).max() < 1e-12


def test_two_token_closed_form():
    # n = 2: o = sigmoid(x0 - x1) v0 + sigmoid(x1 - x0) v1 -- sign and K/V-role errors show here
    q = np.array([[[1.0, 2.0]]], dtype=np.float32)
    K = [np.array([[[0.5, -1.0]], [[-0.25, 0.75]]], dtype=np.float32)]
    V = [np.array([[[10.0, 0.0]], [[0.0, -4.0]]], dtype=np.float32)]
    kc, vc, tables, cl = paged_from_contiguous(K, V, 2, 1, np.random.default_rng(0))
    scale = 0.5
    x0, x1 = scale * (0.5 - 2.0), scale * (-0.25 + 1.5)
    a0 = 1.0 / (1.0 + math.exp(x1 - x0))
    out = oracle.decode(q, kc, vc, tables, cl, scale, "f32")
    assert np.allclose(out[0, 0], [10.0 * a0, -4.0 * (1 - a0)], rtol=0, atol=1e-15)


def test_logit_shift_invariance():
    rng = np.random.default_rng(8)
    q, K, V = rand_seqs(rng, [40], 1, 4)
    q = np.round(q * 4) / 4                       # exact in fp32 after the shift below
    K[0] = np.round(K[0] * 4) / 4
    kc, vc, tables, cl = paged_from_contiguous(K, V, 8, 6, rng)
    out = oracle.decode(q.astype(np.float32), kc, vc, tables, cl, 0.5, "f32")
    # adding a vector orthogonal-free multiple of e_0 to every key shifts all logits by c*q_0
    K2 = [K[0].copy()]
    K2[0][:, :, 0] += 8.0
    kc2, vc2, t2, cl2 = paged_from_contiguous(K2, V, 8, 6, np.random.default_rng(8 + 1))
    out2 = oracle.decode(q.astype(np.float32), kc2, vc2, t2, cl2, 0.5, "f32")
    assert np.abs(out - out2).max() < 1e-13


def test_query_and_scale_trade_exactly():
    rng = np.random.default_rng(9)
    q, K, V = rand_seqs(rng, [9, 30], 2, 4)
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 12, rng)
    a = oracle.decode(q, kc, vc, tables, cl, 0.25, "f32")
    b = oracle.decode((q * 2).astype(np.float32), kc, vc, tables, cl, 0.125, "f32")
    assert np.array_equal(a, b)


def test_shared_blocks_equal_private_copies():
    # Sec. 4.4: the kernel only sees physical ids; sharing by reference must be invisible
    rng = np.random.default_rng(10)
    H, D, B, NB = 2, 8, 4, 24
    mgr = BlockManager(NB, B, order=rng.permutation(NB))
    parent = mgr.allocate(10)
    kids = [parent, mgr.fork(parent), mgr.fork(parent)]
    kc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f32")
    vc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "f32")
    for k in kids:
        for _ in range(int(rng.integers(1, 9))):
            mgr.append(k)
    oracle.copy_blocks([kc], [vc], np.array(mgr.take_copies(), dtype=np.int64), "f32")
    mb = max(len(k.blocks) for k in kids)
    tables = np.full((3, mb), -1, dtype=np.int32)
    for i, k in enumerate(kids):
        tables[i, :len(k.blocks)] = k.blocks
    cl = np.array([k.length for k in kids], dtype=np.int32)
    q = rng.standard_normal((3, H, D)).astype(np.float32)
    shared = oracle.decode(q, kc, vc, tables, cl, 0.35, "f32")
    assert len(set(tables[:, 0])) == 1            # block 0 really is shared
    # private copies: every sequence gets its own physical blocks in a bigger pool
    kc2 = np.full((3 * mb, H, B, D), np.nan, dtype=np.float32)
    vc2 = np.full_like(kc2, np.nan)
    t2 = np.full_like(tables, -1)
    nxt = 0
    for i, k in enumerate(kids):
        for j, pb in enumerate(k.blocks):
            kc2[nxt], vc2[nxt], t2[i, j] = kc[pb], vc[pb], nxt
            nxt += 1
    private = oracle.decode(q, kc2, vc2, t2, cl, 0.35, "f32")
    assert np.array_equal(shared, private)


def test_poison_outside_context_is_ignored():
    rng = np.random.default_rng(11)
    q, K, V = rand_seqs(rng, [5, 12], 2, 4)
    kc, vc, tables, cl = paged_from_contiguous(K, V, 8, 6, rng, fill=np.nan)
    kz, vz, tz, _ = paged_from_contiguous(K, V, 8, 6, np.random.default_rng(11 + 0), fill=0.0)
    out = oracle.decode(q, kc, vc, tables, cl, 0.5, "f32")
    assert np.isfinite(out).all()
    # shortening the context must drop exactly the trailing tokens
    cl2 = np.array([3, 12], dtype=np.int32)
    K3, V3 = [K[0][:3], K[1]], [V[0][:3], V[1]]
    k3, v3, t3, c3 = paged_from_contiguous(K3, V3, 8, 6, np.random.default_rng(5))
    assert np.array_equal(oracle.decode(q, kc, vc, tables, cl2, 0.5, "f32"),
                          oracle.decode(q, k3, v3, t3, c3, 0.5, "f32"))


def test_context_len_zero_gives_zero_row():
    rng = np.random.default_rng(12)
    q, K, V = rand_seqs(rng, [4, 6], 1, 4)
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 4, rng)
    cl[0] = 0
    out = oracle.decode(q, kc, vc, tables, cl, 0.5, "f32")
    assert np.array_equal(out[0], np.zeros_like(out[0])) and np.abs(out[1]).max() > 0


@pytest.mark.parametrize("ps", [4, 8, 16, 64])
def test_split_context_equals_single_pass(ps):
    rng = np.random.default_rng(13)
    lens = [1, 3, 4, 5, 15, 16, 17, 63, 64, 65, 100]
    q, K, V = rand_seqs(rng, lens, 2, 8)
    q *= 3.0                                       # sharper softmax, partition maxima differ widely
    kc, vc, tables, cl = paged_from_contiguous(K, V, 4, 120, rng)
    single = oracle.decode(q, kc, vc, tables, cl, 0.35, "f32")
    split = oracle.decode(q, kc, vc, tables, cl, 0.35, "f32", partition_size=ps)
    assert np.abs(single - split).max() < 1e-14


def test_rows_subset_matches_full():
    w = W.config1()
    v = W.make_values(w)
    kc, vc = v.k_cache.copy(), v.v_cache.copy()
    oracle.reshape_and_cache(v.k_new, v.v_new, kc, vc, w.write_slots, w.dtype)
    full = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    assert np.isfinite(full).all()
    rows = np.array([[7, 3], [0, 0], [3, 2]], dtype=np.int32)
    sub = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype, rows=rows)
    for r, (s, h) in enumerate(rows):
        assert np.array_equal(sub[r], full[s, h])
    one = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype, threads=1)
    assert np.array_equal(one, full)


def test_multi_query_matches_torch_causal_attention():
    # several new tokens per sequence: against a masked softmax in torch float64 on contiguous K, V
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(18)
    lens, q_lens, H, D, B = [37, 20, 5, 64], [5, 20, 1, 0], 2, 8, 8
    _, K, V = rand_seqs(rng, lens, H, D)
    kc, vc, tables, cl = paged_from_contiguous(K, V, B, 20, rng)
    q_start = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    q = rng.standard_normal((int(q_start[-1]), H, D)).astype(np.float32)
    scale = np.float32(0.3)
    out = oracle.decode_multi(q, kc, vc, tables, cl, q_start, scale, "f32")
    for s, (n, ql) in enumerate(zip(lens, q_lens)):
        if ql == 0:
            continue
        qt = torch.from_numpy(q[q_start[s]:q_start[s + 1]]).double().permute(1, 0, 2)    # [H][ql][D]
        Kt = torch.from_numpy(K[s]).double().permute(1, 0, 2)
        Vt = torch.from_numpy(V[s]).double().permute(1, 0, 2)
        logits = torch.einsum("hqd,hnd->hqn", qt, Kt) * float(scale)
        pos = torch.arange(n - ql, n).view(1, ql, 1)
        logits = logits.masked_fill(torch.arange(n).view(1, 1, n) > pos, float("-inf"))
        ref = torch.einsum("hqn,hnd->hqd", torch.softmax(logits, dim=-1), Vt).permute(1, 0, 2).numpy()
        assert np.abs(out[q_start[s]:q_start[s + 1]] - ref).max() < 1e-13
    # one query per sequence is ordinary decode
    one = np.arange(len(lens) + 1, dtype=np.int32)
    q1 = rng.standard_normal((len(lens), H, D)).astype(np.float32)
    assert np.array_equal(oracle.decode_multi(q1, kc, vc, tables, cl, one, scale, "f32"),
                          oracle.decode(q1, kc, vc, tables, cl, scale, "f32"))
    # the first of the new tokens of a sequence of exactly q_len tokens sees only itself
    qs2 = np.array([0, 5], dtype=np.int32)
    K2, V2 = [K[2]], [V[2]]
    k2, v2, t2, c2 = paged_from_contiguous(K2, V2, B, 3, np.random.default_rng(1))
    o2 = oracle.decode_multi(q[:5].copy(), k2, v2, t2, c2, qs2, scale, "f32")
    assert np.array_equal(o2[0], V[2][0].astype(np.float64))


# ---------------------------------------------------------------------------
# storage decoding: every 16-bit pattern against numpy's own conversions
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_all_16bit_patterns_decode_exactly(dtype):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    if dtype == "f16":
        vals = bits.view(np.float16)
        want = vals.astype(np.float64)
        store = vals
    else:
        want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        store = bits
    ok = np.isfinite(want)
    # one token per pattern, context_len 1 -> the oracle returns the decoded value
    D, B = 8, 4
    n = 65536 // D
    NB = n                                          # one block per sequence, slot 0
    vc = np.zeros((NB, 1, B, D), dtype=store.dtype)
    vc[:, 0, 0, :] = store.reshape(n, D)
    kc = np.zeros_like(vc)
    q = np.zeros((n, 1, D), dtype=store.dtype)
    tables = np.arange(n, dtype=np.int32).reshape(n, 1)
    cl = np.ones(n, dtype=np.int32)
    out = oracle.decode(q, kc, vc, tables, cl, 1.0, dtype).reshape(-1)
    assert np.array_equal(out[ok], want[ok])
    assert np.isnan(out[np.isnan(want)]).all()
    assert np.array_equal(out[np.isinf(want)], want[np.isinf(want)])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_reduced_precision_inputs_match_float64_formula(dtype):
    rng = np.random.default_rng(14)
    lens, H, D, B = [20, 9], 2, 8, 4
    q, K, V = rand_seqs(rng, lens, H, D)
    kc, vc, tables, cl = paged_from_contiguous(K, V, B, 10, rng, dtype)
    qs = W.to_storage(q, dtype)
    out = oracle.decode(qs, kc, vc, tables, cl, 0.35, dtype)
    scale = float(np.float32(0.35))
    for s, n in enumerate(lens):
        qd = W.storage_to_f64(qs[s], dtype)
        Kd = W.storage_to_f64(W.to_storage(K[s], dtype), dtype)
        Vd = W.storage_to_f64(W.to_storage(V[s], dtype), dtype)
        x = np.einsum("hd,nhd->hn", qd, Kd) * scale
        a = np.exp(x - x.max(axis=1, keepdims=True))
        a /= a.sum(axis=1, keepdims=True)
        assert np.abs(out[s] - np.einsum("hn,nhd->hd", a, Vd)).max() < 1e-13


# ---------------------------------------------------------------------------
# cache maintenance
# ---------------------------------------------------------------------------
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_reshape_and_cache_worked_example():
    # Sec. 4.3 walk-through: tokens land at the (physical block, offset) the figure shows
    rows = [[int(x) for x in r] for r in _read_golden("block_table_example.txt") if r[0].isdigit()]
    H, D, B, NB = 3, 2, 4, 8
    T = len(rows)
    k = np.arange(T * H * D, dtype=np.float32).reshape(T, H, D) + 1000
    v = -k
    kc = np.zeros((NB, H, B, D), dtype=np.float32)
    vc = np.zeros_like(kc)
    slots = np.array([r[4] for r in rows], dtype=np.int64)
    oracle.reshape_and_cache(k, v, kc, vc, slots, "f32")
    touched = np.zeros((NB, B), dtype=bool)
    for pos, lb, pb, off, slot in rows:
        assert np.array_equal(kc[pb, :, off, :], k[pos]) and np.array_equal(vc[pb, :, off, :], v[pos])
        touched[pb, off] = True
    assert not kc.transpose(0, 2, 1, 3)[~touched].any() and not vc.transpose(0, 2, 1, 3)[~touched].any()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_reshape_and_cache_matches_numpy_scatter(dtype):
    rng = np.random.default_rng(15)
    T, H, D, B, NB = 37, 3, 8, 4, 20
    st = W.storage_np_dtype(dtype)
    k = W.to_storage(rng.standard_normal((T, H, D)).astype(np.float32), dtype)
    v = W.to_storage(rng.standard_normal((T, H, D)).astype(np.float32), dtype)
    kc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), dtype)
    vc = W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), dtype)
    slots = rng.permutation(NB * B)[:T].astype(np.int64)
    slots[[3, 17]] = -1                              # padding tokens are skipped
    want_k, want_v = kc.copy(), vc.copy()
    keep = slots >= 0
    want_k[slots[keep] // B, :, slots[keep] % B, :] = k[keep]
    want_v[slots[keep] // B, :, slots[keep] % B, :] = v[keep]
    oracle.reshape_and_cache(k, v, kc, vc, slots, dtype)
    assert kc.dtype == st
    assert np.array_equal(kc.view(np.uint8), want_k.view(np.uint8))
    assert np.array_equal(vc.view(np.uint8), want_v.view(np.uint8))


def test_copy_blocks_matches_numpy_and_example():
    rng = np.random.default_rng(16)
    L, NB, H, B, D = 3, 10, 2, 4, 8
    ks = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "bf16") for _ in range(L)]
    vs = [W.to_storage(rng.standard_normal((NB, H, B, D)).astype(np.float32), "bf16") for _ in range(L)]
    # the paper's example pair (1 -> 3) plus a fan-out of one source to several children
    pairs = np.array([[1, 3], [7, 0], [7, 5], [7, 9]], dtype=np.int64)
    wk = [k.copy() for k in ks]
    wv = [v.copy() for v in vs]
    for l in range(L):
        wk[l][pairs[:, 1]] = wk[l][pairs[:, 0]]
        wv[l][pairs[:, 1]] = wv[l][pairs[:, 0]]
    oracle.copy_blocks(ks, vs, pairs, "bf16")
    for l in range(L):
        assert np.array_equal(ks[l], wk[l]) and np.array_equal(vs[l], wv[l])
        assert np.array_equal(ks[l][3], ks[l][1]) and not np.array_equal(ks[l][3], vs[l][3])
    oracle.copy_blocks(ks, vs, np.zeros((0, 2), dtype=np.int64), "bf16")   # empty list is a no-op
    for l in range(L):
        assert np.array_equal(ks[l], wk[l])


def test_swap_blocks_matches_numpy_round_trip():
    # Sec. 4.5: blocks go out to a second pool and come back elsewhere; contents survive bit for bit
    rng = np.random.default_rng(17)
    L, NBG, NBC, H, B, D = 2, 12, 7, 2, 4, 8
    gk = [W.to_storage(rng.standard_normal((NBG, H, B, D)).astype(np.float32), "f16") for _ in range(L)]
    gv = [W.to_storage(rng.standard_normal((NBG, H, B, D)).astype(np.float32), "f16") for _ in range(L)]
    ck = [np.zeros((NBC, H, B, D), dtype=np.float16) for _ in range(L)]
    cv = [np.zeros((NBC, H, B, D), dtype=np.float16) for _ in range(L)]
    keep_k, keep_v = [x.copy() for x in gk], [x.copy() for x in gv]
    out_pairs = np.array([[3, 0], [11, 6], [5, 2]], dtype=np.int64)          # gpu block -> cpu block
    oracle.swap_blocks(gk, gv, ck, cv, out_pairs, "f16")
    for l in range(L):
        want = np.zeros_like(ck[l])
        want[out_pairs[:, 1]] = keep_k[l][out_pairs[:, 0]]
        assert np.array_equal(ck[l], want)
        assert np.array_equal(cv[l][6], keep_v[l][11]) and not np.array_equal(cv[l][6], ck[l][6])
        assert np.array_equal(gk[l], keep_k[l])                                 # the source pool is untouched
    for l in range(L):
        gk[l][:] = 0
        gv[l][:] = 0
    in_pairs = np.array([[0, 9], [6, 1], [2, 4]], dtype=np.int64)             # cpu block -> new gpu block
    oracle.swap_blocks(ck, cv, gk, gv, in_pairs, "f16")
    for l in range(L):
        assert np.array_equal(gk[l][9], keep_k[l][3]) and np.array_equal(gv[l][1], keep_v[l][11])
        assert np.array_equal(gk[l][4], keep_k[l][5]) and not gk[l][0].any()


def test_full_timeline_small_sharing_workload():
    # copy-on-write, writes, then decode on a shrunken parallel-sampling workload:
    # every slot decode reads must have been produced by the timeline (no NaN leaks)
    w = W.config3(num_groups=5, H=2, prompt_median=20, prompt_cap=64, max_out=30)
    v = W.make_values(w)
    kc, vc = v.k_cache.copy(), v.v_cache.copy()
    oracle.copy_blocks([kc], [vc], w.copy_pairs, w.dtype)
    oracle.reshape_and_cache(v.k_new, v.v_new, kc, vc, w.write_slots, w.dtype)
    out = oracle.decode(v.q, kc, vc, w.block_tables, w.context_lens, w.scale, w.dtype)
    assert np.isfinite(out).all()
    # samples of one group agree on the prompt part of the cache
    for g, p in zip(w.meta["groups"], w.meta["prompts"]):
        for t in range(p):
            ref = kc[w.block_tables[g[0], t // 16], :, t % 16]
            for s in g[1:]:
                assert np.array_equal(ref, kc[w.block_tables[s, t // 16], :, t % 16])
