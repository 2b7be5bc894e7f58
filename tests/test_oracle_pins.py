"""Pins for the fp64 CPU oracle (CPU only).

Each test checks the oracle against something fixed by the mathematics of
softmax attention or by the paged layout, never against the oracle itself:
dense brute force written separately in numpy, closed forms, invariants,
hand-worked values.  A dropped term, a wrong sign, a wrong GQA map or a wrong
page/slot formula in the oracle fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

import oracle
from paper_2602_02204_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_form_cases.txt")


# --------------------------------------------------------------------------- helpers
def to_f64(a, dtype):
    return a.astype(np.float64) if dtype == W.F32 else W.bf16_bits_to_f32(a).astype(np.float64)


def dense_bruteforce(wl):
    """Unpaged reference: gather with plain numpy indexing, repeat KV heads G times, softmax(QK^T)V in fp64."""
    out = np.zeros((wl.B, wl.Hq, wl.D))
    kc, vc = to_f64(wl.k_cache, wl.dtype), to_f64(wl.v_cache, wl.dtype)
    q = to_f64(wl.q, wl.dtype)
    for b in range(wl.B):
        L = int(wl.context_lens[b])
        if L == 0:
            continue
        t = np.arange(L)
        pages = wl.block_table[b, t // wl.ps]
        K = kc[pages, :, t % wl.ps, :]                    # [L, Hkv, D]
        V = vc[pages, :, t % wl.ps, :]
        K = np.repeat(K, wl.G, axis=1)                    # [L, Hq, D]: head h uses KV head h // G
        V = np.repeat(V, wl.G, axis=1)
        s = np.einsum("hd,lhd->hl", q[b], K) * np.float64(wl.scale)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[b] = np.einsum("hl,lhd->hd", p, V)
    return out


def run(wl, **kw):
    return oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens,
                                    wl.scale, wl.dtype, **kw)


def small(seed, dtype=W.F32, lens=(1, 5, 16, 17, 33, 40), Hq=6, Hkv=2, D=8, ps=4, **kw):
    return W.build("small", seed, lens, Hq=Hq, Hkv=Hkv, D=D, ps=ps, dtype=dtype, pool_factor=1.5, **kw)


# --------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("hq,hkv", [(6, 2), (4, 4), (7, 1), (8, 2)])
def test_matches_dense_bruteforce(dtype, hq, hkv):
    wl = small(3, dtype=dtype, Hq=hq, Hkv=hkv)
    got, ref = run(wl), dense_bruteforce(wl)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_tiny_config_matches_bruteforce():
    wl = W.make("tiny")
    assert (wl.B, wl.Hq, wl.Hkv, wl.D, wl.ps, wl.P) == (4, 4, 2, 64, 16, 64)
    assert list(wl.context_lens) == [17, 64, 129, 200] and float(wl.scale) == 0.125
    assert np.max(np.abs(run(wl) - dense_bruteforce(wl))) < 1e-13


def test_gqa_map_is_contiguous_groups():
    # Make KV head 0 and KV head 1 carry constant, different V: every query head must return its own group's constant.
    wl = small(5, Hq=6, Hkv=2)
    live = ~np.isnan(wl.v_cache)
    wl.v_cache[:, 0][live[:, 0]] = 10.0
    wl.v_cache[:, 1][live[:, 1]] = 20.0
    out = run(wl)
    assert np.allclose(out[:, 0:3], 10.0, atol=1e-12) and np.allclose(out[:, 3:6], 20.0, atol=1e-12)


# --------------------------------------------------------------------------- special cases and closed forms
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_length_one_returns_v_row_exactly(dtype):
    wl = small(7, dtype=dtype, lens=(1, 1, 1))
    out = run(wl)
    v = to_f64(wl.v_cache, wl.dtype)
    for b in range(wl.B):
        page = wl.block_table[b, 0]
        for h in range(wl.Hq):
            assert np.array_equal(out[b, h], v[page, h // wl.G, 0])


def test_identical_keys_give_mean_of_v():
    wl = small(11, lens=(9, 23))
    live = ~np.isnan(wl.k_cache)
    wl.k_cache[live] = 0.37
    out = run(wl)
    v = to_f64(wl.v_cache, wl.dtype)
    for b in range(wl.B):
        L = int(wl.context_lens[b]); t = np.arange(L)
        V = v[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]
        for h in range(wl.Hq):
            assert np.allclose(out[b, h], V[:, h // wl.G].mean(axis=0), atol=1e-14)


def test_zero_query_gives_mean_of_v():
    wl = small(12, lens=(13,))
    wl.q[...] = 0.0
    out = run(wl)
    v = to_f64(wl.v_cache, wl.dtype)
    t = np.arange(13)
    V = v[wl.block_table[0, t // wl.ps], :, t % wl.ps, :]
    for h in range(wl.Hq):
        assert np.allclose(out[0, h], V[:, h // wl.G].mean(axis=0), atol=1e-14)


def test_length_two_closed_form():
    wl = small(13, lens=(2, 2, 2), Hq=2, Hkv=2)
    out = run(wl)
    q, k, v = (to_f64(a, wl.dtype) for a in (wl.q, wl.k_cache, wl.v_cache))
    for b in range(wl.B):
        pg = wl.block_table[b, 0]
        for h in range(wl.Hq):
            s0 = float(wl.scale) * math.fsum(q[b, h] * k[pg, h, 0])
            s1 = float(wl.scale) * math.fsum(q[b, h] * k[pg, h, 1])
            w0 = 1.0 / (1.0 + math.exp(s1 - s0))
            assert np.allclose(out[b, h], w0 * v[pg, h, 0] + (1 - w0) * v[pg, h, 1], atol=1e-14)


def _parse_vals(txt):
    return [math.log(float(tok[2:])) if tok.startswith("ln") else float(tok) for tok in txt.split()]


def test_golden_hand_worked_cases():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, scale, q, K, V, exp = [f.strip() for f in line.split("|")]
        q = np.array(_parse_vals(q), dtype=np.float32)[None, None, :]
        K = np.array([_parse_vals(r) for r in K.split(";")], dtype=np.float32)
        V = np.array([_parse_vals(r) for r in V.split(";")], dtype=np.float32)
        L, D = K.shape
        ps = 2
        npg = (L + ps - 1) // ps
        kc = np.full((npg + 1, 1, ps, D), np.nan, dtype=np.float32)
        vc = kc.copy()
        table = np.arange(npg, 0, -1, dtype=np.int32)[None, :]           # pages npg..1, page 0 unused
        for t in range(L):
            kc[table[0, t // ps], 0, t % ps] = K[t]
            vc[table[0, t // ps], 0, t % ps] = V[t]
        out = oracle.paged_decode_attn(q, kc, vc, table, np.array([L], np.int32), float(scale), W.F32)
        assert np.allclose(out[0, 0], _parse_vals(exp), atol=2e-6), name
        n += 1
    assert n == 4


def test_golden_hand_worked_causal_chunks():
    """Hand-worked chunks (tests/golden/causal_chunk_cases.txt): rational softmax weights over tokens 0 .. own position."""
    n = 0
    for line in open(os.path.join(os.path.dirname(GOLDEN), "causal_chunk_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, scale, q, K, V, exp = [f.strip() for f in line.split("|")]
        q = np.array([_parse_vals(r) for r in q.split(";")], dtype=np.float32)[:, None, :]      # [n, Hq = 1, D]
        K = np.array([_parse_vals(r) for r in K.split(";")], dtype=np.float32)
        V = np.array([_parse_vals(r) for r in V.split(";")], dtype=np.float32)
        exp = np.array([_parse_vals(r) for r in exp.split(";")])
        L, D = K.shape
        ps = 2
        npg = (L + ps - 1) // ps
        kc = np.full((npg + 1, 1, ps, D), np.nan, dtype=np.float32)
        vc = kc.copy()
        table = np.arange(npg, 0, -1, dtype=np.int32)[None, :]           # pages npg..1, page 0 unused
        for t in range(L):
            kc[table[0, t // ps], 0, t % ps] = K[t]
            vc[table[0, t // ps], 0, t % ps] = V[t]
        out = oracle.paged_prefill_attn(q, kc, vc, table, np.array([L], np.int32), np.array([len(q)], np.int32),
                                        np.array([0], np.int64), float(scale), W.F32)
        assert np.allclose(out[:, 0], exp, atol=4e-6), name
        n += 1
    assert n == 3


# --------------------------------------------------------------------------- invariants
def test_key_shift_invariance_large_shift():
    # Adding u to every key adds the constant scale*q.u to every score of a head: softmax does not move.
    wl = small(17, lens=(31,), Hq=2, Hkv=1, D=8)
    base = run(wl)
    q = wl.q[0].astype(np.float64)
    u = 80.0 / float(wl.scale) * q[0] / np.dot(q[0], q[0])          # shifts head 0 by exactly ~80
    live = ~np.isnan(wl.k_cache)
    k2 = wl.k_cache.astype(np.float64)
    k2[0:wl.P, 0, :, :] += u
    wl2 = small(17, lens=(31,), Hq=2, Hkv=1, D=8)
    wl2.k_cache = np.where(live, k2, np.nan).astype(np.float32)
    shifted = run(wl2)
    assert np.all(np.isfinite(shifted))
    # fp32 rounding of the shifted keys perturbs scores by ~80 * 2^-24: compare at 1e-4
    assert np.max(np.abs(shifted[0, 0] - base[0, 0])) < 1e-4


def test_dominant_key_limit():
    wl = small(19, lens=(25,), Hq=1, Hkv=1, D=8)
    t_star = 9
    pg, sl = wl.block_table[0, t_star // wl.ps], t_star % wl.ps
    qv = wl.q[0, 0].astype(np.float64)
    live = ~np.isnan(wl.k_cache)
    wl.k_cache[live] = 0.0
    wl.k_cache[pg, 0, sl] = (100.0 / float(wl.scale) * qv / np.dot(qv, qv)).astype(np.float32)
    out = run(wl)
    assert np.max(np.abs(out[0, 0] - wl.v_cache[pg, 0, sl].astype(np.float64))) < 1e-20


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_output_in_convex_hull_of_v(dtype):
    wl = small(23, dtype=dtype)
    out = run(wl)
    v = to_f64(wl.v_cache, wl.dtype)
    for b in range(wl.B):
        L = int(wl.context_lens[b]); t = np.arange(L)
        V = v[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]
        for h in range(wl.Hq):
            lo, hi = V[:, h // wl.G].min(axis=0), V[:, h // wl.G].max(axis=0)
            assert np.all(out[b, h] >= lo - 1e-12) and np.all(out[b, h] <= hi + 1e-12)


def test_page_permutation_is_bit_invariant():
    wl = small(29, dtype=W.BF16)
    base = run(wl)
    rng = np.random.default_rng(1)
    perm = rng.permutation(wl.P)                      # new physical id of old page p is perm[p]
    k2, v2 = np.empty_like(wl.k_cache), np.empty_like(wl.v_cache)
    k2[perm] = wl.k_cache
    v2[perm] = wl.v_cache
    t2 = np.where(wl.block_table >= 0, perm[np.maximum(wl.block_table, 0)], -1).astype(np.int32)
    out = oracle.paged_decode_attn(wl.q, k2, v2, t2, wl.context_lens, wl.scale, wl.dtype)
    assert np.array_equal(out, base)


def test_page_size_change_is_bit_invariant():
    lens = (1, 15, 16, 17, 47, 64)
    a = small(31, lens=lens, ps=16, D=16)
    # same logical rows, re-paged at ps = 32 with a different physical assignment
    rng = np.random.default_rng(2)
    ps2 = 32
    npg = [(L + ps2 - 1) // ps2 for L in lens]
    P2 = sum(npg) + 3
    ids = rng.permutation(P2)[: sum(npg)].astype(np.int32)
    table = np.full((len(lens), max(npg)), -1, np.int32)
    kc = np.full((P2, a.Hkv, ps2, a.D), np.nan, np.float32); vc = kc.copy()
    pos = 0
    for b, L in enumerate(lens):
        table[b, : npg[b]] = ids[pos: pos + npg[b]]; pos += npg[b]
        for t in range(L):
            src = (a.block_table[b, t // a.ps], slice(None), t % a.ps)
            dst = (table[b, t // ps2], slice(None), t % ps2)
            kc[dst] = a.k_cache[src]; vc[dst] = a.v_cache[src]
    out = oracle.paged_decode_attn(a.q, kc, vc, table, a.context_lens, a.scale, a.dtype)
    assert np.array_equal(out, run(a))


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_poison_never_reaches_output(dtype):
    wl = small(37, dtype=dtype)
    # unowned slots and pages are NaN by construction; padded table entries are -1
    raw = wl.k_cache if dtype == W.F32 else W.bf16_bits_to_f32(wl.k_cache)
    assert np.isnan(raw).any() and (wl.block_table == -1).any()
    assert np.all(np.isfinite(run(wl)))


def test_empty_request_gives_zero_row():
    wl = small(41, lens=(0, 7, 0))
    out = run(wl)
    assert np.all(out[0] == 0.0) and np.all(out[2] == 0.0) and np.all(np.isfinite(out[1]))


def test_scale_is_the_callers_fp32_value():
    # 1/sqrt(128) is not representable: the oracle must use the fp32 value handed in, widened.
    wl = small(43, lens=(6,), Hq=1, Hkv=1, D=8)
    s32 = np.float32(1.0 / math.sqrt(128.0))
    out = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, s32, wl.dtype)
    wl.scale = s32
    assert np.max(np.abs(out - dense_bruteforce(wl))) < 1e-15


def test_pairs_subset_matches_full():
    wl = small(47)
    full = run(wl)
    pairs = [(0, 0), (3, 5), (5, 2), (2, 4)]
    sub = run(wl, pairs=pairs)
    for i, (b, h) in enumerate(pairs):
        assert np.array_equal(sub[i], full[b, h])


# --------------------------------------------------------------------------- split + merge identity
def test_split_and_merge_equals_unsplit():
    wl = small(53, lens=(40, 33), dtype=W.BF16)
    full = run(wl)
    for b in range(wl.B):
        L = int(wl.context_lens[b])
        for h in (0, wl.Hq - 1):
            for cuts in ([0, L], [0, 1, L], [0, 16, 17, L], [0, 7, 7, 30, L], [0, L, L]):
                parts = [oracle.partial(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.scale, wl.dtype,
                                        b, h, cuts[i], cuts[i + 1]) for i in range(len(cuts) - 1)]
                o = np.stack([p[0] for p in parts]); m = np.array([p[1] for p in parts]); l = np.array([p[2] for p in parts])
                assert np.max(np.abs(oracle.merge(o, m, l) - full[b, h])) < 1e-14


def test_partial_is_the_unnormalised_sum():
    # (o, m, l) of a range, recomputed with numpy from gathered rows
    wl = small(59, lens=(20,), Hq=2, Hkv=1, D=8)
    o, m, l = oracle.partial(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.scale, wl.dtype, 0, 1, 3, 15)
    t = np.arange(3, 15)
    K = wl.k_cache[wl.block_table[0, t // wl.ps], 0, t % wl.ps].astype(np.float64)
    V = wl.v_cache[wl.block_table[0, t // wl.ps], 0, t % wl.ps].astype(np.float64)
    s = K @ wl.q[0, 1].astype(np.float64) * float(wl.scale)
    assert m == s.max() and abs(l - np.exp(s - s.max()).sum()) < 1e-14
    assert np.max(np.abs(o - np.exp(s - s.max()) @ V)) < 1e-13


def test_merge_ignores_empty_partitions():
    o = np.array([[0.0, 0.0], [2.0, 4.0]]); m = np.array([-np.inf, 0.3]); l = np.array([0.0, 2.0])
    assert np.allclose(oracle.merge(o, m, l), [1.0, 2.0])
    assert np.all(oracle.merge(o[:1], m[:1], l[:1]) == 0.0)


# --------------------------------------------------------------------------- append and gather
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_append_writes_exactly_one_row_per_head(dtype):
    wl = small(61, dtype=dtype, lens=(1, 4, 5, 17, 0), append=True)
    k0, v0 = wl.k_cache.copy(), wl.v_cache.copy()
    oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    changed = np.zeros(wl.k_cache.shape[:3], dtype=bool)
    for b in range(wl.B):
        pos = int(wl.positions[b])
        if pos < 0:
            continue
        pg, sl = wl.block_table[b, pos // wl.ps], pos % wl.ps
        assert np.array_equal(wl.k_cache[pg, :, sl], wl.k_new[b])
        assert np.array_equal(wl.v_cache[pg, :, sl], wl.v_new[b])
        changed[pg, :, sl] = True
    same_bits = lambda a, b: np.array_equal(a.view(np.uint8), b.view(np.uint8))
    assert same_bits(wl.k_cache[~changed], k0[~changed]) and same_bits(wl.v_cache[~changed], v0[~changed])
    # after the append every live slot is finite
    assert np.all(np.isfinite(run(wl)))
    g = oracle.gather(wl.k_cache, wl.block_table, wl.context_lens, 3, wl.dtype)
    assert np.array_equal(g[16], wl.k_new[3])


def test_gather_is_token_ordered_bit_copy():
    wl = small(67, dtype=W.BF16)
    for b in range(wl.B):
        g = oracle.gather(wl.v_cache, wl.block_table, wl.context_lens, b, wl.dtype)
        L = int(wl.context_lens[b]); t = np.arange(L)
        assert np.array_equal(g, wl.v_cache[wl.block_table[b, t // wl.ps], :, t % wl.ps, :])


# ---- KV pack / unpack (the dense per-request copies a connector ships between stages)

def _pack_case(seed=11):
    wl = W.make("tiny", seed=seed)
    lens = wl.context_lens.copy()
    lens[1] = 0                                              # an empty request
    order = [2, 0, 3, 1]                                     # dense order differs from batch order
    offs = np.full(wl.B, -1, dtype=np.int64)
    run = 3                                                  # and the dense buffer has rows nobody owns
    for b in order:
        offs[b] = run
        run += int(lens[b]) + 1
    offs[3] = -1                                             # a skipped request
    return wl, lens, offs, run


def test_kv_pack_equals_brute_force_loops():
    wl, lens, offs, total = _pack_case()
    dense = oracle.kv_pack(wl.k_cache, wl.block_table, lens, offs, total)
    want = np.zeros_like(dense)
    for b in range(wl.B):
        if offs[b] < 0:
            continue
        for t in range(int(lens[b])):
            for g in range(wl.Hkv):
                want[offs[b] + t, g] = wl.k_cache[wl.block_table[b, t // wl.ps], g, t % wl.ps]
    assert np.array_equal(dense.view(np.uint8), want.view(np.uint8))
    for b in range(wl.B):                                    # and with the per-request gather of the C oracle
        if offs[b] >= 0 and lens[b] > 0:
            g1 = oracle.gather(wl.k_cache, wl.block_table, lens, b, wl.dtype)
            assert np.array_equal(dense[offs[b]:offs[b] + lens[b]].view(np.uint8), g1.view(np.uint8))


def test_kv_unpack_is_the_inverse_and_touches_nothing_else():
    wl, lens, offs, total = _pack_case(seed=12)
    dense = oracle.kv_pack(wl.v_cache, wl.block_table, lens, offs, total)
    pool = np.full_like(wl.v_cache, np.float32(123.0))       # a different pool: only owned rows may change
    oracle.kv_unpack(dense, pool, wl.block_table, lens, offs)
    owned = np.zeros(wl.v_cache.shape[:3], dtype=bool)       # [page, head, slot]
    for b in range(wl.B):
        if offs[b] < 0:
            continue
        for t in range(int(lens[b])):
            owned[wl.block_table[b, t // wl.ps], :, t % wl.ps] = True
    assert np.array_equal(pool[owned].view(np.uint8), wl.v_cache[owned].view(np.uint8))
    assert np.all(pool[~owned] == np.float32(123.0))
    again = oracle.kv_pack(pool, wl.block_table, lens, offs, total)
    assert np.array_equal(again.view(np.uint8), dense.view(np.uint8))


def test_kv_pack_mutations_are_caught():
    """A transposed slot/page index or a dropped offset must change the result (the pins above would fail)."""
    wl, lens, offs, total = _pack_case(seed=13)
    good = oracle.kv_pack(wl.k_cache, wl.block_table, lens, offs, total)
    shifted = oracle.kv_pack(wl.k_cache, wl.block_table, lens, offs + (offs >= 0), total + 1)[1:]
    assert np.array_equal(shifted.view(np.uint8), good.view(np.uint8))                  # offsets are honoured exactly
    bt2 = wl.block_table.copy()
    bt2[0, 0], bt2[0, 1] = bt2[0, 1], bt2[0, 0]
    assert not np.array_equal(oracle.kv_pack(wl.k_cache, bt2, lens, offs, total).view(np.uint8), good.view(np.uint8))


# ---- multi-token (chunk) queries: causal inside the chunk

def _chunk_case(seed=21, dtype=None):
    lens = [37, 5, 64, 1, 90]
    wl = W.build("chunk", seed, lens, Hq=6, Hkv=2, D=64, ps=16, dtype=dtype or W.F32, pool_factor=1.5)
    ch = W.add_chunk(wl, [7, 5, 1, 1, 33], seed + 1, gap=2)
    return wl, ch


def test_chunk_of_one_token_is_the_decode_definition():
    wl = W.make("tiny")
    ch = W.add_chunk(wl, [1] * wl.B, 3)
    ch.q[:] = wl.q                                           # same query rows as the decode batch
    got = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    ref = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_chunk_equals_dense_causal_brute_force(dtype):
    wl, ch = _chunk_case(dtype=dtype)
    got = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    to64 = (lambda a: a.astype(np.float64)) if dtype == W.F32 else (lambda a: W.bf16_bits_to_f32(a).astype(np.float64))
    G = wl.G
    for b in range(wl.B):
        L, n = int(wl.context_lens[b]), int(ch.q_lens[b])
        K = to64(oracle.gather(wl.k_cache, wl.block_table, wl.context_lens, b, wl.dtype))      # [L, Hkv, D]
        V = to64(oracle.gather(wl.v_cache, wl.block_table, wl.context_lens, b, wl.dtype))
        Q = to64(ch.q[ch.q_offsets[b]:ch.q_offsets[b] + n])                                     # [n, Hq, D]
        Kh, Vh = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)                               # [L, Hq, D]
        S = np.einsum("ihd,thd->hit", Q, Kh) * float(wl.scale)                                  # [Hq, n, L]
        pos = (L - n + np.arange(n))[None, :, None]
        S = np.where(np.arange(L)[None, None, :] <= pos, S, -np.inf)
        Pm = np.exp(S - S.max(axis=2, keepdims=True))
        Pm /= Pm.sum(axis=2, keepdims=True)
        want = np.einsum("hit,thd->ihd", Pm, Vh)
        assert np.max(np.abs(got[ch.q_offsets[b]:ch.q_offsets[b] + n] - want)) < 1e-12, b


def test_chunk_rows_after_a_query_never_reach_it_and_first_token_returns_its_v_row():
    wl, ch = _chunk_case(seed=31)
    args = (wl.block_table, wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale, wl.dtype)
    b, i, h = 4, 10, 5                                       # position 90 - 33 + 10 = 67: 22 later rows exist
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, *args, rows=[(b, i, h)])
    kc, vc = wl.k_cache.copy(), wl.v_cache.copy()
    for t in range(67 + 1, 90):
        kc[wl.block_table[b, t // wl.ps], :, t % wl.ps, :] = np.nan
        vc[wl.block_table[b, t // wl.ps], :, t % wl.ps, :] = np.nan
    got = oracle.paged_prefill_attn(ch.q, kc, vc, *args, rows=[(b, i, h)])
    assert np.array_equal(got, ref) and np.all(np.isfinite(ref))
    kc[wl.block_table[b, 67 // wl.ps], :, 67 % wl.ps, :] = np.nan          # its own position does count
    assert not np.all(np.isfinite(oracle.paged_prefill_attn(ch.q, kc, vc, *args, rows=[(b, i, h)])))
    # request 1 is all chunk (5 of 5 tokens): its first query sees only token 0
    first = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, *args, rows=[(1, 0, 3)])
    assert np.array_equal(first[0], wl.v_cache[wl.block_table[1, 0], 3 // wl.G, 0, :].astype(np.float64))
    # rows in the sampled form equal the rows of the full form
    full = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, *args)
    assert np.array_equal(full[ch.q_offsets[b] + i, h], ref[0])
    assert np.all(full[ch.q_offsets[0] + 7:ch.q_offsets[1]] == 0)          # gap rows between requests stay zero


def test_kv_append_chunk_writes_exactly_the_chunk_rows():
    lens = [37, 5, 64, 1, 90]
    wl = W.build("chunk", 41, lens, Hq=6, Hkv=2, D=64, ps=16, dtype=W.BF16, pool_factor=1.5)
    full_k, full_v = wl.k_cache.copy(), wl.v_cache.copy()
    ch = W.add_chunk(wl, [7, 5, 0, 1, 33], 42, in_cache=False, gap=1)
    changed = (wl.k_cache != full_k).any(axis=(1, 3)).sum()
    assert changed == 7 + 5 + 0 + 1 + 33                     # that many (page, slot) rows were taken out
    oracle.kv_append_chunk(ch.k_new, ch.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                           ch.q_offsets)
    assert np.array_equal(wl.k_cache, full_k) and np.array_equal(wl.v_cache, full_v)
    # one token per request is the single-token append
    wl1 = W.build("chunk", 41, lens, Hq=6, Hkv=2, D=64, ps=16, dtype=W.BF16, pool_factor=1.5, append=True)
    k2, v2 = wl1.k_cache.copy(), wl1.v_cache.copy()
    oracle.kv_append(wl1.k_new, wl1.v_new, wl1.k_cache, wl1.v_cache, wl1.block_table, wl1.positions, wl1.dtype)
    oracle.kv_append_chunk(wl1.k_new, wl1.v_new, k2, v2, wl1.block_table, wl1.context_lens, np.ones(5, np.int32),
                           np.arange(5, dtype=np.int64))
    assert np.array_equal(k2.view(np.uint8), wl1.k_cache.view(np.uint8))
    assert np.array_equal(v2.view(np.uint8), wl1.v_cache.view(np.uint8))


# ---- 8-bit (E4M3) KV cache with per-(page, head) scales

def test_fp8_decode_matches_an_independent_conversion_for_all_bytes():
    import torch
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for b in range(256):
        got = oracle.fp8_e4m3_decode(b)
        assert (math.isnan(got) and math.isnan(ref[b])) or got == ref[b], b
    assert oracle.fp8_e4m3_decode(0x7E) == 448.0 and oracle.fp8_e4m3_decode(0x01) == 2.0 ** -9
    assert oracle.fp8_e4m3_decode(0x38) == 1.0 and oracle.fp8_e4m3_decode(0xB8) == -1.0


def _dequantized(wl, f8):
    """fp32 pools holding decode(byte) * scale, by the library's own cast (NaN bytes stay NaN)."""
    import torch
    def one(c8, sc):
        x = torch.from_numpy(c8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        return (x * sc[:, :, None, None]).astype(np.float32)
    return one(f8.k_cache, f8.k_scale), one(f8.v_cache, f8.v_scale)


def test_fp8_attention_with_power_of_two_scales_is_the_fp32_oracle_on_dequantised_pools():
    wl = W.build("f8", 51, [37, 5, 64, 1, 0, 90], Hq=6, Hkv=2, D=64, ps=16, dtype=W.BF16, pool_factor=1.5)
    f8 = W.quantize_fp8(wl, power_of_two_scales=True)
    got = oracle.paged_decode_attn_fp8(wl.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                       wl.context_lens, wl.scale)
    kd, vd = _dequantized(wl, f8)                            # exact: a 4-bit significand times a power of two
    qf = W.bf16_bits_to_f32(wl.q)
    ref = oracle.paged_decode_attn(qf, kd, vd, wl.block_table, wl.context_lens, wl.scale, W.F32)
    assert np.array_equal(got, ref)
    assert np.all(got[4] == 0)                               # the empty request


def test_fp8_attention_with_general_scales_and_quantisation_error_is_small():
    wl = W.build("f8", 52, [200, 33, 64], Hq=8, Hkv=2, D=128, ps=32, dtype=W.BF16)
    f8 = W.quantize_fp8(wl)
    assert f8.k_cache.dtype == np.uint8 and np.all(f8.k_scale > 0)
    got = oracle.paged_decode_attn_fp8(wl.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                       wl.context_lens, wl.scale)
    import torch
    kd = torch.from_numpy(f8.k_cache).view(torch.float8_e4m3fn).to(torch.float64).numpy() * f8.k_scale.astype(np.float64)[:, :, None, None]
    vd = torch.from_numpy(f8.v_cache).view(torch.float8_e4m3fn).to(torch.float64).numpy() * f8.v_scale.astype(np.float64)[:, :, None, None]
    qf = W.bf16_bits_to_f32(wl.q).astype(np.float64)
    for b in range(wl.B):                                    # dense brute force on the de-quantised rows, fp64
        L = int(wl.context_lens[b]); t = np.arange(L)
        K = kd[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]; V = vd[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]
        Kh, Vh = np.repeat(K, wl.G, axis=1), np.repeat(V, wl.G, axis=1)
        S = np.einsum("hd,thd->ht", qf[b], Kh) * float(wl.scale)
        Pm = np.exp(S - S.max(axis=1, keepdims=True)); Pm /= Pm.sum(axis=1, keepdims=True)
        assert np.max(np.abs(got[b] - np.einsum("ht,thd->hd", Pm, Vh))) < 1e-12
    # and it is attention over a quantised copy of the bf16 pools: close to the bf16 result, not equal to it
    ref16 = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype)
    d = np.max(np.abs(got - ref16))
    assert 1e-5 < d < 0.2


def _fp8_chunk_case(seed, power_of_two):
    wl = W.build("f8c", seed, [70, 5, 33, 1, 0, 90], Hq=6, Hkv=2, D=64, ps=16, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, [40, 5, 1, 1, 0, 17], seed + 1, in_cache=True, gap=2)
    return wl, ch, W.quantize_fp8(wl, power_of_two_scales=power_of_two)


def test_fp8_chunks_of_one_token_are_the_fp8_decode_oracle():
    wl = W.build("f8c", 53, [37, 5, 64, 1, 0, 90], Hq=6, Hkv=2, D=64, ps=16, dtype=W.BF16, pool_factor=1.5)
    f8 = W.quantize_fp8(wl)
    ones = np.where(wl.context_lens > 0, 1, 0).astype(np.int32)
    offs = np.arange(wl.B, dtype=np.int64)
    got = oracle.paged_prefill_attn_fp8(wl.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, ones, offs, wl.scale)
    ref = oracle.paged_decode_attn_fp8(wl.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                       wl.context_lens, wl.scale)
    assert np.array_equal(got, ref)


def test_fp8_chunks_with_power_of_two_scales_are_the_chunk_oracle_on_dequantised_pools():
    wl, ch, f8 = _fp8_chunk_case(54, True)
    got = oracle.paged_prefill_attn_fp8(ch.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale)
    kd, vd = _dequantized(wl, f8)
    ref = oracle.paged_prefill_attn(W.bf16_bits_to_f32(ch.q), kd, vd, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, W.F32)
    assert np.array_equal(got, ref)
    rows = [(0, 0, 0), (0, 39, 5), (5, 16, 3), (2, 0, 1)]
    some = oracle.paged_prefill_attn_fp8(ch.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                         wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale, rows=rows)
    for r, (b, i, h) in enumerate(rows):
        assert np.array_equal(some[r], got[ch.q_offsets[b] + i, h])


def test_fp8_chunks_with_general_scales_against_a_dense_causal_brute_force():
    import torch
    wl, ch, f8 = _fp8_chunk_case(55, False)
    got = oracle.paged_prefill_attn_fp8(ch.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale)
    kd = torch.from_numpy(f8.k_cache).view(torch.float8_e4m3fn).to(torch.float64).numpy() * f8.k_scale.astype(np.float64)[:, :, None, None]
    vd = torch.from_numpy(f8.v_cache).view(torch.float8_e4m3fn).to(torch.float64).numpy() * f8.v_scale.astype(np.float64)[:, :, None, None]
    qf = W.bf16_bits_to_f32(ch.q).astype(np.float64)
    for b in range(wl.B):
        L, n = int(wl.context_lens[b]), int(ch.q_lens[b])
        if n == 0:
            continue
        t = np.arange(L)
        K = np.repeat(kd[wl.block_table[b, t // wl.ps], :, t % wl.ps, :], wl.G, axis=1)
        V = np.repeat(vd[wl.block_table[b, t // wl.ps], :, t % wl.ps, :], wl.G, axis=1)
        Q = qf[ch.q_offsets[b]:ch.q_offsets[b] + n]                                  # [n, Hq, D]
        S = np.einsum("ihd,thd->iht", Q, K) * float(wl.scale)
        pos = L - n + np.arange(n)
        S = np.where(t[None, None, :] <= pos[:, None, None], S, -np.inf)              # causal inside the chunk
        Pm = np.exp(S - S.max(axis=2, keepdims=True)); Pm /= Pm.sum(axis=2, keepdims=True)
        ref = np.einsum("iht,thd->ihd", Pm, np.nan_to_num(V))                          # rows beyond a position weigh 0
        assert np.max(np.abs(got[ch.q_offsets[b]:ch.q_offsets[b] + n] - ref)) < 1e-12


def test_chunk_oracle_rejects_rows_outside_the_chunks():
    wl, ch = _chunk_case(seed=61)
    args = (ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale, wl.dtype)
    with pytest.raises(ValueError):
        oracle.paged_prefill_attn(*args, rows=[(0, 7, 0)])              # request 0 has 7 chunk rows: 0..6
    with pytest.raises(ValueError):
        oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens,
                                  ch.q_lens + 100, ch.q_offsets, wl.scale, wl.dtype)


# --------------------------------------------------------------------------- quantising append (E4M3 encoder)
def _e4m3_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "e4m3_rounding_cases.txt")
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            value, byte = line.split()[:2]
            yield float(value), int(byte, 16)


def test_e4m3_encoder_on_hand_worked_cases():
    n = 0
    for value, byte in _e4m3_golden():
        assert oracle.fp8_e4m3_encode(value) == byte, (value, hex(byte), hex(oracle.fp8_e4m3_encode(value)))
        n += 1
    assert n >= 16
    assert oracle.fp8_e4m3_encode(float("nan")) == 0x7F


def test_e4m3_encoder_round_trips_every_finite_code_and_is_monotonic():
    vals = []
    for code in range(256):
        v = oracle.fp8_e4m3_decode(code)
        if np.isnan(v):
            continue
        assert oracle.fp8_e4m3_encode(v) == code or (v == 0 and oracle.fp8_e4m3_encode(v) in (0x00, 0x80))
        vals.append(v)
    xs = np.linspace(-460.0, 460.0, 20001).astype(np.float32)
    dec = np.array([oracle.fp8_e4m3_decode(oracle.fp8_e4m3_encode(float(x))) for x in xs])
    assert np.all(np.diff(dec) >= 0)                                   # rounding never reorders
    grid = np.array(sorted(vals))
    nearest = np.abs(grid[None, :] - np.clip(xs, -448, 448).astype(np.float64)[:, None]).min(axis=1)
    assert np.array_equal(np.abs(dec - np.clip(xs, -448, 448).astype(np.float64)), nearest)   # and picks a nearest value


def test_e4m3_encoder_agrees_with_the_frameworks_cast():
    """torch's float8_e4m3fn cast (round to nearest even) on every representable value, every midpoint between
    neighbours, values a hair to either side of the midpoints, and random values inside the finite range."""
    import torch
    grid = np.array(sorted({oracle.fp8_e4m3_decode(c) for c in range(0x7F)}), dtype=np.float64)
    mids = (grid[:-1] + grid[1:]) / 2
    xs = np.concatenate([grid, mids, np.nextafter(mids.astype(np.float32), np.float32(0)),
                         np.nextafter(mids.astype(np.float32), np.float32(1e9)),
                         np.random.default_rng(77).uniform(0, 448, 4000), np.random.default_rng(78).normal(0, 1, 4000)])
    xs = np.concatenate([xs, -xs]).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.fp8_e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, want)


def _quant_case(seed, ps=16, Hkv=2, D=128):
    rng = np.random.default_rng(seed)
    lens = np.array([ps + 1, 2 * ps, 5, 3 * ps + 1, 0, 1, ps], dtype=np.int64)       # positions at slot 0 and elsewhere
    wl = W.build("quant", seed, lens, Hq=2 * Hkv, Hkv=Hkv, D=D, ps=ps, dtype=W.BF16, append=True, pool_factor=1.5)
    f8 = W.quantize_fp8(wl)
    # make the new rows span several binades, with a few values beyond what an old page's scale can hold
    kf = (rng.standard_normal(wl.k_new.shape) * np.exp2(rng.integers(-6, 4, size=wl.k_new.shape[:2] + (1,)))).astype(np.float32)
    vf = (rng.standard_normal(wl.v_new.shape) * 3.0).astype(np.float32)
    wl.k_new, wl.v_new = W.f32_to_bf16_bits(kf), W.f32_to_bf16_bits(vf)
    return wl, f8


@pytest.mark.parametrize("headroom", [1.0, 2.0, 1.37])
@pytest.mark.parametrize("ps", [16, 32])
def test_quantising_append_against_a_brute_force_on_the_frameworks_cast(headroom, ps):
    import torch
    wl, f8 = _quant_case(90 + ps, ps=ps)
    k8, v8, ks, vs = f8.k_cache.copy(), f8.v_cache.copy(), f8.k_scale.copy(), f8.v_scale.copy()
    oracle.kv_append_quant_fp8(wl.k_new, wl.v_new, k8, v8, ks, vs, wl.block_table, wl.positions, headroom)
    # brute force, written separately: fp32 arithmetic in numpy, bytes by the framework's cast
    ek, ev, eks, evs = f8.k_cache.copy(), f8.v_cache.copy(), f8.k_scale.copy(), f8.v_scale.copy()
    for cache, scales, new in ((ek, eks, wl.k_new), (ev, evs, wl.v_new)):
        x = W.bf16_bits_to_f32(new)
        for b in range(wl.B):
            pos = int(wl.positions[b])
            if pos < 0:
                continue
            page, slot = int(wl.block_table[b, pos // ps]), pos % ps
            for g in range(wl.Hkv):
                if slot == 0:
                    top = np.float32(np.abs(x[b, g]).max()) * np.float32(headroom)
                    scales[page, g] = np.maximum(top, np.float32(2.0 ** -100)) / np.float32(448.0)
                q = np.clip(x[b, g] / scales[page, g], np.float32(-448.0), np.float32(448.0)).astype(np.float32)
                cache[page, g, slot] = torch.from_numpy(q).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(ks, eks) and np.array_equal(vs, evs)
    assert np.array_equal(k8, ek) and np.array_equal(v8, ev)                   # whole pools: nothing else changed
    touched_scales = int((ks != f8.k_scale).sum())
    assert touched_scales == sum(1 for b in range(wl.B) if wl.positions[b] >= 0 and wl.positions[b] % ps == 0) * wl.Hkv


def test_quantising_append_reconstruction_error_and_saturation():
    wl, f8 = _quant_case(95)
    k8, v8, ks, vs = f8.k_cache.copy(), f8.v_cache.copy(), f8.k_scale.copy(), f8.v_scale.copy()
    oracle.kv_append_quant_fp8(wl.k_new, wl.v_new, k8, v8, ks, vs, wl.block_table, wl.positions, 1.0)
    x = W.bf16_bits_to_f32(wl.k_new).astype(np.float64)
    dec = np.vectorize(oracle.fp8_e4m3_decode)
    for b in range(wl.B):
        pos = int(wl.positions[b])
        if pos < 0:
            continue
        page, slot = int(wl.block_table[b, pos // wl.ps]), pos % wl.ps
        for g in range(wl.Hkv):
            s = float(ks[page, g])
            back = dec(k8[page, g, slot]).astype(np.float64) * s
            inside = np.abs(x[b, g]) <= 448.0 * s
            # inside the page's range: half a unit of the last place of a 4-bit significand (2^-4 relative), or half a
            # subnormal step (2^-10 * scale); outside: the largest value the scale can hold, with the right sign
            assert np.all(np.abs(back - x[b, g])[inside] <= np.maximum(np.abs(x[b, g])[inside] * 2.0 ** -4, s * 2.0 ** -10) + 1e-30)
            assert np.all(back[~inside] == np.sign(x[b, g][~inside]) * 448.0 * s)
            if slot == 0:                                    # headroom 1: the row's largest element lands on +-448 exactly
                assert np.max(np.abs(dec(k8[page, g, slot]))) == 448.0
