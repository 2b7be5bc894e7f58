"""Decode attention with several query tokens per request (OMNI_TUNE_QUERY_TOKENS = T) through the C ABI.

The T new tokens of a request are the last T of its context; query i sees tokens 0 .. L - T + i.  The oracle is the
chunk definition (`oracle.paged_prefill_attn`) with q_lens = T and q rows laid out [B, T, Hq, D].
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, DeviceBatch, to_dev
from test_fp8_gpu import Fp8Batch

pytestmark = pytest.mark.gpu


def queries(wl, T, seed):
    rng = np.random.default_rng(seed)
    return W.f32_to_bf16_bits(rng.standard_normal((wl.B * T, wl.Hq, wl.D)).astype(np.float32))


def chunk_args(wl, T):
    """q_lens / q_offsets of the chunk definition: the last min(T, L) query rows of each request."""
    n = np.minimum(T, wl.context_lens).astype(np.int32)
    offs = (np.arange(wl.B, dtype=np.int64) * T + (T - n)).astype(np.int64)
    return n, offs


def expected(wl, q, T):
    n, offs = chunk_args(wl, T)
    ref = oracle.paged_prefill_attn(q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, n, offs, wl.scale, wl.dtype)
    return ref.reshape(wl.B, T, wl.Hq, wl.D)                # rows no query owns (L < T) stay zero, as the call writes them


def attend(wl, q, T, tuning=None, out_dtype=W.F32):
    tn = {omni.OMNI_TUNE_QUERY_TOKENS: T}
    tn.update(tuning or {})
    dev = DeviceBatch(wl, out_dtype=out_dtype, tuning=tn)
    dq = to_dev(q, wl.dtype)
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), device="cuda",
                     dtype=torch.float32 if out_dtype == W.F32 else torch.bfloat16)
    dev.h.omni_paged_decode_attn(dq, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, float(wl.scale), out)
    torch.cuda.synchronize()
    return dev, out.float().cpu().numpy().astype(np.float64)


LENS = [2, 5, 16, 17, 31, 32, 33, 34, 64, 65, 66, 250, 0, 96, 97, 1, 3]


@pytest.mark.parametrize("G,Hkv,T,ps", [(7, 4, 2, 16), (8, 2, 2, 16), (4, 2, 4, 32), (1, 3, 16, 16), (3, 2, 5, 16),
                                        (5, 1, 3, 32), (16, 1, 1, 16), (2, 2, 7, 16),
                                        # more columns than a pass holds: several passes, the last one ragged
                                        (7, 4, 5, 16), (8, 2, 4, 16), (16, 1, 3, 32), (4, 2, 9, 16), (1, 2, 33, 16)])
@pytest.mark.parametrize("tuning", [{}, {omni.OMNI_TUNE_FORCE_PARTITION: 32}, {omni.OMNI_TUNE_FORCE_PARTITION: 128},
                                    {omni.OMNI_TUNE_TARGET_WORKGROUPS: 64, omni.OMNI_TUNE_MIN_PARTITION: 32}],
                         ids=["default", "force32", "force128", "wg64"])
def test_edge_lengths_and_groups(G, Hkv, T, ps, tuning):
    """Lengths around tile and page boundaries, shorter than T, and zero; one-tile ranges put a request's newest tokens
    into a piece of their own, which the earlier queries of the request must not see anything of."""
    wl = W.build("mt", 2000 + G + T, LENS, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    q = queries(wl, T, 2100 + G)
    dev, got = attend(wl, q, T, tuning)
    ref = expected(wl, q, T)
    assert np.all(np.isfinite(got)), "non-finite output"
    assert np.max(np.abs(got - ref)) <= TOL[wl.dtype]
    empty = LENS.index(0)
    assert np.all(got[empty] == 0)
    one = LENS.index(1)                                       # L = 1: only the last query sees a token: its V row
    if T > 1:
        assert np.all(got[one, :T - 1] == 0)
        v_row = W.bf16_bits_to_f32(wl.v_cache[wl.block_table[one, 0], :, 0, :]).astype(np.float64)
        assert np.max(np.abs(got[one, T - 1] - np.repeat(v_row, G, axis=0))) <= 1e-6


@pytest.mark.parametrize("name,kw,T", [("thinker", dict(batch=12), 2), ("talker", dict(batch=48), 2),
                                       ("mixed", dict(batch=30, len_div=4), 4), ("long", dict(batch=2, len_div=4), 2)])
def test_reduced_configs(name, kw, T):
    wl = W.make(name, append=False, **kw)
    q = queries(wl, T, 2200)
    dev, got = attend(wl, q, T)
    assert np.max(np.abs(got - expected(wl, q, T))) <= TOL[wl.dtype]
    # one token per request through the same handle type equals the plain call on the last query
    dev1 = DeviceBatch(wl)
    dev1.q.copy_(to_dev(q.reshape(wl.B, T, wl.Hq, wl.D)[:, T - 1].copy(), wl.dtype))
    last = dev1.attend()
    assert np.max(np.abs(got[:, T - 1] - last)) <= 1e-5


def test_random_shapes():
    for seed in range(12):
        rng = np.random.default_rng(2300 + seed)
        G = int(rng.choice([1, 2, 3, 4, 7, 8])); T = int(rng.integers(2, 16 // G + 1)) if G < 8 else 2
        Hkv = int(rng.choice([1, 2, 4])); ps = int(rng.choice([16, 32])); B = int(rng.integers(1, 70))
        lens = rng.integers(0, int(rng.choice([40, 300, 1500])), size=B)
        wl = W.build("mt", 2400 + seed, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16,
                     pool_factor=float(rng.choice([1.0, 2.0])), extra_table_cols=int(rng.integers(0, 3)))
        q = queries(wl, T, 2500 + seed)
        tuning = {omni.OMNI_TUNE_TARGET_WORKGROUPS: int(rng.choice([64, 256, 512, 1024])),
                  omni.OMNI_TUNE_MIN_PARTITION: int(rng.choice([32, 128]))}
        dev, got = attend(wl, q, T, tuning)
        err = np.max(np.abs(got - expected(wl, q, T))) if got.size else 0.0
        assert np.all(np.isfinite(got)) and err <= TOL[wl.dtype], f"seed {seed}: G={G} T={T} B={B}: {err:.3e}"


def test_bf16_output_and_rerun_bit_identical():
    wl = W.make("thinker", batch=6, append=False)
    q = queries(wl, 2, 2600)
    _, a = attend(wl, q, 2, out_dtype=W.BF16)
    _, b = attend(wl, q, 2, out_dtype=W.BF16)
    assert np.array_equal(a, b)
    ref = expected(wl, q, 2)
    assert np.all(np.abs(a - ref) <= TOL[W.BF16] + np.abs(ref) * 2.0 ** -8)


def test_over_the_8bit_cache():
    wl = W.make("talker", batch=40, len_div=2, append=False)
    f8 = W.quantize_fp8(wl)
    T = 2
    q = queries(wl, T, 2700)
    fb = Fp8Batch(wl, f8, {omni.OMNI_TUNE_QUERY_TOKENS: T})
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), dtype=torch.float32, device="cuda")
    fb.h.omni_paged_decode_attn_fp8(to_dev(q, wl.dtype), fb.k, fb.v, fb.ks, fb.vs, fb.bt, fb.lens, float(wl.scale), out)
    torch.cuda.synchronize()
    n, offs = chunk_args(wl, T)
    ref = oracle.paged_prefill_attn_fp8(q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, n, offs, wl.scale).reshape(wl.B, T, wl.Hq, wl.D)
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= TOL[W.BF16]


def test_what_the_setting_rejects():
    h = omni.Handle(batch=4, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16, num_pages=64,
                    max_blocks_per_seq=8, kv_dtype=omni.OMNI_BF16)
    before = h.omni_workspace_bytes()
    h.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, 2)
    assert h.omni_workspace_bytes() > before                 # twice the partial rows
    h.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, 5)        # 5 x 7 heads: three passes of up to two tokens
    with pytest.raises(omni.OmniError):
        h.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, 0)
    with pytest.raises(omni.OmniError):
        h.omni_set_tuning(omni.OMNI_TUNE_KERNEL, omni.KERNEL_VALU)       # the vector-ALU kernel takes one token
    f32 = omni.Handle(batch=4, num_q_heads=4, num_kv_heads=2, head_dim=64, page_size=16, num_pages=64,
                      max_blocks_per_seq=8, kv_dtype=omni.OMNI_F32)
    with pytest.raises(omni.OmniError):
        f32.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, 2)


@pytest.mark.parametrize("G,Hkv,T,ps,fp8", [(7, 4, 2, 16, False), (4, 2, 4, 32, False), (1, 2, 16, 16, False),
                                            (8, 2, 2, 16, True), (3, 1, 5, 32, True), (7, 4, 5, 16, False),
                                            (8, 2, 3, 32, True)])
@pytest.mark.parametrize("force_pl", [0, 32])
def test_fused_step_equals_chunk_append_then_attention(G, Hkv, T, ps, fp8, force_pl):
    """omni_decode_step (and its 8-bit form) with T tokens per request: the T new rows land at positions L - T .. L - 1
    (wherever tile and page boundaries fall between them; rows of negative positions are skipped) before the attention
    reads them: same pools and output, bit for bit, as writing the rows first and attending afterwards."""
    lens = [2, 5, 16, 17, 31, 32, 33, 34, 35, 47, 48, 49, 64, 65, 66, 250, 0, 96, 97, 1, 3]
    wl = W.build("mtstep", 2800 + G + T, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    q = queries(wl, T, 2900)
    tuning = {omni.OMNI_TUNE_QUERY_TOKENS: T}
    if force_pl:
        tuning[omni.OMNI_TUNE_FORCE_PARTITION] = force_pl
    rng = np.random.default_rng(2950)
    if fp8:
        f8 = W.quantize_fp8(wl)
        pools_k, pools_v = f8.k_cache, f8.v_cache
        finite = np.array([b for b in range(256) if (b & 0x7F) < 0x60], dtype=np.uint8)
        k_new = rng.choice(finite, size=(wl.B, T, wl.Hkv, wl.D)).astype(np.uint8)
        v_new = rng.choice(finite, size=(wl.B, T, wl.Hkv, wl.D)).astype(np.uint8)
        poison = W.FP8_NAN_BYTE
    else:
        pools_k, pools_v = wl.k_cache, wl.v_cache
        k_new = W.f32_to_bf16_bits(rng.standard_normal((wl.B, T, wl.Hkv, wl.D)).astype(np.float32))
        v_new = W.f32_to_bf16_bits(rng.standard_normal((wl.B, T, wl.Hkv, wl.D)).astype(np.float32))
        poison = np.uint16(0x7fc1)
    want_k, want_v = pools_k.copy(), pools_v.copy()
    for b in range(wl.B):                                    # the newest rows are not in the pools yet
        for i in range(T):
            t = int(wl.context_lens[b]) - T + i
            if t >= 0:
                pg, sl = wl.block_table[b, t // wl.ps], t % wl.ps
                pools_k[pg, :, sl, :] = poison; pools_v[pg, :, sl, :] = poison
                want_k[pg, :, sl, :] = k_new[b, i]; want_v[pg, :, sl, :] = v_new[b, i]
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), dtype=torch.float32, device="cuda")
    dq = to_dev(q, wl.dtype)
    if fp8:
        fb = Fp8Batch(wl, f8, tuning)
        kn, vn = torch.from_numpy(k_new).cuda(), torch.from_numpy(v_new).cuda()
        fb.h.omni_decode_step_fp8(dq, kn, vn, fb.k, fb.v, fb.ks, fb.vs, fb.bt, fb.lens, float(wl.scale), out)
        torch.cuda.synchronize()
        got_k, got_v = fb.k.cpu().numpy(), fb.v.cpu().numpy()
        n, offs = chunk_args(wl, T)
        ref = oracle.paged_prefill_attn_fp8(q, want_k, want_v, f8.k_scale, f8.v_scale, wl.block_table, wl.context_lens,
                                            n, offs, wl.scale).reshape(wl.B, T, wl.Hq, wl.D)
        # attention alone over pools that already hold the rows
        f8.k_cache[:] = want_k; f8.v_cache[:] = want_v
        fb2 = Fp8Batch(wl, f8, tuning)
        out2 = torch.full_like(out, float("nan"))
        fb2.h.omni_paged_decode_attn_fp8(dq, fb2.k, fb2.v, fb2.ks, fb2.vs, fb2.bt, fb2.lens, float(wl.scale), out2)
    else:
        dev = DeviceBatch(wl, tuning=tuning)
        kn, vn = to_dev(k_new, wl.dtype), to_dev(v_new, wl.dtype)
        dev.h.omni_decode_step(dq, kn, vn, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, float(wl.scale), out)
        torch.cuda.synchronize()
        from gpu_util import bits_of
        got_k, got_v = bits_of(dev.k_cache), bits_of(dev.v_cache)
        wl.k_cache[:] = want_k; wl.v_cache[:] = want_v
        ref = expected(wl, q, T)
        dev2 = DeviceBatch(wl, tuning=tuning)
        out2 = torch.full_like(out, float("nan"))
        dev2.h.omni_paged_decode_attn(dq, dev2.k_cache, dev2.v_cache, dev2.block_table, dev2.context_lens, float(wl.scale), out2)
    torch.cuda.synchronize()
    assert np.array_equal(got_k.view(np.uint8), want_k.view(np.uint8)) and np.array_equal(got_v.view(np.uint8), want_v.view(np.uint8))
    got = out.cpu().numpy().astype(np.float64)
    assert np.array_equal(got, out2.cpu().numpy().astype(np.float64))
    bar = TOL[W.BF16] if not fp8 else max(TOL[W.BF16], 2.0 ** -9 * np.max(np.abs(ref)))
    assert np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= bar


# --------------------------------------------------------------------------- a different number of tokens per request
def ragged_expected(wl, q, T, n):
    """Request b brings n[b] <= T tokens in rows 0 .. n[b] - 1 of its T; a query at a negative position and the rows
    behind n[b] give zeros."""
    n_eff = np.minimum(n, wl.context_lens).astype(np.int32)
    offs = (np.arange(wl.B, dtype=np.int64) * T + (n - n_eff)).astype(np.int64)
    ref = oracle.paged_prefill_attn(q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, n_eff, offs, wl.scale, wl.dtype)
    return ref.reshape(wl.B, T, wl.Hq, wl.D)


@pytest.mark.parametrize("G,Hkv,T,ps", [(7, 4, 2, 16), (4, 2, 4, 32), (1, 2, 16, 16), (8, 2, 4, 16), (3, 1, 7, 16)])
@pytest.mark.parametrize("tuning", [{}, {omni.OMNI_TUNE_FORCE_PARTITION: 32}], ids=["default", "force32"])
def test_ragged_numbers_of_query_tokens(G, Hkv, T, ps, tuning):
    rng = np.random.default_rng(3000 + G + T)
    lens = np.array(LENS + [700, 33, 64, 129], dtype=np.int64)
    wl = W.build("mtr", 3100 + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    n = rng.integers(0, T + 1, size=wl.B).astype(np.int32)
    n[:4] = [T, 0, 1, T]                                     # all, none, one, all
    q = queries(wl, T, 3200 + G)
    q4 = q.reshape(wl.B, T, wl.Hq, wl.D)
    for b in range(wl.B):                                    # rows nobody brings hold NaN: they must not matter
        q4[b, n[b]:] = np.uint16(0x7fc0)
    tn = {omni.OMNI_TUNE_QUERY_TOKENS: T}
    tn.update(tuning)
    dev = DeviceBatch(wl, tuning=tn)
    dn = torch.from_numpy(n).cuda()
    dev.h.omni_set_query_lens(dn)
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), device="cuda", dtype=torch.float32)
    dev.h.omni_paged_decode_attn(to_dev(q, wl.dtype), dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens,
                                 float(wl.scale), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    qz = q.copy().reshape(wl.B, T, wl.Hq, wl.D)
    for b in range(wl.B):
        qz[b, n[b]:] = 0
    ref = ragged_expected(wl, qz.reshape(q.shape), T, n)
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref)) <= TOL[wl.dtype]
    for b in range(wl.B):
        assert np.all(got[b, n[b]:] == 0), f"request {b}: rows behind its {n[b]} tokens"
    # the array is read at every launch: new contents, same handle; then back to "every request brings T"
    n2 = np.minimum(n + 1, T).astype(np.int32)
    dn.copy_(torch.from_numpy(n2).cuda())
    q2 = queries(wl, T, 3300 + G)
    dq2 = to_dev(q2, wl.dtype)
    dev.h.omni_paged_decode_attn(dq2, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, float(wl.scale), out)
    torch.cuda.synchronize()
    qz2 = q2.copy().reshape(wl.B, T, wl.Hq, wl.D)
    for b in range(wl.B):
        qz2[b, n2[b]:] = 0
    assert np.max(np.abs(out.cpu().numpy().astype(np.float64) - ragged_expected(wl, qz2.reshape(q2.shape), T, n2))) <= TOL[wl.dtype]
    dev.h.omni_set_query_lens(None)
    dev.h.omni_paged_decode_attn(dq2, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, float(wl.scale), out)
    torch.cuda.synchronize()
    assert np.max(np.abs(out.cpu().numpy().astype(np.float64) - expected(wl, q2, T))) <= TOL[wl.dtype]


@pytest.mark.parametrize("G,Hkv,T,ps", [(7, 4, 2, 16), (4, 2, 4, 32), (2, 2, 9, 16)])
def test_ragged_fused_step_appends_only_the_rows_a_request_brings(G, Hkv, T, ps):
    rng = np.random.default_rng(3400 + G)
    lens = [2, 5, 16, 17, 31, 32, 33, 34, 35, 47, 48, 49, 64, 65, 66, 250, 0, 96, 97, 1, 3]
    wl = W.build("mtrs", 3500 + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    n = np.minimum(rng.integers(0, T + 1, size=wl.B), wl.context_lens).astype(np.int32)
    q = queries(wl, T, 3600)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((wl.B, T, wl.Hkv, wl.D)).astype(np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((wl.B, T, wl.Hkv, wl.D)).astype(np.float32))
    want_k, want_v = wl.k_cache.copy(), wl.v_cache.copy()
    for b in range(wl.B):
        for i in range(int(n[b])):
            t = int(wl.context_lens[b]) - int(n[b]) + i
            pg, sl = wl.block_table[b, t // wl.ps], t % wl.ps
            wl.k_cache[pg, :, sl, :] = np.uint16(0x7fc1); wl.v_cache[pg, :, sl, :] = np.uint16(0x7fc1)
            want_k[pg, :, sl, :] = k_new[b, i]; want_v[pg, :, sl, :] = v_new[b, i]
    dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_QUERY_TOKENS: T})
    dn = torch.from_numpy(n).cuda()
    dev.h.omni_set_query_lens(dn)
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), device="cuda", dtype=torch.float32)
    dev.h.omni_decode_step(to_dev(q, wl.dtype), to_dev(k_new, wl.dtype), to_dev(v_new, wl.dtype), dev.k_cache, dev.v_cache,
                           dev.block_table, dev.context_lens, float(wl.scale), out)
    torch.cuda.synchronize()
    from gpu_util import bits_of
    assert np.array_equal(bits_of(dev.k_cache).view(np.uint8), want_k.view(np.uint8))
    assert np.array_equal(bits_of(dev.v_cache).view(np.uint8), want_v.view(np.uint8))
    wl.k_cache[:] = want_k; wl.v_cache[:] = want_v
    qz = q.copy().reshape(wl.B, T, wl.Hq, wl.D)
    for b in range(wl.B):
        qz[b, n[b]:] = 0
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)) and np.max(np.abs(got - ragged_expected(wl, qz.reshape(q.shape), T, n))) <= TOL[wl.dtype]


def test_ragged_counts_over_the_8bit_cache_and_in_a_replayed_graph():
    """Per-request counts with the 8-bit cache, the call recorded once as a graph: every replay reads the counts (and
    the lengths and queries) of the moment."""
    wl = W.make("talker", batch=40, len_div=2, append=False)
    f8 = W.quantize_fp8(wl)
    T = 2
    fb = Fp8Batch(wl, f8, {omni.OMNI_TUNE_QUERY_TOKENS: T})
    rng = np.random.default_rng(3700)
    dn = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    fb.h.omni_set_query_lens(dn)
    dq = torch.zeros((wl.B * T, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
    out = torch.full((wl.B, T, wl.Hq, wl.D), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.Stream()
    call = lambda: fb.h.omni_paged_decode_attn_fp8(dq, fb.k, fb.v, fb.ks, fb.vs, fb.bt, fb.lens, float(wl.scale), out, stream)
    call()
    torch.cuda.synchronize()
    with omni.Graph(stream) as g:
        call()
    torch.cuda.synchronize()
    for rep in range(3):
        n = rng.integers(0, T + 1, size=wl.B).astype(np.int32)
        q = queries(wl, T, 3800 + rep)
        qz = q.copy().reshape(wl.B, T, wl.Hq, wl.D)
        for b in range(wl.B):
            qz[b, n[b]:] = 0
        dn.copy_(torch.from_numpy(n).cuda()); dq.copy_(to_dev(q, wl.dtype)); out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.launch()
        torch.cuda.synchronize()
        n_eff = np.minimum(n, wl.context_lens).astype(np.int32)
        offs = (np.arange(wl.B, dtype=np.int64) * T + (n - n_eff)).astype(np.int64)
        ref = oracle.paged_prefill_attn_fp8(qz.reshape(q.shape), f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                            wl.context_lens, n_eff, offs, wl.scale).reshape(wl.B, T, wl.Hq, wl.D)
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= TOL[W.BF16], f"replay {rep}"
    g.close()

