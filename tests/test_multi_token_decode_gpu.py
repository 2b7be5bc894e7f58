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
                                        (5, 1, 3, 32), (16, 1, 1, 16), (2, 2, 7, 16)])
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
    for bad in (0, 3):                                       # 3 x 7 heads do not fit 16 columns
        with pytest.raises(omni.OmniError):
            h.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, bad)
    with pytest.raises(omni.OmniError):
        h.omni_set_tuning(omni.OMNI_TUNE_KERNEL, omni.KERNEL_VALU)       # the vector-ALU kernel takes one token
    ws = h.alloc_workspace()
    L = omni.lib()
    import ctypes as C
    assert L.omni_decode_step(h._h, 256, 256, 256, 256, 256, 256, 256, C.c_float(1.0), 256, None) == 4
    f32 = omni.Handle(batch=4, num_q_heads=4, num_kv_heads=2, head_dim=64, page_size=16, num_pages=64,
                      max_blocks_per_seq=8, kv_dtype=omni.OMNI_F32)
    with pytest.raises(omni.OmniError):
        f32.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, 2)
