"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle on the same seeded inputs.

Bars: max |err| <= 1e-5 for fp32 KV, <= 2e-3 for bf16 KV (fp32 output); append / gather / page-table indexing
bit-exact; bit-identical output from run to run and under a physical page permutation.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, DeviceBatch, bits_of, to_dev

pytestmark = pytest.mark.gpu


def oracle_out(wl, **kw):
    return oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale,
                                    wl.dtype, **kw)


def check(wl, tuning=None, label=""):
    dev = DeviceBatch(wl, tuning=tuning)
    got = dev.attend()
    ref = oracle_out(wl)
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    err = np.max(np.abs(got - ref)) if got.size else 0.0
    assert err <= TOL[wl.dtype], f"{label}: max|err| {err:.3e} > {TOL[wl.dtype]}"
    return dev, got, err


def kernels_for(wl):
    ks = [omni.KERNEL_VALU]
    if wl.dtype == W.BF16 and wl.D == 128:
        ks.append(omni.KERNEL_MFMA)
    return ks


# --------------------------------------------------------------------------- hand-worked cases
def test_hand_worked_cases_through_the_c_abi():
    """tests/golden/closed_form_cases.txt (rational softmax weights), zero-padded to head_dim 64 in fp32: both the
    split-free plan and a forced 32-token partition are held to 1e-5 of the hand-worked result."""
    import math
    import os

    def vals(txt):
        return [math.log(float(tok[2:])) if tok.startswith("ln") else float(tok) for tok in txt.split()]

    n = 0
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "closed_form_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, scale, q, K, V, exp = [f.strip() for f in line.split("|")]
        q = np.array(vals(q), dtype=np.float32)
        K = np.array([vals(r) for r in K.split(";")], dtype=np.float32)
        V = np.array([vals(r) for r in V.split(";")], dtype=np.float32)
        exp = np.array(vals(exp))
        L, d = K.shape
        wl = W.build("golden", 7, [L], Hq=1, Hkv=1, D=64, ps=16, dtype=W.F32, scale=float(scale))
        pg = wl.block_table[0, 0]
        wl.k_cache[pg, 0, :L] = 0.0; wl.v_cache[pg, 0, :L] = 0.0; wl.q[0, 0] = 0.0
        wl.k_cache[pg, 0, :L, :d] = K; wl.v_cache[pg, 0, :L, :d] = V; wl.q[0, 0, :d] = q
        for tuning in (None, {omni.OMNI_TUNE_FORCE_PARTITION: 32}):
            got = DeviceBatch(wl, tuning=tuning).attend()
            assert np.max(np.abs(got[0, 0, :d] - exp)) <= 1e-5 and np.all(got[0, 0, d:] == 0.0), name
        n += 1
    assert n == 4


# --------------------------------------------------------------------------- the five configurations
def test_tiny_config_fp32():
    wl = W.make("tiny")
    _, _, err = check(wl, label="tiny")
    print(f"tiny fp32 max|err| = {err:.3e}")
    for pl in (32, 64):
        check(wl, tuning={omni.OMNI_TUNE_FORCE_PARTITION: pl}, label=f"tiny PL={pl}")


REDUCED = [
    ("thinker", dict(batch=12)),                 # full lengths 512..4096, fewer requests
    ("talker", dict(batch=48)),
    ("long", dict(batch=2, len_div=4)),          # 4096..8192
    ("mixed", dict(batch=30, len_div=4)),
]


@pytest.mark.parametrize("name,kw", REDUCED, ids=[r[0] for r in REDUCED])
@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
@pytest.mark.parametrize("force_pl", [0, 160, 1024], ids=["plan", "pl160", "pl1024"])
def test_reduced_configs(name, kw, kernel, force_pl):
    wl = W.make(name, **kw)
    if wl.positions is not None:                  # talker: the appended token must be in the cache for the oracle too
        oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    tuning = {omni.OMNI_TUNE_KERNEL: kernel}
    if force_pl:
        tuning[omni.OMNI_TUNE_FORCE_PARTITION] = force_pl
    dev, _, err = check(wl, tuning=tuning, label=f"{name} k{kernel} pl{force_pl}")
    plan = dev.h.omni_debug_last_plan()
    assert plan["total_tokens"] == wl.total_tokens
    if force_pl:
        assert plan["partition_len"] == force_pl
        tiles = int(sum(-(-int(L) // 32) for L in wl.context_lens))
        assert plan["request_parts"] == -(-tiles // (force_pl // 32))
    print(f"{name} kernel={kernel} plan={plan} max|err|={err:.3e}")


# --------------------------------------------------------------------------- property sweep
EDGE_LENS = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 300, 511, 513, 1000]


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("ps", [16, 32])
@pytest.mark.parametrize("G", [1, 2, 4, 7, 8, 16])
def test_edge_lengths_and_groups(dtype, D, ps, G):
    Hkv = 2 if G < 16 else 1
    seed = 1000 + 7 * G + D + ps + (0 if dtype == W.F32 else 1)
    wl = W.build("edge", seed, EDGE_LENS, Hq=G * Hkv, Hkv=Hkv, D=D, ps=ps, dtype=dtype, pool_factor=1.3)
    ref = oracle_out(wl)
    for kernel in kernels_for(wl):
        for pl in (0, 32, 96):
            tuning = {omni.OMNI_TUNE_KERNEL: kernel}
            if pl:
                tuning[omni.OMNI_TUNE_FORCE_PARTITION] = pl
            got = DeviceBatch(wl, tuning=tuning).attend()
            assert np.all(np.isfinite(got))
            assert np.all(got[0] == 0.0), "empty request must give a zero row"
            err = np.max(np.abs(got - ref))
            assert err <= TOL[dtype], f"kernel {kernel} PL {pl}: {err:.3e}"
            # length 1: the output is the V row itself (exact in fp32)
            v1 = wl.v_cache[wl.block_table[1, 0], :, 0, :]
            v1 = v1.astype(np.float64) if dtype == W.F32 else W.bf16_bits_to_f32(v1).astype(np.float64)
            assert np.array_equal(got[1], np.repeat(v1, G, axis=0))


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes(seed):
    rng = np.random.default_rng(500 + seed)
    B = int(rng.integers(1, 40))
    lens = rng.integers(0, 700, size=B)
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
    Hkv = int(rng.choice([1, 2, 3]))
    ps = int(rng.choice([16, 32]))
    dtype = [W.F32, W.BF16][seed % 2]
    D = int(rng.choice([64, 128]))
    wl = W.build("rand", 900 + seed, lens, Hq=G * Hkv, Hkv=Hkv, D=D, ps=ps, dtype=dtype, pool_factor=2.0,
                 extra_table_cols=int(rng.integers(0, 3)))
    ref = oracle_out(wl)
    for kernel in kernels_for(wl):
        for tw in (1024, 64, 4096):
            got = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_TARGET_WORKGROUPS: tw,
                                          omni.OMNI_TUNE_MIN_PARTITION: 32}).attend()
            err = np.max(np.abs(got - ref))
            assert np.all(np.isfinite(got)) and err <= TOL[dtype], f"seed {seed} kernel {kernel} tw {tw}: {err:.3e}"


@pytest.mark.parametrize("B,G,Hkv,top", [(257, 7, 4, 300), (1000, 8, 2, 120), (4096, 16, 1, 70), (4096, 4, 2, 40)])
def test_large_batches(B, G, Hkv, top):
    """Batches above 256 requests take the workgroup-wide plan; 4096 is the largest batch a handle accepts (with 16
    heads per KV head the ring of segment slots shrinks to what still fits beside the plan)."""
    rng = np.random.default_rng(B + G)
    lens = rng.integers(0, top, size=B)
    lens[rng.integers(0, B, size=B // 50 + 1)] = 0
    wl = W.build("big", 4000 + B + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=16, dtype=W.BF16, pool_factor=1.3)
    ref = oracle_out(wl)
    for kernel in kernels_for(wl):
        got = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_MIN_PARTITION: 32}).attend()
        err = np.max(np.abs(got - ref))
        assert np.all(np.isfinite(got)) and err <= TOL[wl.dtype], f"B {B} kernel {kernel}: {err:.3e}"


@pytest.mark.parametrize("B,G,Hkv,tw", [(200, 8, 2, 8), (256, 7, 4, 16), (600, 16, 1, 8), (90, 4, 2, 2)])
def test_many_requests_per_range(B, G, Hkv, tw):
    """Few workgroups and many short requests: one range holds far more requests than the kernel keeps states for at a
    time, below and above the 256 requests up to which every wave plans for itself."""
    rng = np.random.default_rng(B * 7 + tw)
    lens = rng.integers(0, 100, size=B)
    lens[rng.integers(0, B, size=3)] = 700                      # and a few that span several runs of tiles
    wl = W.build("crowd", 5000 + B, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=16, dtype=W.BF16, pool_factor=1.5)
    ref = oracle_out(wl)
    for kernel in kernels_for(wl):
        got = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_TARGET_WORKGROUPS: tw,
                                      omni.OMNI_TUNE_MIN_PARTITION: 32}).attend()
        err = np.max(np.abs(got - ref))
        assert np.all(np.isfinite(got)) and err <= TOL[wl.dtype], f"B {B} kernel {kernel}: {err:.3e}"


def test_large_scores_and_peaked_softmax():
    # keys 6x larger: |scores| reach ~60, the softmax is nearly one-hot; the running-max rescale must hold up
    wl = W.build("peaked", 77, [700, 33, 1500], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    kf = W.bf16_bits_to_f32(wl.k_cache) * np.float32(6.0)
    wl.k_cache = np.where(np.isnan(kf), W.BF16_NAN_BITS, W.f32_to_bf16_bits(np.nan_to_num(kf))).astype(np.uint16)
    for kernel in kernels_for(wl):
        check(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_FORCE_PARTITION: 128}, label=f"peaked k{kernel}")


# --------------------------------------------------------------------------- bit-exact parts
@pytest.mark.parametrize("dtype,D,ps", [(W.F32, 64, 16), (W.BF16, 128, 16), (W.BF16, 128, 32), (W.F32, 128, 32)])
def test_kv_append_and_gather_bit_exact(dtype, D, ps):
    lens = [1, 16, 17, 33, 0, 250, 64]
    wl = W.build("app", 31, lens, Hq=8, Hkv=2, D=D, ps=ps, dtype=dtype, pool_factor=1.5, append=True)
    dev = DeviceBatch(wl)
    dev.append()
    torch.cuda.synchronize()
    oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    as_bytes = lambda a: a.view(np.uint8)
    assert np.array_equal(as_bytes(bits_of(dev.k_cache)), as_bytes(wl.k_cache))     # whole pool, NaN poison included
    assert np.array_equal(as_bytes(bits_of(dev.v_cache)), as_bytes(wl.v_cache))
    for b in (0, 3, 5):
        for cache_d, cache_h in ((dev.k_cache, wl.k_cache), (dev.v_cache, wl.v_cache)):
            ref = oracle.gather(cache_h, wl.block_table, wl.context_lens, b, wl.dtype)
            dense = torch.zeros((lens[b], wl.Hkv, D), dtype=cache_d.dtype, device="cuda")
            dev.h.omni_debug_gather(cache_d, dev.block_table, dev.context_lens, b, dense)
            torch.cuda.synchronize()
            assert np.array_equal(as_bytes(bits_of(dense)), as_bytes(ref))
    # attention after the append matches the oracle after its append
    got = dev.attend()
    assert np.max(np.abs(got - oracle_out(wl))) <= TOL[dtype]


@pytest.mark.parametrize("name,kw", [("thinker", dict(batch=10)), ("talker", dict(batch=40)), ("mixed", dict(batch=20, len_div=4))])
@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
@pytest.mark.parametrize("force_pl", [0, 64], ids=["plan", "pl64"])
def test_decode_step_equals_append_then_attention(name, kw, kernel, force_pl):
    """omni_decode_step == omni_kv_append at context_lens - 1 followed by omni_paged_decode_attn: same pool bits, same
    output bits; and both match the oracle's append + attention."""
    wl = W.make(name, append=True, **kw)
    lens = wl.context_lens.copy()
    lens[0] = 0                                        # an empty request: nothing is appended for it
    wl.context_lens = lens
    wl.positions = (lens - 1).astype(np.int32)
    tuning = {omni.OMNI_TUNE_KERNEL: kernel}
    if force_pl:
        tuning[omni.OMNI_TUNE_FORCE_PARTITION] = force_pl
    two = DeviceBatch(wl, tuning=tuning)
    two.context_lens.copy_(torch.from_numpy(lens).cuda())
    two.positions.copy_(torch.from_numpy(wl.positions).cuda())
    two.append()
    out_two = two.attend().copy()
    one = DeviceBatch(wl, tuning=tuning)
    one.context_lens.copy_(torch.from_numpy(lens).cuda())
    one.out.fill_(float("nan"))
    one.h.omni_decode_step(one.q, one.k_new, one.v_new, one.k_cache, one.v_cache, one.block_table, one.context_lens,
                           float(wl.scale), one.out)
    torch.cuda.synchronize()
    out_one = one.out.float().cpu().numpy().astype(np.float64)
    as_bytes = lambda a: a.view(np.uint8)
    assert np.array_equal(as_bytes(bits_of(one.k_cache)), as_bytes(bits_of(two.k_cache)))
    assert np.array_equal(as_bytes(bits_of(one.v_cache)), as_bytes(bits_of(two.v_cache)))
    assert np.array_equal(out_one, out_two)
    oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    assert np.array_equal(as_bytes(bits_of(one.k_cache)), as_bytes(wl.k_cache))
    assert np.max(np.abs(out_one - oracle_out(wl))) <= TOL[wl.dtype]


@pytest.mark.parametrize("seed", range(8))
def test_decode_step_random_shapes(seed):
    """The fused step on random batches whose lengths sit on and around tile and page boundaries (the new token first
    or last of a page, of a 32-token tile, alone in its request), any group size and page size, few and many
    workgroups: the pools come out as the oracle's append leaves them, bit for bit, and the output is the attention
    over them."""
    rng = np.random.default_rng(800 + seed)
    B = int(rng.integers(1, 48))
    G = int(rng.choice([1, 2, 4, 7, 8, 16]))
    Hkv = int(rng.choice([1, 2, 4]))
    ps = int(rng.choice([16, 32]))
    base = rng.integers(0, 12, size=B) * 32
    lens = np.maximum(base + rng.choice([0, 1, 2, 15, 16, 17, 31, 32, 33], size=B), 0)
    lens[rng.integers(0, B)] = 0
    wl = W.build("step", 6000 + seed, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5, append=True)
    tuning = {omni.OMNI_TUNE_TARGET_WORKGROUPS: int(rng.choice([16, 128, 512])), omni.OMNI_TUNE_MIN_PARTITION: 32}
    one = DeviceBatch(wl, tuning=tuning)
    one.out.fill_(float("nan"))
    one.h.omni_decode_step(one.q, one.k_new, one.v_new, one.k_cache, one.v_cache, one.block_table, one.context_lens,
                           float(wl.scale), one.out)
    torch.cuda.synchronize()
    got = one.out.float().cpu().numpy().astype(np.float64)
    oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    as_bytes = lambda a: a.view(np.uint8)
    assert np.array_equal(as_bytes(bits_of(one.k_cache)), as_bytes(wl.k_cache))
    assert np.array_equal(as_bytes(bits_of(one.v_cache)), as_bytes(wl.v_cache))
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - oracle_out(wl))) <= TOL[wl.dtype], (seed, B, G, Hkv, ps)


@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
def test_bit_identical_rerun_and_page_permutation(kernel):
    wl = W.make("thinker", batch=6)
    tuning = {omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_FORCE_PARTITION: 512}
    dev = DeviceBatch(wl, tuning=tuning)
    a = dev.attend().copy()
    b = dev.attend()
    assert np.array_equal(a, b), "run-to-run difference"
    rng = np.random.default_rng(5)
    perm = rng.permutation(wl.P)
    k2, v2 = np.empty_like(wl.k_cache), np.empty_like(wl.v_cache)
    k2[perm] = wl.k_cache
    v2[perm] = wl.v_cache
    wl2 = W.make("thinker", batch=6)
    wl2.k_cache, wl2.v_cache = k2, v2
    wl2.block_table = np.where(wl.block_table >= 0, perm[np.maximum(wl.block_table, 0)], -1).astype(np.int32)
    c = DeviceBatch(wl2, tuning=tuning).attend()
    assert np.array_equal(a, c), "output depends on the physical page assignment"


@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
def test_workspace_reuse_with_changing_inputs(kernel):
    """The same handle and workspace serve many calls: partial rows of an earlier call must never leak into a later
    one (the merge reads rows that another compute die wrote; a stale cached copy would show up here)."""
    wl = W.make("long", batch=3, len_div=4)
    dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_FORCE_PARTITION: 256})
    rng = np.random.default_rng(9)
    for it in range(6):
        qf = rng.standard_normal(wl.q.shape, dtype=np.float32) * np.float32(1.0 + it)
        wl.q = W.f32_to_bf16_bits(qf)
        dev.q.copy_(to_dev(wl.q, wl.dtype))
        if it % 2:                                            # lengths change too: fewer partitions than before
            wl.context_lens = np.maximum(1, wl.context_lens // 2).astype(np.int32)
            dev.context_lens.copy_(torch.from_numpy(wl.context_lens).cuda())
        got = dev.attend()
        err = np.max(np.abs(got - oracle_out(wl)))
        assert err <= TOL[wl.dtype], f"call {it}: {err:.3e}"


@pytest.mark.parametrize("dtype,D,kernel,G,Hkv", [(W.F32, 64, omni.KERNEL_VALU, 3, 3), (W.BF16, 128, omni.KERNEL_MFMA, 7, 4),
                                                   (W.BF16, 128, omni.KERNEL_VALU, 7, 4)], ids=["f32-valu", "bf16-mfma", "bf16-valu"])
def test_merge_never_reads_stale_partial_rows(dtype, D, kernel, G, Hkv):
    """One-tile ranges: every request is merged from up to 22 pieces written by workgroups on other compute dies.
    The query changes on every call and the partial-row area is refilled with NaN between calls, so a piece that the
    merging workgroup sees late (a missing device-scope release/acquire) shows up as NaN or as a wrong value."""
    rng = np.random.default_rng(504)
    lens = rng.integers(0, 700, size=35)
    wl = W.build("stale", 904, lens, Hq=G * Hkv, Hkv=Hkv, D=D, ps=16, dtype=dtype, pool_factor=2.0, extra_table_cols=1)
    dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel, omni.OMNI_TUNE_TARGET_WORKGROUPS: 4096,
                                  omni.OMNI_TUNE_MIN_PARTITION: 32})
    first_row = 256                                                      # behind the 256 bytes of plan words
    for rep in range(120):
        qf = rng.standard_normal(wl.q.shape, dtype=np.float32) * np.float32(1 + rep % 3)
        wl.q = qf if dtype == W.F32 else W.f32_to_bf16_bits(qf)
        dev.q.copy_(to_dev(wl.q, dtype))
        if rep % 2 == 0:
            dev.ws[first_row:].view(torch.float32).fill_(float("nan"))
        got = dev.attend()
        err = np.max(np.abs(got - oracle_out(wl)))
        assert np.all(np.isfinite(got)) and err <= TOL[dtype], f"call {rep}: {err}"


def test_bf16_output_is_rounded_fp32_result():
    wl = W.make("talker", batch=16, append=False)
    f32 = DeviceBatch(wl).attend()
    dev = DeviceBatch(wl, out_dtype=W.BF16)
    dev.attend()
    got_bits = bits_of(dev.out).astype(np.int32)
    want_bits = W.f32_to_bf16_bits(f32.astype(np.float32)).astype(np.int32)
    assert np.array_equal(got_bits, want_bits)


def test_max_context_hint_and_wide_table():
    # a block table far wider than any request (large max_blocks_per_seq) with a tight hint from the caller
    wl = W.build("wide", 3, [40, 700, 5], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16, extra_table_cols=4000)
    ref = oracle_out(wl)
    for hint in (0, 704):
        got = DeviceBatch(wl, max_context_hint=hint).attend()
        assert np.max(np.abs(got - ref)) <= TOL[wl.dtype]


@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
@pytest.mark.parametrize("B", [5, 64, 67, 300])
def test_lengths_at_any_four_byte_alignment(B, kernel):
    """context_lens needs 4-byte alignment only: the plan reads it in 16-byte pieces where the address allows and
    word by word otherwise (and for a batch that is no multiple of four); same bits either way."""
    rng = np.random.default_rng(40 + B)
    wl = W.build("align", 41 + B, rng.integers(0, 400, size=B), Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16)
    dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel})
    ref = oracle_out(wl)
    outs = []
    for off in range(4):
        buf = torch.zeros(B + 4, dtype=torch.int32, device="cuda")
        buf[off:off + B] = torch.from_numpy(wl.context_lens).cuda()
        dev.context_lens = buf[off:off + B]
        assert dev.context_lens.data_ptr() % 16 == 4 * off
        got = dev.attend()
        assert np.max(np.abs(got - ref)) <= TOL[wl.dtype], f"offset {off}"
        outs.append(got)
    assert all(np.array_equal(outs[0], o) for o in outs[1:])


def test_handles_with_different_shared_memory_needs_take_turns():
    """Two live handles on the same kernel variant whose ring layouts differ in size (the larger one above the 64 KB a
    kernel gets without asking): launches alternate, neither may lower what the other was granted."""
    rng = np.random.default_rng(600)
    big = W.build("lds-big", 601, rng.integers(1, 300, size=300), Hq=16, Hkv=2, D=128, ps=16, dtype=W.BF16)
    small = W.build("lds-small", 602, rng.integers(1, 300, size=16), Hq=16, Hkv=2, D=128, ps=16, dtype=W.BF16)
    a, b = DeviceBatch(big), DeviceBatch(small)
    ra, rb = oracle_out(big), oracle_out(small)
    for _ in range(3):
        assert np.max(np.abs(a.attend() - ra)) <= TOL[W.BF16]
        assert np.max(np.abs(b.attend() - rb)) <= TOL[W.BF16]


# --------------------------------------------------------------------------- full-size configurations, every row
FULL = ["thinker", "talker", "long", "mixed"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_every_row(name):
    """Benchmark launch configuration (default plan, auto kernel, fused and separate append) at full size, every
    output element against the oracle (OpenMP over (request, head): a fraction of a second per batch)."""
    wl = W.make(name)
    dev = DeviceBatch(wl)
    if wl.positions is not None:
        dev.append()
        oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)
    got = dev.attend()
    assert np.all(np.isfinite(got))
    plan = dev.h.omni_debug_last_plan()
    assert plan["total_tokens"] == wl.total_tokens
    ref = oracle_out(wl)
    err = float(np.max(np.abs(got - ref)))
    print(f"{name}: plan={plan} all {wl.B * wl.Hq} rows, max|err|={err:.3e}")
    assert err <= TOL[wl.dtype]
    if wl.positions is not None:
        # the step the benchmark times: the append fused into the attention kernel, on pools that lack the new rows
        dev2 = DeviceBatch(W.make(name))
        dev2.out.fill_(float("nan"))
        dev2.h.omni_decode_step(dev2.q, dev2.k_new, dev2.v_new, dev2.k_cache, dev2.v_cache, dev2.block_table,
                                dev2.context_lens, float(wl.scale), dev2.out)
        torch.cuda.synchronize()
        assert np.array_equal(dev2.out.cpu().numpy().astype(np.float64), got)
        for fused, separate in ((dev2.k_cache, dev.k_cache), (dev2.v_cache, dev.v_cache)):      # same pools, byte for byte
            assert np.array_equal(bits_of(fused).view(np.uint8), bits_of(separate).view(np.uint8))
