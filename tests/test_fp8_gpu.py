"""Decode attention over an 8-bit (E4M3) KV cache with per-(page, head) scales, through the C ABI, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, to_dev

pytestmark = pytest.mark.gpu


class Fp8Batch:
    def __init__(self, wl: W.Workload, f8: W.Fp8Pools, tuning=None, out_dtype=omni.OMNI_F32):
        self.wl, self.f8 = wl, f8
        self.h = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                             num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=omni.OMNI_FP8_E4M3,
                             q_dtype=omni.OMNI_BF16, out_dtype=out_dtype)
        for k, v in (tuning or {}).items():
            self.h.omni_set_tuning(k, v)
        self.ws = self.h.alloc_workspace()
        self.q = to_dev(wl.q, wl.dtype)
        self.k, self.v = torch.from_numpy(f8.k_cache).cuda(), torch.from_numpy(f8.v_cache).cuda()
        self.ks, self.vs = torch.from_numpy(f8.k_scale).cuda(), torch.from_numpy(f8.v_scale).cuda()
        self.bt = torch.from_numpy(wl.block_table).cuda()
        self.lens = torch.from_numpy(wl.context_lens).cuda()
        self.out = torch.full((wl.B, wl.Hq, wl.D), float("nan"), dtype=torch.float32, device="cuda")

    def attend(self):
        self.out.fill_(float("nan"))
        self.h.omni_paged_decode_attn_fp8(self.q, self.k, self.v, self.ks, self.vs, self.bt, self.lens,
                                          float(self.wl.scale), self.out)
        torch.cuda.synchronize()
        return self.out.cpu().numpy().astype(np.float64)


def ref_of(wl, f8, pairs=None):
    return oracle.paged_decode_attn_fp8(wl.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, wl.scale, pairs=pairs)


@pytest.mark.parametrize("name,kw", [("thinker", dict(batch=12)), ("talker", dict(batch=48)), ("long", dict(batch=2, len_div=4)),
                                     ("mixed", dict(batch=30, len_div=4))])
@pytest.mark.parametrize("force_pl", [0, 128])
def test_reduced_configs_fp8(name, kw, force_pl):
    wl = W.make(name, append=False, **kw)
    f8 = W.quantize_fp8(wl)
    tuning = {omni.OMNI_TUNE_FORCE_PARTITION: force_pl} if force_pl else {}
    got = Fp8Batch(wl, f8, tuning).attend()
    err = np.max(np.abs(got - ref_of(wl, f8)))
    assert np.all(np.isfinite(got)) and err <= TOL[W.BF16], f"{name}: {err:.3e}"


@pytest.mark.parametrize("G,Hkv,ps", [(1, 3, 16), (16, 1, 16), (5, 2, 32), (7, 4, 16)])
def test_edge_lengths_fp8(G, Hkv, ps):
    lens = [1, 0, 16, 17, 31, 32, 33, 250, 64, 2]
    wl = W.build("f8edge", 60 + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.7)
    f8 = W.quantize_fp8(wl)
    for tw in (None, 64):
        tuning = {omni.OMNI_TUNE_MIN_PARTITION: 32}
        if tw:
            tuning[omni.OMNI_TUNE_TARGET_WORKGROUPS] = tw
        got = Fp8Batch(wl, f8, tuning).attend()
        ref = ref_of(wl, f8)
        assert np.all(got[1] == 0)                           # the empty request
        assert np.max(np.abs(got - ref)) <= TOL[W.BF16]
    # a one-token context returns its de-quantised V row (weight 1, scale split into two bf16 terms)
    import torch as _t
    v_row = _t.from_numpy(f8.v_cache[wl.block_table[0, 0], :, 0, :]).view(_t.float8_e4m3fn).to(_t.float64).numpy()
    v_row = v_row * f8.v_scale[wl.block_table[0, 0]].astype(np.float64)[:, None]
    assert np.max(np.abs(got[0] - np.repeat(v_row, G, axis=0))) <= 1e-4 * np.max(np.abs(v_row))


def test_full_size_thinker_fp8_sampled_rows():
    wl = W.make("thinker", append=False)
    f8 = W.quantize_fp8(wl)
    got = Fp8Batch(wl, f8).attend()
    rng = np.random.default_rng(4)
    pairs = [(int(b), int(h)) for b, h in zip(rng.integers(0, wl.B, 12), rng.integers(0, wl.Hq, 12))]
    ref = ref_of(wl, f8, pairs)
    for i, (b, h) in enumerate(pairs):
        assert np.max(np.abs(got[b, h] - ref[i])) <= TOL[W.BF16], (b, h)
    assert np.all(np.isfinite(got))


def test_fp8_handle_moves_bytes_and_rejects_16_bit_calls():
    wl = W.build("f8mv", 71, [40, 3, 64], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16, pool_factor=1.5)
    f8 = W.quantize_fp8(wl)
    fb = Fp8Batch(wl, f8)
    L = omni.lib()
    assert L.omni_paged_decode_attn(fb.h._h, fb.q.data_ptr(), fb.k.data_ptr(), fb.v.data_ptr(), fb.bt.data_ptr(),
                                    fb.lens.data_ptr(), 1.0, fb.out.data_ptr(), None) == 4
    with pytest.raises(omni.OmniError):
        fb.h.omni_set_tuning(omni.OMNI_TUNE_KERNEL, omni.KERNEL_VALU)
    # append: one byte row per (request, KV head), a bit copy
    rng = np.random.default_rng(1)
    k_new = rng.integers(0, 0x7F, size=(wl.B, wl.Hkv, wl.D), dtype=np.uint8)
    v_new = rng.integers(0, 0x7F, size=(wl.B, wl.Hkv, wl.D), dtype=np.uint8)
    pos = (wl.context_lens - 1).astype(np.int32)
    fb.h.omni_kv_append(torch.from_numpy(k_new).cuda(), torch.from_numpy(v_new).cuda(), fb.k, fb.v, fb.bt,
                        torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    want_k, want_v = f8.k_cache.copy(), f8.v_cache.copy()
    for b in range(wl.B):
        want_k[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = k_new[b]
        want_v[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = v_new[b]
    assert np.array_equal(fb.k.cpu().numpy(), want_k) and np.array_equal(fb.v.cpu().numpy(), want_v)
    # pack: dense byte rows
    offs = np.concatenate([[0], np.cumsum(wl.context_lens[:-1])]).astype(np.int64)
    total = int(wl.context_lens.sum())
    kd = torch.zeros((total, wl.Hkv, wl.D), dtype=torch.uint8, device="cuda")
    vd = torch.zeros_like(kd)
    fb.h.omni_kv_pack(fb.k, fb.v, fb.bt, fb.lens, torch.from_numpy(offs).cuda(), kd, vd)
    torch.cuda.synchronize()
    assert np.array_equal(kd.cpu().numpy(), oracle.kv_pack(want_k, wl.block_table, wl.context_lens, offs, total))
    # and a 16-bit handle rejects the fp8 call
    hb = omni.Handle(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=128, page_size=16, num_pages=8,
                     max_blocks_per_seq=4, kv_dtype=omni.OMNI_BF16)
    assert L.omni_paged_decode_attn_fp8(hb._h, 256, 256, 256, 256, 256, 256, 256, 1.0, 256, None) == 4


# --------------------------------------------------------------------------- multi-token queries over the 8-bit cache
def run_chunk_fp8(wl, f8, ch, max_q_len=None, tuning=None, split_workspace=False):
    fb = Fp8Batch(wl, f8, tuning)
    mq = max_q_len or max(ch.max_q_len, 1)
    if split_workspace:
        n = max(fb.h.omni_workspace_bytes(), fb.h.omni_prefill_workspace_bytes(mq))
        fb.ws = torch.full((n // 4,), float("nan"), dtype=torch.float32, device="cuda")
        fb.h.omni_set_workspace(fb.ws)
    q = to_dev(ch.q, wl.dtype)
    q_lens, q_offs = torch.from_numpy(ch.q_lens).cuda(), torch.from_numpy(ch.q_offsets).cuda()
    out = torch.full((ch.total, wl.Hq, wl.D), float("nan"), dtype=torch.float32, device="cuda")
    fb.h.omni_paged_prefill_attn_fp8(q, fb.k, fb.v, fb.ks, fb.vs, fb.bt, fb.lens, q_lens, q_offs, mq, float(wl.scale), out)
    torch.cuda.synchronize()
    return fb, out.cpu().numpy().astype(np.float64)


def check_chunk_fp8(wl, f8, ch, label="", **kw):
    fb, got = run_chunk_fp8(wl, f8, ch, **kw)
    ref = oracle.paged_prefill_attn_fp8(ch.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale)
    owned = np.zeros(ch.total, dtype=bool)
    for b in range(wl.B):
        owned[ch.q_offsets[b]:ch.q_offsets[b] + ch.q_lens[b]] = True
    assert np.all(np.isnan(got[~owned])), f"{label}: rows nobody owns were written"
    err = np.max(np.abs(got[owned] - ref[owned])) if owned.any() else 0.0
    assert np.all(np.isfinite(got[owned])) and err <= TOL[W.BF16], f"{label}: max|err| {err:.3e}"
    return got, ref


@pytest.mark.parametrize("G,Hkv,ps", [(7, 4, 16), (8, 2, 16), (4, 8, 32), (16, 1, 16), (1, 2, 16), (3, 2, 32)])
def test_chunks_of_many_shapes_fp8(G, Hkv, ps):
    lens = [300, 64, 1, 0, 33, 257, 96, 40]
    q_lens = [300, 1, 1, 0, 17, 100, 37, 40]                 # whole prompt, one token, nothing, ragged pieces
    wl = W.build("f8chunk", 720 + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, q_lens, 820 + G, in_cache=True, gap=3)
    f8 = W.quantize_fp8(wl)
    got, ref = check_chunk_fp8(wl, f8, ch, label=f"G{G} Hkv{Hkv} ps{ps}")
    # the first query of the whole-prompt request sees token 0 only: its de-quantised V row, rounded once to fp16
    v0 = torch.from_numpy(f8.v_cache[wl.block_table[0, 0], :, 0, :]).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    v0 = v0 * f8.v_scale[wl.block_table[0, 0]].astype(np.float64)[:, None]
    assert np.max(np.abs(got[ch.q_offsets[0]] - np.repeat(v0, G, axis=0))) <= 2.0 ** -11 * np.max(np.abs(v0))


def test_one_token_chunks_agree_with_the_decode_call_fp8():
    wl = W.make("talker", batch=24, len_div=2, append=False)
    f8 = W.quantize_fp8(wl)
    ch = W.add_chunk(wl, [1] * wl.B, 5, in_cache=True)
    ch.q[:] = wl.q                                            # the decode batch's own queries, one row per request
    got, _ = check_chunk_fp8(wl, f8, ch, label="one-token")
    dec = Fp8Batch(wl, f8).attend()
    assert np.max(np.abs(got[ch.q_offsets] - dec)) <= 2 * TOL[W.BF16]


@pytest.mark.parametrize("splits,min_split", [(0, 256), (3, 64), (16, 128)], ids=lambda v: str(v))
def test_context_split_fp8(splits, min_split):
    wl = W.build("f8split", 1600, [2100, 64, 700, 1, 0], Hq=28, Hkv=4, D=128, ps=16, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, [37, 64, 400, 1, 0], 1601, in_cache=True, gap=2)
    f8 = W.quantize_fp8(wl)
    check_chunk_fp8(wl, f8, ch, label=f"splits={splits}", split_workspace=True,
                    tuning={omni.OMNI_TUNE_PREFILL_SPLITS: splits, omni.OMNI_TUNE_PREFILL_MIN_SPLIT: min_split})


def test_every_byte_value_and_uneven_scales_fp8():
    """K and V pools that hold every finite E4M3 byte, page scales spread over 2^-6 .. 2^3 (not powers of two):
    a wrong decode of any byte, or a scale applied to the wrong half of a tile, shows against the oracle."""
    rng = np.random.default_rng(77)
    wl = W.build("f8bytes", 1700, [130, 47], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [50, 47], 1701, in_cache=True)
    f8 = W.quantize_fp8(wl)
    finite = np.array([b for b in range(256) if (b & 0x7F) != 0x7F], dtype=np.uint8)
    live = f8.k_cache != W.FP8_NAN_BYTE
    f8.k_cache[live] = rng.choice(finite, size=int(live.sum()))
    live = f8.v_cache != W.FP8_NAN_BYTE
    f8.v_cache[live] = rng.choice(finite, size=int(live.sum()))
    f8.k_scale[:] = np.exp2(rng.uniform(-9, -5, size=f8.k_scale.shape)).astype(np.float32)     # scores stay moderate
    f8.v_scale[:] = np.exp2(rng.uniform(-6, 3, size=f8.v_scale.shape)).astype(np.float32)
    fb, got = run_chunk_fp8(wl, f8, ch)
    ref = oracle.paged_prefill_attn_fp8(ch.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                                        wl.context_lens, ch.q_lens, ch.q_offsets, wl.scale)
    # V reaches 448 * 8 here: the bar scales with the values (weights and V both carry 2^-12 relative rounding)
    bound = 2.0 ** -10 * np.max(np.abs(ref))
    assert np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= max(bound, TOL[W.BF16])


def test_fp8_prefill_argument_checks():
    wl = W.build("f8args", 1800, [40], Hq=4, Hkv=2, D=128, ps=16, dtype=W.BF16)
    f8 = W.quantize_fp8(wl)
    fb = Fp8Batch(wl, f8)
    L = omni.lib()
    assert L.omni_paged_prefill_attn_fp8(fb.h._h, 256, 256, 256, None, 256, 256, 256, 256, 256, 8, 1.0, 256, None) == 1
    assert L.omni_paged_prefill_attn_fp8(fb.h._h, 256, 256, 256, 256, 256, 256, 256, 256, 256, 0, 1.0, 256, None) == 2
    assert L.omni_paged_prefill_attn_fp8(fb.h._h, 256, 256, 256, 256, 256, 256, 256, 256, 256, 8, 0.0, 256, None) == 2
    hb = omni.Handle(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=128, page_size=16, num_pages=8,
                     max_blocks_per_seq=4, kv_dtype=omni.OMNI_BF16)
    assert L.omni_paged_prefill_attn_fp8(hb._h, 256, 256, 256, 256, 256, 256, 256, 256, 256, 8, 1.0, 256, None) == 4
    assert L.omni_paged_prefill_attn(fb.h._h, 256, 256, 256, 256, 256, 256, 256, 8, 1.0, 256, None) == 4


@pytest.mark.parametrize("name,kw,force_pl", [("thinker", dict(batch=12), 0), ("talker", dict(batch=48), 0),
                                              ("mixed", dict(batch=30, len_div=4), 128), ("long", dict(batch=2, len_div=4), 0)])
def test_decode_step_fp8_equals_append_then_attention(name, kw, force_pl):
    """omni_decode_step_fp8 = omni_kv_append of the new byte rows at context_lens - 1, then omni_paged_decode_attn_fp8:
    same pools and same output bit for bit, and the output within the bar of the oracle over the appended pools."""
    wl = W.make(name, append=False, **kw)
    f8 = W.quantize_fp8(wl)
    rng = np.random.default_rng(3)
    finite = np.array([b for b in range(256) if (b & 0x7F) != 0x7F], dtype=np.uint8)
    k_new = rng.choice(finite[(finite & 0x7F) < 0x60], size=(wl.B, wl.Hkv, wl.D)).astype(np.uint8)   # moderate magnitudes
    v_new = rng.choice(finite, size=(wl.B, wl.Hkv, wl.D)).astype(np.uint8)
    pos = (wl.context_lens - 1).astype(np.int32)
    # the last token's rows are not in the pools yet
    for b in range(wl.B):
        if pos[b] >= 0:
            f8.k_cache[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = W.FP8_NAN_BYTE
            f8.v_cache[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = W.FP8_NAN_BYTE
    tuning = {omni.OMNI_TUNE_FORCE_PARTITION: force_pl} if force_pl else {}
    two, one = Fp8Batch(wl, f8, tuning), Fp8Batch(wl, f8, tuning)
    kn, vn = torch.from_numpy(k_new).cuda(), torch.from_numpy(v_new).cuda()
    two.h.omni_kv_append(kn, vn, two.k, two.v, two.bt, torch.from_numpy(pos).cuda())
    ref_two = two.attend()
    one.out.fill_(float("nan"))
    one.h.omni_decode_step_fp8(one.q, kn, vn, one.k, one.v, one.ks, one.vs, one.bt, one.lens, float(wl.scale), one.out)
    torch.cuda.synchronize()
    got = one.out.cpu().numpy().astype(np.float64)
    assert np.array_equal(one.k.cpu().numpy(), two.k.cpu().numpy()) and np.array_equal(one.v.cpu().numpy(), two.v.cpu().numpy())
    assert np.array_equal(got, ref_two)
    want_k, want_v = f8.k_cache.copy(), f8.v_cache.copy()
    for b in range(wl.B):
        if pos[b] >= 0:
            want_k[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = k_new[b]
            want_v[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :] = v_new[b]
    assert np.array_equal(one.k.cpu().numpy(), want_k) and np.array_equal(one.v.cpu().numpy(), want_v)
    ref = oracle.paged_decode_attn_fp8(wl.q, want_k, want_v, f8.k_scale, f8.v_scale, wl.block_table, wl.context_lens, wl.scale)
    bar = max(TOL[W.BF16], 2.0 ** -9 * np.max(np.abs(ref)))           # V bytes reach 448 times the page scale here
    assert np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= bar



# --------------------------------------------------------------------------- the append that quantises
def _append_quant_on_gpu(wl, f8, headroom):
    dev = Fp8Batch(wl, f8)
    k_new, v_new = to_dev(wl.k_new, wl.dtype), to_dev(wl.v_new, wl.dtype)
    pos = torch.from_numpy(wl.positions).cuda()
    dev.h.omni_kv_append_quant_fp8(k_new, v_new, dev.k, dev.v, dev.ks, dev.vs, dev.bt, pos, headroom)
    torch.cuda.synchronize()
    return dev


def test_hardware_e4m3_conversion_equals_the_oracles_encoder_on_every_boundary():
    """Rows made of every representable E4M3 magnitude, every midpoint between neighbours and the bf16 values next to
    each midpoint, both signs, plus values beyond the range and NaN, written at a slot other than 0 into pages whose
    scale is 1: the bytes are the encoder's, bit for bit (round to nearest even, saturation, NaN byte)."""
    grid = np.array(sorted({oracle.fp8_e4m3_decode(c) for c in range(0x7F)}), dtype=np.float64)
    mids = ((grid[:-1] + grid[1:]) / 2).astype(np.float32)
    up = W.bf16_bits_to_f32((W.f32_to_bf16_bits(mids).astype(np.uint32) + 1).astype(np.uint16))      # next bf16 above
    dn = W.bf16_bits_to_f32((W.f32_to_bf16_bits(mids).astype(np.uint32) - 1).astype(np.uint16))      # next bf16 below
    vals = np.concatenate([grid.astype(np.float32), mids, up, dn[1:], [450.0, 464.0, 2.0 ** 20, 2.0 ** 127, np.nan]]).astype(np.float32)
    vals = np.concatenate([vals, -vals])
    assert np.array_equal(W.bf16_bits_to_f32(W.f32_to_bf16_bits(vals[~np.isnan(vals)])), vals[~np.isnan(vals)])  # all are bf16 values
    D, Hkv = 128, 2
    B = -(-vals.size // (D * Hkv))
    flat = np.zeros(B * Hkv * D, dtype=np.float32)
    flat[:vals.size] = vals
    lens = np.full(B, 5, dtype=np.int64)                              # position 4: never slot 0
    wl = W.build("cvt", 300, lens, Hq=2 * Hkv, Hkv=Hkv, D=D, ps=16, dtype=W.BF16, append=True)
    f8 = W.quantize_fp8(wl)
    f8.k_scale[:] = 1.0
    f8.v_scale[:] = 0.5                                               # V: the same values through a scale of one half
    wl.k_new = W.f32_to_bf16_bits(flat.reshape(B, Hkv, D))
    wl.v_new = W.f32_to_bf16_bits((flat * np.float32(0.5)).reshape(B, Hkv, D))
    dev = _append_quant_on_gpu(wl, f8, 1.0)
    k8, v8, ks, vs = f8.k_cache.copy(), f8.v_cache.copy(), f8.k_scale.copy(), f8.v_scale.copy()
    oracle.kv_append_quant_fp8(wl.k_new, wl.v_new, k8, v8, ks, vs, wl.block_table, wl.positions, 1.0)
    assert np.array_equal(dev.k.cpu().numpy(), k8) and np.array_equal(dev.v.cpu().numpy(), v8)
    assert np.array_equal(dev.ks.cpu().numpy(), ks) and np.array_equal(dev.vs.cpu().numpy(), vs)
    page, slot = wl.block_table[0, 0], 4
    want = np.array([oracle.fp8_e4m3_encode(float(x)) for x in flat[:D]], dtype=np.uint8)
    assert np.array_equal(dev.k.cpu().numpy()[page, 0, slot], want)


@pytest.mark.parametrize("headroom", [1.0, 2.0, 1.37])
@pytest.mark.parametrize("ps,Hkv", [(16, 2), (32, 4), (16, 1)])
def test_quantising_append_whole_pools_and_scales(headroom, ps, Hkv):
    """Rows spanning several binades, positions at slot 0 (the page's scale is set from the row) and elsewhere (the
    page's scale is used, values beyond it saturate), empty requests skipped: pools and scales byte for byte."""
    rng = np.random.default_rng(400 + ps + Hkv)
    lens = np.concatenate([[ps + 1, 2 * ps, 5, 3 * ps + 1, 0, 1, ps], rng.integers(1, 200, size=40)]).astype(np.int64)
    wl = W.build("quant", 401 + ps, lens, Hq=4 * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, append=True, pool_factor=1.5)
    f8 = W.quantize_fp8(wl)
    kf = (rng.standard_normal(wl.k_new.shape) * np.exp2(rng.integers(-6, 4, size=wl.k_new.shape[:2] + (1,)))).astype(np.float32)
    vf = (rng.standard_normal(wl.v_new.shape) * 3.0).astype(np.float32)
    kf[3, 0, 7] = np.nan                                              # a NaN element: NaN byte, and it never sets a scale
    wl.k_new, wl.v_new = W.f32_to_bf16_bits(kf), W.f32_to_bf16_bits(vf)
    wl.k_new[3, 0, 7] = W.BF16_NAN_BITS
    dev = _append_quant_on_gpu(wl, f8, headroom)
    k8, v8, ks, vs = f8.k_cache.copy(), f8.v_cache.copy(), f8.k_scale.copy(), f8.v_scale.copy()
    oracle.kv_append_quant_fp8(wl.k_new, wl.v_new, k8, v8, ks, vs, wl.block_table, wl.positions, headroom)
    assert np.array_equal(dev.ks.cpu().numpy(), ks) and np.array_equal(dev.vs.cpu().numpy(), vs)
    assert np.array_equal(dev.k.cpu().numpy(), k8) and np.array_equal(dev.v.cpu().numpy(), v8)


def test_decode_over_rows_the_library_quantised_itself():
    """A talker-shaped batch whose newest token is quantised by omni_kv_append_quant_fp8, then attended to: equal to
    the oracle's append followed by the oracle's attention over the 8-bit cache."""
    wl = W.make("talker", batch=40, append=True)
    f8 = W.quantize_fp8(wl)
    dev = _append_quant_on_gpu(wl, f8, 1.5)
    got = dev.attend()
    oracle.kv_append_quant_fp8(wl.k_new, wl.v_new, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl.block_table,
                               wl.positions, 1.5)
    err = np.max(np.abs(got - ref_of(wl, f8)))
    assert np.all(np.isfinite(got)) and err <= TOL[W.BF16], f"{err:.3e}"


def test_quantising_append_argument_checks():
    wl = W.make("talker", batch=4, append=True)
    f8 = W.quantize_fp8(wl)
    dev = Fp8Batch(wl, f8)
    for bad in (0.5, float("nan"), 1e9):
        with pytest.raises(omni.OmniError) as e:
            dev.h.omni_kv_append_quant_fp8(dev.q, dev.q, dev.k, dev.v, dev.ks, dev.vs, dev.bt, dev.lens, bad)
        assert e.value.status == 2
    bf = omni.Handle(batch=4, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, num_pages=64,
                     max_blocks_per_seq=8, kv_dtype=omni.OMNI_BF16)
    with pytest.raises(omni.OmniError) as e:
        bf.omni_kv_append_quant_fp8(dev.q, dev.q, dev.k, dev.v, dev.ks, dev.vs, dev.bt, dev.lens, 1.0)
    assert e.value.status == 4
