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
