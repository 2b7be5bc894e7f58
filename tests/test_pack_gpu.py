"""omni_kv_pack / omni_kv_unpack through the C ABI against the oracle: bit-exact, and nothing else is written."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import workloads as W
from gpu_util import DeviceBatch, bits_of, to_dev

pytestmark = pytest.mark.gpu


def as_bytes(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint8)


def sentinel_like(a: np.ndarray) -> np.ndarray:
    return np.full_like(a, np.uint16(0x4321) if a.dtype == np.uint16 else np.float32(-7.25))


def layout(wl: W.Workload, rng, skip=(), gap=2):
    """Dense offsets in a shuffled request order with unowned rows between the requests."""
    offs = np.full(wl.B, -1, dtype=np.int64)
    run = 1
    for b in rng.permutation(wl.B):
        if b in skip:
            continue
        offs[b] = run
        run += int(wl.context_lens[b]) + gap
    return offs, run


CASES = [("tiny", {}), ("thinker", dict(batch=8, len_div=4)), ("talker", dict(batch=24, len_div=2)),
         ("mixed", dict(batch=16, len_div=8)), ("long", dict(batch=2, len_div=16))]


@pytest.mark.parametrize("name,kw", CASES)
def test_pack_and_unpack_match_oracle(name, kw):
    wl = W.make(name, append=False, **kw)
    rng = np.random.default_rng(5)
    lens = wl.context_lens.copy()
    lens[min(1, wl.B - 1)] = 0                               # an empty request
    wl.context_lens = lens
    offs, total = layout(wl, rng, skip=(0,))                 # request 0 is skipped
    dev = DeviceBatch(wl)
    offs_d = torch.from_numpy(offs).cuda()
    kd = to_dev(sentinel_like(np.zeros((total, wl.Hkv, wl.D), dtype=wl.k_cache.dtype)), wl.dtype)
    vd = kd.clone()
    dev.h.omni_kv_pack(dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, offs_d, kd, vd)
    torch.cuda.synchronize()
    for got, cache in ((kd, wl.k_cache), (vd, wl.v_cache)):
        want = oracle.kv_pack(cache, wl.block_table, lens, offs, total)
        owned = np.zeros(total, dtype=bool)
        for b in range(wl.B):
            if offs[b] >= 0:
                owned[offs[b]:offs[b] + lens[b]] = True
        g = bits_of(got)
        assert np.array_equal(as_bytes(g[owned]), as_bytes(want[owned]))
        assert np.array_equal(as_bytes(g[~owned]), as_bytes(sentinel_like(g[~owned])))      # rows nobody owns are untouched

    # unpack the dense copies into sentinel-filled pools: the oracle does the same on the host
    k_pool, v_pool = sentinel_like(wl.k_cache), sentinel_like(wl.v_cache)
    k_pool_d, v_pool_d = to_dev(k_pool, wl.dtype), to_dev(v_pool, wl.dtype)
    dev.h.omni_kv_unpack(kd, vd, k_pool_d, v_pool_d, dev.block_table, dev.context_lens, offs_d)
    torch.cuda.synchronize()
    oracle.kv_unpack(bits_of(kd), k_pool, wl.block_table, lens, offs)
    oracle.kv_unpack(bits_of(vd), v_pool, wl.block_table, lens, offs)
    assert np.array_equal(as_bytes(bits_of(k_pool_d)), as_bytes(k_pool))
    assert np.array_equal(as_bytes(bits_of(v_pool_d)), as_bytes(v_pool))


def test_moved_requests_attend_to_the_same_bits():
    """Pack a batch out of one pool and unpack it into another pool under a different block table (a request handed
    from a prefill engine to a decode engine): attention over the second pool returns the same bits."""
    wl = W.make("thinker", batch=8, len_div=4, append=False)
    src = DeviceBatch(wl)
    out_src = src.attend()
    rng = np.random.default_rng(9)
    perm = rng.permutation(wl.P).astype(np.int32)            # new physical page of every old page
    wl2 = W.make("thinker", batch=8, len_div=4, append=False)
    wl2.block_table = np.where(wl.block_table >= 0, perm[np.maximum(wl.block_table, 0)], -1).astype(np.int32)
    poison = np.uint16(0x7fc1)
    wl2.k_cache = np.full_like(wl.k_cache, poison)
    wl2.v_cache = np.full_like(wl.v_cache, poison)
    dst = DeviceBatch(wl2)
    offs = np.concatenate([[0], np.cumsum(wl.context_lens[:-1])]).astype(np.int64)
    total = int(wl.context_lens.sum())
    offs_d = torch.from_numpy(offs).cuda()
    kd = torch.empty((total, wl.Hkv, wl.D), dtype=torch.bfloat16, device="cuda")
    vd = torch.empty_like(kd)
    src.h.omni_kv_pack(src.k_cache, src.v_cache, src.block_table, src.context_lens, offs_d, kd, vd)
    dst.h.omni_kv_unpack(kd, vd, dst.k_cache, dst.v_cache, dst.block_table, dst.context_lens, offs_d)
    out_dst = dst.attend()
    assert np.array_equal(out_src, out_dst)


def test_pack_full_thinker_batch():
    wl = W.make("thinker", append=False)
    dev = DeviceBatch(wl)
    offs = np.concatenate([[0], np.cumsum(wl.context_lens[:-1])]).astype(np.int64)
    total = int(wl.context_lens.sum())
    offs_d = torch.from_numpy(offs).cuda()
    kd = torch.empty((total, wl.Hkv, wl.D), dtype=torch.bfloat16, device="cuda")
    vd = torch.empty_like(kd)
    dev.h.omni_kv_pack(dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, offs_d, kd, vd)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(kd), oracle.kv_pack(wl.k_cache, wl.block_table, wl.context_lens, offs, total))
    assert np.array_equal(bits_of(vd), oracle.kv_pack(wl.v_cache, wl.block_table, wl.context_lens, offs, total))
