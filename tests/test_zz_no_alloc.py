"""omni_paged_decode_attn_static (no workspace from the caller, nothing allocated) against omni_paged_decode_attn and
the oracle, through the C ABI: two calls in a row, the second on a smaller batch, so the second call finds the first
one's plan words and partial rows in the shared array."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, DeviceBatch

pytestmark = pytest.mark.gpu


def static_call(dev: DeviceBatch) -> np.ndarray:
    dev.out.fill_(float("nan"))
    dev.h.omni_paged_decode_attn_static(dev.q, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens,
                                        float(dev.wl.scale), dev.out)
    torch.cuda.synchronize()
    return dev.out.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("kernel", [omni.KERNEL_MFMA, omni.KERNEL_VALU], ids=["mfma", "valu"])
def test_static_scratch_matches_the_workspace_call_twice_in_a_row(kernel):
    big = W.make("thinker", batch=12, len_div=2)            # several ranges per request: every request is merged
    small = W.make("thinker", seed=7, batch=5, len_div=4)
    for wl in (big, small):                                 # the second call is the smaller one
        dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel})
        want = dev.attend()                                 # the entry point with a registered workspace
        ref = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype)
        bare = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                           num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=omni.OMNI_BF16)
        bare.omni_set_tuning(omni.OMNI_TUNE_KERNEL, kernel)
        dev.h = bare                                        # a handle that never saw a workspace
        got = static_call(dev)
        assert np.all(np.isfinite(got))
        assert np.max(np.abs(got - ref)) <= TOL[wl.dtype]
        assert np.array_equal(got, want)                    # same kernels, same plan: the same bits


def test_static_scratch_holds_a_large_batch():
    """Above 256 requests the attention kernel leaves the tile offsets for the merge kernel in the workspace: here in
    the static array, twice in a row with different lengths."""
    for seed in (1, 2):
        rng = np.random.default_rng(40 + seed)
        lens = rng.integers(0, 200, size=300)
        wl = W.build("crowd", 7000 + seed, lens, Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16, pool_factor=1.2)
        dev = DeviceBatch(wl)
        want = dev.attend()
        ref = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype)
        bare = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                           num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=omni.OMNI_BF16)
        assert bare.omni_workspace_bytes() <= (8 << 20)
        dev.h = bare
        got = static_call(dev)
        assert np.max(np.abs(got - ref)) <= TOL[wl.dtype]
        assert np.array_equal(got, want)


def test_static_scratch_rejects_what_does_not_fit():
    h = omni.Handle(batch=4096, num_q_heads=64, num_kv_heads=4, head_dim=128, page_size=16, num_pages=4096,
                    max_blocks_per_seq=4, kv_dtype=omni.OMNI_BF16)
    assert h.omni_workspace_bytes() > (8 << 20)
    with pytest.raises(omni.OmniError) as e:
        h.omni_paged_decode_attn_static(256, 256, 256, 256, 256, 1.0, 256)
    assert e.value.status == 5
    f8 = omni.Handle(batch=4, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, num_pages=64,
                     max_blocks_per_seq=8, kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_BF16)
    with pytest.raises(omni.OmniError) as e:
        f8.omni_paged_decode_attn_static(256, 256, 256, 256, 256, 1.0, 256)
    assert e.value.status == 4
