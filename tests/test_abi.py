"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and rejects bad arguments."""
import ctypes as C
import os
import re

import pytest

from paper_2602_02204_amd import binding as omni

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good(**over):
    kw = dict(batch=4, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, num_pages=64,
              max_blocks_per_seq=8, kv_dtype=omni.OMNI_BF16)
    kw.update(over)
    return kw


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "omni_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(omni_[a-z0-9_]+)\s*\(", text))
    assert declared == set(omni.EXPORTS)
    L = omni.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    assert omni.status_string(0) == "ok"
    assert len({omni.status_string(i) for i in range(8)}) == 8


@pytest.mark.parametrize("over,status", [
    (dict(batch=0), 2), (dict(num_q_heads=7), 2), (dict(num_kv_heads=0), 2), (dict(num_pages=-1), 2),
    (dict(kv_dtype=5), 3), (dict(q_dtype=omni.OMNI_F32), 3), (dict(kv_dtype=omni.OMNI_F32, out_dtype=omni.OMNI_BF16), 3),
    (dict(head_dim=96), 4), (dict(page_size=8), 4), (dict(num_q_heads=34, num_kv_heads=2), 4), (dict(batch=5000), 4),
])
def test_create_rejects(over, status):
    with pytest.raises(omni.OmniError) as e:
        omni.Handle(**good(**over))
    assert e.value.status == status


def test_create_null_and_struct_size():
    L = omni.lib()
    h = C.c_void_p()
    assert L.omni_create(None, C.byref(h)) == 1
    d = omni.omni_attn_desc_t(4, 4, 8, 2, 128, 16, 64, 8, 1, 1, 0, 0)      # wrong struct_size
    assert L.omni_create(C.byref(d), C.byref(h)) == 2 and not h.value


def test_workspace_and_null_argument_errors_without_touching_the_gpu():
    h = omni.Handle(**good())
    n = h.omni_workspace_bytes()
    assert n > 0 and n % 256 == 0
    L = omni.lib()
    # no workspace yet
    assert L.omni_paged_decode_attn(h._h, 256, 256, 256, 256, 256, C.c_float(1.0), 256, None) == 5
    assert L.omni_set_workspace(h._h, None, n) == 1
    assert L.omni_set_workspace(h._h, 4096 + 8, n) == 5          # misaligned
    assert L.omni_set_workspace(h._h, 4096, n - 1) == 5          # too small
    assert L.omni_paged_decode_attn(h._h, None, 256, 256, 256, 256, C.c_float(1.0), 256, None) == 1
    assert L.omni_kv_append(h._h, None, 256, 256, 256, 256, 256, None) == 1
    assert L.omni_kv_append(None, 256, 256, 256, 256, 256, 256, None) == 1
    assert L.omni_debug_gather(h._h, 256, 256, 256, 99, 256, None) == 2
    assert L.omni_kv_append(h._h, 256 + 8, 256, 256, 256, 256, 256, None) == 2        # rows move in 16-byte pieces
    assert L.omni_kv_append(h._h, 256, 256, 256, 256, 256 + 2, 256, None) == 2        # int32 array off by 2 bytes


def test_tuning_validation_and_plan():
    h = omni.Handle(**good())
    plan = h.omni_get_plan()
    assert plan["kernel"] == omni.KERNEL_MFMA and plan["threads_per_workgroup"] == 256
    assert plan["merge_grid"] == 4 * 2 and plan["partition_grid"] == 512 and plan["max_request_parts"] == 256 + 4
    h.omni_set_tuning(omni.OMNI_TUNE_KERNEL, omni.KERNEL_VALU)
    assert h.omni_get_plan()["kernel"] == omni.KERNEL_VALU
    for key, val in [(omni.OMNI_TUNE_KERNEL, 3), (omni.OMNI_TUNE_TARGET_WORKGROUPS, 0),
                     (omni.OMNI_TUNE_MIN_PARTITION, 48), (omni.OMNI_TUNE_FORCE_PARTITION, 40), (99, 1)]:
        with pytest.raises(omni.OmniError):
            h.omni_set_tuning(key, val)
    # context split of multi-token queries: no workspace where the grid fills the chip or the split is switched off
    one = omni.Handle(**good(batch=1, max_blocks_per_seq=2048))
    assert one.omni_prefill_workspace_bytes(512) > 0
    assert omni.Handle(**good(batch=64, max_blocks_per_seq=2048)).omni_prefill_workspace_bytes(512) == 0
    assert omni.Handle(**good(batch=1, max_blocks_per_seq=8)).omni_prefill_workspace_bytes(64) == 0    # 128 tokens at most
    one.omni_set_tuning(omni.OMNI_TUNE_PREFILL_SPLITS, 1)
    assert one.omni_prefill_workspace_bytes(512) == 0
    one.omni_set_tuning(omni.OMNI_TUNE_PREFILL_SPLITS, 3)
    Hq, D = good()["num_q_heads"], good()["head_dim"]
    assert one.omni_prefill_workspace_bytes(100) >= 100 * Hq * 3 * (D + 2) * 4
    with pytest.raises(omni.OmniError):
        one.omni_prefill_workspace_bytes(0)
    for key, val in [(omni.OMNI_TUNE_PREFILL_SPLITS, 17), (omni.OMNI_TUNE_PREFILL_MIN_SPLIT, 0),
                     (omni.OMNI_TUNE_PREFILL_MIN_SPLIT, 96)]:
        with pytest.raises(omni.OmniError):
            one.omni_set_tuning(key, val)
    short = omni.Handle(**good(batch=1, max_blocks_per_seq=8))
    short.omni_set_tuning(omni.OMNI_TUNE_PREFILL_MIN_SPLIT, 64)               # 128 tokens: two shares of 64
    assert short.omni_prefill_workspace_bytes(64) >= 64 * Hq * 2 * (D + 2) * 4
    big = omni.Handle(**good(max_blocks_per_seq=4096))
    before = big.omni_workspace_bytes()
    big.omni_set_tuning(omni.OMNI_TUNE_FORCE_PARTITION, 32)
    assert big.omni_workspace_bytes() > before                  # more partitions -> more partial rows
    f32 = omni.Handle(**good(kv_dtype=omni.OMNI_F32))
    assert f32.omni_get_plan()["kernel"] == omni.KERNEL_VALU
    with pytest.raises(omni.OmniError):
        f32.omni_set_tuning(omni.OMNI_TUNE_KERNEL, omni.KERNEL_MFMA)


@pytest.mark.parametrize("kv", [omni.OMNI_BF16, omni.OMNI_FP8_E4M3], ids=["bf16", "fp8"])
def test_shared_memory_layout_fits_for_every_batch_and_group(kv):
    """Over the whole (batch, columns) range the library accepts: the dynamic and static shared memory of the
    matrix-core kernel fit two workgroups per compute unit (half of 160 KB each) wherever the layout says so, never
    exceed what the launch may ask for, and K is staged only where its staging area leaves room for five states."""
    for B in (1, 64, 256, 257, 1024, 2048, 3000, 4096):
        for G in (1, 4, 7, 8, 16):
            for T in (1, 2, 16 // G if G < 16 else 1):
                h = omni.Handle(**good(batch=B, num_q_heads=2 * G, kv_dtype=kv,
                                       q_dtype=omni.OMNI_BF16 if kv == omni.OMNI_FP8_E4M3 else None))
                if T > 1:
                    h.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, T)
                lay = h.omni_debug_lds_layout()
                used = lay["dynamic_bytes"] + lay["static_bytes"] + 512
                assert 4 <= lay["ring_states"] <= 16, (B, G, T, lay)
                assert lay["dynamic_bytes"] <= lay["max_dynamic_bytes"] and used <= 160 * 1024, (B, G, T, lay)
                if lay["two_workgroups_per_cu"]:
                    assert used <= 80 * 1024, (B, G, T, lay)
                assert (lay["static_bytes"] > 0) == lay["k_staged"]
                if lay["k_staged"]:
                    assert lay["two_workgroups_per_cu"] and lay["ring_states"] >= 5, (B, G, T, lay)
    # the benchmark shapes keep two workgroups per compute unit
    for B, Hq, Hkv in ((64, 28, 4), (256, 16, 2), (8, 28, 4), (128, 32, 8)):
        assert omni.Handle(**good(batch=B, num_q_heads=Hq, num_kv_heads=Hkv)).omni_debug_lds_layout()["two_workgroups_per_cu"]


def test_fp8_cache_descriptions():
    h = omni.Handle(**good(kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_BF16))
    plan = h.omni_get_plan()
    assert plan["kernel"] == omni.KERNEL_MFMA
    with pytest.raises(omni.OmniError) as e:
        omni.Handle(**good(kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_F32))
    assert e.value.status == 3
    with pytest.raises(omni.OmniError) as e:
        omni.Handle(**good(kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_BF16, head_dim=64))
    assert e.value.status == 4
    with pytest.raises(omni.OmniError) as e:
        omni.Handle(**good(kv_dtype=3))
    assert e.value.status == 3


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
