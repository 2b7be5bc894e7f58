"""omni_paged_prefill_attn / omni_kv_append_chunk through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, DeviceBatch, bits_of, to_dev

pytestmark = pytest.mark.gpu


def as_bytes(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint8)


class ChunkOnDevice:
    def __init__(self, dev: DeviceBatch, ch: W.Chunk, out_dtype=torch.float32):
        wl = dev.wl
        self.q = to_dev(ch.q, wl.dtype)
        self.k_new, self.v_new = to_dev(ch.k_new, wl.dtype), to_dev(ch.v_new, wl.dtype)
        self.q_lens = torch.from_numpy(ch.q_lens).cuda()
        self.q_offsets = torch.from_numpy(ch.q_offsets).cuda()
        self.out = torch.full((ch.total, wl.Hq, wl.D), float("nan"), dtype=out_dtype, device="cuda")


def run_chunk(wl, ch, max_q_len=None, out_dtype=W.F32, tuning=None, split_workspace=False):
    """Append the chunk's rows, then attend; returns (DeviceBatch, fp64 output with NaN in rows nobody owns).
    split_workspace: register a workspace large enough for the context split (poisoned with NaN first)."""
    dev = DeviceBatch(wl, out_dtype=out_dtype, tuning=tuning)
    c = ChunkOnDevice(dev, ch, torch.float32 if out_dtype == W.F32 else torch.bfloat16)
    mq = max_q_len or max(ch.max_q_len, 1)
    if split_workspace:
        n = max(dev.h.omni_workspace_bytes(), dev.h.omni_prefill_workspace_bytes(mq))
        dev.ws = torch.full((n // 4,), float("nan"), dtype=torch.float32, device="cuda")
        dev.h.omni_set_workspace(dev.ws)
    dev.h.omni_kv_append_chunk(c.k_new, c.v_new, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens,
                               c.q_lens, c.q_offsets, mq)
    dev.h.omni_paged_prefill_attn(c.q, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, c.q_lens,
                                  c.q_offsets, mq, float(wl.scale), c.out)
    torch.cuda.synchronize()
    return dev, c.out.float().cpu().numpy().astype(np.float64)


def check_chunk(wl, ch, label="", **kw):
    dev, got = run_chunk(wl, ch, **kw)
    oracle.kv_append_chunk(ch.k_new, ch.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                           ch.q_offsets)
    assert np.array_equal(as_bytes(bits_of(dev.k_cache)), as_bytes(wl.k_cache)), label      # the append is a bit copy
    assert np.array_equal(as_bytes(bits_of(dev.v_cache)), as_bytes(wl.v_cache)), label
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    owned = np.zeros(ch.total, dtype=bool)
    for b in range(wl.B):
        owned[ch.q_offsets[b]:ch.q_offsets[b] + ch.q_lens[b]] = True
    assert np.all(np.isnan(got[~owned])), f"{label}: rows nobody owns were written"
    err = np.max(np.abs(got[owned] - ref[owned])) if owned.any() else 0.0
    assert np.all(np.isfinite(got[owned])) and err <= TOL[wl.dtype], f"{label}: max|err| {err:.3e}"
    return got, ref


@pytest.mark.parametrize("G,Hkv,ps", [(7, 4, 16), (8, 2, 16), (4, 8, 32), (16, 1, 16), (1, 2, 16), (3, 2, 32), (5, 1, 16)])
def test_chunks_of_many_shapes(G, Hkv, ps):
    lens = [300, 64, 1, 0, 33, 257, 96, 40]
    q_lens = [300, 1, 1, 0, 17, 100, 37, 40]                 # whole prompt, one token, nothing, ragged pieces
    wl = W.build("chunk", 700 + G, lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, q_lens, 800 + G, in_cache=False, gap=3)
    got, ref = check_chunk(wl, ch, label=f"G{G} Hkv{Hkv} ps{ps}")
    # request 0 is all chunk: its first query sees only token 0 and returns that V row (the weight is exp2 of a
    # rounding residue: 1 to within a few ulp)
    v0 = W.bf16_bits_to_f32(wl.v_cache[wl.block_table[0, 0], :, 0, :]).astype(np.float64)
    assert np.max(np.abs(got[ch.q_offsets[0]] - np.repeat(v0, G, axis=0))) <= 1e-5


@pytest.mark.parametrize("dtype,D,G,Hkv,ps", [(W.F32, 64, 2, 2, 16), (W.F32, 64, 7, 1, 32), (W.F32, 128, 4, 2, 16),
                                              (W.BF16, 64, 5, 2, 16), (W.BF16, 64, 16, 1, 32)])
def test_chunks_on_every_other_dtype_and_head_size(dtype, D, G, Hkv, ps):
    """fp32 caches and head_dim 64 go through the vector-ALU kernel (fp32 caches to 1e-5)."""
    lens = [300, 64, 1, 0, 33, 257, 96, 40]
    q_lens = [300, 1, 1, 0, 17, 100, 37, 40]
    wl = W.build("chunk", 800 + G + D, lens, Hq=G * Hkv, Hkv=Hkv, D=D, ps=ps, dtype=dtype, pool_factor=1.5)
    ch = W.add_chunk(wl, q_lens, 801 + G, in_cache=False, gap=3)
    check_chunk(wl, ch, label=f"{dtype} D={D} G={G} ps={ps}")


def test_vector_alu_kernel_agrees_with_the_matrix_core_kernel_on_bf16():
    """The same bf16 / head_dim 128 chunks through both kernels (kernel choice 1 = vector ALU): each within the bar of
    the oracle, and within twice the bar of each other."""
    wl = W.build("chunk", 950, [700, 129, 64], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [260, 129, 1], 951, in_cache=True)
    got_mfma, ref = check_chunk(wl, ch, label="mfma")
    got_valu, _ = check_chunk(wl, ch, label="valu", tuning={omni.OMNI_TUNE_KERNEL: 1})
    assert np.nanmax(np.abs(got_mfma - got_valu)) <= 2 * TOL[W.BF16]
    assert np.nanmax(np.abs(got_valu - ref)) <= 1e-5                      # fp32 arithmetic on exact bf16 inputs


def test_one_token_chunks_agree_with_the_decode_call():
    wl = W.make("talker", batch=24, len_div=2, append=False)
    ch = W.add_chunk(wl, [1] * wl.B, 5)
    ch.q[:] = wl.q
    got, ref = check_chunk(wl, ch, label="decode")
    dec = DeviceBatch(wl).attend()
    assert np.max(np.abs(got - dec)) <= 2 * TOL[wl.dtype]
    assert np.array_equal(ref, oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens,
                                                        wl.scale, wl.dtype))


def test_chunk_longer_than_max_q_len_hint_is_cut_and_bf16_output_rounds():
    wl = W.build("chunk", 900, [200, 150], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [64, 150], 901, in_cache=True)
    dev, got = run_chunk(wl, ch, out_dtype=W.BF16)
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    rounded = W.bf16_bits_to_f32(W.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
    ulp = np.maximum(np.abs(rounded), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(got - rounded) <= ulp + 2e-3)


def test_peaked_softmax_and_large_scores_in_a_chunk():
    wl = W.build("chunk", 910, [500, 90], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    kf = W.bf16_bits_to_f32(wl.k_cache) * np.float32(6.0)
    wl.k_cache = np.where(np.isnan(kf), W.BF16_NAN_BITS, W.f32_to_bf16_bits(np.nan_to_num(kf))).astype(np.uint16)
    ch = W.add_chunk(wl, [130, 90], 911, in_cache=False)
    check_chunk(wl, ch, label="peaked")


def _map_pool(cache, fn):
    """Apply fn to the values of a bf16 pool, keeping the NaN of slots nobody owns."""
    f = W.bf16_bits_to_f32(cache)
    g = fn(np.nan_to_num(f)).astype(np.float32)
    return np.where(np.isnan(f), W.BF16_NAN_BITS, W.f32_to_bf16_bits(g)).astype(np.uint16)


def test_scores_that_grow_along_the_context_move_the_reference_many_times():
    """All-positive q and K whose rows grow with the token position: the running maximum of every column keeps rising
    (by some 30 log2 units over the context), so the kernel's softmax reference moves again and again, inside the
    pipelined steps too, with accumulated and pending weights to rescale each time."""
    lens = [900, 333]
    wl = W.build("chunk", 920, lens, Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    wl.k_cache = _map_pool(wl.k_cache, np.abs)
    for b, L in enumerate(lens):
        t = np.arange(L)
        pages, slots = wl.block_table[b, t // wl.ps], t % wl.ps
        rows = W.bf16_bits_to_f32(wl.k_cache[pages, :, slots, :]) * (0.2 + 2.8 * t / L)[:, None, None].astype(np.float32)
        wl.k_cache[pages, :, slots, :] = W.f32_to_bf16_bits(rows)
    ch = W.add_chunk(wl, [200, 333], 921, in_cache=True)
    ch.q = W.f32_to_bf16_bits(np.abs(W.bf16_bits_to_f32(ch.q)))
    check_chunk(wl, ch, label="growing")


@pytest.mark.parametrize("log2_factor", [-12, 13])
def test_v_magnitudes_near_both_ends_of_the_fp16_range(log2_factor):
    """The kernel multiplies V as fp16: exact for 2^-14 <= |V| <= 65504, an absolute error of at most 2^-25 per value
    below that.  V scaled by 2^-12 straddles the lower end, by 2^13 comes close to the upper one."""
    f = np.float32(2.0 ** log2_factor)
    wl = W.build("chunk", 930, [400, 77], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16)
    wl.v_cache = _map_pool(wl.v_cache, lambda v: v * f)
    assert np.nanmax(np.abs(W.bf16_bits_to_f32(wl.v_cache))) < 65504
    ch = W.add_chunk(wl, [150, 77], 931, in_cache=True)
    dev, got = run_chunk(wl, ch)
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    err = np.max(np.abs(got - ref))
    assert np.all(np.isfinite(got)) and err <= TOL[wl.dtype] * float(f) + 2.0 ** -24, f"max|err| {err:.3e}"


def test_v_values_that_are_fp16_subnormals_are_not_flushed():
    """Every V element is 2^-20, an fp16 subnormal: a softmax-weighted mean of equal rows is that value again, so the
    output is 2^-20 up to fp32 rounding; flushing subnormal operands to zero anywhere on the way would give 0."""
    wl = W.build("chunk", 960, [300, 45], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    v = np.float32(2.0 ** -20)
    wl.v_cache = _map_pool(wl.v_cache, lambda x: np.full_like(x, v))
    ch = W.add_chunk(wl, [120, 45], 961, in_cache=True)
    dev, got = run_chunk(wl, ch)
    assert np.max(np.abs(got / float(v) - 1.0)) <= 1e-3


def test_a_v_value_beyond_the_fp16_range_shows_as_non_finite_output():
    """Such a value is outside the documented range of the call; the queries that attend to it must not get a wrong
    finite number (earlier queries of the same tile may see it too, as 0 * inf; the other dims stay clean)."""
    wl = W.build("chunk", 940, [96], Hq=4, Hkv=1, D=128, ps=16, dtype=W.BF16)
    page, slot, dim = wl.block_table[0, 2], 5, 17                            # token 37, seen by queries 37 .. 95
    wl.v_cache[page, 0, slot, dim] = W.f32_to_bf16_bits(np.array([1e5], dtype=np.float32))[0]
    ch = W.add_chunk(wl, [96], 941, in_cache=True)
    dev, got = run_chunk(wl, ch)
    assert np.all(np.isfinite(np.delete(got, dim, axis=2)))
    assert not np.any(np.isfinite(got[37:, :, dim]))


def test_hand_worked_causal_chunks_through_the_c_abi():
    """The hand-worked cases of tests/golden/causal_chunk_cases.txt, zero-padded to head_dim 64 in fp32 (the vector-ALU
    kernel, held to 1e-5 of the rational result) and to head_dim 128 in bf16 (the matrix-core kernel: the logarithms
    among the keys round to bf16, which moves the exact answer by up to a few 1e-2, so it is held to 2e-3 of the
    oracle on the rounded inputs and to 6e-2 of the rational result)."""
    import math
    import os

    def vals(txt):
        return [math.log(float(tok[2:])) if tok.startswith("ln") else float(tok) for tok in txt.split()]

    n = 0
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "causal_chunk_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, scale, q, K, V, exp = [f.strip() for f in line.split("|")]
        q = np.array([vals(r) for r in q.split(";")], dtype=np.float32)
        K = np.array([vals(r) for r in K.split(";")], dtype=np.float32)
        V = np.array([vals(r) for r in V.split(";")], dtype=np.float32)
        exp = np.array([vals(r) for r in exp.split(";")])
        L, nq = len(K), len(q)
        for dtype, D, tol in ((W.F32, 64, 1e-5), (W.BF16, 128, 6e-2)):
            wl = W.build("golden", 5, [L], Hq=1, Hkv=1, D=D, ps=16, dtype=dtype, scale=float(scale))
            ch = W.add_chunk(wl, [nq], 6, in_cache=True)
            enc = (lambda a: a) if dtype == W.F32 else W.f32_to_bf16_bits
            pad = lambda a: np.concatenate([a, np.zeros((len(a), D - a.shape[1]), np.float32)], axis=1)
            pg = wl.block_table[0, 0]
            wl.k_cache[pg, 0, :L] = enc(pad(K)); wl.v_cache[pg, 0, :L] = enc(pad(V))
            ch.q[:nq, 0] = enc(pad(q))
            ch.k_new[:nq, 0] = wl.k_cache[pg, 0, L - nq:L]; ch.v_new[:nq, 0] = wl.v_cache[pg, 0, L - nq:L]
            dev, got = run_chunk(wl, ch)
            ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                            ch.q_offsets, wl.scale, wl.dtype)
            assert np.max(np.abs(got[:nq] - ref[:nq])) <= TOL[dtype], (name, dtype)
            assert np.max(np.abs(got[:nq, 0, :exp.shape[1]] - exp)) <= tol, (name, dtype)
            assert np.all(got[:nq, 0, exp.shape[1]:] == 0.0), (name, dtype)
        n += 1
    assert n == 3


def test_full_size_prefill_chunk_sampled_rows():
    """Eight thinker-sized requests, each with a 512-token chunk at the end of a 512..4096-token context."""
    wl = W.make("thinker", batch=8, append=False)
    ch = W.add_chunk(wl, [512] * wl.B, 77, in_cache=False)
    dev, got = run_chunk(wl, ch)
    oracle.kv_append_chunk(ch.k_new, ch.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                           ch.q_offsets)
    assert np.array_equal(as_bytes(bits_of(dev.k_cache)), as_bytes(wl.k_cache))
    rng = np.random.default_rng(3)
    rows = [(int(b), int(i), int(h)) for b, i, h in zip(rng.integers(0, wl.B, 24), rng.integers(0, 512, 24),
                                                        rng.integers(0, wl.Hq, 24))]
    rows += [(0, 0, 0), (wl.B - 1, 511, wl.Hq - 1)]
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype, rows=rows)
    for r, (b, i, h) in enumerate(rows):
        assert np.max(np.abs(got[ch.q_offsets[b] + i, h] - ref[r])) <= TOL[wl.dtype], (b, i, h)
    assert np.all(np.isfinite(got))


def test_prefill_argument_errors():
    h = omni.Handle(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=128, page_size=16, num_pages=8,
                    max_blocks_per_seq=4, kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_BF16)
    L = omni.lib()
    assert L.omni_paged_prefill_attn(h._h, 256, 256, 256, 256, 256, 256, 256, 8, 1.0, 256, None) == 4     # 8-bit cache
    hb = omni.Handle(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=128, page_size=16, num_pages=8,
                     max_blocks_per_seq=4, kv_dtype=omni.OMNI_BF16)
    assert L.omni_paged_prefill_attn(hb._h, 256, 256, 256, 256, 256, 256, 256, 0, 1.0, 256, None) == 2
    assert L.omni_paged_prefill_attn(hb._h, 256, 256, 256, 256, 256, None, 256, 8, 1.0, 256, None) == 1
    assert L.omni_kv_append_chunk(hb._h, 256, 256, 256, 256, 256, 256, 256, 256 + 4, 8, None) == 2        # int64 array off by 4


# --------------------------------------------------------------------------- context split
SPLIT_CASES = {
    # name: (context lengths, chunk lengths, G, Hkv, page size)
    "one-long-request": ([3000], [300], 7, 4, 16),
    "whole-prompt": ([1500], [1500], 4, 2, 32),
    "ragged-batch": ([2100, 64, 1, 0, 700, 129, 65], [37, 64, 1, 0, 400, 1, 65], 7, 2, 16),
    "short-contexts": ([40, 100, 63, 64, 65, 200], [40, 3, 63, 1, 65, 130], 8, 1, 16),     # fewer steps than splits
    "group-16": ([900, 333], [90, 333], 16, 1, 32),
}


@pytest.mark.parametrize("splits,min_split", [(0, 1024), (0, 64), (2, 64), (3, 128), (7, 64), (16, 64), (16, 256)],
                         ids=lambda v: str(v))
@pytest.mark.parametrize("case", list(SPLIT_CASES))
def test_context_split_against_the_oracle_and_the_unsplit_kernel(case, splits, min_split):
    """The matrix-core kernel with every workgroup's context dealt to several workgroups and merged afterwards:
    within the bar of the oracle for every split count (0 = the library's own choice) and smallest share (64 tokens:
    every split the context has steps for is used; requests with fewer steps are shared by fewer workgroups or by
    none, whose rows the merge must leave alone), and within a quarter of the
    bar of the unsplit result (every piece rounds its weights to fp16 against a reference of its own, so the two
    differ by rounding errors of the weights, not only by the order of summation).  The workspace starts out as NaN."""
    lens, q_lens, G, Hkv, ps = SPLIT_CASES[case]
    wl = W.build("split", 1300 + len(lens), lens, Hq=G * Hkv, Hkv=Hkv, D=128, ps=ps, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, q_lens, 1301, in_cache=True, gap=2)
    one, _ = check_chunk(wl, ch, label=f"{case} unsplit", tuning={omni.OMNI_TUNE_PREFILL_SPLITS: 1})
    got, _ = check_chunk(wl, ch, label=f"{case} splits={splits}", split_workspace=True,
                         tuning={omni.OMNI_TUNE_PREFILL_SPLITS: splits, omni.OMNI_TUNE_PREFILL_MIN_SPLIT: min_split})
    assert np.nanmax(np.abs(got - one)) <= TOL[W.BF16] / 4


def test_context_split_needs_its_workspace_and_is_repeatable():
    """Without a workspace of omni_prefill_workspace_bytes the call does not split (bit-identical to splits = 1); with
    it the result is bit-identical from call to call, also after the workspace was overwritten in between."""
    wl = W.build("split", 1400, [2500, 900], Hq=28, Hkv=4, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [128, 200], 1401, in_cache=True)
    _, unsplit = run_chunk(wl, ch, tuning={omni.OMNI_TUNE_PREFILL_SPLITS: 1})
    dev, small_ws = run_chunk(wl, ch)                                     # decode-sized workspace only
    need = dev.h.omni_prefill_workspace_bytes(ch.max_q_len)
    assert need > dev.h.omni_workspace_bytes() and dev.h.omni_get_plan()["kernel"] == omni.KERNEL_MFMA
    assert np.array_equal(small_ws, unsplit, equal_nan=True)
    dev, a = run_chunk(wl, ch, split_workspace=True)
    assert not np.array_equal(a, unsplit, equal_nan=True)                 # it did split
    c = ChunkOnDevice(dev, ch)
    for poison in (0.0, float("inf")):
        dev.ws.fill_(poison)
        dev.h.omni_paged_prefill_attn(c.q, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, c.q_lens,
                                      c.q_offsets, ch.max_q_len, float(wl.scale), c.out)
        torch.cuda.synchronize()
        assert np.array_equal(c.out.cpu().numpy().astype(np.float64), a, equal_nan=True)


def test_context_split_with_bf16_output_and_a_larger_max_q_len():
    wl = W.build("split", 1500, [1800, 70], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [100, 70], 1501, in_cache=True)
    got, ref = None, None
    dev, got = run_chunk(wl, ch, max_q_len=160, out_dtype=W.BF16, split_workspace=True,
                         tuning={omni.OMNI_TUNE_PREFILL_SPLITS: 4})
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    owned = np.zeros(ch.total, dtype=bool)
    for b in range(wl.B):
        owned[ch.q_offsets[b]:ch.q_offsets[b] + ch.q_lens[b]] = True
    err = np.abs(got[owned] - ref[owned])
    assert np.all(err <= TOL[W.BF16] + np.abs(ref[owned]) * 2.0 ** -8)    # the bar plus a bf16 rounding of the result
    assert np.all(np.isnan(got[~owned]))


def test_longest_first_order_changes_nothing_but_the_schedule():
    """More than 256 workgroups and a workspace: the requests are ranked by context length on the device (ties, empty
    requests and one-token chunks included) and taken longest first; every output bit is as in batch order."""
    rng = np.random.default_rng(1900)
    lens = np.concatenate([rng.integers(1, 900, size=40), [0, 0, 300, 300, 300, 1, 64]]).astype(np.int64)
    q_lens = np.minimum(lens, rng.integers(0, 200, size=lens.size)).astype(np.int64)
    q_lens[-5:-2] = [300, 17, 300]
    wl = W.build("order", 1901, lens, Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16, pool_factor=1.5)
    ch = W.add_chunk(wl, q_lens, 1902, in_cache=True, gap=1)
    assert ((ch.max_q_len + 35) // 36) * wl.Hkv * wl.B > 256
    got_sorted, _ = check_chunk(wl, ch, label="sorted")
    _, in_order = run_chunk(wl, ch, tuning={omni.OMNI_TUNE_PREFILL_SORT: 0})
    assert np.array_equal(got_sorted, in_order, equal_nan=True)



@pytest.mark.parametrize("split", [False, True], ids=["one-launch", "context-split"])
@pytest.mark.parametrize("kernel", [omni.KERNEL_AUTO, omni.KERNEL_VALU], ids=["mfma", "valu"])
def test_chunks_longer_than_max_q_len_are_cut_off_there(split, kernel):
    """q_lens above the host's bound: query tokens 0 .. max_q_len - 1 of every chunk are computed (each still at its
    position in the full chunk), the others are not touched.  Group size 7 makes a query block 36 tokens, so a bound of
    40 ends inside the second block; with the context split the pieces of tokens beyond the bound would land in the
    next request's rows, and those of the last request behind the workspace: a guard area there must stay as it was."""
    if split and kernel == omni.KERNEL_VALU:
        pytest.skip("the vector-ALU kernel never splits the context")
    wl = W.build("cut", 1600, [1500, 900, 700], Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [100, 90, 50], 1601, in_cache=True)
    mq = 40
    dev = DeviceBatch(wl, tuning={omni.OMNI_TUNE_KERNEL: kernel} if kernel else None)
    c = ChunkOnDevice(dev, ch)
    guard = 1 << 20
    need = max(dev.h.omni_workspace_bytes(), dev.h.omni_prefill_workspace_bytes(mq) if split else 0)
    if split:
        assert dev.h.omni_prefill_workspace_bytes(mq) > 0
    buf = torch.full(((need + guard) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    buf[need // 4:] = 12345.0
    dev.ws = buf
    dev.h.omni_set_workspace(buf, need)
    dev.h.omni_paged_prefill_attn(c.q, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens, c.q_lens,
                                  c.q_offsets, mq, float(wl.scale), c.out)
    torch.cuda.synchronize()
    assert bool(torch.all(buf[need // 4:] == 12345.0)), "wrote behind the registered workspace"
    got = c.out.cpu().numpy().astype(np.float64)
    ref = oracle.paged_prefill_attn(ch.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, ch.q_lens,
                                    ch.q_offsets, wl.scale, wl.dtype)
    for b in range(wl.B):
        o, n = int(ch.q_offsets[b]), int(ch.q_lens[b])
        assert np.max(np.abs(got[o:o + mq] - ref[o:o + mq])) <= TOL[wl.dtype], f"request {b}"
        assert np.all(np.isnan(got[o + mq:o + n])), f"request {b}: tokens beyond the bound were written"


def test_chunk_append_is_cut_off_at_max_q_len_too():
    wl = W.build("cut", 1610, [300, 120], Hq=8, Hkv=2, D=128, ps=16, dtype=W.BF16)
    ch = W.add_chunk(wl, [70, 50], 1611, in_cache=False)
    mq = 40
    dev = DeviceBatch(wl)
    c = ChunkOnDevice(dev, ch)
    dev.h.omni_kv_append_chunk(c.k_new, c.v_new, dev.k_cache, dev.v_cache, dev.block_table, dev.context_lens,
                               c.q_lens, c.q_offsets, mq)
    torch.cuda.synchronize()
    # the first mq rows of each chunk, at their positions in the full chunk: the same as a chunk of mq tokens that ends
    # q_lens - mq tokens before the context does
    cut = np.minimum(ch.q_lens, mq).astype(np.int32)
    oracle.kv_append_chunk(ch.k_new, ch.v_new, wl.k_cache, wl.v_cache, wl.block_table,
                           (wl.context_lens - (ch.q_lens - cut)).astype(np.int32), cut, ch.q_offsets)
    assert np.array_equal(as_bytes(bits_of(dev.k_cache)), as_bytes(wl.k_cache))
    assert np.array_equal(as_bytes(bits_of(dev.v_cache)), as_bytes(wl.v_cache))
