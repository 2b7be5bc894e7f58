"""A recorded decode step (append + attention + merge) replayed as a HIP graph.

The graph is captured once and replayed for four consecutive decode iterations of the same batch: each replay appends
one more token per request and attends over the longer context, with eager work and synchronisations between the
replays.  Every replay is checked against the fp64 oracle and, bit for bit, against the same step run eagerly on a
copy of the pools.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from gpu_util import TOL, DeviceBatch, bits_of, to_dev

pytestmark = pytest.mark.gpu

STEPS = 4


def as_bytes(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint8)           # the pools hold NaN poison: compare bits, not values


def rows_at(cache: np.ndarray, wl: W.Workload, pos: np.ndarray) -> np.ndarray:
    """cache[page of token pos[b] of request b, :, slot, :] for every request: the rows a decode step appends."""
    out = np.zeros((wl.B, wl.Hkv, wl.D), dtype=cache.dtype)
    for b in range(wl.B):
        if pos[b] >= 0:
            out[b] = cache[wl.block_table[b, pos[b] // wl.ps], :, pos[b] % wl.ps, :]
    return out


def blank_rows(cache: np.ndarray, wl: W.Workload, first: np.ndarray, last: np.ndarray) -> None:
    """Poison the rows of tokens first[b] .. last[b]-1: they are not in the cache yet."""
    poison = np.uint16(0x7fc1) if cache.dtype == np.uint16 else np.float32("nan")
    for b in range(wl.B):
        for t in range(max(first[b], 0), last[b]):
            cache[wl.block_table[b, t // wl.ps], :, t % wl.ps, :] = poison


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("thinker", dict(batch=8, len_div=4)), ("talker", dict(batch=24, len_div=2)),
                                     ("mixed", dict(batch=16, len_div=8))])
def test_replayed_decode_steps_match_oracle_and_eager(name, kw):
    wl = W.make(name, append=False, **kw)
    final = wl.context_lens.astype(np.int64)                 # lengths after the last replayed step
    start = np.maximum(final - STEPS, 0)                     # tokens in the cache before the first step
    k_full, v_full = wl.k_cache.copy(), wl.v_cache.copy()
    blank_rows(wl.k_cache, wl, start, final)
    blank_rows(wl.v_cache, wl, start, final)

    graph_side = DeviceBatch(wl)
    eager_side = DeviceBatch(wl)
    stream = torch.cuda.Stream()
    k_new = torch.zeros((wl.B, wl.Hkv, wl.D), dtype=graph_side.k_cache.dtype, device="cuda")
    v_new = torch.zeros_like(k_new)
    lens = torch.zeros(wl.B, dtype=torch.int32, device="cuda")

    def call(side, s):
        side.h.omni_decode_step(side.q, k_new, v_new, side.k_cache, side.v_cache, side.block_table, lens,
                                float(wl.scale), side.out, s)

    # the first launch of a handle configures its kernel: do it before recording (lens = 0: nothing is written)
    call(graph_side, stream)
    torch.cuda.synchronize()
    with omni.Graph(stream) as g:
        call(graph_side, stream)
    torch.cuda.synchronize()

    rng = np.random.default_rng(7)
    for step in range(STEPS):
        cur = np.minimum(start + step + 1, final).astype(np.int32)     # context including the token of this step
        live = start + step < final
        cur = np.where(live, cur, 0).astype(np.int32)                  # requests that ran out of tokens sit this step out
        pos = np.where(live, start + step, -1)
        q_step = rng.standard_normal(wl.q.shape).astype(np.float32)
        q_host = W.f32_to_bf16_bits(q_step) if wl.dtype == W.BF16 else q_step
        # eager work between replays: new inputs written in place, a reduction, a synchronisation
        for side in (graph_side, eager_side):
            side.q.copy_(to_dev(q_host, wl.dtype))
            side.out.fill_(float("nan"))
        k_new.copy_(to_dev(rows_at(k_full, wl, pos), wl.dtype))
        v_new.copy_(to_dev(rows_at(v_full, wl, pos), wl.dtype))
        lens.copy_(torch.from_numpy(cur).cuda())
        _ = float(graph_side.q.float().abs().sum())
        torch.cuda.synchronize()

        g.launch()
        call(eager_side, None)
        torch.cuda.synchronize()

        got = graph_side.out.cpu().numpy().astype(np.float64)
        assert np.array_equal(got, eager_side.out.cpu().numpy().astype(np.float64)), f"step {step}: replay != eager"
        assert np.array_equal(as_bytes(bits_of(graph_side.k_cache)), as_bytes(bits_of(eager_side.k_cache)))
        assert np.array_equal(as_bytes(bits_of(graph_side.v_cache)), as_bytes(bits_of(eager_side.v_cache)))
        ref = oracle.paged_decode_attn(q_host, k_full, v_full, wl.block_table, cur, wl.scale, wl.dtype)
        assert np.max(np.abs(got - ref)) <= TOL[wl.dtype], f"step {step}"
    # after the last step the graph side's pools hold every row of the full pools
    assert np.array_equal(as_bytes(bits_of(graph_side.k_cache)), as_bytes(k_full))
    assert np.array_equal(as_bytes(bits_of(graph_side.v_cache)), as_bytes(v_full))
    g.close()


def test_replayed_chunk_steps_with_a_split_context_match_oracle_and_eager():
    """omni_kv_append_chunk + omni_paged_prefill_attn with the context shared between workgroups (attention and merge
    kernels) recorded once and replayed for three consecutive chunks of the same requests: lengths, chunk lengths,
    offsets, queries and new rows change in place between the replays."""
    chunks = [np.array([64, 17, 0], dtype=np.int32), np.array([33, 64, 1], dtype=np.int32),
              np.array([1, 40, 64], dtype=np.int32)]
    start = np.array([900, 300, 0], dtype=np.int64)
    final = start + sum(c.astype(np.int64) for c in chunks)
    wl = W.build("graph-chunks", 77, final, Hq=14, Hkv=2, D=128, ps=16, dtype=W.BF16, pool_factor=1.5)
    k_full, v_full = wl.k_cache.copy(), wl.v_cache.copy()
    blank_rows(wl.k_cache, wl, start, final)
    blank_rows(wl.v_cache, wl, start, final)
    MQ, ROWS = 64, 3 * 64 + 8
    tuning = {omni.OMNI_TUNE_PREFILL_SPLITS: 4, omni.OMNI_TUNE_PREFILL_MIN_SPLIT: 128}
    sides = [DeviceBatch(wl, tuning=tuning), DeviceBatch(wl, tuning=tuning)]
    for side in sides:
        side.ws = side.h.alloc_workspace(prefill_max_q_len=MQ)
        assert side.h.omni_prefill_workspace_bytes(MQ) > 0
    graph_side, eager_side = sides
    stream = torch.cuda.Stream()
    dt = graph_side.k_cache.dtype
    q = torch.zeros((ROWS, wl.Hq, wl.D), dtype=dt, device="cuda")
    k_new = torch.zeros((ROWS, wl.Hkv, wl.D), dtype=dt, device="cuda")
    v_new = torch.zeros_like(k_new)
    lens = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    q_lens = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    q_offs = torch.zeros(wl.B, dtype=torch.int64, device="cuda")
    outs = [torch.zeros((ROWS, wl.Hq, wl.D), dtype=torch.float32, device="cuda") for _ in sides]

    def call(side, out, s):
        side.h.omni_kv_append_chunk(k_new, v_new, side.k_cache, side.v_cache, side.block_table, lens, q_lens, q_offs, MQ, s)
        side.h.omni_paged_prefill_attn(q, side.k_cache, side.v_cache, side.block_table, lens, q_lens, q_offs, MQ,
                                       float(wl.scale), out, s)

    call(graph_side, outs[0], stream)                        # nothing to do yet (all lengths zero)
    torch.cuda.synchronize()
    with omni.Graph(stream) as g:
        call(graph_side, outs[0], stream)
    torch.cuda.synchronize()

    rng = np.random.default_rng(8)
    done = start.copy()
    for step, n in enumerate(chunks):
        cur = (done + n).astype(np.int32)
        offs = np.array([0, 64 + step, 128 + 2 * step], dtype=np.int64)      # rows of the requests inside the row buffers
        qf = rng.standard_normal((ROWS, wl.Hq, wl.D)).astype(np.float32)
        q_host = W.f32_to_bf16_bits(qf)
        kn = np.zeros((ROWS, wl.Hkv, wl.D), dtype=np.uint16); vn = np.zeros_like(kn)
        for b in range(wl.B):
            for i in range(int(n[b])):
                t = int(done[b]) + i
                kn[offs[b] + i] = k_full[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]
                vn[offs[b] + i] = v_full[wl.block_table[b, t // wl.ps], :, t % wl.ps, :]
        q.copy_(to_dev(q_host, wl.dtype)); k_new.copy_(to_dev(kn, wl.dtype)); v_new.copy_(to_dev(vn, wl.dtype))
        lens.copy_(torch.from_numpy(cur).cuda()); q_lens.copy_(torch.from_numpy(n).cuda()); q_offs.copy_(torch.from_numpy(offs).cuda())
        for o in outs:
            o.fill_(float("nan"))
        _ = float(q.float().abs().sum())
        torch.cuda.synchronize()

        g.launch()
        call(eager_side, outs[1], None)
        torch.cuda.synchronize()

        got = outs[0].cpu().numpy().astype(np.float64)
        assert np.array_equal(got, outs[1].cpu().numpy().astype(np.float64), equal_nan=True), f"chunk {step}: replay != eager"
        assert np.array_equal(as_bytes(bits_of(graph_side.k_cache)), as_bytes(bits_of(eager_side.k_cache)))
        ref = oracle.paged_prefill_attn(q_host, k_full, v_full, wl.block_table, cur, n, offs, wl.scale, wl.dtype)
        owned = np.zeros(ROWS, dtype=bool)
        for b in range(wl.B):
            owned[offs[b]:offs[b] + n[b]] = True
        assert np.all(np.isnan(got[~owned]))
        assert np.max(np.abs(got[owned] - ref[owned])) <= TOL[wl.dtype], f"chunk {step}"
        done = done + n
    assert np.array_equal(as_bytes(bits_of(graph_side.k_cache)), as_bytes(k_full))
    assert np.array_equal(as_bytes(bits_of(graph_side.v_cache)), as_bytes(v_full))
    g.close()


def test_graph_rejects_the_null_stream():
    L = omni.lib()
    assert L.omni_graph_begin(None) == 4
    assert L.omni_graph_launch(None, None) == 1
    L.omni_graph_destroy(None)
