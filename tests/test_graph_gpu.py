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


def test_graph_rejects_the_null_stream():
    L = omni.lib()
    assert L.omni_graph_begin(None) == 4
    assert L.omni_graph_launch(None, None) == 1
    L.omni_graph_destroy(None)
