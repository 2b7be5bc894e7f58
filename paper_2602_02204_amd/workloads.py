"""Seeded synthetic decode batches (host numpy arrays only).

This module serves both the HIP path and the CPU oracle with *inputs*; it holds
none of the method's arithmetic (no dot products, no softmax, no page walk).  It
imports neither of them.

The batches stand in for the per-stage decode batches of the paper's
autoregressive stages (Section 3.3, "AR stage support": each engine batches its
own requests and keeps its own paged KV cache; Section 4.2 gives the only
published shape statistics: about 842 prompt tokens including video tokens, 151
generated text tokens and 545 generated audio tokens per request).  Head counts,
head size and page sizes are those of the five benchmark configurations.

Draw order for one seed (numpy ``Generator(PCG64(seed))``):
lengths -> physical page assignment -> q -> K rows -> V rows -> (k_new, v_new).
Floating-point values are drawn as fp32 normals; bf16 tensors are the
round-to-nearest-even truncation of those, stored as uint16 bit patterns.
Every cache slot that no live token owns holds NaN and every unused block-table
entry holds -1: neither may ever influence a result.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

F32 = "f32"
BF16 = "bf16"

BF16_NAN_BITS = np.uint16(0x7FC0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One decode batch.  Cache layout is [P, Hkv, ps, D]; q/out are [B, Hq, D]."""
    name: str
    seed: int
    B: int
    Hq: int
    Hkv: int
    D: int
    ps: int
    dtype: str                      # F32 or BF16: dtype of q, K, V
    P: int                          # pages in the pool
    MB: int                         # block-table row length
    scale: np.float32
    q: np.ndarray                   # [B, Hq, D]  float32 or uint16 (bf16 bits)
    k_cache: np.ndarray             # [P, Hkv, ps, D]
    v_cache: np.ndarray
    block_table: np.ndarray         # [B, MB] int32, -1 beyond the owned pages
    context_lens: np.ndarray        # [B] int32, counts the appended token if there is one
    k_new: Optional[np.ndarray] = None   # [B, Hkv, D] rows to append at `positions`
    v_new: Optional[np.ndarray] = None
    positions: Optional[np.ndarray] = None  # [B] int32
    meta: dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def total_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self) -> int:
        """Algorithmic KV bytes of one attention call: a K row and a V row per live token per KV head."""
        return self.total_tokens * 2 * self.Hkv * self.D * self.elem_size

    def np_dtype(self):
        return np.float32 if self.dtype == F32 else np.uint16


def _draw(rng: np.random.Generator, shape, dtype: str, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x if dtype == F32 else f32_to_bf16_bits(x)


def _poison(shape, dtype: str) -> np.ndarray:
    if dtype == F32:
        return np.full(shape, np.nan, dtype=np.float32)
    return np.full(shape, BF16_NAN_BITS, dtype=np.uint16)


def build(name: str, seed: int, lens: Sequence[int], Hq: int, Hkv: int, D: int, ps: int,
          dtype: str, *, pool_pages: Optional[int] = None, pool_factor: float = 1.0,
          v_std: float = 1.0, append: bool = False, scale: Optional[float] = None,
          rng: Optional[np.random.Generator] = None, extra_table_cols: int = 0) -> Workload:
    """Lay out one batch.

    lens[b] is the context length the query attends to.  With ``append`` the last
    of those tokens is *not* in the cache yet: its K/V rows come back as
    ``k_new``/``v_new`` with ``positions[b] = lens[b] - 1`` (requests of length 0
    get position -1, meaning "skip"), and its slot holds NaN until appended.
    The pool has ``pool_pages`` pages (default: ceil(pool_factor * pages needed));
    the batch owns a uniformly random subset of them in random order.
    """
    if rng is None:
        rng = np.random.default_rng(np.random.PCG64(seed))
    lens = np.asarray(lens, dtype=np.int64)
    B = int(lens.shape[0])
    assert Hq % Hkv == 0
    npages = (lens + ps - 1) // ps
    need = int(npages.sum())
    if pool_pages is None:
        pool_pages = max(1, int(np.ceil(pool_factor * need)))
    assert pool_pages >= need, "pool too small for the batch"
    P = int(pool_pages)
    MB = int(max(1, npages.max() if B else 1)) + int(extra_table_cols)

    # physical page assignment
    owned = rng.permutation(P)[:need].astype(np.int32)
    block_table = np.full((B, MB), -1, dtype=np.int32)
    starts = np.concatenate([[0], np.cumsum(npages)])
    for b in range(B):
        block_table[b, : npages[b]] = owned[starts[b]: starts[b + 1]]

    q = _draw(rng, (B, Hq, D), dtype)

    T = int(lens.sum())
    k_cache = _poison((P, Hkv, ps, D), dtype)
    v_cache = _poison((P, Hkv, ps, D), dtype)
    # token -> (page, slot)
    if T > 0:
        req = np.repeat(np.arange(B), lens)
        tok = np.arange(T) - np.repeat(np.cumsum(lens) - lens, lens)
        page = block_table[req, tok // ps]
        slot = (tok % ps).astype(np.int64)
        is_last = tok == (np.repeat(lens, lens) - 1)
    k_rows = _draw(rng, (T, Hkv, D), dtype)
    v_rows = _draw(rng, (T, Hkv, D), dtype, std=v_std)
    k_new = v_new = positions = None
    if append:
        positions = (lens - 1).astype(np.int32)          # -1 for empty requests
        k_new = _draw(rng, (B, Hkv, D), dtype)
        v_new = _draw(rng, (B, Hkv, D), dtype, std=v_std)
        if T > 0:
            keep = ~is_last
            k_cache[page[keep], :, slot[keep], :] = k_rows[keep]
            v_cache[page[keep], :, slot[keep], :] = v_rows[keep]
    elif T > 0:
        k_cache[page, :, slot, :] = k_rows
        v_cache[page, :, slot, :] = v_rows
    del k_rows, v_rows

    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    return Workload(name=name, seed=seed, B=B, Hq=Hq, Hkv=Hkv, D=D, ps=ps, dtype=dtype, P=P, MB=MB,
                    scale=np.float32(scale), q=q, k_cache=k_cache, v_cache=v_cache,
                    block_table=block_table, context_lens=lens.astype(np.int32),
                    k_new=k_new, v_new=v_new, positions=positions,
                    meta={"pages_needed": need, "append": append})


def _uniform_int(rng, lo, hi, n):
    """Integers uniform on [lo, hi], both ends included."""
    return rng.integers(lo, hi + 1, size=n, dtype=np.int64)


CONFIG_NAMES = ("tiny", "thinker", "talker", "long", "mixed")
DEFAULT_SEED = {"tiny": 0, "thinker": 1, "talker": 2, "long": 3, "mixed": 4}


def make(name: str, seed: Optional[int] = None, *, append: Optional[bool] = None,
         batch: Optional[int] = None, len_div: int = 1) -> Workload:
    """The five benchmark configurations.

    ``append`` overrides whether the last token arrives through k_new/v_new
    (default: only "talker").  ``batch`` and ``len_div`` shrink a configuration
    (fewer requests, lengths divided) for tests that run the full oracle; the
    defaults give the configuration at full size.
    """
    if seed is None:
        seed = DEFAULT_SEED[name]
    rng = np.random.default_rng(np.random.PCG64(seed))

    def shrink(lo, hi):
        return max(1, lo // len_div), max(1, hi // len_div)

    if name == "tiny":
        lens = [17, 64, 129, 200]
        return build(name, seed, lens, Hq=4, Hkv=2, D=64, ps=16, dtype=F32, pool_pages=64,
                     append=bool(append), scale=0.125, rng=rng)
    if name == "thinker":
        B = batch or 64
        lens = _uniform_int(rng, *shrink(512, 4096), B)
        return build(name, seed, lens, Hq=28, Hkv=4, D=128, ps=16, dtype=BF16,
                     append=bool(append), rng=rng)
    if name == "talker":
        B = batch or 256
        lens_old = _uniform_int(rng, *shrink(128, 1024), B)
        use_append = True if append is None else append
        return build(name, seed, lens_old + 1, Hq=16, Hkv=2, D=128, ps=16, dtype=BF16,
                     append=use_append, rng=rng)
    if name == "long":
        B = batch or 8
        lens = _uniform_int(rng, *shrink(16384, 32768), B)
        return build(name, seed, lens, Hq=28, Hkv=4, D=128, ps=16, dtype=BF16,
                     append=bool(append), rng=rng)
    if name == "mixed":
        B = batch or 128
        n_long = int(round(0.1 * B))
        short = _uniform_int(rng, *shrink(64, 512), B - n_long)
        long_ = _uniform_int(rng, *shrink(8192, 16384), n_long)
        lens = np.concatenate([short, long_])
        lens = lens[rng.permutation(B)]
        return build(name, seed, lens, Hq=32, Hkv=8, D=128, ps=32, dtype=BF16,
                     pool_factor=2.0, v_std=0.5, append=bool(append), rng=rng)
    raise KeyError(name)


@dataclass
class Chunk:
    """Multi-token queries for a batch (chunked prefill): request b brings q_lens[b] new tokens, the last
    q_lens[b] of its context_lens[b] tokens.  q / k_new / v_new hold the chunk rows of all requests back to back."""
    q_lens: np.ndarray              # [B] int32
    q_offsets: np.ndarray           # [B] int64: first row of request b in q / out / k_new / v_new
    total: int                      # rows in q
    q: np.ndarray                   # [total, Hq, D]
    k_new: np.ndarray               # [total, Hkv, D]: the K rows of the chunk tokens (taken out of the pool)
    v_new: np.ndarray

    @property
    def max_q_len(self) -> int:
        return int(self.q_lens.max()) if self.q_lens.size else 0


def add_chunk(wl: Workload, q_lens: Sequence[int], seed: int, *, in_cache: bool = True, gap: int = 0) -> Chunk:
    """Turn the last q_lens[b] tokens of every request of ``wl`` into a chunk of new tokens.

    Query rows are drawn from ``seed``.  The chunk's K/V rows are copied out of the pools into k_new / v_new; with
    ``in_cache=False`` their pool slots are poisoned with NaN afterwards (they are "not appended yet").  ``gap`` leaves
    that many unused rows between the requests' row ranges.
    """
    rng = np.random.default_rng(np.random.PCG64(seed))
    ql = np.minimum(np.asarray(q_lens, dtype=np.int64), wl.context_lens.astype(np.int64))
    ql = np.maximum(ql, 0)
    offs = np.zeros(wl.B, dtype=np.int64)
    run = 0
    for b in range(wl.B):
        offs[b] = run
        run += int(ql[b]) + gap
    total = max(run, 1)
    q = _draw(rng, (total, wl.Hq, wl.D), wl.dtype)
    k_new = np.zeros((total, wl.Hkv, wl.D), dtype=wl.np_dtype())
    v_new = np.zeros_like(k_new)
    for b in range(wl.B):
        n, L = int(ql[b]), int(wl.context_lens[b])
        if n <= 0:
            continue
        t = np.arange(L - n, L)
        pages, slots = wl.block_table[b, t // wl.ps], t % wl.ps
        k_new[offs[b]:offs[b] + n] = wl.k_cache[pages, :, slots, :]
        v_new[offs[b]:offs[b] + n] = wl.v_cache[pages, :, slots, :]
        if not in_cache:
            wl.k_cache[pages, :, slots, :] = _poison((n, wl.Hkv, wl.D), wl.dtype)
            wl.v_cache[pages, :, slots, :] = _poison((n, wl.Hkv, wl.D), wl.dtype)
    return Chunk(ql.astype(np.int32), offs, int(total), q, k_new, v_new)


FP8_NAN_BYTE = np.uint8(0x7F)
FP8_MAX = 448.0


@dataclass
class Fp8Pools:
    """The K/V pools of a workload re-encoded as 8-bit E4M3 bytes with one fp32 scale per (page, KV head)."""
    k_cache: np.ndarray             # [P, Hkv, ps, D] uint8; slots no live token owns hold the NaN byte
    v_cache: np.ndarray
    k_scale: np.ndarray             # [P, Hkv] float32
    v_scale: np.ndarray

    @property
    def kv_bytes_per_token_head(self) -> int:
        return 2 * self.k_cache.shape[-1]


def quantize_fp8(wl: Workload, *, power_of_two_scales: bool = False) -> Fp8Pools:
    """Encode the pools of ``wl`` (bf16 or fp32) in E4M3: scale = largest live magnitude of the (page, head) / 448
    (rounded up to a power of two on request; 1 for an all-dead page), bytes by the library's round-to-nearest cast."""
    import torch

    def one(cache):
        x = cache.astype(np.float32) if cache.dtype == np.float32 else bf16_bits_to_f32(cache)
        live = ~np.isnan(x)
        amax = np.where(live, np.abs(x), 0.0).max(axis=(2, 3))                       # [P, Hkv]
        scale = np.where(amax > 0, amax / FP8_MAX, 1.0).astype(np.float32)
        if power_of_two_scales:
            scale = np.exp2(np.ceil(np.log2(scale))).astype(np.float32)
        y = np.where(live, x / scale[:, :, None, None], 0.0).astype(np.float32)
        b = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()
        b[~live] = FP8_NAN_BYTE
        return b, scale

    k8, ks = one(wl.k_cache)
    v8, vs = one(wl.v_cache)
    return Fp8Pools(k8, v8, ks, vs)
