"""fp64 CPU oracle for paged decode attention: ctypes front end of oracle_attn.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It imports nothing from the HIP package; inputs
come in as host numpy arrays (fp32, or uint16 bf16 bit patterns).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_DT = {"f32": 0, "bf16": 1}


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "ps", "MB", "q_dtype", "kv_dtype")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # ORACLE_SANITIZED=1: the address / undefined-behaviour instrumented build (the process must preload its runtime)
        path = _build.build(force=False, sanitize=os.environ.get("ORACLE_SANITIZED") == "1")
        L = C.CDLL(path)
        L.oracle_paged_decode_attn.restype = C.c_int
        L.oracle_paged_decode_attn.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 5 + [C.c_float, C.c_void_p,
                                                                                       C.c_void_p, C.c_int32, C.c_int32]
        L.oracle_partial.restype = None
        L.oracle_partial.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 4 + [C.c_float] + [C.c_int32] * 4 + [C.c_void_p] * 3
        L.oracle_merge.restype = None
        L.oracle_merge.argtypes = [C.c_int32, C.c_int32] + [C.c_void_p] * 4
        L.oracle_kv_append.restype = None
        L.oracle_kv_append.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 6
        L.oracle_paged_prefill_attn.restype = C.c_int
        L.oracle_paged_prefill_attn.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 7 + [C.c_float, C.c_void_p, C.c_void_p,
                                                                                        C.c_int64, C.c_int32]
        L.oracle_fp8_e4m3_decode.restype = C.c_double
        L.oracle_fp8_e4m3_decode.argtypes = [C.c_uint8]
        L.oracle_paged_decode_attn_fp8.restype = C.c_int
        L.oracle_paged_decode_attn_fp8.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 7 + [C.c_float, C.c_void_p,
                                                                                           C.c_void_p, C.c_int32, C.c_int32]
        L.oracle_paged_prefill_attn_fp8.restype = C.c_int
        L.oracle_paged_prefill_attn_fp8.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 9 + [C.c_float, C.c_void_p,
                                                                                            C.c_void_p, C.c_int64, C.c_int32]
        L.oracle_fp8_e4m3_encode.restype = C.c_uint8
        L.oracle_fp8_e4m3_encode.argtypes = [C.c_float]
        L.oracle_kv_append_quant_fp8.restype = None
        L.oracle_kv_append_quant_fp8.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 8 + [C.c_float]
        L.oracle_gather.restype = None
        L.oracle_gather.argtypes = [C.POINTER(_Shape)] + [C.c_void_p] * 3 + [C.c_int32, C.c_void_p]
        _lib = L
    return _lib


def _check(a: np.ndarray, dtype: str, what: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    if a.dtype != want or not a.flags.c_contiguous:
        raise TypeError(f"{what}: need C-contiguous {want.__name__} array for dtype {dtype}, got {a.dtype}")
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _shape(q, k_cache, block_table, dtype, q_dtype=None) -> _Shape:
    B, Hq, D = q.shape
    P, Hkv, ps, D2 = k_cache.shape
    assert D == D2 and Hq % Hkv == 0
    assert block_table.dtype == np.int32 and block_table.flags.c_contiguous and block_table.shape[0] == B
    return _Shape(B, Hq, Hkv, D, ps, block_table.shape[1], _DT[q_dtype or dtype], _DT[dtype])


def paged_decode_attn(q, k_cache, v_cache, block_table, context_lens, scale, dtype: str,
                      pairs: Optional[Sequence[Tuple[int, int]]] = None, num_threads: int = 0,
                      return_threads: bool = False):
    """softmax(scale q K^T) V per (request, query head) in fp64.

    Returns [B, Hq, D] float64, or [len(pairs), D] when `pairs` lists (b, h) to compute.
    """
    _check(q, dtype, "q"); _check(k_cache, dtype, "k_cache"); _check(v_cache, dtype, "v_cache")
    s = _shape(q, k_cache, block_table, dtype)
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    if pairs is None:
        out = np.zeros((s.B, s.Hq, s.D), dtype=np.float64)
        pr, n = None, 0
    else:
        pr = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
        n = pr.shape[0]
        out = np.zeros((n, s.D), dtype=np.float64)
    used = lib().oracle_paged_decode_attn(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(block_table), _p(lens),
                                          C.c_float(float(scale)), _p(out), _p(pr), n, int(num_threads))
    return (out, used) if return_threads else out


def partial(q, k_cache, v_cache, block_table, scale, dtype: str, b: int, h: int, t0: int, t1: int):
    """Unnormalised (o[D], m, l) of (b, h) over tokens [t0, t1)."""
    s = _shape(q, k_cache, block_table, dtype)
    o = np.zeros(s.D, dtype=np.float64)
    m = np.zeros(1, dtype=np.float64)
    l = np.zeros(1, dtype=np.float64)
    lib().oracle_partial(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(block_table), C.c_float(float(scale)),
                         b, h, t0, t1, _p(o), _p(m), _p(l))
    return o, float(m[0]), float(l[0])


def merge(o: np.ndarray, m: np.ndarray, l: np.ndarray) -> np.ndarray:
    """Log-sum-exp merge of partitions: o [n, D], m [n], l [n] -> [D]."""
    o = np.ascontiguousarray(o, dtype=np.float64)
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    out = np.zeros(o.shape[1], dtype=np.float64)
    lib().oracle_merge(o.shape[0], o.shape[1], _p(o), _p(m), _p(l), _p(out))
    return out


def kv_append(k_new, v_new, k_cache, v_cache, block_table, positions, dtype: str) -> None:
    """In-place bit copy of the new rows into their page slots (positions < 0 are skipped)."""
    for a, w in ((k_new, "k_new"), (v_new, "v_new"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _check(a, dtype, w)
    B, Hkv, D = k_new.shape
    P, Hkv2, ps, D2 = k_cache.shape
    assert (Hkv, D) == (Hkv2, D2)
    s = _Shape(B, Hkv, Hkv, D, ps, block_table.shape[1], _DT[dtype], _DT[dtype])
    pos = np.ascontiguousarray(positions, dtype=np.int32)
    lib().oracle_kv_append(C.byref(s), _p(k_new), _p(v_new), _p(k_cache), _p(v_cache), _p(block_table), _p(pos))


def gather(cache, block_table, context_lens, b: int, dtype: str) -> np.ndarray:
    """Request b's rows in token order, [L_b, Hkv, D], same dtype as the cache (bit copy)."""
    _check(cache, dtype, "cache")
    P, Hkv, ps, D = cache.shape
    s = _Shape(block_table.shape[0], Hkv, Hkv, D, ps, block_table.shape[1], _DT[dtype], _DT[dtype])
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    out = np.zeros((int(lens[b]), Hkv, D), dtype=cache.dtype)
    lib().oracle_gather(C.byref(s), _p(cache), _p(block_table), _p(lens), b, _p(out))
    return out


def kv_pack(cache, block_table, context_lens, token_offsets, total_tokens: int) -> np.ndarray:
    """Dense copy of every request's rows (Section 3.4: the connector moves a request's KV cache between stages).

    dense[token_offsets[b] + t, g, :] = cache[block_table[b, t // ps], g, t % ps, :] for t < context_lens[b];
    requests with token_offsets[b] < 0 are skipped; rows of `dense` that no request owns stay zero.  A bit copy.
    Pins: brute-force triple loop, pack/unpack round trip into a poisoned pool, agreement with `gather`.
    """
    P, Hkv, ps, D = cache.shape
    dense = np.zeros((int(total_tokens), Hkv, D), dtype=cache.dtype)
    for b in range(block_table.shape[0]):
        L, off = int(context_lens[b]), int(token_offsets[b])
        if off < 0 or L <= 0:
            continue
        t = np.arange(L)
        dense[off:off + L] = cache[block_table[b, t // ps], :, t % ps, :]
    return dense


def kv_unpack(dense, cache, block_table, context_lens, token_offsets) -> None:
    """Inverse of kv_pack, in place: cache[block_table[b, t // ps], g, t % ps, :] = dense[token_offsets[b] + t, g, :]
    for t < context_lens[b] of every request with token_offsets[b] >= 0.  No other byte of `cache` changes."""
    P, Hkv, ps, D = cache.shape
    for b in range(block_table.shape[0]):
        L, off = int(context_lens[b]), int(token_offsets[b])
        if off < 0 or L <= 0:
            continue
        t = np.arange(L)
        cache[block_table[b, t // ps], :, t % ps, :] = dense[off:off + L]


def paged_prefill_attn(q, k_cache, v_cache, block_table, context_lens, q_lens, q_offsets, scale, dtype: str,
                       rows: Optional[Sequence[Tuple[int, int, int]]] = None, num_threads: int = 0) -> np.ndarray:
    """Multi-token (chunk) queries, causal inside the chunk: fp64 [Tq, Hq, D], or [len(rows), D] for (b, i, h) triples.

    q is [Tq, Hq, D]; request b's chunk is rows q_offsets[b] .. +q_lens[b]; its query i sits at position
    context_lens[b] - q_lens[b] + i and attends to every token up to and including itself.
    """
    _check(q, dtype, "q"); _check(k_cache, dtype, "k_cache"); _check(v_cache, dtype, "v_cache")
    Tq, Hq, D = q.shape
    P, Hkv, ps, D2 = k_cache.shape
    assert D == D2 and Hq % Hkv == 0
    s = _Shape(block_table.shape[0], Hq, Hkv, D, ps, block_table.shape[1], _DT[dtype], _DT[dtype])
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    ql = np.ascontiguousarray(q_lens, dtype=np.int32)
    qo = np.ascontiguousarray(q_offsets, dtype=np.int64)
    for b in range(block_table.shape[0]):                    # the C code trusts these
        if ql[b] > 0 and (ql[b] > lens[b] or qo[b] < 0 or qo[b] + ql[b] > Tq):
            raise ValueError(f"request {b}: chunk of {ql[b]} rows at {qo[b]} does not fit (context {lens[b]}, {Tq} rows)")
    if rows is not None:
        r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
        for b, i, h in r:
            if not (0 <= b < block_table.shape[0] and 0 <= i < ql[b] and 0 <= h < Hq):
                raise ValueError(f"row ({b}, {i}, {h}) is outside the chunks")
        out = np.zeros((len(r), D), dtype=np.float64)
        lib().oracle_paged_prefill_attn(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(bt), _p(lens), _p(ql), _p(qo),
                                        C.c_float(scale), _p(out), _p(r), len(r), num_threads)
    else:
        out = np.zeros((Tq, Hq, D), dtype=np.float64)
        lib().oracle_paged_prefill_attn(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(bt), _p(lens), _p(ql), _p(qo),
                                        C.c_float(scale), _p(out), None, 0, num_threads)
    return out


def kv_append_chunk(k_new, v_new, k_cache, v_cache, block_table, context_lens, q_lens, q_offsets) -> None:
    """Bit copy of every chunk token's K/V rows into the pools: row q_offsets[b] + i of k_new / v_new [Tq, Hkv, D]
    goes to position context_lens[b] - q_lens[b] + i of request b.  Requests with q_lens[b] <= 0 are skipped."""
    P, Hkv, ps, D = k_cache.shape
    for b in range(block_table.shape[0]):
        n, L = int(q_lens[b]), int(context_lens[b])
        if n <= 0:
            continue
        t = np.arange(L - n, L)
        src = slice(int(q_offsets[b]), int(q_offsets[b]) + n)
        k_cache[block_table[b, t // ps], :, t % ps, :] = k_new[src]
        v_cache[block_table[b, t // ps], :, t % ps, :] = v_new[src]


def fp8_e4m3_decode(byte: int) -> float:
    """Value of one OCP E4M3 byte (NaN for 0x7f / 0xff)."""
    return float(lib().oracle_fp8_e4m3_decode(int(byte) & 0xff))


def fp8_e4m3_encode(x: float) -> int:
    """E4M3 code nearest to x (fp32), ties to the even code, magnitudes above 448 saturate, NaN gives 0x7f."""
    return int(lib().oracle_fp8_e4m3_encode(C.c_float(float(np.float32(x)))))


def kv_append_quant_fp8(k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, positions, headroom: float) -> None:
    """In place: quantise the bf16 rows k_new / v_new [B, Hkv, D] into the E4M3 pools at `positions` (< 0 skips).  A row
    at slot 0 of its page sets that (page, KV head) scale to max(amax * headroom, 2^-100) / 448; other rows use the
    page's scale.  k_cache / v_cache uint8 [P, Hkv, ps, D]; k_scale / v_scale float32 [P, Hkv]."""
    _check(k_new, "bf16", "k_new"); _check(v_new, "bf16", "v_new")
    for a, what in ((k_cache, "k_cache"), (v_cache, "v_cache")):
        if a.dtype != np.uint8 or not a.flags.c_contiguous:
            raise TypeError(f"{what}: need C-contiguous uint8")
    for a, what in ((k_scale, "k_scale"), (v_scale, "v_scale")):
        if a.dtype != np.float32 or not a.flags.c_contiguous:
            raise TypeError(f"{what}: need C-contiguous float32")
    P, Hkv, ps, D = k_cache.shape
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    pos = np.ascontiguousarray(positions, dtype=np.int32)
    sh = _Shape(bt.shape[0], Hkv, Hkv, D, ps, bt.shape[1], _DT["bf16"], _DT["bf16"])
    lib().oracle_kv_append_quant_fp8(C.byref(sh), k_new.ctypes.data, v_new.ctypes.data, k_cache.ctypes.data,
                                     v_cache.ctypes.data, k_scale.ctypes.data, v_scale.ctypes.data, bt.ctypes.data,
                                     pos.ctypes.data, C.c_float(float(headroom)))


def paged_decode_attn_fp8(q, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, scale,
                          pairs: Optional[Sequence[Tuple[int, int]]] = None, num_threads: int = 0) -> np.ndarray:
    """Decode attention over an 8-bit (E4M3) KV cache with one fp32 scale per (page, KV head); q is bf16 bits.

    k_cache / v_cache are uint8 [P, Hkv, ps, D]; k_scale / v_scale float32 [P, Hkv].  fp64 [B, Hq, D] (or
    [len(pairs), D])."""
    _check(q, "bf16", "q")
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8 and k_cache.flags.c_contiguous
    B, Hq, D = q.shape
    P, Hkv, ps, D2 = k_cache.shape
    assert D == D2 and Hq % Hkv == 0 and k_scale.shape == (P, Hkv) and v_scale.shape == (P, Hkv)
    s = _Shape(B, Hq, Hkv, D, ps, block_table.shape[1], _DT["bf16"], 2)
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    ks = np.ascontiguousarray(k_scale, dtype=np.float32)
    vs = np.ascontiguousarray(v_scale, dtype=np.float32)
    if pairs is not None:
        pr = np.ascontiguousarray(np.asarray(pairs, dtype=np.int32).reshape(-1, 2))
        out = np.zeros((len(pr), D), dtype=np.float64)
        lib().oracle_paged_decode_attn_fp8(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(ks), _p(vs), _p(bt), _p(lens),
                                           C.c_float(scale), _p(out), _p(pr), len(pr), num_threads)
    else:
        out = np.zeros((B, Hq, D), dtype=np.float64)
        lib().oracle_paged_decode_attn_fp8(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(ks), _p(vs), _p(bt), _p(lens),
                                           C.c_float(scale), _p(out), None, 0, num_threads)
    return out


def paged_prefill_attn_fp8(q, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, q_lens, q_offsets, scale,
                           rows: Optional[Sequence[Tuple[int, int, int]]] = None, num_threads: int = 0) -> np.ndarray:
    """Multi-token (chunk) queries over the 8-bit (E4M3) cache with one fp32 scale per (page, KV head); q is bf16 bits
    [Tq, Hq, D].  fp64 [Tq, Hq, D], or [len(rows), D] for (b, i, h) triples."""
    _check(q, "bf16", "q")
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8 and k_cache.flags.c_contiguous
    Tq, Hq, D = q.shape
    P, Hkv, ps, D2 = k_cache.shape
    assert D == D2 and Hq % Hkv == 0 and k_scale.shape == (P, Hkv) and v_scale.shape == (P, Hkv)
    s = _Shape(block_table.shape[0], Hq, Hkv, D, ps, block_table.shape[1], _DT["bf16"], 2)
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    ql = np.ascontiguousarray(q_lens, dtype=np.int32)
    qo = np.ascontiguousarray(q_offsets, dtype=np.int64)
    ks = np.ascontiguousarray(k_scale, dtype=np.float32)
    vs = np.ascontiguousarray(v_scale, dtype=np.float32)
    for b in range(block_table.shape[0]):                    # the C code trusts these
        if ql[b] > 0 and (ql[b] > lens[b] or qo[b] < 0 or qo[b] + ql[b] > Tq):
            raise ValueError(f"request {b}: chunk of {ql[b]} rows at {qo[b]} does not fit (context {lens[b]}, {Tq} rows)")
    r, n = None, 0
    if rows is not None:
        r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
        for b, i, h in r:
            if not (0 <= b < block_table.shape[0] and 0 <= i < ql[b] and 0 <= h < Hq):
                raise ValueError(f"row ({b}, {i}, {h}) is outside the chunks")
        n = len(r)
    out = np.zeros((n, D) if rows is not None else (Tq, Hq, D), dtype=np.float64)
    lib().oracle_paged_prefill_attn_fp8(C.byref(s), _p(q), _p(k_cache), _p(v_cache), _p(ks), _p(vs), _p(bt), _p(lens),
                                        _p(ql), _p(qo), C.c_float(scale), _p(out), _p(r), n, num_threads)
    return out

