"""Thin ctypes binding of libomni_attn.so: argument marshalling only.

Names mirror the C ABI (include/omni_attn.h).  PyTorch supplies device memory
and the stream; every step of the path runs in the library's HIP kernels.  There
is no fallback: if the library has not been built, or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("OMNI_ATTN_LIB") or os.path.join(_HERE, "libomni_attn.so")

OMNI_F32, OMNI_BF16, OMNI_FP8_E4M3 = 0, 1, 2
OMNI_TUNE_KERNEL, OMNI_TUNE_TARGET_WORKGROUPS, OMNI_TUNE_MIN_PARTITION, OMNI_TUNE_FORCE_PARTITION = 0, 1, 2, 3
OMNI_TUNE_PREFILL_SPLITS, OMNI_TUNE_PREFILL_MIN_SPLIT, OMNI_TUNE_QUERY_TOKENS = 4, 5, 6
OMNI_TUNE_PREFILL_SORT = 7
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA = 0, 1, 2

EXPORTS = (
    "omni_create", "omni_destroy", "omni_set_tuning", "omni_workspace_bytes", "omni_prefill_workspace_bytes",
    "omni_set_workspace", "omni_set_query_lens",
    "omni_paged_decode_attn", "omni_paged_decode_attn_static", "omni_paged_decode_attn_fp8", "omni_kv_append", "omni_decode_step", "omni_decode_step_fp8", "omni_kv_append_quant_fp8", "omni_kv_pack", "omni_kv_unpack", "omni_paged_prefill_attn", "omni_paged_prefill_attn_fp8", "omni_kv_append_chunk", "omni_get_plan",
    "omni_status_string",
    "omni_debug_last_plan", "omni_debug_lds_layout", "omni_debug_kernel_resources", "omni_debug_gather", "omni_debug_stream_read", "omni_debug_profile_begin",
    "omni_debug_profile_end", "omni_graph_begin", "omni_graph_end", "omni_graph_launch", "omni_graph_destroy",
)


class OmniError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class omni_attn_desc_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_int32) for n in (
        "batch", "num_q_heads", "num_kv_heads", "head_dim", "page_size", "num_pages", "max_blocks_per_seq",
        "q_dtype", "kv_dtype", "out_dtype", "max_context_hint")]


_lib = None


def lib():
    """Open the HIP library (built by paper_2602_02204_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'` (needs hipcc)")
        L = C.CDLL(LIB_PATH)
        vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
        L.omni_create.argtypes = [C.POINTER(omni_attn_desc_t), C.POINTER(vp)]
        L.omni_destroy.argtypes = [vp]; L.omni_destroy.restype = None
        L.omni_set_tuning.argtypes = [vp, C.c_int32, C.c_int32]
        L.omni_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        L.omni_prefill_workspace_bytes.argtypes = [vp, C.c_int32, C.POINTER(C.c_size_t)]
        L.omni_set_workspace.argtypes = [vp, vp, C.c_size_t]
        L.omni_set_query_lens.argtypes = [vp, vp]
        L.omni_paged_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, C.c_float, vp, vp]
        L.omni_paged_decode_attn_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_float, vp, vp]
        L.omni_paged_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, C.c_float, vp, vp]
        L.omni_kv_append.argtypes = [vp] * 8
        L.omni_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_float, vp, vp]
        L.omni_decode_step_fp8.argtypes = [vp] * 10 + [C.c_float, vp, vp]
        L.omni_kv_append_quant_fp8.argtypes = [vp] * 9 + [C.c_float, vp]
        L.omni_kv_pack.argtypes = [vp] * 9
        L.omni_kv_unpack.argtypes = [vp] * 9
        L.omni_paged_prefill_attn.argtypes = [vp] * 8 + [C.c_int32, C.c_float, vp, vp]
        L.omni_paged_prefill_attn_fp8.argtypes = [vp] * 10 + [C.c_int32, C.c_float, vp, vp]
        L.omni_kv_append_chunk.argtypes = [vp] * 9 + [C.c_int32, vp]
        L.omni_get_plan.argtypes = [vp] + [i32p] * 5
        L.omni_status_string.argtypes = [C.c_int]; L.omni_status_string.restype = C.c_char_p
        L.omni_debug_last_plan.argtypes = [vp, i32p, vp]
        L.omni_debug_lds_layout.argtypes = [vp, i32p]
        L.omni_debug_kernel_resources.argtypes = [vp, C.c_int32, i32p]
        L.omni_debug_gather.argtypes = [vp, vp, vp, vp, C.c_int32, vp, vp]
        L.omni_debug_stream_read.argtypes = [vp, C.c_size_t, vp, C.c_size_t, vp, vp]
        L.omni_debug_profile_begin.argtypes = [vp, C.c_int32, C.c_int32]
        L.omni_debug_profile_end.argtypes = [vp, C.POINTER(C.c_float), i32p]
        L.omni_graph_begin.argtypes = [vp]
        L.omni_graph_end.argtypes = [vp, C.POINTER(vp)]
        L.omni_graph_launch.argtypes = [vp, vp]
        L.omni_graph_destroy.argtypes = [vp]; L.omni_graph_destroy.restype = None
        for name in EXPORTS:
            if name not in ("omni_destroy", "omni_status_string", "omni_graph_destroy"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def omni_debug_stream_read(a, b, sink, stream=None) -> None:
    """Plain streaming read of tensors a and b (b may be None); sink is a device tensor of at least 4 bytes."""
    nbytes = lambda t: 0 if t is None else t.numel() * t.element_size()
    _ck(lib().omni_debug_stream_read(_ptr(a), nbytes(a), _ptr(b) if b is not None else None, nbytes(b), _ptr(sink),
                                     _stream(stream)), "omni_debug_stream_read")


class Graph:
    """A recorded sequence of library calls on one stream: `with Graph(stream) as g: ...calls...`, then g.launch()."""

    def __init__(self, stream):
        self._stream = stream
        self._g = None

    def __enter__(self):
        _ck(lib().omni_graph_begin(_stream(self._stream)), "omni_graph_begin")
        return self

    def __exit__(self, exc_type, exc, tb):
        g = C.c_void_p()
        status = lib().omni_graph_end(_stream(self._stream), C.byref(g))      # ends the capture also after an error
        if exc_type is None:
            _ck(status, "omni_graph_end")
            self._g = g
        elif g:
            lib().omni_graph_destroy(g)
        return False

    def launch(self, stream=None) -> None:
        _ck(lib().omni_graph_launch(self._g, _stream(stream if stream is not None else self._stream)), "omni_graph_launch")

    def close(self) -> None:
        if self._g is not None and _lib is not None:
            _lib.omni_graph_destroy(self._g)
        self._g = None

    def __del__(self):
        self.close()


def status_string(status: int) -> str:
    return lib().omni_status_string(int(status)).decode()


def _ck(status: int, where: str) -> None:
    if status != 0:
        raise OmniError(status, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / raw int; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Handle:
    """Owns an omni_handle_t.  Methods are the C entry points with the handle bound."""

    def __init__(self, *, batch, num_q_heads, num_kv_heads, head_dim, page_size, num_pages, max_blocks_per_seq,
                 kv_dtype, out_dtype=OMNI_F32, q_dtype=None, max_context_hint=0):
        d = omni_attn_desc_t(C.sizeof(omni_attn_desc_t), batch, num_q_heads, num_kv_heads, head_dim, page_size,
                             num_pages, max_blocks_per_seq, kv_dtype if q_dtype is None else q_dtype, kv_dtype,
                             out_dtype, max_context_hint)
        self.desc = d
        self._h = C.c_void_p()
        _ck(lib().omni_create(C.byref(d), C.byref(self._h)), "omni_create")
        self._ws = None

    def close(self):
        if getattr(self, "_h", None) is not None and self._h and _lib is not None:
            _lib.omni_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close

    def omni_set_tuning(self, key: int, value: int) -> None:
        _ck(lib().omni_set_tuning(self._h, key, value), "omni_set_tuning")

    def omni_workspace_bytes(self) -> int:
        n = C.c_size_t()
        _ck(lib().omni_workspace_bytes(self._h, C.byref(n)), "omni_workspace_bytes")
        return n.value

    def omni_prefill_workspace_bytes(self, max_q_len: int) -> int:
        n = C.c_size_t()
        _ck(lib().omni_prefill_workspace_bytes(self._h, int(max_q_len), C.byref(n)), "omni_prefill_workspace_bytes")
        return n.value

    def omni_set_workspace(self, tensor_or_ptr, nbytes: Optional[int] = None) -> None:
        if nbytes is None:
            nbytes = tensor_or_ptr.numel() * tensor_or_ptr.element_size()
        self._ws = tensor_or_ptr                     # keep the caller's tensor alive
        _ck(lib().omni_set_workspace(self._h, _ptr(tensor_or_ptr), nbytes), "omni_set_workspace")

    def omni_set_query_lens(self, tensor_or_none) -> None:
        self._q_lens = tensor_or_none                # keep the caller's tensor alive
        _ck(lib().omni_set_query_lens(self._h, _ptr(tensor_or_none) if tensor_or_none is not None else None),
            "omni_set_query_lens")

    def omni_paged_decode_attn(self, q, k_cache, v_cache, block_table, context_lens, scale, out, stream=None) -> None:
        _ck(lib().omni_paged_decode_attn(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                         _ptr(context_lens), C.c_float(float(scale)), _ptr(out), _stream(stream)),
            "omni_paged_decode_attn")

    def omni_paged_decode_attn_static(self, q, k_cache, v_cache, block_table, context_lens, scale, out, stream=None) -> None:
        _ck(lib().omni_paged_decode_attn_static(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                                _ptr(context_lens), C.c_float(float(scale)), _ptr(out), _stream(stream)),
            "omni_paged_decode_attn_static")

    def omni_paged_decode_attn_fp8(self, q, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, scale, out,
                                   stream=None) -> None:
        _ck(lib().omni_paged_decode_attn_fp8(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                                             _ptr(block_table), _ptr(context_lens), C.c_float(float(scale)), _ptr(out),
                                             _stream(stream)), "omni_paged_decode_attn_fp8")

    def omni_kv_append(self, k_new, v_new, k_cache, v_cache, block_table, positions, stream=None) -> None:
        _ck(lib().omni_kv_append(self._h, _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                 _ptr(positions), _stream(stream)), "omni_kv_append")

    def omni_decode_step(self, q, k_new, v_new, k_cache, v_cache, block_table, context_lens, scale, out,
                         stream=None) -> None:
        _ck(lib().omni_decode_step(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                   _ptr(block_table), _ptr(context_lens), C.c_float(float(scale)), _ptr(out),
                                   _stream(stream)), "omni_decode_step")

    def omni_get_plan(self) -> dict:
        v = [C.c_int32() for _ in range(5)]
        _ck(lib().omni_get_plan(self._h, *[C.byref(x) for x in v]), "omni_get_plan")
        keys = ("kernel", "partition_grid", "merge_grid", "max_request_parts", "threads_per_workgroup")
        return dict(zip(keys, (x.value for x in v)))

    def omni_kv_pack(self, k_cache, v_cache, block_table, context_lens, token_offsets, k_dense, v_dense, stream=None) -> None:
        _ck(lib().omni_kv_pack(self._h, _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(context_lens),
                               _ptr(token_offsets), _ptr(k_dense), _ptr(v_dense), _stream(stream)), "omni_kv_pack")

    def omni_kv_unpack(self, k_dense, v_dense, k_cache, v_cache, block_table, context_lens, token_offsets, stream=None) -> None:
        _ck(lib().omni_kv_unpack(self._h, _ptr(k_dense), _ptr(v_dense), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                 _ptr(context_lens), _ptr(token_offsets), _stream(stream)), "omni_kv_unpack")

    def omni_paged_prefill_attn(self, q, k_cache, v_cache, block_table, context_lens, q_lens, q_offsets, max_q_len: int,
                                scale: float, out, stream=None) -> None:
        _ck(lib().omni_paged_prefill_attn(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                          _ptr(context_lens), _ptr(q_lens), _ptr(q_offsets), int(max_q_len),
                                          C.c_float(scale), _ptr(out), _stream(stream)), "omni_paged_prefill_attn")

    def omni_decode_step_fp8(self, q, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, scale,
                             out, stream=None) -> None:
        _ck(lib().omni_decode_step_fp8(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(k_scale), _ptr(v_scale), _ptr(block_table), _ptr(context_lens),
                                       C.c_float(float(scale)), _ptr(out), _stream(stream)), "omni_decode_step_fp8")

    def omni_kv_append_quant_fp8(self, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, positions,
                                 headroom: float, stream=None) -> None:
        _ck(lib().omni_kv_append_quant_fp8(self._h, _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale),
                                           _ptr(v_scale), _ptr(block_table), _ptr(positions), C.c_float(float(headroom)),
                                           _stream(stream)), "omni_kv_append_quant_fp8")

    def omni_paged_prefill_attn_fp8(self, q, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, q_lens,
                                    q_offsets, max_q_len: int, scale, out, stream=None) -> None:
        _ck(lib().omni_paged_prefill_attn_fp8(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                                              _ptr(block_table), _ptr(context_lens), _ptr(q_lens), _ptr(q_offsets),
                                              int(max_q_len), C.c_float(float(scale)), _ptr(out), _stream(stream)),
            "omni_paged_prefill_attn_fp8")

    def omni_kv_append_chunk(self, k_new, v_new, k_cache, v_cache, block_table, context_lens, q_lens, q_offsets,
                             max_q_len: int, stream=None) -> None:
        _ck(lib().omni_kv_append_chunk(self._h, _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                       _ptr(context_lens), _ptr(q_lens), _ptr(q_offsets), int(max_q_len), _stream(stream)),
            "omni_kv_append_chunk")

    def omni_debug_last_plan(self, stream=None) -> dict:
        arr = (C.c_int32 * 4)()
        _ck(lib().omni_debug_last_plan(self._h, arr, _stream(stream)), "omni_debug_last_plan")
        return {"partition_len": arr[0], "request_parts": arr[1], "total_tokens": arr[2]}

    def omni_debug_lds_layout(self) -> dict:
        arr = (C.c_int32 * 6)()
        _ck(lib().omni_debug_lds_layout(self._h, arr), "omni_debug_lds_layout")
        return {"dynamic_bytes": arr[0], "static_bytes": arr[1], "ring_states": arr[2], "k_staged": bool(arr[3]),
                "two_workgroups_per_cu": bool(arr[4]), "max_dynamic_bytes": arr[5]}

    def omni_debug_kernel_resources(self, which: int = 0) -> dict:
        arr = (C.c_int32 * 6)()
        _ck(lib().omni_debug_kernel_resources(self._h, int(which), arr), "omni_debug_kernel_resources")
        return {"registers_per_lane": arr[0], "static_lds_bytes": arr[1], "dynamic_lds_bytes": arr[2],
                "max_threads_per_workgroup": arr[3], "scratch_bytes_per_lane": arr[4], "threads_launched": arr[5]}

    def omni_debug_gather(self, cache, block_table, context_lens, request: int, dense_out, stream=None) -> None:
        _ck(lib().omni_debug_gather(self._h, _ptr(cache), _ptr(block_table), _ptr(context_lens), int(request),
                                    _ptr(dense_out), _stream(stream)), "omni_debug_gather")

    def omni_debug_profile_begin(self, capacity: int, stride: int = 1) -> None:
        self._prof_cap = int(capacity)
        _ck(lib().omni_debug_profile_begin(self._h, int(capacity), int(stride)), "omni_debug_profile_begin")

    def omni_debug_profile_end(self) -> list:
        buf = (C.c_float * self._prof_cap)()
        n = C.c_int32()
        _ck(lib().omni_debug_profile_end(self._h, buf, C.byref(n)), "omni_debug_profile_end")
        return [buf[i] for i in range(n.value)]

    def alloc_workspace(self, device="cuda", prefill_max_q_len: int = 0):
        """Convenience for callers that use torch for memory: allocate and register the workspace (large enough for
        the context split of multi-token queries of up to prefill_max_q_len tokens, if given)."""
        import torch
        n = self.omni_workspace_bytes()
        if prefill_max_q_len > 0:
            n = max(n, self.omni_prefill_workspace_bytes(prefill_max_q_len))
        ws = torch.empty(n, dtype=torch.uint8, device=device)
        self.omni_set_workspace(ws)
        return ws
