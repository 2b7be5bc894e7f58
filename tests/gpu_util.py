"""Helpers for GPU tests: move a host workload to the device and run the HIP path through the C ABI binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_02204_amd import binding as omni
from paper_2602_02204_amd import workloads as W
from paper_2602_02204_amd.devmem import bits_of, to_dev  # noqa: F401  (re-exported for the tests)


class DeviceBatch:
    def __init__(self, wl: W.Workload, out_dtype: str = W.F32, max_context_hint: int = 0, tuning: dict | None = None):
        self.wl = wl
        kv = omni.OMNI_F32 if wl.dtype == W.F32 else omni.OMNI_BF16
        od = omni.OMNI_F32 if out_dtype == W.F32 else omni.OMNI_BF16
        self.h = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                             num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=kv, out_dtype=od,
                             max_context_hint=max_context_hint)
        for k, v in (tuning or {}).items():
            self.h.omni_set_tuning(k, v)
        self.ws = self.h.alloc_workspace()
        self.q = to_dev(wl.q, wl.dtype)
        self.k_cache = to_dev(wl.k_cache, wl.dtype)
        self.v_cache = to_dev(wl.v_cache, wl.dtype)
        self.block_table = torch.from_numpy(wl.block_table).cuda()
        self.context_lens = torch.from_numpy(wl.context_lens).cuda()
        self.out = torch.full((wl.B, wl.Hq, wl.D), float("nan"), device="cuda",
                              dtype=torch.float32 if out_dtype == W.F32 else torch.bfloat16)
        if wl.k_new is not None:
            self.k_new = to_dev(wl.k_new, wl.dtype)
            self.v_new = to_dev(wl.v_new, wl.dtype)
            self.positions = torch.from_numpy(wl.positions).cuda()

    def append(self):
        self.h.omni_kv_append(self.k_new, self.v_new, self.k_cache, self.v_cache, self.block_table, self.positions)

    def attend(self) -> np.ndarray:
        self.out.fill_(float("nan"))
        self.h.omni_paged_decode_attn(self.q, self.k_cache, self.v_cache, self.block_table, self.context_lens,
                                      float(self.wl.scale), self.out)
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64)


TOL = {W.F32: 1e-5, W.BF16: 2e-3}       # max |err| against the fp64 oracle (fp32 output)
