#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: omni_decode_step, i.e. the new token's K/V rows
written into their pages (kv_append), the device-side plan, the split-context attention over the paged cache and the
log-sum-exp merge (two kernel launches: attention with the append fused in, then the merge).  --unfused times
omni_kv_append + omni_paged_decode_attn instead (three launches).
Inputs are resident in HBM before the timed region.  The KV pools are replicated and the steps rotate over the
replicas so that the 256 MB memory-side cache cannot serve the reads of the next step.

Prints ONE JSON line: metric/value (tokens/s = requests decoded per second, one token each) and ms_per_step from
exactly --steps timed steps with nothing else in the stream; the roofline of the dominant kernel (algorithmic KV bytes
per launch / its average duration over at least 32 launches, each with a HIP event pair in its own dispatch, in an
untimed loop after the timed region) with the whole-step fraction beside it; the same figures for the other three
stage-shaped batches and for the thinker and talker shapes at four times the batch (extra.other_workloads); and the
fp64 CPU oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
# HBM bytes per launch of the attention kernel, from two rocprofv3 counter runs per workload (FETCH_SIZE scaled by
# 2.000, WRITE_SIZE by 1.000, the factors a plain 1 GiB copy gives); see profiles/decode_mfma_kernel_<workload>.txt.
# Not measured by this script; valid only for the launch plan of the counter run, so the key holds that plan:
# (workload, seed, range length in tokens, ranges, workgroups) -> bytes.  Anything else reports null.
MEASURED_TRAFFIC_BYTES = {("thinker", 1, 1152, 126, 512): 300.2e6, ("talker", 2, 608, 254, 512): 162.6e6,
                          ("long", 3, 1536, 126, 512): 397.1e6, ("mixed", 4, 3104, 64, 512): 812.9e6}
KERNEL_EVENT_LAUNCHES = 48      # launches of the attention kernel that carry an event pair (untimed loop)
STEADY_STEPS = 300              # steps of the steady-state loop reported beside the --steps figure
OTHER_STEPS = 200               # timed steps for each of the other workloads
LARGER_BATCHES = (("thinker", 256), ("talker", 1024))   # also measured: the two stage shapes at four times the batch


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="thinker", choices=["thinker", "talker", "long", "mixed"])
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--replicas", type=int, default=0, help="KV pool replicas to rotate over (0 = enough for >= 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 vector-ALU, 2 MFMA")
    ap.add_argument("--target-wgs", type=int, default=0)
    ap.add_argument("--min-partition", type=int, default=0)
    ap.add_argument("--force-partition", type=int, default=0)
    ap.add_argument("--unfused", action="store_true", help="time omni_kv_append + omni_paged_decode_attn instead")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the talker / long / mixed figures")
    ap.add_argument("--timed-only", action="store_true",
                    help="skip the extra record-keeping loops, so that a profiler sees only warm-up and timed steps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, so that a counter run has a kernel of known traffic in it")
    ap.add_argument("--verbose", action="store_true")
    return ap.parse_args()


class DecodeSetup:
    """One workload resident on the device: handle, workspace, replicated KV pools, and the step functions."""

    def __init__(self, wl, args, torch, np, omni, W, tuned=True):
        from paper_2602_02204_amd.devmem import to_dev
        self.wl, self.torch, self.np, self.omni = wl, torch, np, omni
        self.kvd = omni.OMNI_BF16 if wl.dtype == W.BF16 else omni.OMNI_F32
        h = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                        num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=self.kvd, out_dtype=omni.OMNI_F32)
        if tuned:
            for key, val in ((omni.OMNI_TUNE_KERNEL, args.kernel), (omni.OMNI_TUNE_TARGET_WORKGROUPS, args.target_wgs),
                             (omni.OMNI_TUNE_MIN_PARTITION, args.min_partition),
                             (omni.OMNI_TUNE_FORCE_PARTITION, args.force_partition)):
                if val:
                    h.omni_set_tuning(key, val)
        self.h = h
        self.ws = h.alloc_workspace()
        self.kv_bytes = wl.kv_bytes
        self.pool_bytes = 2 * wl.k_cache.nbytes
        R = args.replicas or max(2, int(np.ceil((1 << 30) / max(self.kv_bytes, 1))))
        self.R = R = min(R, max(1, int(150e9 // self.pool_bytes)))
        self.q = to_dev(wl.q)
        k0, v0 = to_dev(wl.k_cache), to_dev(wl.v_cache)
        self.kc = [k0] + [k0.clone() for _ in range(R - 1)]
        self.vc = [v0] + [v0.clone() for _ in range(R - 1)]
        self.bt = torch.from_numpy(wl.block_table).cuda()
        self.lens = torch.from_numpy(wl.context_lens).cuda()
        self.k_new, self.v_new = to_dev(wl.k_new), to_dev(wl.v_new)
        self.pos = torch.from_numpy(wl.positions).cuda()
        self.out = torch.empty((wl.B, wl.Hq, wl.D), dtype=torch.float32, device="cuda")
        self.scale = float(wl.scale)
        self.stream = torch.cuda.current_stream()
        for r in range(R):                   # every replica holds the appended token before anything is timed
            h.omni_kv_append(self.k_new, self.v_new, self.kc[r], self.vc[r], self.bt, self.pos, self.stream)

    def step_two_launches(self, i):
        r = i % self.R
        self.h.omni_kv_append(self.k_new, self.v_new, self.kc[r], self.vc[r], self.bt, self.pos, self.stream)
        self.h.omni_paged_decode_attn(self.q, self.kc[r], self.vc[r], self.bt, self.lens, self.scale, self.out, self.stream)

    def attention_only(self, i):
        r = i % self.R
        self.h.omni_paged_decode_attn(self.q, self.kc[r], self.vc[r], self.bt, self.lens, self.scale, self.out, self.stream)

    def step_fused(self, i):
        r = i % self.R
        self.h.omni_decode_step(self.q, self.k_new, self.v_new, self.kc[r], self.vc[r], self.bt, self.lens, self.scale,
                                self.out, self.stream)

    def timed(self, fn, K, fixed_replica=False):
        """Milliseconds per step over exactly K steps, synchronised on both sides, nothing else in the stream."""
        self.torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(K):
            fn(0 if fixed_replica else i)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - a) * 1e3 / K

    def kernel_times_ms(self, fn, n=KERNEL_EVENT_LAUNCHES):
        """Durations of the attention kernel alone over n launches: the library attaches a HIP event pair to the kernel's
        own dispatch (on the stream the kernel runs on), in an untimed loop of n steps over the rotating replicas."""
        self.h.omni_debug_profile_begin(n, 1)
        for i in range(n):
            fn(i)
        self.torch.cuda.synchronize()
        return self.h.omni_debug_profile_end()

    def stream_read_ceiling(self, k_avg_us, n=32):
        """The memory system's ceiling for a kernel of this size: a plain streaming read of one replica's K and V pools
        (pool bytes >= the algorithmic bytes: it also reads the unused tail slots and, where the pool is larger than
        the batch, the pages nobody owns), timed with event pairs over the rotating replicas."""
        torch, np, omni = self.torch, self.np, self.omni
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for i in range(8):
            omni.omni_debug_stream_read(self.kc[i % self.R], self.vc[i % self.R], sink, self.stream)
        for i, (a, b) in enumerate(evs):
            a.record(self.stream)
            omni.omni_debug_stream_read(self.kc[i % self.R], self.vc[i % self.R], sink, self.stream)
            b.record(self.stream)
        torch.cuda.synchronize()
        us = float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e3
        return {"kernel": "stream_read_kernel", "bytes": self.pool_bytes, "avg_us": us, "GB/s": self.pool_bytes / us / 1e3,
                "attention_vs_stream_read": (self.kv_bytes / k_avg_us) / (self.pool_bytes / us)}

    def plan(self):
        plan = self.h.omni_debug_last_plan()
        plan.update(self.h.omni_get_plan())
        return plan

    def resources(self):
        res = {"merge_kernel": self.h.omni_debug_kernel_resources(1)}
        if self.h.omni_get_plan()["kernel"] == self.omni.KERNEL_MFMA:
            res["decode_mfma_kernel"] = self.h.omni_debug_kernel_resources(0)
            res["decode_mfma_kernel"]["shared_memory_layout"] = self.h.omni_debug_lds_layout()
        return res

    def check_parity(self, oracle, W, n_pairs=4):
        """Sampled rows of the last step against the oracle (on a host copy of the pools with the token appended)."""
        wl, np = self.wl, self.np
        kf, vf = wl.k_cache.copy(), wl.v_cache.copy()
        oracle.kv_append(wl.k_new, wl.v_new, kf, vf, wl.block_table, wl.positions, wl.dtype)
        rng = np.random.default_rng(0)
        pairs = [(int(b), int(hh)) for b, hh in zip(rng.integers(0, wl.B, n_pairs), rng.integers(0, wl.Hq, n_pairs))]
        ref = oracle.paged_decode_attn(wl.q, kf, vf, wl.block_table, wl.context_lens, wl.scale, wl.dtype, pairs=pairs)
        got = self.out.cpu().numpy().astype(np.float64)
        err = float(max(np.max(np.abs(got[b, hh] - ref[i])) for i, (b, hh) in enumerate(pairs)))
        tol = 2e-3 if wl.dtype == W.BF16 else 1e-5
        if not (err <= tol):
            print(f"bench.py: parity check failed on {wl.name}, max|err|={err:.3e} > {tol}", file=sys.stderr)
            sys.exit(1)
        return err


def traffic_for(wl, plan):
    if plan["kernel"] != 2:
        return None
    return MEASURED_TRAFFIC_BYTES.get((wl.name, wl.seed, plan["partition_len"], plan["request_parts"], plan["partition_grid"]))


def measure_other(name, args, torch, np, omni, W, oracle, batch=None):
    """One of the other stage-shaped batches through the same step, default tuning: step time over OTHER_STEPS timed
    steps, the attention kernel over KERNEL_EVENT_LAUNCHES event-carrying launches, the stream-read ceiling.
    `batch`: the same shape and length distribution with that many requests."""
    wl = W.make(name, append=True, batch=batch)
    d = DecodeSetup(wl, args, torch, np, omni, W, tuned=False)
    for i in range(10):
        d.step_fused(i)
    ms = d.timed(d.step_fused, OTHER_STEPS)
    km = d.kernel_times_ms(d.step_fused)
    k_avg_us, k_med_us = float(np.mean(km)) * 1e3, float(np.median(km)) * 1e3
    plan = d.plan()
    res = {"config": f"{wl.name}: B={wl.B}, Hq={wl.Hq}, Hkv={wl.Hkv}, D={wl.D}, page={wl.ps}, seed {wl.seed}, "
                     f"pool {wl.P} pages ({d.pool_bytes / 1e6:.0f} MB of K+V)",
           "total_context_tokens": wl.total_tokens, "kv_bytes_per_step": d.kv_bytes, "pool_replicas": d.R,
           "steps": OTHER_STEPS, "ms_per_step": ms, "tokens_per_s": wl.B / (ms * 1e-3),
           "kv_gbs_per_step": d.kv_bytes / (ms * 1e-3) / 1e9, "step_frac": d.kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "kernel": "decode_mfma_kernel" if plan["kernel"] == 2 else "decode_valu_kernel",
           "kernel_avg_us": k_avg_us, "kernel_median_us": k_med_us, "kernel_launches_timed": len(km),
           "kernel_GB/s": d.kv_bytes / k_avg_us / 1e3, "frac": d.kv_bytes / k_avg_us / 1e3 / HBM_PEAK_GBS,
           "traffic": traffic_for(wl, plan), "stream_read_ceiling": d.stream_read_ceiling(k_avg_us, n=24),
           "plan": plan, "kernel_resources": d.resources(),
           "parity_max_abs_err_sampled": d.check_parity(oracle, W)}
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); nothing here shards across devices.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_02204_amd import binding as omni
    from paper_2602_02204_amd import workloads as W
    from paper_2602_02204_amd.devmem import to_dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    log = (lambda *a: print(*a, file=sys.stderr, flush=True)) if args.verbose else (lambda *a: None)

    wl = W.make(args.workload, seed=args.seed, append=True)
    kv_bytes = wl.kv_bytes
    log(f"workload {wl.name}: B={wl.B} Hq={wl.Hq} Hkv={wl.Hkv} D={wl.D} ps={wl.ps} T={wl.total_tokens} "
        f"KV bytes/call={kv_bytes / 1e6:.1f} MB pool pages={wl.P}")

    dec = DecodeSetup(wl, args, torch, np, omni, W)
    h, kvd, R, pool_bytes = dec.h, dec.kvd, dec.R, dec.pool_bytes
    q, kc, vc, bt, lens, k_new, v_new, out = dec.q, dec.kc, dec.vc, dec.bt, dec.lens, dec.k_new, dec.v_new, dec.out
    scale, stream = dec.scale, dec.stream
    step_fused, step_two_launches = dec.step_fused, dec.step_two_launches
    step = step_two_launches if args.unfused else step_fused

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    plan = dec.plan()

    # ---- timed region: exactly K steps between two synchronisations, nothing else in the stream
    K = args.steps
    ms_per_step = dec.timed(step, K)
    tokens_per_s = wl.B / (ms_per_step * 1e-3)

    # ---- the attention kernel alone (untimed loop, an event pair in every launch's own dispatch)
    kernel_ms = dec.kernel_times_ms(step)
    k_avg_ms = float(np.mean(kernel_ms))
    k_med_ms = float(np.median(kernel_ms))
    achieved = kv_bytes / (k_avg_ms * 1e-3) / 1e9

    def timed(fn, fixed_replica=False, steps=None):
        return dec.timed(fn, steps or K, fixed_replica)

    # ---- for the record: a longer steady-state loop, the same K steps as two launches, and on a single replica
    ms_steady = ms_other = ms_warm = ms_graph = host_us_graph = host_us_eager = ms_attn = None
    if not args.timed_only:
        ms_steady = timed(step, steps=max(K, STEADY_STEPS))
        ms_other = timed(step_fused if args.unfused else step_two_launches)
        # one omni_paged_decode_attn call (attention + merge; every token already in the pools): no append in it
        ms_attn = timed(dec.attention_only, steps=max(K, STEADY_STEPS))
        ms_warm = timed(step, fixed_replica=True)
        # the same steps recorded once as a HIP graph (one step per pool replica) and replayed: what is left of the
        # step time when the host issues one call per R steps instead of one per kernel
        gs = torch.cuda.Stream()
        for r in range(R):
            h.omni_decode_step(q, k_new, v_new, kc[r], vc[r], bt, lens, scale, out, gs)
        torch.cuda.synchronize()
        with omni.Graph(gs) as graph:
            for r in range(R):
                h.omni_decode_step(q, k_new, v_new, kc[r], vc[r], bt, lens, scale, out, gs)
        for _ in range(3):
            graph.launch()
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(max(1, K // R)):
            graph.launch()
        issued = time.perf_counter()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - a) * 1e3 / (max(1, K // R) * R)
        host_us_graph = (issued - a) * 1e6 / (max(1, K // R) * R)
        graph.close()
        # host time to issue a step eagerly (python + ctypes + two launches), GPU idle-free queue not awaited
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(64):
            step(i)
        host_us_eager = (time.perf_counter() - a) * 1e6 / 64
        torch.cuda.synchronize()

    # ---- several query tokens per request (speculative decoding / multi-token prediction): the same batch with T
    # tokens per request through the same kernel, T * (Hq / Hkv) <= 16 columns; attention + merge over rotating replicas
    multi = None
    if not args.timed_only and h.omni_get_plan()["kernel"] == omni.KERNEL_MFMA and 2 * (wl.Hq // wl.Hkv) <= 16:
        T = 16 // (wl.Hq // wl.Hkv)
        hT = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                         num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=kvd, out_dtype=omni.OMNI_F32)
        hT.omni_set_tuning(omni.OMNI_TUNE_QUERY_TOKENS, T)
        wsT = hT.alloc_workspace()
        qT_host = W.f32_to_bf16_bits(np.random.default_rng(5).standard_normal((wl.B * T, wl.Hq, wl.D)).astype(np.float32))
        qT = to_dev(qT_host, wl.dtype)
        outT = torch.empty((wl.B, T, wl.Hq, wl.D), dtype=torch.float32, device="cuda")
        stepT = lambda i: hT.omni_paged_decode_attn(qT, kc[i % R], vc[i % R], bt, lens, scale, outT, stream)
        for i in range(8):
            stepT(i)
        msT = timed(stepT)
        # parity on sampled rows: the chunk definition with q_lens = T (the appended token is in every replica)
        import oracle as _oracle
        kfull, vfull = wl.k_cache.copy(), wl.v_cache.copy()
        _oracle.kv_append(wl.k_new, wl.v_new, kfull, vfull, wl.block_table, wl.positions, wl.dtype)
        nT = np.full(wl.B, T, dtype=np.int32)
        oT = np.arange(wl.B, dtype=np.int64) * T
        rowsT = [(0, 0, 0), (wl.B - 1, T - 1, wl.Hq - 1), (wl.B // 2, T // 2, 3)]
        refT = _oracle.paged_prefill_attn(qT_host, kfull, vfull, wl.block_table, wl.context_lens, nT, oT, wl.scale, wl.dtype,
                                          rows=rowsT)
        gotT = outT.cpu().numpy().astype(np.float64)
        errT = float(max(np.max(np.abs(gotT[b, i, hh] - refT[r])) for r, (b, i, hh) in enumerate(rowsT)))
        if not (errT <= 2e-3):
            print(f"bench.py: multi-token parity check failed, max|err|={errT:.3e}", file=sys.stderr)
            sys.exit(1)
        multi = {"query_tokens_per_request": T, "ms_per_step": msT, "query_tokens_per_s": wl.B * T / (msT * 1e-3),
                 "parity_max_abs_err_sampled": errT, "note": "omni_paged_decode_attn with OMNI_TUNE_QUERY_TOKENS: attention + merge, no append"}
        del qT, outT, wsT

    # ---- the memory system's ceiling for a kernel of this size (plain streaming read of one replica's pools)
    ceiling = None if args.timed_only else dec.stream_read_ceiling(k_avg_ms * 1e3, n=40)

    # ---- the dense copies a connector ships (whole batch packed out of the pools, and unpacked back in)
    pack = None
    if not args.timed_only:
        offs = torch.from_numpy(np.concatenate([[0], np.cumsum(wl.context_lens[:-1])]).astype(np.int64)).cuda()
        kd = torch.empty((wl.total_tokens, wl.Hkv, wl.D), dtype=kc[0].dtype, device="cuda")
        vd = torch.empty_like(kd)
        pack = {"bytes_read_plus_written": 2 * kv_bytes}
        for nm, fn in (("pack", lambda r: h.omni_kv_pack(kc[r], vc[r], bt, lens, offs, kd, vd, stream)),
                       ("unpack", lambda r: h.omni_kv_unpack(kd, vd, kc[r], vc[r], bt, lens, offs, stream))):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(24)]
            for i in range(4):
                fn(i % R)
            for i, (a, b) in enumerate(evs):
                a.record(stream)
                fn(i % R)
                b.record(stream)
            torch.cuda.synchronize()
            us = float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e3
            pack[nm + "_avg_us"] = us
            pack[nm + "_GB/s"] = 2 * kv_bytes / us / 1e3
        # yardstick: the runtime's own device-to-device copy of the same dense buffers
        kd2, vd2 = torch.empty_like(kd), torch.empty_like(vd)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
        for i, (a, b) in enumerate(evs):
            a.record(stream)
            kd2.copy_(kd)
            vd2.copy_(vd)
            b.record(stream)
        torch.cuda.synchronize()
        us = float(np.mean([a.elapsed_time(b) for a, b in evs[2:]])) * 1e3
        pack["plain_copy_avg_us"] = us
        pack["plain_copy_GB/s"] = 2 * kv_bytes / us / 1e3
        del kd, vd, kd2, vd2

    # ---- multi-token queries (chunked prefill) on the matrix cores; useful flops = 4 * D * Hq per (query, visible
    # token) pair.  (a) 32 thinker-shaped requests, each with a chunk of 512 new tokens at the end of its context: the
    # query blocks fill the chip.  (b) ONE long request (about 30k tokens of context) with a 512-token chunk: 60
    # workgroups unless the context is split, measured both ways.
    def measure_prefill(pw, chunk, split, fp8=False):
        ch = W.add_chunk(pw, [chunk] * pw.B, 77, in_cache=True)
        ph = omni.Handle(batch=pw.B, num_q_heads=pw.Hq, num_kv_heads=pw.Hkv, head_dim=pw.D, page_size=pw.ps,
                         num_pages=pw.P, max_blocks_per_seq=pw.MB, kv_dtype=omni.OMNI_FP8_E4M3 if fp8 else kvd,
                         q_dtype=omni.OMNI_BF16, out_dtype=omni.OMNI_F32)
        if not split:
            ph.omni_set_tuning(omni.OMNI_TUNE_PREFILL_SPLITS, 1)
        pws = ph.alloc_workspace(prefill_max_q_len=ch.max_q_len)
        pq = to_dev(ch.q, pw.dtype)
        if fp8:
            p8 = W.quantize_fp8(pw)
            pk, pv = torch.from_numpy(p8.k_cache).cuda(), torch.from_numpy(p8.v_cache).cuda()
            pks, pvs = torch.from_numpy(p8.k_scale).cuda(), torch.from_numpy(p8.v_scale).cuda()
        else:
            pk, pv = to_dev(pw.k_cache, pw.dtype), to_dev(pw.v_cache, pw.dtype)
        pbt, plens = torch.from_numpy(pw.block_table).cuda(), torch.from_numpy(pw.context_lens).cuda()
        pql, pqo = torch.from_numpy(ch.q_lens).cuda(), torch.from_numpy(ch.q_offsets).cuda()
        pout = torch.empty((ch.total, pw.Hq, pw.D), dtype=torch.float32, device="cuda")
        Lh, nh = pw.context_lens.astype(np.int64), ch.q_lens.astype(np.int64)
        pairs = int(np.sum(nh * (Lh - nh) + nh * (nh + 1) // 2))
        flops = 4.0 * pw.D * pw.Hq * pairs
        if fp8:
            run = lambda: ph.omni_paged_prefill_attn_fp8(pq, pk, pv, pks, pvs, pbt, plens, pql, pqo, ch.max_q_len,
                                                         float(pw.scale), pout, stream)
        else:
            run = lambda: ph.omni_paged_prefill_attn(pq, pk, pv, pbt, plens, pql, pqo, ch.max_q_len, float(pw.scale), pout, stream)
        for _ in range(3):
            run()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for a, b in evs:
            a.record(stream)
            run()
            b.record(stream)
        torch.cuda.synchronize()
        us = float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e3
        live = [b for b in range(pw.B) if ch.q_lens[b] > 0]
        rows = [(live[0], 0, 0), (live[-1], int(ch.q_lens[live[-1]]) - 1, pw.Hq - 1),
                (live[len(live) // 2], int(ch.q_lens[live[len(live) // 2]]) // 2, 3)]
        import oracle as _oracle
        if fp8:
            pref = _oracle.paged_prefill_attn_fp8(ch.q, p8.k_cache, p8.v_cache, p8.k_scale, p8.v_scale, pw.block_table,
                                                  pw.context_lens, ch.q_lens, ch.q_offsets, pw.scale, rows=rows)
        else:
            pref = _oracle.paged_prefill_attn(ch.q, pw.k_cache, pw.v_cache, pw.block_table, pw.context_lens, ch.q_lens,
                                              ch.q_offsets, pw.scale, pw.dtype, rows=rows)
        pgot = pout.cpu().numpy().astype(np.float64)
        perr = float(max(np.max(np.abs(pgot[ch.q_offsets[b] + i, hh] - pref[r])) for r, (b, i, hh) in enumerate(rows)))
        if not (perr <= 2e-3):
            print(f"bench.py: prefill parity check failed, max|err|={perr:.3e}", file=sys.stderr)
            sys.exit(1)
        return {"query_token_pairs": pairs, "useful_flops": flops, "avg_us": us, "TFLOP/s": flops / us / 1e6,
                "peak_TFLOP/s": 2500.0, "frac": flops / us / 1e6 / 2500.0, "parity_max_abs_err_sampled": perr,
                "context_split_workspace_MB": ph.omni_prefill_workspace_bytes(ch.max_q_len) / 1e6}

    prefill = None
    prefill_one = None
    if not args.timed_only and wl.dtype == W.BF16 and wl.D == 128:
        pw = W.make(wl.name, batch=min(32, wl.B), append=False)
        prefill = {"kernel": "prefill_mfma_kernel", "workload": f"{pw.B} {pw.name}-shaped requests, chunk of 512 tokens each"}
        prefill.update(measure_prefill(pw, 512, True))
        prefill["over_8bit_kv_cache"] = measure_prefill(pw, 512, True, fp8=True)
        p1 = W.make("long", batch=1, append=False)
        prefill_one = {"kernel": "prefill_mfma_kernel + prefill_merge_kernel",
                       "workload": f"one request of {int(p1.context_lens[0])} tokens, chunk of 512 tokens",
                       "context_split": measure_prefill(p1, 512, True), "no_split": measure_prefill(p1, 512, False)}
        del pw, p1

    # ---- the same batch over an 8-bit (E4M3) KV cache with per-page scales: half the bytes per token
    fp8 = None
    if not args.timed_only and wl.dtype == W.BF16 and wl.D == 128:
        wl8 = W.make(args.workload, seed=args.seed, append=False)       # the same batch with every token in the pools
        f8 = W.quantize_fp8(wl8)
        h8 = omni.Handle(batch=wl.B, num_q_heads=wl.Hq, num_kv_heads=wl.Hkv, head_dim=wl.D, page_size=wl.ps,
                         num_pages=wl.P, max_blocks_per_seq=wl.MB, kv_dtype=omni.OMNI_FP8_E4M3, q_dtype=omni.OMNI_BF16,
                         out_dtype=omni.OMNI_F32)
        ws8 = h8.alloc_workspace()
        k8 = [torch.from_numpy(f8.k_cache).cuda()]
        v8 = [torch.from_numpy(f8.v_cache).cuda()]
        R8 = max(2, int(np.ceil((1 << 30) / max(kv_bytes // 2, 1))))
        k8 += [k8[0].clone() for _ in range(R8 - 1)]
        v8 += [v8[0].clone() for _ in range(R8 - 1)]
        ks8, vs8 = torch.from_numpy(f8.k_scale).cuda(), torch.from_numpy(f8.v_scale).cuda()
        out8 = torch.empty_like(out)
        # the step appends the last token's byte rows (the ones the pools already hold, so every replica stays as it is)
        pos8 = wl8.context_lens.astype(np.int64) - 1
        pg8 = wl8.block_table[np.arange(wl.B), pos8 // wl.ps]
        kn8 = torch.from_numpy(np.ascontiguousarray(f8.k_cache[pg8, :, pos8 % wl.ps, :])).cuda()
        vn8 = torch.from_numpy(np.ascontiguousarray(f8.v_cache[pg8, :, pos8 % wl.ps, :])).cuda()
        step8 = lambda i: h8.omni_decode_step_fp8(q, kn8, vn8, k8[i % R8], v8[i % R8], ks8, vs8, bt, lens, scale, out8, stream)
        for i in range(args.warmup):
            step8(i)
        ms8 = timed(step8, steps=max(K, STEADY_STEPS))
        h8.omni_debug_profile_begin(KERNEL_EVENT_LAUNCHES, 1)
        for i in range(KERNEL_EVENT_LAUNCHES):
            step8(i)
        torch.cuda.synchronize()
        kern8 = float(np.mean(h8.omni_debug_profile_end())) * 1e3
        import oracle as _oracle
        pr8 = [(0, 0), (wl.B - 1, wl.Hq - 1), (wl.B // 2, 3)]
        ref8 = _oracle.paged_decode_attn_fp8(wl8.q, f8.k_cache, f8.v_cache, f8.k_scale, f8.v_scale, wl8.block_table,
                                             wl8.context_lens, wl8.scale, pairs=pr8)
        got8 = out8.cpu().numpy().astype(np.float64)
        err8 = float(max(np.max(np.abs(got8[b, hh] - ref8[i])) for i, (b, hh) in enumerate(pr8)))
        if not (err8 <= 2e-3):
            print(f"bench.py: fp8 parity check failed, max|err|={err8:.3e}", file=sys.stderr)
            sys.exit(1)
        fp8 = {"kv_bytes_per_step": kv_bytes // 2, "ms_per_step": ms8, "tokens_per_s": wl.B / (ms8 * 1e-3),
               "kernel_avg_us": kern8, "kernel_launches_timed": KERNEL_EVENT_LAUNCHES, "kernel_GB/s": kv_bytes / 2 / kern8 / 1e3,
               "kernel_frac_of_hbm_peak": kv_bytes / 2 / kern8 / 1e3 / HBM_PEAK_GBS, "pool_replicas": R8,
               "parity_max_abs_err_sampled": err8, "note": "omni_decode_step_fp8: append fused into the attention kernel, then the merge"}
        del k8, v8

    if args.calibrate_copy:                  # 1 GiB read + 1 GiB written per copy: the yardstick for FETCH_SIZE / WRITE_SIZE
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- validity: sampled rows of the last step against the oracle (the appended token is in the pools now)
    import oracle
    for i in range(2):
        step(i)
    torch.cuda.synchronize()
    max_err = dec.check_parity(oracle, W)
    oracle.kv_append(wl.k_new, wl.v_new, wl.k_cache, wl.v_cache, wl.block_table, wl.positions, wl.dtype)

    # ---- the other stage-shaped batches through the same step (default tuning)
    resources = dec.resources()
    others = None
    if not args.timed_only and not args.no_other_workloads:
        others = {}
        for name in ("thinker", "talker", "long", "mixed"):
            if name != wl.name:
                log(f"other workload: {name}")
                others[name] = measure_other(name, args, torch, np, omni, W, oracle)
                torch.cuda.empty_cache()
        # the same shapes with four times the requests (what a fuller engine would hand over per step)
        for name, batch in LARGER_BATCHES:
            log(f"larger batch: {name} x {batch}")
            others[f"{name}_batch_{batch}"] = measure_other(name, args, torch, np, omni, W, oracle, batch=batch)
            torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle as it stands, all host threads, whole batch, one warm-up slice then timed passes
    cpu = None
    if not args.no_cpu_baseline:
        oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype,
                                 pairs=[(0, 0)])
        reps, spent, used = 0, 0.0, 1
        while reps < 1 or (spent < 1.5 and reps < 25):     # about 20 core-seconds of oracle work
            c0 = time.perf_counter()
            _, used = oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens,
                                               wl.scale, wl.dtype, return_threads=True)
            spent += time.perf_counter() - c0
            reps += 1
        cpu_s = spent / reps
        # the same oracle on one thread, on a slice of the batch (the first 8 requests)
        nb = min(8, wl.B)
        one_pairs = [(b, hh) for b in range(nb) for hh in range(wl.Hq)]
        c0 = time.perf_counter()
        oracle.paged_decode_attn(wl.q, wl.k_cache, wl.v_cache, wl.block_table, wl.context_lens, wl.scale, wl.dtype,
                                 pairs=one_pairs, num_threads=1)
        one_s = time.perf_counter() - c0
        one_tokens = float(wl.context_lens[:nb].astype(np.int64).sum())
        cpu = {"value": wl.B / cpu_s, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
               "single_thread_tokens_per_s": nb / one_s,
               "single_thread_sample": f"first {nb} requests ({int(one_tokens)} context tokens) in {one_s:.2f} s on 1 thread",
               "sample": f"whole {wl.name} batch ({wl.B} requests, {wl.total_tokens} context tokens), "
                         f"{reps} pass(es) of {cpu_s:.2f} s, fp64, OpenMP over (request, head)",
               "kv_gbs": kv_bytes / cpu_s / 1e9}

    result = {
        "metric": "decode-attention tokens/s (one token per request per step; kv_append + paged decode attention, "
                  + ("separate append kernel)" if args.unfused else "append fused into the attention kernel)"),
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == W.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B}, context U[512,4096], Hq={wl.Hq}, Hkv={wl.Hkv}, D={wl.D}, "
                               f"page={wl.ps}, bf16 KV/Q, fp32 accumulate and output" if wl.name == "thinker" else
                               f"{wl.name}: B={wl.B}, Hq={wl.Hq}, Hkv={wl.Hkv}, D={wl.D}, page={wl.ps}",
                   "seed": wl.seed, "total_context_tokens": wl.total_tokens, "kv_bytes_per_step": kv_bytes,
                   "pool_replicas": R, "plan": plan},
        "kv_gbs_per_step": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_for(wl, plan),
                     "kernel": "decode_mfma_kernel" if plan["kernel"] == 2 else "decode_valu_kernel",
                     "kernel_avg_us": k_avg_ms * 1e3, "kernel_median_us": k_med_ms * 1e3,
                     "kernel_launches_timed": len(kernel_ms),
                     "algorithmic_bytes_per_launch": kv_bytes,
                     "step_frac": kv_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "step_frac_steady": kv_bytes / (ms_steady * 1e-3) / 1e9 / HBM_PEAK_GBS if ms_steady else None,
                     "steady_steps": max(K, STEADY_STEPS) if ms_steady else None,
                     "note": "frac = the attention kernel alone (event pairs in its dispatch); step_frac = the same bytes "
                             "over the whole step of the timed region (attention + merge + launch gaps + the two "
                             "synchronisations, which weigh 1/steps); step_frac_steady = the same over steady_steps steps. "
                             "The 0.70 target of this workload is defined on the call, merge included: read step_frac_steady.",
                     "stream_read_ceiling": ceiling},
        "cpu_baseline": cpu,
        "extra": {"ms_per_step_steady": ms_steady,
                  "kernel_resources": resources,
                  "other_workloads": others,
                  ("ms_per_step_fused" if args.unfused else "ms_per_step_separate_append"): ms_other,
                  "ms_per_call_attention_only": ms_attn,
                  "frac_per_call_attention_only": kv_bytes / (ms_attn * 1e-3) / 1e9 / HBM_PEAK_GBS if ms_attn else None,
                  "ms_per_step_single_replica_cache_warm": ms_warm,
                  "ms_per_step_replayed_as_hip_graph": ms_graph,
                  "host_us_to_issue_a_step_eager": host_us_eager, "host_us_to_issue_a_step_in_graph": host_us_graph,
                  "kv_gbs_cache_warm": kv_bytes / (ms_warm * 1e-3) / 1e9 if ms_warm else None,
                  "kv_pack_unpack": pack,
                  "multi_token_decode": multi,
                  "prefill_chunk": prefill,
                  "prefill_chunk_one_long_request": prefill_one,
                  "fp8_kv_cache": fp8,
                  "parity_max_abs_err_sampled": max_err},
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
