#!/usr/bin/env python3
"""Benchmark of the librap hot path on one MI355X.

A step is one pass of the whole path over one batch: rap_rope_append of the new token(s) of every
sequence, then rap_decode_attn over the compact cache.  Headline workload: the Llama-3.1-8B-shaped
configuration at rho = 0.7 (cfg2: batch 16, 32/8 heads, 8192 rows, d_k = d_v = 90, 1 % of K rows
x8), seeded synthetic bf16 data already resident in HBM.  Successive steps rotate over several
distinct copies of the cache so that the working set exceeds L2 + Infinity Cache and the bytes
really come from HBM.

Every timed figure is the MEDIAN over REPS repetitions of a block of exactly --steps steps (device
synchronised on both sides of each block), with the fastest and slowest block beside it.

Prints ONE compact JSON line: whole-job throughput in algorithmic GB/s (K and V bytes that a decode
step must read once, divided by the step time), the roofline object of the dominant kernel measured
with HIP events on the launch stream, the other four configurations and the rho = 1.0 controls from
the same code (`configs`), the follow-up calls (one-call step, fp8 caches, several tokens, prefill)
and the float64 oracle timed on the host cores.  The same figures with every detail go to
gpurun_out/bench_detail.json when that directory can be written.
"""
from __future__ import annotations

import argparse
import ctypes as C
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
REPS = 11                        # repetitions of the --steps block behind every median


class HipEvents:
    """hipEvent_t handles through the HIP runtime's own C API (torch events are tied to torch's
    current stream; these are recorded by librap on the stream it launches on)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self) -> C.c_void_p:
        ev = C.c_void_p()
        rc = self.hip.hipEventCreate(C.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev

    def elapsed_ms(self, a, b) -> float:
        self.hip.hipEventSynchronize(b)
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def kv_bytes(w, seq_lens) -> int:
    """Algorithmic bytes of one decode step: every K and V row of every KV head once."""
    return int(np.sum(seq_lens)) * w.n_kv_heads * (w.d_k + w.d_v) * 2


def blocks(fn, steps, warmup, sync, reps=REPS):
    """Seconds per step of `reps` blocks of exactly `steps` calls of fn(i), after `warmup` calls:
    (median, min, max)."""
    i = 0
    for _ in range(warmup):
        fn(i)
        i += 1
    out = []
    for _ in range(reps):
        sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn(i)
            i += 1
        sync()
        out.append((time.perf_counter() - t0) / steps)
    return float(np.median(out)), float(np.min(out)), float(np.max(out))


class Job:
    """One workload with n_buf distinct cache copies, ready to step."""

    def __init__(self, rap, I, name, n_buf, device):
        import torch
        self.torch = torch
        self.rap = rap
        self.w = I.WORKLOADS[name]
        if self.w.ragged_min is not None:
            n_buf = 1     # ragged lengths differ from copy to copy (and so do the capacities); one copy is far beyond any cache
        self.cases = [I.make_case(I.scaled(self.w, seed=self.w.seed + 100 * i), device=device) for i in range(n_buf)]
        c0 = self.cases[0]
        w = self.w
        self.shape = rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, c0.cap, w.rope_theta)
        self.max_len = int(max(int(c.seq_lens.max().item()) for c in self.cases))
        self.ws = rap.new_workspace(self.shape, self.max_len, None, device=device)
        self.out = torch.empty((w.batch, w.n_q_heads, w.d_v), dtype=torch.float32, device=device)
        self.bytes_per_step = float(np.mean([kv_bytes(w, c.seq_lens.cpu().numpy()) for c in self.cases]))
        for c in self.cases:
            c.k_new1, c.v_new1 = c.k_new[:, -1].contiguous(), c.v_new[:, -1].contiguous()
            c.pos1 = c.pos[:, -1].contiguous()

    def step(self, i, tuning=None, mode="two"):
        """One decode step.  mode "step": one rap_decode_step call (query already rotated);
        "step_rope": the same with the query rotation fused in; "two": rap_rope_append then
        rap_decode_attn.  Workloads that append several tokens per step always take "two"."""
        c = self.cases[i % len(self.cases)]
        w = self.w
        if w.n_new != 1 or mode == "two":
            self.rap.rap_rope_append(self.shape, w.n_new, c.k_new, c.v_new, c.pos, c.keep, c.k_cache, c.v_cache)
            self.rap.rap_decode_attn(self.shape, c.q, c.k_cache, c.v_cache, c.seq_lens, self.max_len, self.out,
                                     float(w.scale), self.ws, tuning)
        else:
            self.rap.rap_decode_step(self.shape, c.k_new1, c.v_new1, c.pos1, c.keep, c.q, mode == "step", c.k_cache,
                                     c.v_cache, c.seq_lens, self.max_len, self.out, float(w.scale), self.ws, tuning)

    def timed(self, steps, warmup, mode="two"):
        return blocks(lambda i: self.step(i, mode=mode), steps, warmup, self.torch.cuda.synchronize)

    def kernel_ms(self, steps, ev):
        """Duration of the partial-attention kernel alone (mean, min over `steps` launches), HIP
        events recorded by librap around that launch on the launch stream."""
        pairs = [(ev.create(), ev.create()) for _ in range(steps)]
        for i, (a, b) in enumerate(pairs):
            self.step(i, self.rap.tuning(ev_main_start=a, ev_main_stop=b))
        self.torch.cuda.synchronize()
        ms = [ev.elapsed_ms(a, b) for a, b in pairs]
        for a, b in pairs:
            ev.destroy(a)
            ev.destroy(b)
        return float(np.mean(ms)), float(np.min(ms))

    def figures(self, steps, warmup, ev):
        """Step time (median of REPS blocks, with spread) and kernel time of this workload."""
        med, lo, hi = self.timed(steps, warmup)
        k_mean, k_min = self.kernel_ms(max(steps, 10), ev)
        gbps = self.bytes_per_step / med / 1e9
        k_gbps = self.bytes_per_step / (k_mean * 1e-3) / 1e9
        return {"ms": med * 1e3, "ms_min": lo * 1e3, "ms_max": hi * 1e3, "GBps": gbps, "frac": gbps / HBM_PEAK_GBPS,
                "k_ms": k_mean, "k_ms_min": k_min, "k_GBps": k_gbps, "k_frac": k_gbps / HBM_PEAK_GBPS,
                "kv_bytes": int(self.bytes_per_step), "tokens_per_s": self.w.batch / med}

    def stream_read_gbps(self, reps=10):
        """What a trivial read-only kernel reaches over this job's cache bytes, same run."""
        torch = self.torch
        flat = torch.cat([c.k_cache.view(-1) for c in self.cases] + [c.v_cache.view(-1) for c in self.cases]) \
            if len(self.cases) > 1 else None
        bufs = [flat.view(torch.uint8)] if flat is not None else [self.cases[0].k_cache.view(-1).view(torch.uint8),
                                                                  self.cases[0].v_cache.view(-1).view(torch.uint8)]
        bufs = [b[:b.numel() // 16 * 16] for b in bufs]
        sink = torch.zeros(16, dtype=torch.uint8, device=self.out.device)
        for _ in range(3):
            for b in bufs:
                self.rap.rap_stream_read(b, sink)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            for b in bufs:
                self.rap.rap_stream_read(b, sink)
        torch.cuda.synchronize()
        return sum(b.numel() for b in bufs) * reps / (time.perf_counter() - t0) / 1e9


def cpu_baseline(I, case, min_seconds=10.0):
    """The oracle as it stands, on the host cores, over whole decode steps of the same workload
    (append of the new token + attention), repeated until min_seconds have passed."""
    from oracle import rap_oracle as O
    w = case.w
    q, kc, vc = I.bits(case.q), I.bits(case.k_cache), I.bits(case.v_cache)
    k_new, v_new = I.bits(case.k_new), I.bits(case.v_new)
    pos, keep, lens = case.pos.cpu().numpy(), case.keep.cpu().numpy(), case.seq_lens.cpu().numpy()
    n = 0
    t0 = time.perf_counter()
    while True:
        O.append_ref(k_new, v_new, pos, keep, kc, vc, w.rope_theta, w.d_head)
        O.attn_ref(q, kc, vc, lens, w.scale)
        n += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or n >= 50:
            break
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    threads = min(threads, len(os.sched_getaffinity(0)))
    return {"value": round(kv_bytes(w, lens) * n / dt / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d whole steps of %s (append + attention), NumPy float64, %.1f s" % (n, w.name, dt),
            "tokens_per_s": round(w.batch * n / dt, 2)}


def prefill_figure(rap, torch, w, dev, reps=5):
    """Causal prefill attention (rap_prefill_attn) at the workload's shape: every sequence prefilled
    from scratch, HIP-event timing on torch's stream (the call is issued there).  Algorithmic
    flops: 2 (d_k + d_v) per (query token, visible row, query head).  Returns (median ms, flops)."""
    B, S = w.batch, w.ctx
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    kc = torch.randn((B, w.n_kv_heads, S, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((B, w.n_kv_heads, S, w.d_v), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((B, S, w.n_q_heads, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.full((B,), S, dtype=torch.int32, device=dev)
    out = torch.empty((B, S, w.n_q_heads, w.d_v), dtype=torch.float32, device=dev)
    shp = rap.shape(B, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, S, w.rope_theta)
    for _ in range(2):
        rap.rap_prefill_attn(shp, S, q, kc, vc, sl, S, out, float(w.scale))
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        rap.rap_prefill_attn(shp, S, q, kc, vc, sl, S, out, float(w.scale))
        b.record()
    torch.cuda.synchronize()
    ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
    flops = B * w.n_q_heads * (S * (S + 1) / 2) * 2 * (w.d_k + w.d_v)
    del kc, vc, q, out
    torch.cuda.empty_cache()
    return ms, flops


def chunk_figure(rap, torch, w, dev, n_new=64, reps=10):
    """A chunk of n_new tokens at the end of every sequence of the workload (chunked prefill,
    drafted tokens beyond what rap_decode_attn_multi takes): rap_prefill_attn_ex as one launch
    against rap_prefill_attn_split, which also cuts the context into key ranges.  ms of each."""
    B, S = w.batch, w.ctx
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 3)
    kc = torch.randn((B, w.n_kv_heads, S, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((B, w.n_kv_heads, S, w.d_v), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((B, n_new, w.n_q_heads, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    sl = torch.full((B,), S, dtype=torch.int32, device=dev)
    out = torch.empty((B, n_new, w.n_q_heads, w.d_v), dtype=torch.float32, device=dev)
    shp = rap.shape(B, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, S, w.rope_theta)
    need = rap.rap_prefill_attn_split_workspace_bytes(shp, n_new, S)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    calls = (lambda: rap.rap_prefill_attn_ex(shp, kc, vc, None, None, None, n_new, q, sl, S, out, float(w.scale)),
             lambda: rap.rap_prefill_attn_split(shp, kc, vc, None, None, None, n_new, q, sl, S, out, float(w.scale),
                                                ws if need else None))
    ms = []
    for fn in calls:
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms.append(a.elapsed_time(b) / reps)
    del kc, vc, q, out, ws
    torch.cuda.empty_cache()
    return ms


def q8_figure(rap, torch, job, steps, warmup):
    """rap_decode_attn_q8 over fp8 (E4M3) caches of the same shape and lengths (random finite
    codes) and rap_decode_attn over the bf16 caches, each attention call alone: seconds per call
    (medians), and the one-byte rows actually read."""
    w = job.w
    dev = job.out.device
    cap = (max(c.cap for c in job.cases) + 15) // 16 * 16
    shp = rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, cap, w.rope_theta)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 7)
    pools = []
    for _ in job.cases:
        k8 = torch.randint(0, 0x78, (w.batch, w.n_kv_heads, cap, w.d_k), generator=gen, device=dev, dtype=torch.uint8)
        k8 |= torch.randint(0, 2, k8.shape, generator=gen, device=dev, dtype=torch.uint8) << 7
        v8 = torch.randint(0, 0x78, (w.batch, w.n_kv_heads, cap, w.d_v), generator=gen, device=dev, dtype=torch.uint8)
        pools.append((k8, v8))
    ks = torch.full((w.n_kv_heads,), 0.0125, dtype=torch.float32, device=dev)
    vs = ks.clone()
    ws = rap.new_workspace(shp, job.max_len, None, device=dev)
    n = len(job.cases)

    def call(i):
        c = job.cases[i % n]
        rap.rap_decode_attn_q8(shp, c.q, None, None, pools[i % n][0], pools[i % n][1], ks, vs, c.seq_lens, job.max_len,
                               job.out, float(w.scale), ws, None)

    def call16(i):
        c = job.cases[i % n]
        rap.rap_decode_attn(job.shape, c.q, c.k_cache, c.v_cache, c.seq_lens, job.max_len, job.out, float(w.scale), job.ws, None)

    s8 = blocks(call, steps, warmup + 3 * n, torch.cuda.synchronize)[0]
    s16 = blocks(call16, steps, warmup + 3 * n, torch.cuda.synchronize)[0]
    del pools
    torch.cuda.empty_cache()
    return s8, s16, job.bytes_per_step / 2


def mx4_figure(rap, torch, job, steps, warmup):
    """rap_decode_attn_mx4 over 4-bit caches of the same shape and lengths (random codes, scale
    bytes around 2^-2): seconds per attention call (median) and the code and scale bytes read."""
    w = job.w
    dev = job.out.device
    cap = max(c.cap for c in job.cases)
    shp = rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, cap, w.rope_theta)
    nbk, nbv = (w.d_k + 31) // 32, (w.d_v + 31) // 32
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 13)
    pools = []
    for _ in job.cases:
        kc = torch.randint(0, 256, (w.batch, w.n_kv_heads, cap, 16 * nbk), generator=gen, device=dev, dtype=torch.uint8)
        vc = torch.randint(0, 256, (w.batch, w.n_kv_heads, cap, 16 * nbv), generator=gen, device=dev, dtype=torch.uint8)
        ks = torch.randint(123, 127, (w.batch, w.n_kv_heads, cap, 4), generator=gen, device=dev, dtype=torch.uint8)
        vs = torch.randint(123, 127, (w.batch, w.n_kv_heads, cap, 4), generator=gen, device=dev, dtype=torch.uint8)
        pools.append((kc, ks, vc, vs))
    ws = rap.new_workspace(shp, job.max_len, None, device=dev)
    n = len(job.cases)

    def call(i):
        c = job.cases[i % n]
        kc, ks, vc, vs = pools[i % n]
        rap.rap_decode_attn_mx4(shp, c.q, kc, ks, vc, vs, c.seq_lens, job.max_len, job.out, float(w.scale), ws, None)

    s4 = blocks(call, steps, warmup + 3 * n, torch.cuda.synchronize)[0]
    del pools
    torch.cuda.empty_cache()
    rows = job.bytes_per_step / (2 * (w.d_k + w.d_v))                 # cache rows read per step (K and V counted once each)
    return s4, rows * (16 * (nbk + nbv) + nbk + nbv)


def next_rows_figure(rap, torch, job, steps, warmup):
    """The other calls of the path at the headline shape, each alone (medians): the attention with
    the query rotation fused in, the attention over paged pools (pages of 128 rows behind a
    shuffled table), and a prefill-sized append (every row of every sequence in one call; bytes
    read + written)."""
    w = job.w
    c = job.cases[0]
    dev = job.out.device
    sync = torch.cuda.synchronize
    qpos = (c.seq_lens - 1).clamp(min=0).to(torch.int32)
    s_rope = blocks(lambda i: rap.rap_decode_attn_rope(job.shape, c.q, qpos, c.keep, c.k_cache, c.v_cache, c.seq_lens, job.max_len,
                                                       job.out, float(w.scale), job.ws, None), steps, warmup, sync, reps=5)[0]
    page_rows = 128
    max_pages = (job.max_len + page_rows - 1) // page_rows
    cap = max_pages * page_rows
    n_pages = w.batch * max_pages
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 17)
    perm = torch.randperm(n_pages, generator=gen, device=dev)

    def to_pool(x, d):      # dense [B, H, cap_d, d] -> pool [n_pages, H, page_rows, d] through the table
        xd = torch.zeros((w.batch, w.n_kv_heads, cap, d), dtype=x.dtype, device=dev)
        n = min(cap, x.shape[2])
        xd[:, :, :n] = x[:, :, :n]
        xp = xd.reshape(w.batch, w.n_kv_heads, max_pages, page_rows, d).permute(0, 2, 1, 3, 4).reshape(n_pages, w.n_kv_heads, page_rows, d)
        pool = torch.empty_like(xp)
        pool[perm] = xp
        return pool.contiguous()

    kp, vp = to_pool(c.k_cache, w.d_k), to_pool(c.v_cache, w.d_v)
    table = perm.reshape(w.batch, max_pages).to(torch.int32).contiguous()
    shp = rap.shape(w.batch, w.n_q_heads, w.n_kv_heads, w.d_head, w.n_pairs, w.d_v, cap, w.rope_theta)
    pg = rap.paging(page_rows, n_pages, table)
    wsp = rap.new_workspace(shp, job.max_len, None, device=dev)
    s_paged = blocks(lambda i: rap.rap_decode_attn_paged(shp, pg, c.q, None, None, kp, vp, c.seq_lens, job.max_len, job.out,
                                                         float(w.scale), wsp, None), steps, warmup, sync, reps=5)[0]
    del kp, vp
    n_new = int(min(job.max_len, c.cap))
    gen.manual_seed(w.seed + 19)
    k_new = torch.randn((w.batch, n_new, w.n_kv_heads, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_new = torch.randn((w.batch, n_new, w.n_kv_heads, w.d_v), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    pos = torch.arange(n_new, dtype=torch.int32, device=dev).repeat(w.batch, 1).contiguous()
    kc, vc = c.k_cache.clone(), c.v_cache.clone()
    s_bulk = blocks(lambda i: rap.rap_rope_append(job.shape, n_new, k_new, v_new, pos, c.keep, kc, vc), 5, 2, sync, reps=5)[0]
    nbytes = 2.0 * w.batch * n_new * w.n_kv_heads * (w.d_k + w.d_v) * 2
    del k_new, v_new, kc, vc
    torch.cuda.empty_cache()
    return {"rope_ms": r(s_rope * 1e3, 5), "paged_ms": r(s_paged * 1e3, 5), "bulk_append_ms": r(s_bulk * 1e3, 4),
            "bulk_append_GBps": r(nbytes / s_bulk / 1e9, 1)}


def multi_figure(rap, torch, job, steps, warmup):
    """rap_decode_attn_multi over the job's caches: the causal attention of the last n_tok rows of
    every sequence, n_tok = 16 // G of them (the most one launch takes), the attention call alone."""
    w = job.w
    dev = job.out.device
    n_tok = max(1, 16 // (w.n_q_heads // w.n_kv_heads))
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 11)
    q = torch.randn((w.batch, n_tok, w.n_q_heads, w.d_k), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty((w.batch, n_tok, w.n_q_heads, w.d_v), dtype=torch.float32, device=dev)
    ws = rap.new_workspace(job.shape, job.max_len, None, device=dev, n_tok=n_tok)
    n = len(job.cases)

    def call(i):
        c = job.cases[i % n]
        rap.rap_decode_attn_multi(job.shape, c.k_cache, c.v_cache, None, None, None, n_tok, q, c.seq_lens, job.max_len, out,
                                  float(w.scale), ws)

    return n_tok, blocks(call, steps, warmup + 3 * n, torch.cuda.synchronize)[0]


KERNEL_SOURCES = ("rap_decode_kernel.h", "rap_decode_mfma.hip", "rap_device.h", "rap_arith.h")


def kernel_source_id():
    """Short hash of the sources of the dominant kernel (what a committed counter summary was measured on)."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_02599_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:12]


def read_traffic(path):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, and
    the kernel-source hash that summary was measured on; the figure is dropped (None) when the
    kernel's sources have changed since."""
    try:
        kv = {}
        with open(path) as f:
            for line in f:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    kv[k.strip()] = v.strip()
        if kv.get("kernel_source_id") != kernel_source_id():
            return None, "stale: %s was measured on other kernel sources" % os.path.basename(path)
        return float(kv["hbm_bytes_per_launch"]), "profiles/%s (rocprofv3 FETCH_SIZE + WRITE_SIZE, kernel sources %s)" % (
            os.path.basename(path), kv["kernel_source_id"])
    except Exception:
        return None, "no counter summary"


def r(x, n=4):
    return round(float(x), n)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", help="headline workload (default cfg2)")
    ap.add_argument("--buffers", type=int, default=4, help="distinct cache copies rotated through")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-control", action="store_true", help="skip the rho = 1.0 controls")
    ap.add_argument("--no-prefill", action="store_true", help="skip the causal prefill attention figures")
    ap.add_argument("--no-q8", action="store_true", help="skip the fp8-cache and several-token figures")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-valu", action="store_true", help="skip the vector-ALU kernel comparison")
    ap.add_argument("--only-prefill", action="store_true",
                    help="run nothing but the causal prefill attention figure (for profiling that kernel)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain copies of 256 MiB (known-size reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every box here has one); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_02599_amd as pkg
    import rap_inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    rap = pkg.load()
    ev = HipEvents()

    if args.only_prefill:
        w = I.WORKLOADS[args.workload]
        pms, pflops = prefill_figure(rap, torch, w, dev)
        print(json.dumps({"metric": "causal prefill attention (rap_prefill_attn), useful TFLOP/s", "workload": w.name,
                          "ms": round(pms, 4), "value": round(pflops / pms / 1e9, 1), "unit": "TFLOP/s",
                          "frac_of_mfma_peak": round(pflops / pms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}))
        return

    detail = {}
    job = Job(rap, I, args.workload, args.buffers, dev)
    w = job.w
    head = job.figures(args.steps, args.warmup, ev)
    sec_one = job.timed(args.steps, args.warmup, mode="step")[0] if w.n_new == 1 else None
    sec_rope = job.timed(args.steps, args.warmup, mode="step_rope")[0] if w.n_new == 1 else None
    detail[w.name] = head
    stream_gbps = job.stream_read_gbps()
    # the plain vector-ALU kernel on the same step (why the default kernel uses the matrix cores)
    valu = None
    if not args.no_valu and w.n_q_heads // w.n_kv_heads <= 8:
        tun1 = rap.tuning(kernel=1)
        vsec = blocks(lambda i: job.step(i, tuning=tun1), max(2, args.steps // 4), 2, torch.cuda.synchronize, reps=5)[0]
        valu = {"ms": r(vsec * 1e3, 5), "GBps": r(job.bytes_per_step / vsec / 1e9, 1)}

    q8 = multi = mx4 = others = None
    if not args.no_q8:
        s8, s16, b8 = q8_figure(rap, torch, job, args.steps, args.warmup)
        q8 = {"ms": r(s8 * 1e3, 5), "GBps": r(b8 / s8 / 1e9, 1), "frac": r(b8 / s8 / 1e9 / HBM_PEAK_GBPS), "bf16_ms": r(s16 * 1e3, 5),
              "x_bf16": r(s16 / s8)}
        s4, b4 = mx4_figure(rap, torch, job, args.steps, args.warmup)
        mx4 = {"ms": r(s4 * 1e3, 5), "GBps": r(b4 / s4 / 1e9, 1), "x_bf16": r(s16 / s4)}
        n_tok, sm = multi_figure(rap, torch, job, args.steps, args.warmup)
        multi = {"n_tok": n_tok, "ms": r(sm * 1e3, 5)}
        others = next_rows_figure(rap, torch, job, args.steps, args.warmup) if w.ragged_min is None and w.n_new == 1 else None

    if args.copy_calibration:
        csrc = torch.full((256 << 20,), 3, dtype=torch.uint8, device=dev)
        cdst = torch.empty_like(csrc)
        for _ in range(3):
            rap.rap_stream_copy(cdst, csrc)
        torch.cuda.synchronize()
        del csrc, cdst

    traffic, traffic_from = read_traffic(os.path.join(ROOT, "profiles", "traffic_decode_mfma_%s.txt" % w.name))
    result = {
        "metric": "decode-attention HBM GB/s (fraction of peak) and tokens/s at rho=0.7, 1 MI355X",
        "value": r(head["GBps"], 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r(head["ms"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": "%s: B=%d, %d/%d heads, ctx=%d, d_k=%d, d_v=%d, rho=%.1f; step = rap_rope_append + rap_decode_attn"
                               % (w.name, w.batch, w.n_q_heads, w.n_kv_heads, w.ctx, w.d_k, w.d_v, w.n_pairs / (w.d_head / 2)),
                   "copies": len(job.cases), "kv_bytes": head["kv_bytes"]},
        "spread": {"stat": "median of %d blocks of --steps steps" % REPS, "ms_min": r(head["ms_min"], 5), "ms_max": r(head["ms_max"], 5)},
        "frac_of_hbm_peak": r(head["frac"]), "tokens_per_s": r(head["tokens_per_s"], 1), "stream_read_GBps": r(stream_gbps, 1),
        "roofline": {"bound": "hbm", "kernel": "decode_mfma_kernel", "achieved": r(head["k_GBps"], 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": r(head["k_frac"]), "traffic": traffic, "traffic_from": traffic_from,
                     "k_ms": r(head["k_ms"], 5), "k_ms_min": r(head["k_ms_min"], 5)},
    }
    if sec_one is not None:
        result["one_call_step_ms"] = [r(sec_one * 1e3, 5), r(sec_rope * 1e3, 5)]     # query rotated / rotation fused in
    if q8 is not None:
        result["fp8"] = q8
        result["mx4"] = mx4
        result["multi"] = multi
        result["other_calls"] = others
    if valu is not None:
        result["valu_kernel"] = valu

    def compact(f):
        return {"ms": r(f["ms"], 5), "GBps": r(f["GBps"], 1), "frac": r(f["frac"]), "k_ms": r(f["k_ms"], 5), "k_frac": r(f["k_frac"])}

    case0 = job.cases[0]
    del job.cases[1:]
    torch.cuda.empty_cache()

    # ---- rho = 1.0 control of the headline workload, same code
    speedups = {}
    configs = {}
    if not args.no_control and (w.name + "_rho1") in I.WORKLOADS:
        ctl = Job(rap, I, w.name + "_rho1", args.buffers, dev)
        cf = ctl.figures(args.steps, args.warmup, ev)
        detail[ctl.w.name] = cf
        configs[ctl.w.name] = compact(cf)
        speedups[w.name] = [r(cf["ms"] / head["ms"]), r(cf["kv_bytes"] / head["kv_bytes"])]
        del ctl
        torch.cuda.empty_cache()

    # ---- causal prefill attention at the headline shape (next row of the path, not part of `value`)
    if not args.no_prefill and w.ragged_min is None and w.batch * w.ctx * w.n_q_heads * w.d_v * 4 <= 8 << 30:
        pms, pflops = prefill_figure(rap, torch, w, dev)
        pf = {"ms": r(pms), "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": r(pflops / pms / 1e9, 1),
                                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                         "frac": r(pflops / pms / 1e9 / MFMA_BF16_PEAK_TFLOPS), "traffic": None}}
        if not args.no_control and (w.name + "_rho1") in I.WORKLOADS:
            cms, cflops = prefill_figure(rap, torch, I.WORKLOADS[w.name + "_rho1"], dev)
            pf["rho1_ms"] = r(cms)
        pf["chunk64_ms"] = [r(x) for x in chunk_figure(rap, torch, w, dev)]      # one launch / key ranges
        result["prefill"] = pf

    # ---- the other configurations, one at a time (caches freed in between)
    if not args.no_configs and args.workload == "cfg2":
        del job
        torch.cuda.empty_cache()
        for name in ("cfg1", "cfg3", "cfg4", "cfg5", "cfg5_rho1"):
            if name.endswith("_rho1") and args.no_control:
                continue
            j = Job(rap, I, name, args.buffers if name == "cfg1" else 1, dev)
            f = j.figures(args.steps, args.warmup, ev)
            f["stream_read_GBps"] = j.stream_read_gbps(reps=3)
            detail[name] = f
            configs[name] = compact(f)
            del j
            torch.cuda.empty_cache()
        if "cfg5" in detail and "cfg5_rho1" in detail:
            speedups["cfg5"] = [r(detail["cfg5_rho1"]["ms"] / detail["cfg5"]["ms"]), r(detail["cfg5_rho1"]["kv_bytes"] / detail["cfg5"]["kv_bytes"])]
    if configs:
        result["configs"] = configs
    if speedups:
        result["speedup_vs_rho1"] = speedups          # [time ratio, KV-byte ratio] of the rho = 1.0 control over the pruned run

    result["cpu_baseline"] = None if args.no_cpu else cpu_baseline(I, case0)
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_detail.json"), "w") as f:
            json.dump({"line": result, "detail": detail}, f, indent=1)
    except OSError:
        pass
    print(json.dumps(result))


if __name__ == "__main__":
    main()
