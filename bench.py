#!/usr/bin/env python3
"""Benchmark of the Shift Parallelism attention hot path on one MI355X.

A "step" is one pass of the whole hot path at the Llama-3.3-70B head-shard shape (8 query
heads / 1 KV head, head_dim 128), inputs resident in HBM:

    sp_kv_append (32768 tokens) ->  sp_attn_prefill   [C5a: SP-mode prefill, one 32768-token
                                                       sequence, causal]
    sp_kv_append (64 tokens)    ->  sp_attn_decode    [C3: TP-mode decode, 64 sequences with
                                                       contexts U{512..8192}; split + combine]

Every phase is bracketed by HIP events on the launch stream inside the timed region, so the
prefill TFLOP/s and the decode GB/s are per-phase figures (mean, median and minimum over the
timed steps); ``ms_per_step`` is the wall time of the whole step.  The decode phase rotates over
several copies of its KV pool so that its working set (about 140 MB, smaller than the 256 MB
last-level cache) is read cold from HBM; the same step on a single pool copy is timed beside it
("warm").

Prints ONE JSON line.  ``value`` is the prefill attention TFLOP/s of C5a (algorithmic flops /
mean prefill-phase duration); the decode GB/s rides along in ``roofline_decode``.  Side
workloads (C2, C4, C5b, C5c, the verification batch, other shard shapes, a mixed batch, the head
exchange) and the oracle's timing on the machine's host cores follow in the same line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled by
# what the same counters read for the 1 GiB copy of `--workload copy` (FETCH_SIZE x2.000,
# WRITE_SIZE x1.000); figures and commands in profiles/pmc_hbm_traffic_and_mfma.md.
TRAFFIC_PREFILL_C5A = int(359105.0 * 1024 * 2.0 + 65852.2 * 1024)
TRAFFIC_DECODE_C3 = int((68028.5 + 3678.5) * 1024 * 2.0 + (3889.6 + 128.0) * 1024)


def _dev_bf16(u16):
    import torch

    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def _dev_i32(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _bits(t) -> np.ndarray:
    import torch

    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _stats(ms):
    ms = np.asarray(ms, dtype=np.float64)
    return {"mean": float(ms.mean()), "median": float(np.median(ms)), "min": float(ms.min())}


def time_phases(fns, steps, warmup):
    """Runs the phase functions in order `steps` times.  Returns (wall ms/step, [per-phase array of
    ms, one entry per step]) from HIP events recorded on the launch stream around every phase."""
    import torch

    for _ in range(warmup):
        for f in fns:
            f()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        ev[s][0].record()
        for i, f in enumerate(fns):
            f()
            ev[s][i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    per = [np.array([ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)]) for i in range(len(fns))]
    return wall, per


def time_one(fn, iters, warmup=3):
    _, per = time_phases([fn], iters, warmup)
    return _stats(per[0])


def randn_bf16(shape, gen):
    import torch

    return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)


class LongPrefillJob:
    """C5a: one 32768-token causal prefill at 8q/1kv, d=128 (block table from the seeded workload
    recipe, values from torch's seeded GPU generator: N(0,1) rounded to bf16)."""

    def __init__(self, sp, T=32768, Hq=8, Hkv=1, d=128, batch=1, seed=5):
        import torch
        import workloads as W

        self.sp, self.T, self.Hq, self.Hkv, self.d, self.batch = sp, T, Hq, Hkv, d, batch
        g = torch.Generator(device="cuda").manual_seed(seed)
        total = np.full(batch, T, dtype=np.int32)
        if batch == 1 and T == 32768 and Hkv == 1 and d == 128:
            w = W.c5_long(decode_steps=0)
            self.block_table, self.num_pages = w.block_table, w.num_pages
        else:
            self.block_table, self.num_pages = W.make_block_table(np.random.default_rng(seed), total)
        self.scale = float(np.float32(1.0) / np.sqrt(np.float32(d)))
        self.k, self.v = randn_bf16((batch * T, Hkv, d), g), randn_bf16((batch * T, Hkv, d), g)
        self.q = randn_bf16((batch * T, Hq, d), g)
        self.out = torch.empty_like(self.q)
        self.cache = sp.KVCache.empty(self.num_pages, Hkv, d)
        self.bt = _dev_i32(self.block_table)
        self.cu_host = np.arange(batch + 1, dtype=np.int32) * T
        self.cu, self.ctx = _dev_i32(self.cu_host), _dev_i32(np.zeros(batch))
        self.flops = batch * 4 * d * Hq * T * (T + 1) // 2
        self.append_bytes = W.append_bytes(batch * T, Hkv, d)

    def append(self):
        self.sp.sp_kv_append(self.cache, self.k, self.v, self.cu, self.ctx, self.bt)

    def attend(self):
        self.sp.sp_attn_prefill(self.cache, self.q, self.out, self.cu, self.ctx, self.bt, self.T, self.T, self.scale)


class PrefillJob:
    """A seeded prefill workload (numpy recipe) resident on the device."""

    def __init__(self, sp, w):
        import torch
        import workloads as W

        self.sp, self.w = sp, w
        st = next(w.steps())
        self.st = st
        self.cache = sp.KVCache.empty(w.num_pages, w.Hkv, w.d)
        self.bt = _dev_i32(w.block_table)
        self.k, self.v, self.q = _dev_bf16(st.k_new), _dev_bf16(st.v_new), _dev_bf16(st.q)
        self.out = torch.empty_like(self.q)
        self.cu, self.ctx = _dev_i32(st.cu_new), _dev_i32(st.ctx_lens)
        self.max_q, self.max_kv = int(st.new_lens.max()), int(st.seq_lens.max())
        self.flops = W.prefill_flops(st, w.Hq, w.d)

    def append(self):
        self.sp.sp_kv_append(self.cache, self.k, self.v, self.cu, self.ctx, self.bt)

    def attend(self):
        self.sp.sp_attn_prefill(self.cache, self.q, self.out, self.cu, self.ctx, self.bt, self.max_q,
                                self.max_kv, float(self.w.scale))


class DecodeJob:
    """TP-mode decode workload: `copies` independent KV pools, rotated so reads come from HBM."""

    def __init__(self, sp, w, copies):
        import torch
        import workloads as W

        self.sp, self.w = sp, w
        steps = list(w.steps())
        fill, dec = steps[0], steps[1]
        self.fill, self.dec = fill, dec
        self.bt = _dev_i32(w.block_table)
        self.caches = []
        k_fill, v_fill = _dev_bf16(fill.k_new), _dev_bf16(fill.v_new)
        cu_f, ctx_f = _dev_i32(fill.cu_new), _dev_i32(fill.ctx_lens)
        for _ in range(copies):
            c = sp.KVCache.empty(w.num_pages, w.Hkv, w.d)
            sp.sp_kv_append(c, k_fill, v_fill, cu_f, ctx_f, self.bt)
            self.caches.append(c)
        del k_fill, v_fill
        self.k, self.v, self.q = _dev_bf16(dec.k_new), _dev_bf16(dec.v_new), _dev_bf16(dec.q)
        self.out = torch.empty_like(self.q)
        self.cu, self.ctx = _dev_i32(dec.cu_new), _dev_i32(dec.ctx_lens)
        self.seq_lens = _dev_i32(dec.seq_lens)
        self.max_len = int(dec.seq_lens.max())
        need = sp.sp_attn_decode_workspace_size(w.batch, self.max_len, w.Hq, w.d)
        self.ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
        self.bytes = W.decode_bytes(dec.seq_lens, w.Hq, w.Hkv, w.d)
        self.i = 0

    def next_cache(self):
        self.i = (self.i + 1) % len(self.caches)
        return self.caches[self.i]

    def append(self, cache):
        self.sp.sp_kv_append(cache, self.k, self.v, self.cu, self.ctx, self.bt)

    def attend(self, cache):
        self.sp.sp_attn_decode(cache, self.q, self.out, self.seq_lens, self.bt, self.max_len,
                               float(self.w.scale), self.ws)

    def fused_step(self, cache):
        """Append + decode in one call (the append runs inside the attention kernel)."""
        self.sp.sp_decode_step(cache, self.k, self.v, self.q, self.out, self.seq_lens, self.bt, self.max_len,
                               float(self.w.scale), self.ws)


# ------------------------------------------------------------------ the oracle on the host cores
def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(long_job, c2_job, c3_job, with_c5a=True):
    """The fp64 oracle as it stands, timed on this machine's host cores on the FULL output of C2, C3
    and (unless switched off) C5a — the same inputs the GPU just ran, its outputs compared on the
    way.  A reported baseline, never a target."""
    import oracle
    import workloads as W

    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    per = {}

    # C2: 4 x 2048-token prefill
    w, st = c2_job.w, c2_job.st
    kp, vp = w.empty_cache()
    oracle.kv_append(kp, vp, st.k_new, st.v_new, st.cu_new, st.ctx_lens, w.block_table)
    t0 = time.perf_counter()
    want = oracle.attn_prefill(kp, vp, st.q, st.cu_new, st.ctx_lens, w.block_table, w.scale)
    t = time.perf_counter() - t0
    c2_job.append()
    c2_job.attend()
    err = float(np.abs(W.bf16_bits_to_f64(_bits(c2_job.out)) - want).max())
    per["C2"] = {"seconds": t, "TFLOPs": c2_job.flops / t / 1e12, "max_abs_err_gpu": err}

    # C3: 64-sequence decode
    w, fill, dec = c3_job.w, c3_job.fill, c3_job.dec
    kp, vp = w.empty_cache()
    oracle.kv_append(kp, vp, fill.k_new, fill.v_new, fill.cu_new, fill.ctx_lens, w.block_table)
    oracle.kv_append(kp, vp, dec.k_new, dec.v_new, dec.cu_new, dec.ctx_lens, w.block_table)
    t0 = time.perf_counter()
    want = oracle.attn_decode(kp, vp, dec.q, dec.seq_lens, w.block_table, w.scale)
    t = time.perf_counter() - t0
    c = c3_job.caches[0]
    c3_job.append(c)
    c3_job.attend(c)
    err = float(np.abs(W.bf16_bits_to_f64(_bits(c3_job.out)) - want).max())
    per["C3"] = {"seconds": t, "GBps": c3_job.bytes / t / 1e9, "max_abs_err_gpu": err}

    head = per["C2"]
    sample = "full outputs of C2 and C3"
    if with_c5a:
        j = long_job
        j.append()
        j.attend()
        got = W.bf16_bits_to_f64(_bits(j.out))
        kp = np.full((j.num_pages, j.Hkv, 16, j.d), W.CANARY, np.uint16)
        vp = kp.copy()
        ctx0 = np.zeros(j.batch, np.int32)
        oracle.kv_append(kp, vp, _bits(j.k), _bits(j.v), j.cu_host, ctx0, j.block_table)
        t0 = time.perf_counter()
        want = oracle.attn_prefill(kp, vp, _bits(j.q), j.cu_host, ctx0, j.block_table, j.scale)
        t = time.perf_counter() - t0
        per["C5a"] = {"seconds": t, "TFLOPs": j.flops / t / 1e12, "max_abs_err_gpu": float(np.abs(got - want).max())}
        head = per["C5a"]
        sample = "full outputs of C5a (headline), C2 and C3"
    return {"value": head["TFLOPs"], "unit": "TFLOP/s", "cores": cores, "kind": "oracle", "sample": "full",
            "what": sample + ", fp64, one run each", "cpu_model": _cpu_model(), "per_config": per}


# ------------------------------------------------------------------ side workloads
def extra_long_prefill(sp, iters=30):
    j = LongPrefillJob(sp)
    j.append()
    t = time_one(j.attend, iters, 2)
    return {"id": "c5a", "workload": "C5a 1x32768-token causal prefill, 8q/1kv, d=128", "ms": t,
            "TFLOPs": j.flops / t["mean"] / 1e9, "frac": j.flops / t["mean"] / 1e9 / PEAK_BF16_TFLOPS}


def fill_random_pools(cache, gen):
    import torch

    for pool in (cache.k_pages, cache.v_pages):       # fill in slabs to bound temporary memory
        flat = pool.view(-1)
        slab = 1 << 28
        for a in range(0, flat.numel(), slab):
            n = min(slab, flat.numel() - a)
            flat[a:a + n] = torch.randn(n, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)


def extra_big_decode(sp, iters=30):
    """Llama-3.1-8B shape decode batch: 128 sequences, 32q/8kv, contexts U{1024..16384} (~4.7 GB of
    KV, far beyond the last-level cache).  Values from torch's seeded GPU generator."""
    import torch
    import workloads as W

    w = W.c5c_decode_8b()
    lens = w.total_lens
    cache = sp.KVCache.empty(w.num_pages, 8, 128)
    g = torch.Generator(device="cuda").manual_seed(6)
    fill_random_pools(cache, g)
    q = randn_bf16((w.batch, 32, 128), g)
    out = torch.empty_like(q)
    bt, sl = _dev_i32(w.block_table), _dev_i32(lens)
    mx = int(lens.max())
    ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, 32, 128), dtype=torch.uint8, device="cuda")
    t = time_one(lambda: sp.sp_attn_decode(cache, q, out, sl, bt, mx, float(w.scale), ws), iters, 2)
    nbytes = W.decode_bytes(lens, 32, 8, 128)
    return {"id": "c5c", "workload": "C5c 128-sequence decode, 32q/8kv, d=128, contexts U{1024..16384}", "ms": t,
            "GBps": nbytes / t["mean"] / 1e6, "frac": nbytes / t["mean"] / 1e6 / PEAK_HBM_GBPS, "kv_bytes": nbytes}


def extra_other_shapes(sp, iters=30):
    """Other shard shapes of the SP x TP = P family and head_dim 64, sized like the headline
    workloads: (32q, 8kv) 4 x 8192-token prefill, (16q, 2kv) d=64 32768-token prefill, and a d=64
    decode batch on C3's contexts."""
    import torch
    import workloads as W

    res = []
    for name, kw in (("32q8kv_4x8192", dict(T=8192, Hq=32, Hkv=8, d=128, batch=4, seed=11)),
                     ("16q2kv_d64_1x32768", dict(T=32768, Hq=16, Hkv=2, d=64, batch=1, seed=12))):
        j = LongPrefillJob(sp, **kw)
        j.append()
        t = time_one(j.attend, iters, 2)
        res.append({"id": "prefill_" + name, "ms": t, "TFLOPs": j.flops / t["mean"] / 1e9,
                    "frac": j.flops / t["mean"] / 1e9 / PEAK_BF16_TFLOPS})
        del j
    w = W.c3_decode(Hq=16, Hkv=2, d=64, n=8, name="d64_decode")
    copies = 8
    lens = w.total_lens
    g = torch.Generator(device="cuda").manual_seed(13)
    caches = []
    for _ in range(copies):
        c = sp.KVCache.empty(w.num_pages, 2, 64)
        fill_random_pools(c, g)
        caches.append(c)
    q = randn_bf16((w.batch, 16, 64), g)
    out = torch.empty_like(q)
    bt, sl = _dev_i32(w.block_table), _dev_i32(lens)
    mx = int(lens.max())
    ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, 16, 64), dtype=torch.uint8, device="cuda")
    i = {"i": 0}

    def step():
        i["i"] = (i["i"] + 1) % copies
        sp.sp_attn_decode(caches[i["i"]], q, out, sl, bt, mx, float(w.scale), ws)

    t = time_one(step, iters, 3)
    nbytes = W.decode_bytes(lens, 16, 2, 64)
    res.append({"id": "decode_16q2kv_d64_cold", "ms": t, "GBps": nbytes / t["mean"] / 1e6,
                "frac": nbytes / t["mean"] / 1e6 / PEAK_HBM_GBPS, "kv_bytes": nbytes})
    return res


def extra_spec_verify(sp, iters=30):
    """Speculative-decoding verification on the C3 batch shape: 4 query tokens per sequence (causal
    inside the chunk) through sp_attn_prefill, which hands such batches to the decode kernels; the
    general prefill kernel on the same input beside it."""
    import torch
    import workloads as W

    w = W.spec_verify()
    cache = sp.KVCache.empty(w.num_pages, w.Hkv, w.d)
    bt = _dev_i32(w.block_table)
    for st in w.steps():
        cu, ctx = _dev_i32(st.cu_new), _dev_i32(st.ctx_lens)
        sp.sp_kv_append(cache, _dev_bf16(st.k_new), _dev_bf16(st.v_new), cu, ctx, bt)
    q = _dev_bf16(st.q)
    kn, vn = _dev_bf16(st.k_new), _dev_bf16(st.v_new)
    out = torch.empty_like(q)
    mq, mkv = int(st.new_lens.max()), int(st.seq_lens.max())
    ms = {}
    for name, mode in (("short_chunk_path", 0), ("prefill_kernel", 1)):
        sp.sp_debug_set_tuning("prefill_short_chunk", mode)
        try:
            need = sp.sp_attn_prefill_workspace_size(w.batch, q.shape[0], mq, mkv, w.Hq, w.Hkv, w.d)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
            fn = lambda: sp.sp_attn_prefill(cache, q, out, cu, ctx, bt, mq, mkv, float(w.scale), workspace=ws)
            ms[name] = time_one(fn, iters)["mean"]
            if mode == 0:   # the whole step: append + attention in two calls, and fused in one (idempotent: same rows, same slots)
                app = lambda: sp.sp_kv_append(cache, kn, vn, cu, ctx, bt)
                _, per = time_phases([app, fn], iters, 3)
                ms["append_plus_attention"] = float(per[0].mean() + per[1].mean())
                step = lambda: sp.sp_chunk_step(cache, kn, vn, q, out, cu, ctx, bt, mq, mkv, float(w.scale), workspace=ws)
                ms["chunk_step_fused"] = time_one(step, iters)["mean"]
        finally:
            sp.sp_debug_set_tuning("prefill_short_chunk", 0)
    nbytes = W.decode_bytes(st.seq_lens, w.Hq, w.Hkv, w.d)
    return {"id": "spec", "workload": "speculative verification, 64 sequences x 4 query tokens, 8q/1kv, d=128, contexts U{512..8192}",
            "ms": ms["short_chunk_path"], "GBps": nbytes / ms["short_chunk_path"] / 1e6,
            "frac": nbytes / ms["short_chunk_path"] / 1e6 / PEAK_HBM_GBPS, "kv_bytes": nbytes,
            "ms_general_prefill_kernel": ms["prefill_kernel"],
            "ms_step_append_plus_attention": ms["append_plus_attention"], "ms_step_fused_sp_chunk_step": ms["chunk_step_fused"]}


def extra_chunked_prefill(sp, iters=30):
    """C4: 32 sequences with lognormal lengths, second half of each prefilled in chunks of <= 512
    tokens against the cached prefix; every step = append + prefill, both timed."""
    import torch
    import workloads as W

    w = W.c4_chunked()
    cache = sp.KVCache.empty(w.num_pages, w.Hkv, w.d)
    bt = _dev_i32(w.block_table)
    steps, flops, t_att, t_app = 0, 0, 0.0, 0.0
    per_step = []
    for st in w.steps():
        k, v = _dev_bf16(st.k_new), _dev_bf16(st.v_new)
        cu, ctx = _dev_i32(st.cu_new), _dev_i32(st.ctx_lens)
        if st.kind == "fill":
            sp.sp_kv_append(cache, k, v, cu, ctx, bt)
            continue
        q = _dev_bf16(st.q)
        out = torch.empty_like(q)
        mq, mkv = int(st.new_lens.max()), int(st.seq_lens.max())
        need = sp.sp_attn_prefill_workspace_size(w.batch, q.shape[0], mq, mkv, w.Hq, w.Hkv, w.d)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        app = lambda: sp.sp_kv_append(cache, k, v, cu, ctx, bt)      # idempotent: same rows, same slots
        att = lambda: sp.sp_attn_prefill(cache, q, out, cu, ctx, bt, mq, mkv, float(w.scale), workspace=ws)
        _, per = time_phases([app, att], iters, 2)
        f = W.prefill_flops(st, w.Hq, w.d)
        a_ms = float(per[1].mean())
        per_step.append({"tokens": int(st.new_lens.sum()), "ms": a_ms, "TFLOPs": f / a_ms / 1e9})
        steps += 1
        flops += f
        t_app += float(per[0].mean())
        t_att += a_ms
    return {"id": "c4", "workload": f"C4 mixed chunked prefill, 32 sequences, {steps} steps of <=512-token chunks on cached "
                                    "prefixes, 8q/1kv, d=128", "ms": t_att, "ms_kv_append": t_app, "TFLOPs": flops / t_att / 1e9,
            "frac": flops / t_att / 1e9 / PEAK_BF16_TFLOPS, "per_step": per_step}


def extra_mixed_batch(sp, iters=30):
    """A continuous-batching step: 63 single-token sequences on C3-like contexts plus one
    2048-token prefill chunk, attended in ONE sp_attn_prefill call and, for comparison, in two
    calls on the two sub-ranges."""
    import torch
    import workloads as W

    rng = np.random.default_rng(20250711)
    ctx = np.concatenate([rng.integers(512, 8193, size=63), [0]]).astype(np.int32)
    new = np.concatenate([np.ones(63, np.int32), [2048]]).astype(np.int32)
    total = ctx + new
    block_table, num_pages = W.make_block_table(rng, total)
    g = torch.Generator(device="cuda").manual_seed(14)
    cache = sp.KVCache.empty(num_pages, 1, 128)
    fill_random_pools(cache, g)
    T = int(new.sum())
    q = randn_bf16((T, 8, 128), g)
    out = torch.empty_like(q)
    cu_h = np.zeros(65, np.int32)
    cu_h[1:] = np.cumsum(new)
    cu, cx, bt = _dev_i32(cu_h), _dev_i32(ctx), _dev_i32(block_table)
    scale = float(np.float32(1.0) / np.sqrt(np.float32(128)))
    mq, mkv = int(new.max()), int(total.max())
    need = sp.sp_attn_prefill_workspace_size(64, T, mq, mkv, 8, 1, 128)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    one = time_one(lambda: sp.sp_attn_prefill(cache, q, out, cu, cx, bt, mq, mkv, scale, workspace=ws), iters)
    need_a = sp.sp_attn_prefill_workspace_size(63, T, 1, int(total[:63].max()), 8, 1, 128)
    ws_a = torch.empty(need_a, dtype=torch.uint8, device="cuda") if need_a else None

    need_b = sp.sp_attn_prefill_workspace_size(1, T, 2048, 2048, 8, 1, 128)
    ws_b = torch.empty(need_b, dtype=torch.uint8, device="cuda") if need_b else None

    def two():
        sp.sp_attn_prefill(cache, q, out, cu[:64], cx[:63], bt[:63], 1, int(total[:63].max()), scale, workspace=ws_a)
        sp.sp_attn_prefill(cache, q, out, cu[63:], cx[63:], bt[63:], 2048, 2048, scale, workspace=ws_b)

    two_t = time_one(two, iters)
    flops = 4 * 128 * 8 * int((new.astype(np.int64) * ctx + new.astype(np.int64) * (new + 1) // 2).sum())
    return {"id": "mixed", "workload": "63 single-token sequences (contexts U{512..8192}) + one 2048-token chunk, 8q/1kv, d=128",
            "ms_one_call": one, "ms_two_calls": two_t, "flops": flops}


def extra_shift_decode(sp, steps=64):
    """C5b: right after a 32768-token prefill, decode steps on the SAME cache and block table
    (append one token, then attend over 32769+t keys).  The 16.8 MB of K/V stay in the
    last-level cache, so this is a launch- and latency-bound figure, not an HBM one."""
    import torch
    import workloads as W

    w = W.c5_long(decode_steps=0)
    g = torch.Generator(device="cuda").manual_seed(7)
    T = 32768
    cache = sp.KVCache.empty(w.num_pages, 1, 128)
    bt = _dev_i32(w.block_table)
    k, v = randn_bf16((T + steps, 1, 128), g), randn_bf16((T + steps, 1, 128), g)
    q = randn_bf16((steps, 8, 128), g)
    out = torch.empty((1, 8, 128), device="cuda", dtype=torch.bfloat16)
    sp.sp_kv_append(cache, k[:T], v[:T], _dev_i32([0, T]), _dev_i32([0]), bt)
    ws = torch.empty(sp.sp_attn_decode_workspace_size(1, T + steps, 8, 128), dtype=torch.uint8, device="cuda")
    cu1 = _dev_i32([0, 1])
    ctxs = [_dev_i32([T + t]) for t in range(steps)]
    lens = [_dev_i32([T + t + 1]) for t in range(steps)]
    state = {"t": 0}

    def app():
        t = state["t"]
        sp.sp_kv_append(cache, k[T + t:T + t + 1], v[T + t:T + t + 1], cu1, ctxs[t], bt)

    def att():
        t = state["t"]
        sp.sp_attn_decode(cache, q[t:t + 1], out, lens[t], bt, T + steps, float(w.scale), ws)
        state["t"] = (t + 1) % steps

    _, per = time_phases([app, att], steps, 4)

    def fused():
        t = state["t"]
        sp.sp_decode_step(cache, k[T + t:T + t + 1], v[T + t:T + t + 1], q[t:t + 1], out, lens[t], bt, T + steps,
                          float(w.scale), ws)
        state["t"] = (t + 1) % steps

    state["t"] = 0
    _, per_f = time_phases([fused], steps, 4)
    nbytes = W.decode_bytes(np.array([T + steps // 2]), 8, 1, 128)
    return {"id": "c5b", "workload": f"C5b decode steps on the cache the 32768-token prefill filled (same block table, no "
                                     f"re-layout), {steps} steps", "us_per_step_attn": _stats(per[1] * 1e3),
            "us_per_step_kv_append": _stats(per[0] * 1e3), "us_per_step_fused": _stats(per_f[0] * 1e3),
            "GBps_cache_resident": nbytes / float(per[1].mean()) / 1e6}


def extra_head_exchange(sp, iters=30):
    """Local halves of the SP-mode head exchange at the 70B shape: one rank's 1024 of 8192 prefill
    tokens, q with all 64 heads -> 8 blocks of 8 heads (pack) and back (unpack)."""
    import torch

    T, H, d, P = 1024, 64, 128, 8
    x = torch.randn((T, H, d), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    send = torch.empty((P, T, H // P, d), device="cuda", dtype=torch.bfloat16)
    y = torch.empty_like(x)
    _, per = time_phases([lambda: sp.sp_ulysses_pack(x, send, P), lambda: sp.sp_ulysses_unpack(send, y)], iters, 3)
    nbytes = 2 * x.numel() * 2
    return {"id": "head_exchange", "workload": "SP-mode head exchange, local pack / unpack of [1024][64][128] bf16 over 8 ranks",
            "us_pack": float(per[0].mean()) * 1e3, "us_unpack": float(per[1].mean()) * 1e3,
            "GBps_pack_read_plus_write": nbytes / float(per[0].mean()) / 1e6,
            "GBps_unpack_read_plus_write": nbytes / float(per[1].mean()) / 1e6}


def ceilings(c3_bytes):
    """What this machine delivers for the two bounding resources (reference kernels of the separate
    libspceilings.so): a register-resident bf16 MFMA loop, and a 16 B/lane streaming read — over
    2 GiB, and over buffers the size of C3's KV working set rotated like its pool copies (cold);
    the best of several launch shapes each."""
    import torch
    from paper_2507_11830_amd import ceilings as C

    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    iters = 20000
    out = {}
    for name, rnd in (("mfma_loop", False), ("mfma_loop_random_operands", True)):
        fl = {}

        def mf():
            fl["f"] = C.ceiling_mfma(iters, sink, random_operands=rnd)

        t = time_one(mf, 5, 2)
        clk = sink[:16].view(torch.int64).cpu().numpy()
        out[name + "_TFLOPs"] = fl["f"] / t["mean"] / 1e9
        out[name + "_shader_clock_MHz"] = float(clk[0]) / (float(clk[1]) / 100e6) / 1e6 if clk[1] > 0 else None
    buf = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    shapes = [(b, u) for b in (4, 8, 16, 32) for u in (4, 8)]
    best = 0.0
    for b, u in shapes:
        t = time_one(lambda: C.ceiling_stream(buf, sink, b, u), 5, 2)
        best = max(best, float(buf.numel()) / t["min"] / 1e6)
    out["stream_read_2GiB_GBps"] = best
    n = (c3_bytes + 255) // 256 * 256
    copies = max(8, (1 << 30) // n + 1)
    parts = [buf[i * n:(i + 1) * n] for i in range(min(copies, buf.numel() // n))]
    best_med, best_min = 0.0, 0.0
    for b, u in shapes:
        i = {"i": 0}

        def rd():
            i["i"] = (i["i"] + 1) % len(parts)
            C.ceiling_stream(parts[i["i"]], sink, b, u)

        t = time_one(rd, 30, 3)
        best_med, best_min = max(best_med, n / t["median"] / 1e6), max(best_min, n / t["min"] / 1e6)
    out["stream_read_c3_sized_cold_GBps"] = {"median": best_med, "best": best_min, "bytes": int(n), "buffers": len(parts)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the ceiling kernels and the side workloads")
    ap.add_argument("--workload", default="main",
                    choices=["main", "c2", "c5a", "c5b", "c5c", "spec", "c4", "mixed", "shapes", "copy"],
                    help="main = the step described above; the others = only that side workload (used for "
                         "per-kernel profiles); copy = a plain 1 GiB device copy, the known-size kernel the HBM "
                         "byte counters are calibrated against")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-oracle-c5a", action="store_true",
                    help="time the oracle on C2 and C3 only (its full C5a run takes about a minute of host time)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="sp_debug_set_tuning override for this run (profiling of non-default launch shapes)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs one GPU's head shard only (no collectives, no sharding); "
                 "use --gpus 1")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    import paper_2507_11830_amd as sp
    import workloads as W

    sp.lib()   # fail loudly if the HIP library is missing
    for kv in args.tune:
        key, _, value = kv.partition("=")
        sp.sp_debug_set_tuning(key, int(value))
    if args.workload == "copy":
        n = 1 << 30
        src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        t = time_one(lambda: dst.copy_(src), args.steps, 2)
        print(json.dumps({"workload": "plain device copy", "bytes_read": n, "bytes_written": n, "ms": t,
                          "GBps_read_plus_write": 2 * n / t["mean"] / 1e6}))
        return
    if args.workload != "main":
        if args.workload == "c2":
            j = PrefillJob(sp, W.c2_prefill())
            j.append()
            t = time_one(j.attend, args.steps)
            print(json.dumps({"id": "c2", "ms": t, "TFLOPs": j.flops / t["mean"] / 1e9}))
            return
        fn = {"c5a": extra_long_prefill, "c5c": extra_big_decode, "spec": extra_spec_verify, "c5b": extra_shift_decode,
              "c4": extra_chunked_prefill, "mixed": extra_mixed_batch, "shapes": extra_other_shapes}[args.workload]
        print(json.dumps(fn(sp, args.steps)))
        return

    long_job = LongPrefillJob(sp)
    wd = W.c3_decode()
    copies = 8
    dec = DecodeJob(sp, wd, copies)
    state = {}

    def ph_append_p():
        long_job.append()

    def ph_prefill():
        long_job.attend()

    def ph_append_d():
        state["c"] = dec.next_cache()
        dec.append(state["c"])

    def ph_decode():
        dec.attend(state["c"])

    wall, per = time_phases([ph_append_p, ph_prefill, ph_append_d, ph_decode], args.steps, args.warmup)
    t_app_p, t_pre, t_app_d, t_dec = (_stats(p) for p in per)
    tflops = long_job.flops / t_pre["mean"] / 1e9
    gbps = dec.bytes / t_dec["mean"] / 1e6
    # the same decode step on ONE pool copy: its 140 MB stay in the 256 MB last-level cache
    warm = time_one(lambda: dec.attend(dec.caches[0]), args.steps, args.warmup)
    res = {
        "metric": "prefill attn TFLOP/s (value) + decode KV GB/s (roofline_decode) at 70B head shard",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C5a 1x32768-token causal prefill + C3 64-seq decode (cold KV), 8q/1kv heads, d=128",
                   "prefill_tokens": long_job.T, "decode_batch": wd.batch,
                   "decode_kv_tokens": int(dec.dec.seq_lens.sum()), "decode_pool_copies": copies},
        "prefill_frac": tflops / PEAK_BF16_TFLOPS,
        "decode_frac": gbps / PEAK_HBM_GBPS,
        "phases_ms": {"kv_append_prefill": t_app_p, "attn_prefill": t_pre, "kv_append_decode": t_app_d,
                      "attn_decode": t_dec},
        "kv_append_GBps": long_job.append_bytes / t_app_p["mean"] / 1e6,
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_PREFILL_C5A, "kernel": "prefill_kernel",
                     "workload": "C5a", "algorithmic_flops": long_job.flops,
                     "median": long_job.flops / t_pre["median"] / 1e9, "best": long_job.flops / t_pre["min"] / 1e9},
        "roofline_decode": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": gbps / PEAK_HBM_GBPS, "traffic": TRAFFIC_DECODE_C3,
                            "kernel": "decode_split_kernel + combine_kernel", "workload": "C3 cold",
                            "algorithmic_bytes": dec.bytes,
                            "median": dec.bytes / t_dec["median"] / 1e6, "best": dec.bytes / t_dec["min"] / 1e6},
        "decode_warm": {"ms": warm, "GBps": dec.bytes / warm["mean"] / 1e6,
                        "note": "C3 on a single pool copy: served by the last-level cache, not HBM"},
    }
    # the same decode with the combine pass folded into the split kernel (last-arriving wave merges;
    # off by default: the device-scope release every wave then needs costs far more than a launch)
    sp.sp_debug_set_tuning("decode_fuse", 2)
    fus = time_one(lambda: dec.attend(dec.next_cache()), args.steps, args.warmup)
    sp.sp_debug_set_tuning("decode_fuse", 0)
    res["decode_combine_in_split_kernel"] = {"ms": fus, "GBps": dec.bytes / fus["mean"] / 1e6}
    fz = time_one(lambda: dec.fused_step(dec.next_cache()), args.steps, args.warmup)
    # the same step captured once per KV-pool copy in a HIP graph and replayed (the library only
    # enqueues, so it is capture-safe; a graph takes the host out of the launch path)
    graphs = []
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for c in dec.caches:
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=side):
                dec.fused_step(c)
            graphs.append(gph)
    torch.cuda.current_stream().wait_stream(side)
    gi = {"i": 0}

    def replay():
        gi["i"] = (gi["i"] + 1) % len(graphs)
        graphs[gi["i"]].replay()

    gr = time_one(replay, args.steps, args.warmup)
    # ... and one graph that holds a step on every pool copy in turn (what a serving loop captures
    # is many launches per graph; the graph's own launch cost is then shared)
    with torch.cuda.stream(side):
        big = torch.cuda.CUDAGraph()
        with torch.cuda.graph(big, stream=side):
            for c in dec.caches:
                dec.fused_step(c)
    torch.cuda.current_stream().wait_stream(side)
    bg = time_one(big.replay, max(args.steps // len(dec.caches), 4), 1)
    per_b_step = bg["mean"] / len(dec.caches)
    res["decode_step_fused"] = {"ms": fz, "GBps": dec.bytes / fz["mean"] / 1e6,
                                "hip_graph_replay_ms": gr["mean"],
                                "hip_graph_of_%d_steps_ms_per_step" % len(dec.caches): per_b_step,
                                "hip_graph_of_%d_steps_GBps" % len(dec.caches): dec.bytes / per_b_step / 1e6,
                                "separate_append_plus_decode_ms": t_app_d["mean"] + t_dec["mean"]}
    c2_job = PrefillJob(sp, W.c2_prefill())
    if not args.no_extras:
        c2_job.append()
        t2 = time_one(c2_job.attend, args.steps, args.warmup)
        side_wl = [{"id": "c2", "workload": "C2 4x2048-token causal prefill, 8q/1kv, d=128", "ms": t2,
                    "TFLOPs": c2_job.flops / t2["mean"] / 1e9, "frac": c2_job.flops / t2["mean"] / 1e9 / PEAK_BF16_TFLOPS}]
        ceil = ceilings(dec.bytes)
        res["ceilings"] = ceil
        res["roofline"]["frac_of_mfma_loop"] = tflops / ceil["mfma_loop_TFLOPs"]
        res["roofline"]["frac_of_mfma_loop_rand"] = tflops / ceil["mfma_loop_random_operands_TFLOPs"]
        res["roofline_decode"]["frac_of_stream_c3_sized"] = gbps / ceil["stream_read_c3_sized_cold_GBps"]["median"]
        side_wl += [extra_big_decode(sp), extra_chunked_prefill(sp), extra_shift_decode(sp), extra_spec_verify(sp),
                    extra_mixed_batch(sp), *extra_other_shapes(sp), extra_head_exchange(sp)]
        res["side"] = side_wl
        res["c2_frac"] = side_wl[0]["frac"]
        res["c5c_frac"] = side_wl[1]["frac"]
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(long_job, c2_job, dec, with_c5a=not args.no_oracle_c5a)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
