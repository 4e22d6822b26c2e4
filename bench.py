#!/usr/bin/env python3
"""Benchmark of the Shift Parallelism attention hot path on one MI355X.

A "step" is one pass of the whole hot path at the Llama-3.3-70B head-shard shape (8 query
heads / 1 KV head, head_dim 128), inputs resident in HBM:

    sp_kv_append (8192 tokens)  ->  sp_attn_prefill   [SP-mode prefill, 4 x 2048 tokens, causal]
    sp_kv_append (64 tokens)    ->  sp_attn_decode    [TP-mode decode, 64 sequences with
                                                       contexts U{512..8192}; split + combine]

Every phase is bracketed by HIP events on the launch stream inside the timed region, so the
prefill TFLOP/s and the decode GB/s are per-phase figures; ``ms_per_step`` is the wall time
of the whole step.  The decode phase rotates over several copies of its KV pool so that its
working set (about 140 MB, smaller than the 256 MB last-level cache) is read cold from HBM.

Prints ONE JSON line.  ``value`` is the prefill attention TFLOP/s (algorithmic flops of the
step's prefill / mean prefill-phase duration); the decode GB/s rides along in ``decode``.
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
TRAFFIC_PREFILL_C2 = int(17416.8 * 1024 * 2.0 + 16384.3 * 1024)
TRAFFIC_DECODE_C3 = int((68030.6 + 3666.5) * 1024 * 2.0 + (3892.0 + 128.0) * 1024)


def _dev_bf16(u16):
    import torch

    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def _dev_i32(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


class PrefillJob:
    """SP-mode prefill workload resident on the device."""

    def __init__(self, sp, w):
        import torch

        self.sp, self.w = sp, w
        st = next(w.steps())
        self.st = st
        self.cache = sp.KVCache.empty(w.num_pages, w.Hkv, w.d)
        self.bt = _dev_i32(w.block_table)
        self.k, self.v, self.q = _dev_bf16(st.k_new), _dev_bf16(st.v_new), _dev_bf16(st.q)
        self.out = torch.empty_like(self.q)
        self.cu, self.ctx = _dev_i32(st.cu_new), _dev_i32(st.ctx_lens)
        self.max_q, self.max_kv = int(st.new_lens.max()), int(st.seq_lens.max())
        import workloads as W

        self.flops = W.prefill_flops(st, w.Hq, w.d)
        self.append_bytes = W.append_bytes(int(st.new_lens.sum()), w.Hkv, w.d)

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
        self.dec = dec
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


def time_phases(fns, steps, warmup):
    """Runs the phase functions in order `steps` times; returns (wall ms/step, [mean ms per phase])."""
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
    per = [float(np.mean([ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)])) for i in range(len(fns))]
    return wall, per


def cpu_baseline(w, st, budget_s=1.5):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a bounded sample of the
    prefill rows (rows drawn uniformly; work = 4*d flops per visible (query, key) pair)."""
    import oracle
    import workloads as W

    kp, vp = w.empty_cache()
    oracle.kv_append(kp, vp, st.k_new, st.v_new, st.cu_new, st.ctx_lens, w.block_table)
    rng = np.random.default_rng(0)
    lens = st.new_lens

    def draw(n):
        rs = rng.integers(0, len(lens), size=n).astype(np.int32)
        rt = np.array([rng.integers(0, lens[s]) for s in rs], dtype=np.int32)
        rh = rng.integers(0, w.Hq, size=n).astype(np.int32)
        flops = int(sum(4 * w.d * (int(st.ctx_lens[s]) + int(t) + 1) for s, t in zip(rs, rt)))
        return rs, rt, rh, flops

    def run(n):
        rs, rt, rh, flops = draw(n)
        t0 = time.perf_counter()
        oracle.attn_prefill_rows(kp, vp, st.q, st.cu_new, st.ctx_lens, w.block_table, w.scale, rs, rt, rh)
        return flops, time.perf_counter() - t0

    f, t = run(2048)                       # pilot
    n = int(max(2048, 2048 * budget_s / max(t, 1e-3)))   # about budget_s of wall time on all cores
    f, t = run(n)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": f / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} (sequence, token, head) rows drawn uniformly with replacement from the same 4x2048 "
                      f"prefill, fp64, {t:.1f} s wall on {cores} threads"}


def extra_long_prefill(sp, iters=5):
    """32768-token single-sequence prefill (values from torch's seeded GPU generator)."""
    import torch
    import workloads as W

    w = W.c5_long(decode_steps=0)
    g = torch.Generator(device="cuda").manual_seed(5)
    T = 32768
    k = torch.randn((T, 1, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((T, 1, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((T, 8, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    cache = sp.KVCache.empty(w.num_pages, 1, 128)
    bt, cu, ctx = _dev_i32(w.block_table), _dev_i32([0, T]), _dev_i32([0])
    sp.sp_kv_append(cache, k, v, cu, ctx, bt)
    fn = lambda: sp.sp_attn_prefill(cache, q, out, cu, ctx, bt, T, T, float(w.scale))
    _, per = time_phases([fn], iters, 1)
    flops = 4 * 128 * 8 * T * (T + 1) // 2
    return {"workload": "C5a 1x32768-token causal prefill, 8q/1kv, d=128", "ms": per[0],
            "TFLOPs": flops / per[0] / 1e9, "frac_of_bf16_peak": flops / per[0] / 1e9 / PEAK_BF16_TFLOPS}


def extra_big_decode(sp, iters=10):
    """Llama-3.1-8B shape decode batch: 128 sequences, 32q/8kv, contexts U{1024..16384} (~4.7 GB of
    KV, far beyond the last-level cache).  Values from torch's seeded GPU generator."""
    import torch
    import workloads as W

    w = W.c5c_decode_8b()
    lens = w.total_lens
    cache = sp.KVCache.empty(w.num_pages, 8, 128)
    g = torch.Generator(device="cuda").manual_seed(6)
    for pool in (cache.k_pages, cache.v_pages):       # fill in slabs to bound temporary memory
        flat = pool.view(-1)
        slab = 1 << 28
        for a in range(0, flat.numel(), slab):
            n = min(slab, flat.numel() - a)
            flat[a:a + n] = torch.randn(n, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((w.batch, 32, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    bt, sl = _dev_i32(w.block_table), _dev_i32(lens)
    mx = int(lens.max())
    ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, 32, 128), dtype=torch.uint8, device="cuda")
    fn = lambda: sp.sp_attn_decode(cache, q, out, sl, bt, mx, float(w.scale), ws)
    _, per = time_phases([fn], iters, 2)
    nbytes = W.decode_bytes(lens, 32, 8, 128)
    return {"workload": "C5c 128-sequence decode, 32q/8kv, d=128, contexts U{1024..16384}", "ms": per[0],
            "GBps": nbytes / per[0] / 1e6, "frac_of_hbm_peak": nbytes / per[0] / 1e6 / PEAK_HBM_GBPS,
            "kv_bytes": nbytes}


def extra_spec_verify(sp, iters=20):
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
            _, per = time_phases([fn], iters, 3)
            ms[name] = per[0]
            if mode == 0:   # the whole step: append + attention in two calls, and fused in one (idempotent: same rows, same slots)
                app = lambda: sp.sp_kv_append(cache, kn, vn, cu, ctx, bt)
                _, per = time_phases([app, fn], iters, 3)
                ms["append_plus_attention"] = per[0] + per[1]
                step = lambda: sp.sp_chunk_step(cache, kn, vn, q, out, cu, ctx, bt, mq, mkv, float(w.scale), workspace=ws)
                _, per = time_phases([step], iters, 3)
                ms["chunk_step_fused"] = per[0]
        finally:
            sp.sp_debug_set_tuning("prefill_short_chunk", 0)
    nbytes = W.decode_bytes(st.seq_lens, w.Hq, w.Hkv, w.d)
    return {"workload": "speculative verification, 64 sequences x 4 query tokens, 8q/1kv, d=128, contexts U{512..8192}",
            "ms": ms["short_chunk_path"], "GBps": nbytes / ms["short_chunk_path"] / 1e6,
            "frac_of_hbm_peak": nbytes / ms["short_chunk_path"] / 1e6 / PEAK_HBM_GBPS, "kv_bytes": nbytes,
            "ms_general_prefill_kernel": ms["prefill_kernel"],
            "ms_step_append_plus_attention": ms["append_plus_attention"], "ms_step_fused_sp_chunk_step": ms["chunk_step_fused"]}


def extra_chunked_prefill(sp):
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
        _, per = time_phases([app, att], 5, 1)
        f = W.prefill_flops(st, w.Hq, w.d)
        per_step.append({"tokens": int(st.new_lens.sum()), "ms": per[1], "TFLOPs": f / per[1] / 1e9})
        steps += 1
        flops += f
        t_app += per[0]
        t_att += per[1]
    return {"workload": f"C4 mixed chunked prefill, 32 sequences, {steps} steps of <=512-token chunks on cached "
                        "prefixes, 8q/1kv, d=128", "ms": t_att, "ms_kv_append": t_app, "TFLOPs": flops / t_att / 1e9,
            "frac_of_bf16_peak": flops / t_att / 1e9 / PEAK_BF16_TFLOPS, "per_step": per_step}


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
    k = torch.randn((T + steps, 1, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((T + steps, 1, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((steps, 8, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
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
    return {"workload": f"C5b decode steps on the cache the 32768-token prefill filled (same block table, no re-layout), "
                        f"{steps} steps", "us_per_step_attn": per[1] * 1e3, "us_per_step_kv_append": per[0] * 1e3,
            "us_per_step_fused": per_f[0] * 1e3,
            "GBps_cache_resident": nbytes / per[1] / 1e6}


def extra_head_exchange(sp):
    """Local halves of the SP-mode head exchange at the 70B shape: one rank's 1024 of 8192 prefill
    tokens, q with all 64 heads -> 8 blocks of 8 heads (pack) and back (unpack)."""
    import torch

    T, H, d, P = 1024, 64, 128, 8
    x = torch.randn((T, H, d), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    send = torch.empty((P, T, H // P, d), device="cuda", dtype=torch.bfloat16)
    y = torch.empty_like(x)
    _, per = time_phases([lambda: sp.sp_ulysses_pack(x, send, P), lambda: sp.sp_ulysses_unpack(send, y)], 20, 3)
    nbytes = 2 * x.numel() * 2
    return {"workload": "SP-mode head exchange, local pack / unpack of [1024][64][128] bf16 over 8 ranks",
            "us_pack": per[0] * 1e3, "us_unpack": per[1] * 1e3, "GBps_pack_read_plus_write": nbytes / per[0] / 1e6,
            "GBps_unpack_read_plus_write": nbytes / per[1] / 1e6}


def ceilings(sp):
    """What this machine delivers for the two bounding resources: a register-resident bf16 MFMA loop
    and a 16 B/lane streaming read of 2 GiB (both kernels live in the library)."""
    import torch

    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    iters = 20000
    out = {}
    for name, rnd in (("mfma_loop", False), ("mfma_loop_random_operands", True)):
        fl = {}

        def mf():
            fl["f"] = sp.sp_debug_ceiling_mfma(iters, sink, random_operands=rnd)

        _, per = time_phases([mf], 5, 2)
        clk = sink[:16].view(torch.int64).cpu().numpy()
        out[name + "_TFLOPs"] = fl["f"] / per[0] / 1e9
        out[name + "_shader_clock_MHz"] = float(clk[0]) / (float(clk[1]) / 100e6) / 1e6 if clk[1] > 0 else None
    buf = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    _, per2 = time_phases([lambda: sp.sp_debug_ceiling_stream(buf, sink)], 5, 2)
    out["stream_read_GBps"] = float(buf.numel()) / per2[0] / 1e6
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the ceiling kernels and the C5a / C5c / C4 / C5b side measurements")
    ap.add_argument("--workload", default="main", choices=["main", "c5a", "c5b", "c5c", "spec", "copy"],
                    help="main = the step described above; c5a / c5b / c5c / spec = only that side workload "
                         "(used for per-kernel profiles); copy = a plain 1 GiB device copy, the "
                         "known-size kernel the HBM byte counters are calibrated against")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
        _, per = time_phases([lambda: dst.copy_(src)], args.steps, 2)
        print(json.dumps({"workload": "plain device copy", "bytes_read": n, "bytes_written": n, "ms": per[0],
                          "GBps_read_plus_write": 2 * n / per[0] / 1e6}))
        return
    if args.workload != "main":
        if args.workload == "c5b":
            print(json.dumps(extra_shift_decode(sp, steps=args.steps)))
            return
        fn = {"c5a": extra_long_prefill, "c5c": extra_big_decode, "spec": extra_spec_verify}[args.workload]
        print(json.dumps(fn(sp, iters=args.steps)))
        return
    wp, wd = W.c2_prefill(), W.c3_decode()
    pre = PrefillJob(sp, wp)
    copies = 8
    dec = DecodeJob(sp, wd, copies)
    state = {}

    def ph_append_p():
        pre.append()

    def ph_prefill():
        pre.attend()

    def ph_append_d():
        state["c"] = dec.next_cache()
        dec.append(state["c"])

    def ph_decode():
        dec.attend(state["c"])

    wall, per = time_phases([ph_append_p, ph_prefill, ph_append_d, ph_decode], args.steps, args.warmup)
    t_app_p, t_pre, t_app_d, t_dec = per
    tflops = pre.flops / t_pre / 1e9
    gbps = dec.bytes / t_dec / 1e6
    res = {
        "metric": "prefill attn TFLOP/s (value) + decode KV GB/s (decode.value) at 70B head shard",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2 (4x2048-token causal prefill) + C3 (64-sequence decode, contexts U{512..8192}, "
                               "cold KV) at 8 q heads / 1 kv head, head_dim 128, 16-token pages",
                   "prefill_tokens": int(pre.st.new_lens.sum()), "decode_batch": wd.batch,
                   "decode_kv_tokens": int(dec.dec.seq_lens.sum()), "decode_pool_copies": copies},
        "phases_ms": {"kv_append_prefill": t_app_p, "attn_prefill": t_pre, "kv_append_decode": t_app_d,
                      "attn_decode_split_plus_combine": t_dec},
        "decode": {"value": gbps, "unit": "GB/s", "frac_of_hbm_peak": gbps / PEAK_HBM_GBPS,
                   "algorithmic_bytes": dec.bytes},
        "kv_append_GBps": pre.append_bytes / t_app_p / 1e6,
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_PREFILL_C2, "kernel": "prefill_kernel",
                     "algorithmic_flops": pre.flops},
        "roofline_decode": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": gbps / PEAK_HBM_GBPS, "traffic": TRAFFIC_DECODE_C3,
                            "kernel": "decode_split_kernel + combine_kernel"},
    }
    _, per_f = time_phases([lambda: dec.fused_step(dec.next_cache())], args.steps, args.warmup)
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

    _, per_g = time_phases([replay], args.steps, args.warmup)
    # ... and one graph that holds a step on every pool copy in turn (what a serving loop captures
    # is many launches per graph; the graph's own launch cost is then shared)
    with torch.cuda.stream(side):
        big = torch.cuda.CUDAGraph()
        with torch.cuda.graph(big, stream=side):
            for c in dec.caches:
                dec.fused_step(c)
    torch.cuda.current_stream().wait_stream(side)
    _, per_b = time_phases([big.replay], max(args.steps // len(dec.caches), 2), 1)
    per_b_step = per_b[0] / len(dec.caches)
    res["decode_step_fused"] = {"ms": per_f[0], "GBps": dec.bytes / per_f[0] / 1e6,
                                "hip_graph_replay_ms": per_g[0], "hip_graph_replay_GBps": dec.bytes / per_g[0] / 1e6,
                                "hip_graph_of_%d_steps_ms_per_step" % len(dec.caches): per_b_step,
                                "hip_graph_of_%d_steps_GBps" % len(dec.caches): dec.bytes / per_b_step / 1e6,
                                "separate_append_plus_decode_ms": t_app_d + t_dec,
                                "note": "sp_decode_step: same work as kv_append_decode + attn_decode in two launches "
                                        "instead of three"}
    if not args.no_extras:
        ceil = ceilings(sp)
        res["ceilings"] = ceil
        res["roofline"]["frac_of_measured_mfma_loop"] = tflops / ceil["mfma_loop_TFLOPs"]
        res["roofline"]["frac_of_measured_mfma_loop_random_operands"] = tflops / ceil["mfma_loop_random_operands_TFLOPs"]
        res["roofline_decode"]["frac_of_measured_stream_read"] = gbps / ceil["stream_read_GBps"]
        res["other_workloads"] = [extra_long_prefill(sp), extra_big_decode(sp), extra_chunked_prefill(sp),
                                  extra_shift_decode(sp), extra_spec_verify(sp), extra_head_exchange(sp)]
        for o in res["other_workloads"]:
            if "TFLOPs" in o:
                o["frac_of_measured_mfma_loop"] = o["TFLOPs"] / ceil["mfma_loop_TFLOPs"]
                o["frac_of_measured_mfma_loop_random_operands"] = o["TFLOPs"] / ceil["mfma_loop_random_operands_TFLOPs"]
            if "GBps" in o:
                o["frac_of_measured_stream_read"] = o["GBps"] / ceil["stream_read_GBps"]
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wp, pre.st)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
