"""Test plumbing: run the same seeded Workload steps through the HIP library (via the Python
binding of the C ABI) and through the fp64 oracle, and compare.  No arithmetic of the method
lives here."""
from __future__ import annotations

import numpy as np

import workloads as W

TOL = 1e-2   # max abs error GPU(bf16 out) vs fp64 oracle; bf16 inputs, fp32 accumulation


def to_dev(u16: np.ndarray):
    import torch

    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def dev_i32(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def bits_of(t) -> np.ndarray:
    import torch

    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class GpuRunner:
    """Owns the device cache of a workload and feeds steps to the library."""

    def __init__(self, w: W.Workload):
        import paper_2507_11830_amd as sp

        self.sp, self.w = sp, w
        self.cache = sp.KVCache.empty(w.num_pages, w.Hkv, w.d, fill_bits=W.CANARY)
        self.bt = dev_i32(w.block_table)
        self.ws = None
        self.prefill_workspace = True   # hand sp_attn_prefill the scratch that lets it split key ranges

    def append(self, st: W.Step):
        self.sp.sp_kv_append(self.cache, to_dev(st.k_new), to_dev(st.v_new), dev_i32(st.cu_new),
                             dev_i32(st.ctx_lens), self.bt)

    def attend(self, st: W.Step):
        import torch

        w, sp = self.w, self.sp
        q = to_dev(st.q)
        out = torch.full_like(q, float("nan"))   # a row the kernels never write cannot pass by accident
        if st.kind == "prefill":
            need = sp.sp_attn_prefill_workspace_size(w.batch, q.shape[0], int(st.new_lens.max()),
                                                     int(st.seq_lens.max()), w.Hq, w.Hkv, w.d) if self.prefill_workspace else 0
            ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
            sp.sp_attn_prefill(self.cache, q, out, dev_i32(st.cu_new), dev_i32(st.ctx_lens), self.bt,
                               int(st.new_lens.max()), int(st.seq_lens.max()), float(w.scale), workspace=ws)
        else:
            seq_lens = st.seq_lens
            mx = int(seq_lens.max())
            need = sp.sp_attn_decode_workspace_size(w.batch, mx, w.Hq, w.d)
            if self.ws is None or self.ws.numel() < need:
                self.ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
            sp.sp_attn_decode(self.cache, q, out, dev_i32(seq_lens), self.bt, mx, float(w.scale), self.ws)
        torch.cuda.synchronize()
        return bits_of(out)

    def chunk_step(self, st: W.Step):
        """Fused append + attention of a chunk step (any chunk lengths)."""
        import torch

        w, sp = self.w, self.sp
        assert st.kind == "prefill"
        q = to_dev(st.q)
        out = torch.full_like(q, float("nan"))
        mq, mkv = int(st.new_lens.max()), int(st.seq_lens.max())
        need = sp.sp_attn_prefill_workspace_size(w.batch, q.shape[0], mq, mkv, w.Hq, w.Hkv, w.d) if self.prefill_workspace else 0
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        sp.sp_chunk_step(self.cache, to_dev(st.k_new), to_dev(st.v_new), q, out, dev_i32(st.cu_new),
                         dev_i32(st.ctx_lens), self.bt, mq, mkv, float(w.scale), workspace=ws)
        torch.cuda.synchronize()
        return bits_of(out)

    def decode_step(self, st: W.Step):
        """Fused append + decode of a step in which every sequence has exactly one new token."""
        import torch

        w, sp = self.w, self.sp
        assert st.kind == "decode" and (st.new_lens == 1).all()
        q = to_dev(st.q)
        out = torch.full_like(q, float("nan"))   # a row the kernels never write cannot pass by accident
        mx = int(st.seq_lens.max())
        need = sp.sp_attn_decode_workspace_size(w.batch, mx, w.Hq, w.d)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
        sp.sp_decode_step(self.cache, to_dev(st.k_new), to_dev(st.v_new), q, out, dev_i32(st.seq_lens), self.bt, mx,
                          float(w.scale), self.ws)
        torch.cuda.synchronize()
        return bits_of(out)

    def cache_bits(self):
        return bits_of(self.cache.k_pages), bits_of(self.cache.v_pages)


class OracleRunner:
    def __init__(self, w: W.Workload):
        import oracle

        self.o, self.w = oracle, w
        self.kp, self.vp = w.empty_cache()

    def append(self, st: W.Step):
        self.o.kv_append(self.kp, self.vp, st.k_new, st.v_new, st.cu_new, st.ctx_lens, self.w.block_table)

    def attend(self, st: W.Step) -> np.ndarray:
        w = self.w
        if st.kind == "prefill":
            return self.o.attn_prefill(self.kp, self.vp, st.q, st.cu_new, st.ctx_lens, w.block_table, w.scale)
        return self.o.attn_decode(self.kp, self.vp, st.q, st.seq_lens, w.block_table, w.scale)


def report_err(name, got_bits, want):
    got = W.bf16_bits_to_f64(got_bits)
    err = np.abs(got - want)
    assert np.isfinite(got).all(), f"{name}: non-finite GPU output"
    idx = np.unravel_index(np.argmax(err), err.shape)
    print(f"[parity] {name}: max abs err {err.max():.5f} at {idx} (gpu {got[idx]:.5f} oracle {want[idx]:.5f})",
          flush=True)
    return float(err.max())
