"""Workgroup timeline of the prefill kernel (measurement aid, not part of the product path).

Needs a library built with the kernel's trace switch:

    SP_HIPCC_EXTRA="-DSP_PREFILL_TRACE" python -m paper_2507_11830_amd.build
    python -m paper_2507_11830_amd.trace_prefill c5a        # or c2; optional: split mode 0 / 1 / 2

With that switch a launch that has no other use for the caller's workspace writes, per workgroup,
the 100 MHz wall clock at its start, after the prologue's barrier, at the end of either wave
group's tile loop and at its end, its tile count and the CU it ran on, and for every eighth tile
period the wall clock and the shader clock.  This script runs one launch of a seeded workload and
prints what the records say: the prologue and epilogue of a workgroup, the time per tile period,
the gaps between workgroups on a CU, and shader cycles per period next to the clock they imply.
"""
from __future__ import annotations

import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

WGS, REC, PER = 8192, 8, 64   # the kernel's kTraceWgs, kTraceRec, kTracePer


def main(argv) -> int:
    import torch

    import bench as B
    import paper_2507_11830_amd as sp
    import workloads as W

    wl = argv[1] if len(argv) > 1 else "c5a"
    w = W.c2_prefill() if wl == "c2" else W.c5_long(decode_steps=0)
    torch.cuda.set_device(0)
    job = B.PrefillJob(sp, w)
    job.append()
    sp.sp_debug_set_tuning("prefill_kv_splits", 1)   # key-range pieces would use the workspace themselves
    if len(argv) > 2:
        sp.sp_debug_set_tuning("prefill_split", int(argv[2]))
    ws = torch.zeros(WGS * (REC + 2 * PER) * 8, dtype=torch.uint8, device="cuda")

    def launch():
        sp.sp_attn_prefill(job.cache, job.q, job.out, job.cu, job.ctx, job.bt, job.max_q, job.max_kv,
                           float(w.scale), workspace=ws)

    for _ in range(5):
        launch()
    torch.cuda.synchronize()
    ws.zero_()
    torch.cuda.synchronize()
    launch()
    torch.cuda.synchronize()
    raw = ws.view(torch.int64).cpu().numpy()
    rec = raw[:WGS * REC].reshape(WGS, REC)
    wall = raw[WGS * REC:][:WGS * PER].reshape(WGS, PER)
    clk = raw[WGS * REC + WGS * PER:][:WGS * PER].reshape(WGS, PER)
    idx = np.nonzero(rec[:, 4] > 0)[0]
    if len(idx) == 0:
        print("no records: the library was not built with -DSP_PREFILL_TRACE")
        return 1
    r = rec[idx]
    t0 = r[:, 0].min()
    us = lambda x: (x - t0) / 100.0
    T = r[:, 5]
    hw, xcc = r[:, 6] & 0xFFFFFFFF, r[:, 6] >> 32
    cu = xcc * 1000 + ((hw >> 13) & 7) * 100 + ((hw >> 12) & 1) * 10 + ((hw >> 8) & 0xF)
    print(f"{wl}: {len(r)} workgroups with work on {len(np.unique(cu))} CUs, launch span {us(r[:, 4].max()):.1f} us")
    pro = (r[:, 1] - r[:, 0]) / 100.0
    loop_end = np.maximum(r[:, 2], r[:, 3])
    loop = (loop_end - r[:, 1]) / 100.0
    epi = (r[:, 4] - loop_end) / 100.0
    print("prologue (start -> first barrier) us: mean %.2f min %.2f max %.2f | after the tile loop us: mean %.2f max %.2f"
          % (pro.mean(), pro.min(), pro.max(), epi.mean(), epi.max()))
    for lo, hi in ((1, 8), (9, 32), (33, 128), (129, 100000)):
        m = (T >= lo) & (T <= hi)
        if m.any():
            print(f"  workgroups of {lo}..{min(hi, int(T.max()))} key tiles: n={int(m.sum())}, prologue {pro[m].mean():.2f} us, "
                  f"tile loop {loop[m].mean():.2f} us = {(loop[m] / T[m]).mean():.3f} us per tile, rest {epi[m].mean():.2f} us")
    gaps, busy = [], []
    for c in np.unique(cu):
        m = cu == c
        s, e = np.sort(us(r[m, 0])), np.sort(us(r[m, 4]))
        busy.append(((r[m, 4] - r[m, 0]) / 100.0).sum())
        gaps.extend(list(s[1:] - e[:-1]))
    print("per CU: busy %.1f us of the span on average, %.2f workgroups, gap between workgroups mean %.2f us max %.2f us"
          % (np.mean(busy), len(r) / len(np.unique(cu)), np.mean(gaps) if gaps else 0.0, np.max(gaps) if gaps else 0.0))
    order = np.argsort(-T)
    picks = [order[0], order[len(order) // 3], order[2 * len(order) // 3]]
    for k in picks:
        g = idx[k]
        ks = [i for i in range(1, PER - 1) if wall[g, i] > 0 and wall[g, i + 1] > 0]
        if not ks:
            continue
        cyc = [(clk[g, i + 1] - clk[g, i]) / 8.0 for i in ks]
        ghz = [(clk[g, i + 1] - clk[g, i]) / ((wall[g, i + 1] - wall[g, i]) * 10.0) for i in ks]
        print(f"  workgroup {g} ({int(T[k])} tiles, started at {us(r[k, 0]):.0f} us): shader cycles per tile period "
              f"min {min(cyc):.0f} max {max(cyc):.0f}; clock GHz over its life: "
              + " ".join(f"{x:.2f}" for x in ghz[:: max(1, len(ghz) // 12)]))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
