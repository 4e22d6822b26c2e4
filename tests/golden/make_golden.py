#!/usr/bin/env python3
"""Writes tests/golden/c1_oracle_outputs.txt: the fp64 oracle's outputs for configuration C1
(tiny GQA: 128-token causal prefill, then 16 decode steps; seeded inputs from workloads.py).

The paper prints no worked numerical example for the attention path (it gives no formula for
it at all), so there are no paper values to store.  This file is a CHANGE DETECTOR for the
oracle, not a pin of it: it records what the oracle, as pinned by tests/test_oracle_pins.py,
produced when the file was written, so that a later edit of the oracle's arithmetic or of the
input generator shows up as a diff.  It calls only oracle/ and workloads.py.

Run from the repository root:  python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as W  # noqa: E402


def oracle_outputs():
    w = W.c1_tiny()
    kp, vp = w.empty_cache()
    outs = []
    for st in w.steps():
        oracle.kv_append(kp, vp, st.k_new, st.v_new, st.cu_new, st.ctx_lens, w.block_table)
        if st.kind == "prefill":
            outs.append(oracle.attn_prefill(kp, vp, st.q, st.cu_new, st.ctx_lens, w.block_table, w.scale))
        elif st.kind == "decode":
            outs.append(oracle.attn_decode(kp, vp, st.q, st.seq_lens, w.block_table, w.scale))
    return outs, kp, vp


def render() -> str:
    outs, kp, vp = oracle_outputs()
    lines = ["# configuration C1, fp64 oracle; written by tests/golden/make_golden.py",
             f"cache_sha256 {hashlib.sha256(kp.tobytes() + vp.tobytes()).hexdigest()}"]
    for i, o in enumerate(outs):
        flat = o.reshape(-1)
        # a few probe values at full precision plus a digest of the rounded tensor
        probes = " ".join(f"{flat[j]:.17g}" for j in (0, len(flat) // 3, len(flat) - 1))
        digest = hashlib.sha256(np.round(o, 12).tobytes()).hexdigest()[:16]
        lines.append(f"step {i} shape {'x'.join(map(str, o.shape))} probes {probes} digest12 {digest}")
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_outputs.txt")
    with open(path, "w") as f:
        f.write(render())
    print("wrote", path)
