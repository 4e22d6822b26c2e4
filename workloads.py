"""Seeded synthetic inputs for the paged-attention hot path (shared by oracle tests, GPU
tests and the bench).  This module holds NO attention arithmetic: it only draws random bits,
lengths and block tables, and describes each workload as a cache shape plus a list of steps.

Recipe (same for every workload):
  * values: float32 N(0,1) from numpy ``Generator(PCG64)`` -> round-to-nearest-even to bf16;
    those exact bits (uint16) go to both the oracle and the GPU;
  * seed of workload Cn is 20250711*10 + n, sub-streams from ``SeedSequence.spawn`` in the
    fixed order (lengths, block table, values);
  * block table: pool of ceil(1.25 * pages_needed) physical pages, one seeded permutation of
    the pool dealt out to the sequences in order (shuffled physical order, holes, interleaving);
  * untouched cache slots hold the bf16 canary 0x7FC0.

The five workloads stand in for the paper's request mixes (ShareGPT / HumanEval / SWE-bench /
production traces, none of which is reproduced here): they take only their shapes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Iterator, List, Optional

import numpy as np

PAGE = 16
CANARY = 0x7FC0
BASE_SEED = 20250711 * 10


# ----------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit pattern (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for a in range(0, n, step):
        b = min(n, a + step)
        out[a:b] = f32_to_bf16_bits(rng.standard_normal(b - a, dtype=np.float32))
    return out.reshape(shape)


# ----------------------------------------------------------------------------- structures
@dataclass
class Step:
    """One forward-pass step: append ``k_new``/``v_new`` then (unless kind == 'fill') attend.

    kind 'fill'    : append only (cache warm-up, no attention);
    kind 'prefill' : q is [T_new, Hq, d], one query per new token (causal, sees the prefix);
    kind 'decode'  : exactly one new token per sequence, q is [B, Hq, d].
    """
    kind: str
    cu_new: np.ndarray          # int32 [B+1]
    ctx_lens: np.ndarray        # int32 [B]  tokens cached before this step
    k_new: np.ndarray           # uint16 [T_new, Hkv, d]
    v_new: np.ndarray           # uint16 [T_new, Hkv, d]
    q: Optional[np.ndarray]     # uint16, see kind

    @property
    def new_lens(self) -> np.ndarray:
        return np.diff(self.cu_new).astype(np.int32)

    @property
    def seq_lens(self) -> np.ndarray:
        return (self.ctx_lens + self.new_lens).astype(np.int32)


@dataclass
class Workload:
    name: str
    Hq: int
    Hkv: int
    d: int
    num_pages: int
    block_table: np.ndarray     # int32 [B, max_pages]
    total_lens: np.ndarray      # int32 [B] final length of every sequence
    make_steps: Callable[[], Iterator[Step]] = field(repr=False, default=None)

    @property
    def scale(self) -> np.float32:
        return np.float32(1.0) / np.sqrt(np.float32(self.d))

    @property
    def batch(self) -> int:
        return int(self.block_table.shape[0])

    def steps(self) -> Iterator[Step]:
        return self.make_steps()

    def empty_cache(self):
        shape = (self.num_pages, self.Hkv, PAGE, self.d)
        return np.full(shape, CANARY, np.uint16), np.full(shape, CANARY, np.uint16)


def _seeds(n: int, k: int = 3):
    """Sub-stream seeds of workload n in the fixed order (lengths, block table, values)."""
    return np.random.SeedSequence(BASE_SEED + n).spawn(k)


def _rng(seed_seq) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_seq))


def make_block_table(rng: np.random.Generator, total_lens, pool_factor: float = 1.25):
    """Deal a permuted page pool to the sequences.  Returns (block_table, num_pages).
    Unused block-table entries are -1."""
    total_lens = np.asarray(total_lens, dtype=np.int64)
    pages = (total_lens + PAGE - 1) // PAGE
    need = int(pages.sum())
    pool = max(1, math.ceil(pool_factor * need))
    perm = rng.permutation(pool).astype(np.int32)
    max_pages = max(1, int(pages.max()) if len(pages) else 1)
    bt = np.full((len(total_lens), max_pages), -1, dtype=np.int32)
    at = 0
    for s, n in enumerate(pages):
        bt[s, :n] = perm[at:at + n]
        at += int(n)
    return bt, pool


def _cu(lens) -> np.ndarray:
    out = np.zeros(len(lens) + 1, dtype=np.int32)
    np.cumsum(np.asarray(lens, dtype=np.int64), out=out[1:])
    return out


def _chunk_step(rng, kind, new_lens, ctx_lens, Hq, Hkv, d, with_q=True) -> Step:
    new_lens = np.asarray(new_lens, dtype=np.int32)
    T = int(new_lens.sum())
    k = normal_bf16(rng, (T, Hkv, d))
    v = normal_bf16(rng, (T, Hkv, d))
    q = None
    if kind == "prefill" and with_q:
        q = normal_bf16(rng, (T, Hq, d))
    elif kind == "decode":
        assert (new_lens == 1).all()
        q = normal_bf16(rng, (len(new_lens), Hq, d))
    return Step(kind, _cu(new_lens), np.asarray(ctx_lens, dtype=np.int32).copy(), k, v, q)


# ----------------------------------------------------------------------------- workloads
def c1_tiny(prefill_len: int = 128, decode_steps: int = 16, Hq: int = 2, Hkv: int = 1,
            d: int = 64) -> Workload:
    """Tiny GQA: one sequence, causal prefill then single-token decode steps."""
    s_len, s_bt, s_val = _seeds(1)
    total = np.array([prefill_len + decode_steps], dtype=np.int32)
    bt, pool = make_block_table(_rng(s_bt), total)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "prefill", [prefill_len], [0], Hq, Hkv, d)
        for t in range(decode_steps):
            yield _chunk_step(rng, "decode", [1], [prefill_len + t], Hq, Hkv, d)

    return Workload("C1_tiny_gqa", Hq, Hkv, d, pool, bt, total, gen)


def c2_prefill(batch: int = 4, seqlen: int = 2048, Hq: int = 8, Hkv: int = 1, d: int = 128) -> Workload:
    """70B head shard, SP-mode prefill: ``batch`` sequences of ``seqlen`` tokens, no prefix."""
    s_len, s_bt, s_val = _seeds(2)
    total = np.full(batch, seqlen, dtype=np.int32)
    bt, pool = make_block_table(_rng(s_bt), total)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "prefill", total, np.zeros(batch), Hq, Hkv, d)

    return Workload("C2_70B_prefill", Hq, Hkv, d, pool, bt, total, gen)


def c3_decode(batch: int = 64, lo: int = 512, hi: int = 8192, Hq: int = 8, Hkv: int = 1,
              d: int = 128, n: int = 3, name: str = "C3_70B_decode") -> Workload:
    """70B head shard, TP-mode decode: context lengths uniform in [lo, hi] (inclusive); the
    cache is filled with L-1 tokens, then one decode step appends the last token and attends."""
    s_len, s_bt, s_val = _seeds(n)
    total = _rng(s_len).integers(lo, hi + 1, size=batch).astype(np.int32)
    bt, pool = make_block_table(_rng(s_bt), total)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "fill", total - 1, np.zeros(batch), Hq, Hkv, d)
        yield _chunk_step(rng, "decode", np.ones(batch), total - 1, Hq, Hkv, d)

    return Workload(name, Hq, Hkv, d, pool, bt, total, gen)


def spec_verify(batch: int = 64, lo: int = 512, hi: int = 8192, q_len: int = 4, Hq: int = 8, Hkv: int = 1,
                d: int = 128, n: int = 7) -> Workload:
    """The decode batch of c3_decode with q_len query tokens per sequence instead of one (a
    speculative-decoding verification step: the last accepted token plus q_len - 1 draft tokens,
    causal inside the chunk).  The cache is filled with L - q_len tokens, then one chunk step
    appends the q_len tokens and attends."""
    s_len, s_bt, s_val = _seeds(n)
    total = _rng(s_len).integers(lo, hi + 1, size=batch).astype(np.int32)
    bt, pool = make_block_table(_rng(s_bt), total)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "fill", total - q_len, np.zeros(batch), Hq, Hkv, d)
        yield _chunk_step(rng, "prefill", np.full(batch, q_len), total - q_len, Hq, Hkv, d)

    return Workload(f"spec_verify_q{q_len}", Hq, Hkv, d, pool, bt, total, gen)


def c4_lengths(batch: int = 32, median: float = 1500.0, sigma: float = 1.0, lo: int = 64,
               hi: int = 8192) -> np.ndarray:
    s_len, _, _ = _seeds(4)
    raw = _rng(s_len).lognormal(mean=math.log(median), sigma=sigma, size=batch)
    return np.clip(np.rint(raw), lo, hi).astype(np.int32)


def c4_chunked(batch: int = 32, median: float = 1500.0, sigma: float = 1.0, lo: int = 64,
               hi: int = 8192, chunk: int = 512, Hq: int = 8, Hkv: int = 1, d: int = 128) -> Workload:
    """Mixed chunked prefill: lognormal lengths (clipped); the first floor(L/2) tokens are
    cached, the rest is prefilled ``chunk`` tokens per step for every unfinished sequence."""
    _, s_bt, s_val = _seeds(4)
    total = c4_lengths(batch, median, sigma, lo, hi)
    bt, pool = make_block_table(_rng(s_bt), total)
    prefix = (total // 2).astype(np.int32)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "fill", prefix, np.zeros(batch), Hq, Hkv, d)
        done = prefix.copy()
        while (done < total).any():
            new = np.minimum(chunk, total - done).astype(np.int32)
            yield _chunk_step(rng, "prefill", new, done, Hq, Hkv, d)
            done = done + new

    return Workload("C4_mixed_chunked", Hq, Hkv, d, pool, bt, total, gen)


def c5_long(prefill_len: int = 32768, decode_steps: int = 256, Hq: int = 8, Hkv: int = 1,
            d: int = 128) -> Workload:
    """Long-context shift: one long causal prefill, then decode steps on the SAME cache and
    block table (no re-layout between the two modes)."""
    s_len, s_bt, s_val = _seeds(5)
    total = np.array([prefill_len + decode_steps], dtype=np.int32)
    bt, pool = make_block_table(_rng(s_bt), total)

    def gen():
        rng = _rng(s_val)
        yield _chunk_step(rng, "prefill", [prefill_len], [0], Hq, Hkv, d)
        for t in range(decode_steps):
            yield _chunk_step(rng, "decode", [1], [prefill_len + t], Hq, Hkv, d)

    return Workload("C5ab_long_shift", Hq, Hkv, d, pool, bt, total, gen)


def c5c_decode_8b(batch: int = 128, lo: int = 1024, hi: int = 16384) -> Workload:
    """Llama-3.1-8B single-GPU shape decode batch (32 query heads / 8 KV heads, d = 128)."""
    return c3_decode(batch, lo, hi, Hq=32, Hkv=8, d=128, n=6, name="C5c_8B_decode")


# ----------------------------------------------------------------------------- work counters
def prefill_flops(step: Step, Hq: int, d: int) -> int:
    """Algorithmic flops of one prefill step: 4*d per visible (query, key) pair per head."""
    n = step.new_lens.astype(np.int64)
    c = step.ctx_lens.astype(np.int64)
    pairs = int((n * c + n * (n + 1) // 2).sum())
    return 4 * d * Hq * pairs


def decode_bytes(seq_lens, Hq: int, Hkv: int, d: int) -> int:
    """Algorithmic bytes of one decode step: every cached K and V element once, plus q, out
    and the block-table entries touched."""
    L = np.asarray(seq_lens, dtype=np.int64)
    B = len(L)
    return int(L.sum()) * Hkv * 2 * d * 2 + 2 * B * Hq * d * 2 + int(((L + PAGE - 1) // PAGE).sum()) * 4


def append_bytes(n_tokens: int, Hkv: int, d: int) -> int:
    return int(n_tokens) * Hkv * d * 2 * 2 * 2
