"""fp64 CPU oracle (TEST INFRASTRUCTURE ONLY) for the paged causal GQA attention path.

Only tests, the smoke check and the bench's cpu_baseline leg may import this package.
It wraps ``attn_oracle.c`` (plain C, fp64, compiled with gcc) through ctypes and shares
nothing with the HIP library.  All tensors cross this boundary as numpy arrays:
bf16 data as ``uint16`` bit patterns, indices as ``int32``, results as ``float64``.

The operation is the plain softmax(scale * q k^T) v definition restricted to the keys a
causal query may see, for the per-GPU head shard described in the paper's section
"Introducing Shift Parallelism" (invariant KV layout, identical attention in TP and SP).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
PAGE = 16

_lib = None


# -O3 for the per-config timing the bench reports; the instruction set is pinned to x86-64-v3
# (AVX2) rather than the build machine's own, because the library is built on one machine and
# loaded on another.  ISO C mode keeps floating-point contraction off, so the fp64 operation
# order is the one written in the source at any optimisation level.
_CFLAGS = ["-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11"]
# SP_ORACLE_SANITIZE=1: an AddressSanitizer + UndefinedBehaviorSanitizer build of the same source
# (host code only; the process must run with gcc's libasan preloaded).  Used by the CPU-only
# sanitizer test, which re-runs the pin tests on it.
_SAN = os.environ.get("SP_ORACLE_SANITIZE", "") == "1"
if _SAN:
    _LIB = os.path.join(_HERE, "_build", "liboracle_attn_san.so")
    _CFLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
               "-fopenmp", "-fPIC", "-shared", "-std=c11"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP on).  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *_CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_kv_append.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def kv_append(k_pages, v_pages, k_new, v_new, cu_new, ctx_lens, block_table):
    """In-place cache image update.  k_pages/v_pages: uint16 [num_pages, Hkv, 16, d]."""
    lib = _load()
    assert k_pages.dtype == np.uint16 and k_pages.flags.c_contiguous
    assert v_pages.dtype == np.uint16 and v_pages.flags.c_contiguous
    num_pages, Hkv, page, d = k_pages.shape
    assert page == PAGE
    k_new, v_new = _u16(k_new), _u16(v_new)
    cu_new, ctx_lens, block_table = _i32(cu_new), _i32(ctx_lens), _i32(block_table)
    batch, max_pages = block_table.shape
    rc = lib.oracle_kv_append(
        _p(k_pages), _p(v_pages), num_pages, Hkv, d, _p(k_new), _p(v_new), _p(cu_new),
        _p(ctx_lens), _p(block_table), batch, max_pages,
    )
    if rc != 0:
        raise ValueError("block table entry out of range")


def attn_prefill(k_pages, v_pages, q, cu_q, ctx_lens, block_table, scale, return_lse=False):
    """q: uint16 [T, Hq, d].  Returns float64 [T, Hq, d] (and lse [T, Hq])."""
    lib = _load()
    k_pages, v_pages, q = _u16(k_pages), _u16(v_pages), _u16(q)
    _, Hkv, _, d = k_pages.shape
    T, Hq, dq = q.shape
    assert dq == d and Hq % Hkv == 0
    cu_q, ctx_lens, block_table = _i32(cu_q), _i32(ctx_lens), _i32(block_table)
    batch, max_pages = block_table.shape
    out = np.zeros((T, Hq, d), dtype=np.float64)
    lse = np.zeros((T, Hq), dtype=np.float64)
    lib.oracle_attn_prefill(
        _p(k_pages), _p(v_pages), Hkv, d, _p(q), _p(cu_q), _p(ctx_lens), _p(block_table),
        batch, max_pages, Hq, ctypes.c_double(float(scale)), _p(out), _p(lse),
    )
    return (out, lse) if return_lse else out


def attn_decode(k_pages, v_pages, q, seq_lens, block_table, scale, return_lse=False):
    """q: uint16 [B, Hq, d]; seq_lens include the current token.  Returns float64 [B, Hq, d]."""
    lib = _load()
    k_pages, v_pages, q = _u16(k_pages), _u16(v_pages), _u16(q)
    _, Hkv, _, d = k_pages.shape
    B, Hq, dq = q.shape
    assert dq == d and Hq % Hkv == 0
    seq_lens, block_table = _i32(seq_lens), _i32(block_table)
    batch, max_pages = block_table.shape
    assert batch == B
    out = np.zeros((B, Hq, d), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    lib.oracle_attn_decode(
        _p(k_pages), _p(v_pages), Hkv, d, _p(q), _p(seq_lens), _p(block_table), batch,
        max_pages, Hq, ctypes.c_double(float(scale)), _p(out), _p(lse),
    )
    return (out, lse) if return_lse else out


def attn_prefill_rows(k_pages, v_pages, q, cu_q, ctx_lens, block_table, scale, row_seq,
                      row_tok, row_head):
    """Sampled rows of the prefill problem: returns float64 [n_rows, d]."""
    lib = _load()
    k_pages, v_pages, q = _u16(k_pages), _u16(v_pages), _u16(q)
    _, Hkv, _, d = k_pages.shape
    _, Hq, _ = q.shape
    cu_q, ctx_lens, block_table = _i32(cu_q), _i32(ctx_lens), _i32(block_table)
    row_seq, row_tok, row_head = _i32(row_seq), _i32(row_tok), _i32(row_head)
    _, max_pages = block_table.shape
    n = row_seq.shape[0]
    out = np.zeros((n, d), dtype=np.float64)
    lib.oracle_attn_prefill_rows(
        _p(k_pages), _p(v_pages), Hkv, d, _p(q), _p(cu_q), _p(ctx_lens), _p(block_table),
        max_pages, Hq, ctypes.c_double(float(scale)), _p(row_seq), _p(row_tok), _p(row_head),
        n, _p(out),
    )
    return out


def attn_row_paged(k_pages, v_pages, bt_row, p, q_row, g, scale):
    """One row through the block table.  Returns (out[d], lse, weights[p+1])."""
    lib = _load()
    k_pages, v_pages, q_row = _u16(k_pages), _u16(v_pages), _u16(q_row)
    _, Hkv, _, d = k_pages.shape
    bt_row = _i32(bt_row)
    out = np.zeros(d, dtype=np.float64)
    lse = np.zeros(1, dtype=np.float64)
    w = np.zeros(p + 1, dtype=np.float64)
    lib.oracle_attn_row_paged(
        _p(k_pages), _p(v_pages), Hkv, d, _p(bt_row), int(p), _p(q_row), int(g),
        ctypes.c_double(float(scale)), _p(out), _p(lse), _p(w),
    )
    return out, float(lse[0]), w


def attn_row_contig(k, v, p, q_row, g, scale):
    """One row over contiguous K, V: uint16 [L, Hkv, d].  Returns (out[d], lse, weights)."""
    lib = _load()
    k, v, q_row = _u16(k), _u16(v), _u16(q_row)
    L, Hkv, d = k.shape
    assert p < L
    out = np.zeros(d, dtype=np.float64)
    lse = np.zeros(1, dtype=np.float64)
    w = np.zeros(p + 1, dtype=np.float64)
    lib.oracle_attn_row_contig(
        _p(k), _p(v), Hkv, d, int(p), _p(q_row), int(g), ctypes.c_double(float(scale)),
        _p(out), _p(lse), _p(w),
    )
    return out, float(lse[0]), w


def attn_row_subset(k_pages, v_pages, bt_row, p, mask, q_row, g, scale):
    """One row restricted to keys with mask[j] != 0.  Returns (out[d], lse)."""
    lib = _load()
    k_pages, v_pages, q_row = _u16(k_pages), _u16(v_pages), _u16(q_row)
    _, Hkv, _, d = k_pages.shape
    bt_row = _i32(bt_row)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.shape[0] == p + 1 and mask.any()
    out = np.zeros(d, dtype=np.float64)
    lse = np.zeros(1, dtype=np.float64)
    lib.oracle_attn_row_subset(
        _p(k_pages), _p(v_pages), Hkv, d, _p(bt_row), int(p), _p(mask), _p(q_row), int(g),
        ctypes.c_double(float(scale)), _p(out), _p(lse),
    )
    return out, float(lse[0])


def ulysses_pack(x, P: int) -> np.ndarray:
    """x: uint16 [T_loc, H, d] (all heads of this rank's tokens) -> send buffer [P, T_loc, H/P, d]
    (block j goes to rank j).  Local half of the pre-attention exchange of the SP mode."""
    x = _u16(x)
    T, H, d = x.shape
    assert H % P == 0
    send = np.empty((P, T, H // P, d), dtype=np.uint16)
    _load().oracle_ulysses_pack(_p(x), _p(send), T, H, d, P)
    return send


def ulysses_unpack(recv) -> np.ndarray:
    """recv: uint16 [P, T_loc, H/P, d] (block j came from rank j) -> [T_loc, H, d].  Local half of
    the post-attention exchange."""
    recv = _u16(recv)
    P, T, hp, d = recv.shape
    y = np.empty((T, P * hp, d), dtype=np.uint16)
    _load().oracle_ulysses_unpack(_p(recv), _p(y), T, P * hp, d, P)
    return y
