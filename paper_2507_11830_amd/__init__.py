"""Python binding of libshiftattn.so — argument marshalling only.

Every step of the hot path (KV append, prefill attention, split decode + combine) runs in the
HIP kernels behind the C ABI declared in ``include/shiftattn.h``; this module converts torch
tensors to raw device pointers, passes the current HIP stream and turns negative status codes
into exceptions.  There is no CPU or PyTorch fallback: if the shared library has not been
built, importing the binding's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshiftattn.so")
if os.environ.get("SP_LIB_SANITIZE", "") == "1":
    # the copy whose host code carries ASan + UBSan instrumentation (CPU-only boundary tests; the
    # process must run with the matching sanitizer runtime preloaded)
    LIB_PATH = os.path.join(_HERE, "_build", "san", "libshiftattn_san.so")

SP_OK = 0
SP_ERR_NULL = -1
SP_ERR_BAD_SHAPE = -2
SP_ERR_UNSUPPORTED = -3
SP_ERR_WORKSPACE = -4
SP_ERR_HIP = -5

EXPORTS = (
    "sp_kv_append", "sp_attn_prefill", "sp_attn_decode", "sp_attn_decode_static", "sp_decode_step", "sp_chunk_step", "sp_ulysses_pack", "sp_ulysses_unpack",
    "sp_attn_prefill_workspace_size",
    "sp_attn_decode_workspace_size", "sp_debug_validate_metadata", "sp_debug_validate_hints", "sp_debug_set_tuning",
    "sp_status_string", "sp_last_error", "sp_version",
)


class SpError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name} ({status}): {detail}")
        self.status = status


class sp_cache_desc(ctypes.Structure):
    _fields_ = [
        ("k_pages", ctypes.c_void_p), ("v_pages", ctypes.c_void_p), ("num_pages", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: run `python -m paper_2507_11830_amd.build` "
                "(or __graft_entry__.build()) first; there is no non-HIP fallback")
        # PyTorch ships its own HIP runtime and owns the device buffers this binding is handed: it
        # has to be in the process before the library binds to a runtime.  Loaded the other way
        # round, the library's first launch fails with "no ROCm-capable device is detected".
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cd = ctypes.POINTER(sp_cache_desc)
        L.sp_kv_append.argtypes = [cd, vp, vp, vp, vp, vp, i32, i32, i32, vp]
        L.sp_kv_append.restype = ctypes.c_int
        L.sp_attn_prefill.argtypes = [cd, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                      ctypes.c_float, i32, vp, sz, vp]
        L.sp_attn_prefill.restype = ctypes.c_int
        L.sp_attn_decode.argtypes = [cd, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, vp, sz, vp]
        L.sp_attn_decode.restype = ctypes.c_int
        L.sp_attn_decode_static.argtypes = [cd, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, vp]
        L.sp_attn_decode_static.restype = ctypes.c_int
        L.sp_decode_step.argtypes = [cd, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, vp, sz, vp]
        L.sp_decode_step.restype = ctypes.c_int
        L.sp_chunk_step.argtypes = [cd, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                    ctypes.c_float, vp, sz, vp]
        L.sp_chunk_step.restype = ctypes.c_int
        L.sp_ulysses_pack.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.sp_ulysses_pack.restype = ctypes.c_int
        L.sp_ulysses_unpack.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.sp_ulysses_unpack.restype = ctypes.c_int
        L.sp_attn_prefill_workspace_size.argtypes = [i32, i32, i32, i32, i32, i32, i32]
        L.sp_attn_prefill_workspace_size.restype = sz
        L.sp_attn_decode_workspace_size.argtypes = [i32, i32, i32, i32]
        L.sp_attn_decode_workspace_size.restype = sz
        L.sp_debug_validate_metadata.argtypes = [cd, vp, vp, i32, i32]
        L.sp_debug_validate_metadata.restype = ctypes.c_int
        L.sp_debug_set_tuning.argtypes = [ctypes.c_char_p, i32]
        L.sp_debug_set_tuning.restype = ctypes.c_int
        L.sp_debug_validate_hints.argtypes = [vp, vp, i32, i32, i32, i32]
        L.sp_debug_validate_hints.restype = ctypes.c_int
        L.sp_status_string.argtypes = [ctypes.c_int]
        L.sp_status_string.restype = ctypes.c_char_p
        L.sp_last_error.restype = ctypes.c_char_p
        L.sp_version.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != SP_OK:
        L = lib()
        raise SpError(status, L.sp_status_string(status).decode(), L.sp_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class KVCache:
    """Owner of the two page pools (torch tensors) plus the C descriptor that names them.
    Layout of both pools: bf16 [num_pages][num_kv_heads][16][head_dim]."""

    def __init__(self, k_pages, v_pages):
        assert k_pages.shape == v_pages.shape and k_pages.dim() == 4
        assert k_pages.is_cuda and k_pages.is_contiguous() and v_pages.is_contiguous()
        assert k_pages.element_size() == 2
        self.k_pages, self.v_pages = k_pages, v_pages
        n, h, p, d = k_pages.shape
        self.desc = sp_cache_desc(k_pages.data_ptr(), v_pages.data_ptr(), n, p, h, d)

    @classmethod
    def empty(cls, num_pages: int, num_kv_heads: int, head_dim: int, device="cuda:0", fill_bits: Optional[int] = None):
        import torch

        shape = (num_pages, num_kv_heads, 16, head_dim)
        if fill_bits is None:
            k = torch.empty(shape, dtype=torch.bfloat16, device=device)
            v = torch.empty(shape, dtype=torch.bfloat16, device=device)
        else:
            signed = fill_bits - 65536 if fill_bits >= 32768 else fill_bits
            k = torch.full(shape, signed, dtype=torch.int16, device=device).view(torch.bfloat16)
            v = torch.full(shape, signed, dtype=torch.int16, device=device).view(torch.bfloat16)
        return cls(k, v)

    @property
    def num_kv_heads(self) -> int:
        return self.desc.num_kv_heads

    @property
    def head_dim(self) -> int:
        return self.desc.head_dim


def sp_version() -> int:
    return lib().sp_version()


def sp_kv_append(cache: KVCache, k_new, v_new, cu_seqlens_new, ctx_lens, block_table, stream=None) -> None:
    """k_new, v_new: bf16 [T, Hkv, d] (cuda); cu_seqlens_new [B+1], ctx_lens [B], block_table
    [B, max_pages]: int32 cuda tensors."""
    batch, max_pages = block_table.shape
    total = k_new.shape[0]
    _check(lib().sp_kv_append(ctypes.byref(cache.desc), _ptr(k_new), _ptr(v_new), _ptr(cu_seqlens_new),
                              _ptr(ctx_lens), _ptr(block_table), batch, max_pages, total, _stream(stream)))


def sp_attn_prefill(cache: KVCache, q, out, cu_seqlens_q, ctx_lens, block_table, max_q_len: int,
                    max_kv_len: int, scale: float, causal: int = 1, workspace=None, stream=None) -> None:
    """q, out: bf16 [T, Hq, d] (cuda).  The chunk's own K/V must already be appended."""
    batch, max_pages = block_table.shape
    total, num_q_heads = q.shape[0], q.shape[1]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sp_attn_prefill(ctypes.byref(cache.desc), _ptr(q), _ptr(out), _ptr(cu_seqlens_q),
                                 _ptr(ctx_lens), _ptr(block_table), batch, max_pages, total, max_q_len,
                                 max_kv_len, num_q_heads, float(scale), causal, _ptr(workspace), ws_bytes,
                                 _stream(stream)))


def sp_attn_decode_workspace_size(batch: int, max_seq_len: int, num_q_heads: int, head_dim: int) -> int:
    return lib().sp_attn_decode_workspace_size(batch, max_seq_len, num_q_heads, head_dim)


def sp_attn_prefill_workspace_size(batch: int, total_q_tokens: int, max_q_len: int, max_kv_len: int,
                                   num_q_heads: int, num_kv_heads: int, head_dim: int) -> int:
    return lib().sp_attn_prefill_workspace_size(batch, total_q_tokens, max_q_len, max_kv_len, num_q_heads,
                                                num_kv_heads, head_dim)


def sp_attn_decode(cache: KVCache, q, out, seq_lens, block_table, max_seq_len: int, scale: float,
                   workspace, stream=None) -> None:
    """q, out: bf16 [B, Hq, d] (cuda); seq_lens include the current token."""
    batch, max_pages = block_table.shape
    num_q_heads = q.shape[1]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sp_attn_decode(ctypes.byref(cache.desc), _ptr(q), _ptr(out), _ptr(seq_lens),
                                _ptr(block_table), batch, max_pages, max_seq_len, num_q_heads, float(scale),
                                _ptr(workspace), ws_bytes, _stream(stream)))


def sp_attn_decode_static(cache: KVCache, q, out, seq_lens, block_table, max_seq_len: int, scale: float, stream=None) -> None:
    """sp_attn_decode with the partials in the library's static device array (no workspace, no
    allocation); shapes whose partials exceed 16 MiB are refused."""
    batch, max_pages = block_table.shape
    _check(lib().sp_attn_decode_static(ctypes.byref(cache.desc), _ptr(q), _ptr(out), _ptr(seq_lens), _ptr(block_table),
                                       batch, max_pages, max_seq_len, q.shape[1], float(scale), _stream(stream)))


def sp_decode_step(cache: KVCache, k_new, v_new, q, out, seq_lens, block_table, max_seq_len: int, scale: float,
                   workspace, stream=None) -> None:
    """Fused append + decode: k_new, v_new bf16 [B, Hkv, d] (the new token of every sequence),
    seq_lens include it; the rest as sp_attn_decode."""
    batch, max_pages = block_table.shape
    num_q_heads = q.shape[1]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sp_decode_step(ctypes.byref(cache.desc), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out),
                                _ptr(seq_lens), _ptr(block_table), batch, max_pages, max_seq_len, num_q_heads,
                                float(scale), _ptr(workspace), ws_bytes, _stream(stream)))


def sp_chunk_step(cache: KVCache, k_new, v_new, q, out, cu_seqlens_q, ctx_lens, block_table, max_q_len: int,
                  max_kv_len: int, scale: float, workspace=None, stream=None) -> None:
    """Fused append + chunk attention: k_new, v_new bf16 [T, Hkv, d] packed like q; the rest as
    sp_attn_prefill."""
    batch, max_pages = block_table.shape
    total, num_q_heads = q.shape[0], q.shape[1]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sp_chunk_step(ctypes.byref(cache.desc), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out),
                               _ptr(cu_seqlens_q), _ptr(ctx_lens), _ptr(block_table), batch, max_pages, total,
                               max_q_len, max_kv_len, num_q_heads, float(scale), _ptr(workspace), ws_bytes,
                               _stream(stream)))


def sp_debug_validate_metadata(cache: KVCache, seq_lens, block_table) -> None:
    batch, max_pages = block_table.shape
    _check(lib().sp_debug_validate_metadata(ctypes.byref(cache.desc), _ptr(seq_lens), _ptr(block_table),
                                            batch, max_pages))


def sp_debug_set_tuning(key: str, value: int) -> None:
    _check(lib().sp_debug_set_tuning(key.encode(), int(value)))


def sp_debug_validate_hints(cu_seqlens, lens, total_tokens: int, max_q_len: int, max_len: int) -> None:
    """Synchronous check of an attention call's host-side hints against its device length arrays
    (cu_seqlens None: a decode call, lens = seq_lens)."""
    _check(lib().sp_debug_validate_hints(_ptr(cu_seqlens), _ptr(lens), lens.shape[0], int(total_tokens),
                                         int(max_q_len), int(max_len)))


def sp_ulysses_pack(x, send, world: int, stream=None) -> None:
    """x: bf16 [T_loc, H, d] -> send: bf16 [world, T_loc, H/world, d] (block j = head slice j)."""
    t, h, d = x.shape
    _check(lib().sp_ulysses_pack(_ptr(x), _ptr(send), t, h, d, int(world), _stream(stream)))


def sp_ulysses_unpack(recv, y, stream=None) -> None:
    """recv: bf16 [world, T_loc, H/world, d] -> y: bf16 [T_loc, H, d]."""
    world, t, hp, d = recv.shape
    _check(lib().sp_ulysses_unpack(_ptr(recv), _ptr(y), t, hp * world, d, world, _stream(stream)))
