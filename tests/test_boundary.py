"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, every symbol
the header declares is exported, and the header and the Python binding agree."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def built_lib():
    import paper_2507_11830_amd as sp
    from paper_2507_11830_amd import build as b

    if not os.path.exists(sp.LIB_PATH):
        b.build()
    return ctypes.CDLL(sp.LIB_PATH)


def header_functions(header="shiftattn.h", prefix="sp_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(%s[a-z_]+)\s*\(" % prefix, text)))


def test_header_declares_the_three_hot_calls():
    names = header_functions()
    for n in ("sp_kv_append", "sp_attn_prefill", "sp_attn_decode"):
        assert n in names


def test_library_exports_every_declared_symbol(built_lib):
    for n in header_functions():
        assert hasattr(built_lib, n), f"{n} declared in shiftattn.h but not exported"


def test_bench_only_library_exports_its_header_and_the_product_library_holds_no_bench_kernels(built_lib):
    """The benchmark's reference kernels live in a shared object of their own."""
    from paper_2507_11830_amd import ceilings

    names = header_functions("sp_ceilings.h", "spc_")
    assert names == sorted(ceilings.EXPORTS)
    L = ctypes.CDLL(ceilings.LIB_PATH)
    for n in names:
        assert hasattr(L, n), f"{n} declared in sp_ceilings.h but not exported"
        assert not hasattr(built_lib, n)
    assert not any("ceiling" in n for n in header_functions())


def test_every_include_header_is_covered():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["shiftattn.h", "sp_ceilings.h"]


def test_binding_names_match_header():
    import paper_2507_11830_amd as sp

    assert sorted(sp.EXPORTS) == header_functions()
    for n in ("sp_kv_append", "sp_attn_prefill", "sp_attn_decode", "sp_attn_decode_workspace_size"):
        assert callable(getattr(sp, n))


def test_status_strings_and_version(built_lib):
    built_lib.sp_status_string.restype = ctypes.c_char_p
    assert built_lib.sp_status_string(0) == b"SP_OK"
    assert built_lib.sp_status_string(-4) == b"SP_ERR_WORKSPACE"
    assert built_lib.sp_version() >= 100


def test_workspace_size_is_host_only_arithmetic(built_lib):
    f = built_lib.sp_attn_decode_workspace_size
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int32] * 4
    assert f(0, 100, 8, 128) == 0 and f(4, 0, 8, 128) == 0
    # one (o[d], m, l) fp32 partial per (sequence, head) and split of 128..1024 keys; the split
    # length depends on the shape, so the size is not monotone in the length
    for batch, mx in ((64, 8192), (64, 16384), (1, 32768), (256, 300)):
        rows = batch * 8
        assert rows * -(-mx // 1024) * 130 * 4 <= f(batch, mx, 8, 128) <= rows * -(-mx // 128) * 130 * 4
    # at least one (o[d], m, l) fp32 partial per (sequence, head)
    assert f(1, 1, 8, 128) >= 8 * 130 * 4


def test_prefill_workspace_size_is_host_only_arithmetic(built_lib):
    f = built_lib.sp_attn_prefill_workspace_size
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int32] * 7   # batch, total_q, max_q_len, max_kv_len, Hq, Hkv, head_dim
    assert f(4, 0, 0, 100, 8, 1, 128) == 0
    # few query rows: room for up to 16 pieces of (head_dim + 2) fp32 per (token, head)
    assert f(4, 100, 25, 4000, 8, 1, 128) == 100 * 8 * 16 * 130 * 4
    # many query rows: key ranges are never cut, no workspace asked for
    assert f(4, 32768, 8192, 8192, 8, 1, 128) == 0
    small, big = f(1, 1000, 1000, 1000, 8, 1, 128), f(1, 8000, 8000, 8000, 8, 1, 128)
    assert small > 0 and big > 0 and big <= 2 * (1 << 17) * 130 * 4
    # chunks of a few tokens (the decode kernels serve them): one partial per 128..1024 keys and row,
    # however many rows there are
    rows = 128 * 4 * 32
    short = f(128, 128 * 4, 4, 16384, 32, 8, 128)
    assert rows * 16 * 130 * 4 <= short <= rows * 128 * 130 * 4
    # ... unless that path is switched off
    import paper_2507_11830_amd as sp
    sp.sp_debug_set_tuning("prefill_short_chunk", 1)
    try:
        assert f(128, 128 * 4, 4, 16384, 32, 8, 128) == rows * 8 * 130 * 4   # the key-range pieces only
    finally:
        sp.sp_debug_set_tuning("prefill_short_chunk", 0)


def test_argument_validation_needs_no_gpu(built_lib):
    """Validation happens before any HIP call, so these return codes are checkable on a CPU machine."""
    import paper_2507_11830_amd as sp

    L = sp.lib()
    d = sp.sp_cache_desc(0x1000, 0x2000, 8, 16, 1, 128)
    one = ctypes.c_void_p(0x4000)
    assert L.sp_kv_append(None, one, one, one, one, one, 1, 1, 1, None) == sp.SP_ERR_NULL
    assert L.sp_kv_append(ctypes.byref(d), one, one, one, one, one, 0, 1, 0, None) == sp.SP_OK
    assert L.sp_kv_append(ctypes.byref(d), None, one, one, one, one, 1, 1, 1, None) == sp.SP_ERR_NULL
    assert L.sp_kv_append(ctypes.byref(d), one, one, one, one, one, -1, 1, 1, None) == sp.SP_ERR_BAD_SHAPE
    bad_page = sp.sp_cache_desc(0x1000, 0x2000, 8, 32, 1, 128)
    assert L.sp_kv_append(ctypes.byref(bad_page), one, one, one, one, one, 1, 1, 1, None) == sp.SP_ERR_UNSUPPORTED
    bad_dim = sp.sp_cache_desc(0x1000, 0x2000, 8, 16, 1, 96)
    assert L.sp_attn_decode(ctypes.byref(bad_dim), one, one, one, one, 1, 1, 16, 8, 0.1, one, 1 << 20, None) == sp.SP_ERR_UNSUPPORTED
    # Hq not a multiple of Hkv
    d3 = sp.sp_cache_desc(0x1000, 0x2000, 8, 16, 3, 128)
    assert L.sp_attn_decode(ctypes.byref(d3), one, one, one, one, 1, 1, 16, 8, 0.1, one, 1 << 20, None) == sp.SP_ERR_BAD_SHAPE
    # non-causal, bad scale
    assert L.sp_attn_prefill(ctypes.byref(d), one, one, one, one, one, 1, 1, 4, 4, 4, 8, 0.1, 0, None, 0, None) == sp.SP_ERR_UNSUPPORTED
    assert L.sp_attn_prefill(ctypes.byref(d), one, one, one, one, one, 1, 1, 4, 4, 4, 8, -1.0, 1, None, 0, None) == sp.SP_ERR_UNSUPPORTED
    # workspace too small / missing
    assert L.sp_attn_decode(ctypes.byref(d), one, one, one, one, 4, 64, 1000, 8, 0.1, one, 16, None) == sp.SP_ERR_WORKSPACE
    assert L.sp_attn_decode(ctypes.byref(d), one, one, one, one, 4, 64, 1000, 8, 0.1, None, 0, None) == sp.SP_ERR_WORKSPACE
    assert b"workspace" in L.sp_last_error()
    # head exchange permutations
    assert L.sp_ulysses_pack(one, one, 4, 8, 128, 3, None) == sp.SP_ERR_BAD_SHAPE       # 8 heads over 3 ranks
    assert L.sp_ulysses_pack(one, one, 4, 8, 100, 2, None) == sp.SP_ERR_UNSUPPORTED     # head_dim % 8
    assert L.sp_ulysses_pack(one, one, 4, 8, 128, 2, None) == sp.SP_ERR_UNSUPPORTED     # in place
    assert L.sp_ulysses_unpack(None, one, 4, 8, 128, 2, None) == sp.SP_ERR_NULL
    assert L.sp_ulysses_unpack(None, None, 0, 8, 128, 2, None) == sp.SP_OK
    assert L.sp_decode_step(ctypes.byref(d), None, one, one, one, one, one, 4, 64, 1000, 8, 0.1, one, 1 << 30, None) == sp.SP_ERR_NULL
    assert L.sp_chunk_step(ctypes.byref(d), None, one, one, one, one, one, one, 4, 64, 16, 4, 1000, 8, 0.1, one, 1 << 30, None) == sp.SP_ERR_NULL
    assert L.sp_chunk_step(ctypes.byref(d), one, one, one, one, one, one, one, 4, 64, 16, 4, 1000, 0, 0.1, one, 1 << 30, None) == sp.SP_ERR_BAD_SHAPE
    assert L.sp_chunk_step(ctypes.byref(d), one, one, one, one, one, one, one, 0, 64, 0, 0, 0, 8, 0.1, None, 0, None) == sp.SP_OK
    # the allocation-free decode: same validation, and shapes beyond its 16 MiB static array are refused
    assert L.sp_attn_decode_static(ctypes.byref(bad_dim), one, one, one, one, 1, 1, 16, 8, ctypes.c_float(0.1), None) == sp.SP_ERR_UNSUPPORTED
    assert L.sp_attn_decode_static(ctypes.byref(d), one, None, one, one, 1, 1, 16, 8, ctypes.c_float(0.1), None) == sp.SP_ERR_NULL
    assert L.sp_attn_decode_static(ctypes.byref(d), one, one, one, one, 0, 1, 16, 8, ctypes.c_float(0.1), None) == sp.SP_OK
    assert sp.sp_attn_decode_workspace_size(4096, 16384, 32, 128) > 16 << 20
    assert L.sp_attn_decode_static(ctypes.byref(d), one, one, one, one, 4096, 1024, 16384, 32, ctypes.c_float(0.1), None) == sp.SP_ERR_WORKSPACE
    assert b"static scratch" in L.sp_last_error()
    # empty batches are legal no-ops
    assert L.sp_attn_prefill(ctypes.byref(d), one, one, one, one, one, 0, 1, 0, 0, 0, 8, 0.1, 1, None, 0, None) == sp.SP_OK
    assert L.sp_attn_decode(ctypes.byref(d), one, one, one, one, 0, 1, 0, 8, 0.1, None, 0, None) == sp.SP_OK


def test_tuning_keys_are_validated(built_lib):
    import paper_2507_11830_amd as sp

    L = sp.lib()
    assert L.sp_debug_set_tuning(None, 0) == sp.SP_ERR_NULL
    assert L.sp_debug_set_tuning(b"no_such_key", 0) == sp.SP_ERR_UNSUPPORTED
    for v, want in [(0, sp.SP_OK), (128, sp.SP_OK), (1024, sp.SP_OK), (320, sp.SP_OK), (300, sp.SP_ERR_UNSUPPORTED),
                    (64, sp.SP_ERR_UNSUPPORTED), (2048, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"decode_chunk", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_OK), (3, sp.SP_ERR_UNSUPPORTED), (-1, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"prefill_split", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_OK), (4, sp.SP_OK), (-1, sp.SP_ERR_UNSUPPORTED), (5, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"decode_ring", v) == want
    for v, want in [(1, sp.SP_OK), (16, sp.SP_OK), (17, sp.SP_ERR_UNSUPPORTED), (-1, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"prefill_kv_splits", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_ERR_UNSUPPORTED), (-1, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"prefill_short_chunk", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_OK), (3, sp.SP_ERR_UNSUPPORTED), (-1, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"prefill_order", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_OK), (3, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"combine_form", v) == want
    for v, want in [(1, sp.SP_OK), (2, sp.SP_OK), (3, sp.SP_ERR_UNSUPPORTED), (-1, sp.SP_ERR_UNSUPPORTED)]:
        assert L.sp_debug_set_tuning(b"decode_fuse", v) == want
    for key in (b"decode_fuse", b"decode_chunk", b"decode_ring", b"prefill_split", b"prefill_kv_splits", b"prefill_short_chunk",
                b"prefill_order", b"combine_form"):
        assert L.sp_debug_set_tuning(key, 0) == sp.SP_OK


def test_tuning_overrides_are_per_thread(built_lib):
    """An override set by one thread changes that thread's workspace sizing only."""
    import threading

    import paper_2507_11830_amd as sp

    f = lambda: sp.sp_attn_decode_workspace_size(64, 8192, 8, 128)
    base = f()
    seen = {}

    def other():
        sp.sp_debug_set_tuning("decode_chunk", 128)
        seen["other"] = f()

    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert seen["other"] == 64 * 8 * (8192 // 128) * 130 * 4
    assert f() == base != seen["other"]


def test_hint_validation_rejects_bad_arguments_without_a_gpu(built_lib):
    import paper_2507_11830_amd as sp

    L = sp.lib()
    one = ctypes.c_void_p(0x4000)
    assert L.sp_debug_validate_hints(None, None, 0, 0, 0, 0) == sp.SP_OK
    assert L.sp_debug_validate_hints(None, None, 3, 0, 0, 0) == sp.SP_ERR_NULL
    assert L.sp_debug_validate_hints(one, one, -1, 0, 0, 0) == sp.SP_ERR_BAD_SHAPE


def test_bench_refuses_more_than_one_gpu():
    """One GPU's shard only: asking bench.py for more must end with a message, before any GPU use."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_prefill_loops_hold_no_spill_code(built_lib):
    """The build refuses a prefill kernel whose one-workgroup-per-query-tile form spills inside its
    loops (a reload on the tile loop's common path costs 5-20 %); this checks the listing that
    the build left behind, with the build's own scanner, and the scanner on a planted case."""
    import glob
    import tempfile

    from paper_2507_11830_amd import build as b

    planted = "\n".join(["_Zk:", ".LBB0_1:   ; in Loop: Header=BB0_1 Depth=1", "\tscratch_load_dword v1, off, off",
                         "; %bb.2:", "\tscratch_store_dword off, v1, off", ".LBB0_3:", "\tscratch_load_dword v1, off, off",
                         ".Lfunc_end0:"])
    with tempfile.NamedTemporaryFile("w", suffix=".s", delete=False) as f:
        f.write(planted)
    try:
        assert b.loop_spills(f.name) == {"_Zk": 2}
    finally:
        os.unlink(f.name)
    listings = glob.glob(os.path.join(os.path.dirname(b.__file__), "_build", "attn_prefill-hip-amdgcn-amd-amdhsa-gfx950.s"))
    if not listings:
        pytest.skip("no assembly listing from this build")
    counts = {k: v for k, v in b.loop_spills(listings[0]).items() if "prefill_kernel" in k}
    assert len(counts) == 6
    for kern, n in counts.items():
        assert n <= (0 if "ELb0ELb0E" in kern else 8), (kern, n)
