"""GPU parity: the HIP library (through the C ABI) against the fp64 oracle on the same seeded
bits.  Floating point: max abs error <= 1e-2 (bf16 in, fp32 accumulate, bf16 out).  Cache
images after sp_kv_append: bit-exact, canaries included."""
import hashlib

import numpy as np
import pytest

import workloads as W
from harness import TOL, GpuRunner, OracleRunner, bits_of, dev_i32, report_err, to_dev

pytestmark = pytest.mark.gpu


def custom_workload(name, lens_total, ctx, Hq, Hkv, d, kind, seed):
    """Sequences with `ctx` tokens cached (a 'fill' step) followed by one `kind` step over the rest."""
    lens_total, ctx = np.asarray(lens_total, np.int32), np.asarray(ctx, np.int32)
    rng = np.random.default_rng(seed)
    bt, pool = W.make_block_table(rng, lens_total)

    def gen():
        r = np.random.default_rng(seed + 1)
        if ctx.sum() > 0:
            yield W._chunk_step(r, "fill", ctx, np.zeros_like(ctx), Hq, Hkv, d)
        yield W._chunk_step(r, kind, lens_total - ctx, ctx, Hq, Hkv, d)

    return W.Workload(name, Hq, Hkv, d, pool, bt, lens_total, gen)


def run_full_compare(w, check_cache=True):
    """Every step on both sides, every attention output compared element by element."""
    g, o = GpuRunner(w), OracleRunner(w)
    worst = 0.0
    for i, st in enumerate(w.steps()):
        g.append(st)
        o.append(st)
        if st.kind != "fill":
            worst = max(worst, report_err(f"{w.name} step {i} {st.kind}", g.attend(st), o.attend(st)))
    if check_cache:
        gk, gv = g.cache_bits()
        assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp), "cache image differs from the oracle's"
    assert worst <= TOL
    return worst


# ------------------------------------------------------------------ sp_kv_append
def test_append_bit_exact_ragged_with_prefix():
    lens = [45, 16, 0, 3, 300, 1]
    ctx = [13, 0, 0, 2, 17, 0]
    for Hkv, d in ((1, 128), (8, 128), (2, 64)):
        w = custom_workload(f"append-{Hkv}-{d}", lens, ctx, 2 * Hkv, Hkv, d, "prefill", seed=11)
        g, o = GpuRunner(w), OracleRunner(w)
        for st in w.steps():
            g.append(st)
            o.append(st)
        gk, gv = g.cache_bits()
        assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp)
        assert (o.kp == W.CANARY).any()            # holes exist and were compared too


def test_append_ignores_out_of_range_pages():
    """A block-table entry outside the pool must not become a wild store."""
    import paper_2507_11830_amd as sp

    w = custom_workload("append-bad", [40], [0], 2, 1, 64, "prefill", seed=12)
    g = GpuRunner(w)
    st = next(w.steps())
    bad = w.block_table.copy()
    bad[0, 1] = w.num_pages + 1000
    g.bt = dev_i32(bad)
    with pytest.raises(sp.SpError):
        sp.sp_debug_validate_metadata(g.cache, dev_i32(st.seq_lens), g.bt)
    g.append(st)
    gk, _ = g.cache_bits()
    good_page = w.block_table[0, 0]
    assert np.array_equal(gk[good_page, 0], st.k_new[:16, 0])
    untouched = np.ones(w.num_pages, bool)
    untouched[[w.block_table[0, 0], w.block_table[0, 2]]] = False
    assert (gk[untouched] == W.CANARY).all()


def test_append_and_chunk_step_on_sub_ranges_of_a_batch():
    """sp_kv_append and sp_chunk_step called on sub-ranges of a batch's sequences (advanced index
    arrays with absolute token offsets, full k_new / v_new / q / out and token total): each call
    writes its own sequences' cache rows and output rows only.  Chunks are too long for the
    short-chunk path, so sp_chunk_step runs append + prefill.  Cache image incl. canaries and
    outputs against the oracle's single pass."""
    import torch
    import paper_2507_11830_amd as sp

    new = np.array([70, 300, 1, 45, 130])
    ctx = np.array([13, 0, 77, 500, 31])
    w = custom_workload("sub-append", ctx + new, ctx, 8, 1, 128, "prefill", seed=101)
    o = OracleRunner(w)
    fill, st = list(w.steps())
    o.append(fill)
    o.append(st)
    want = o.attend(st)
    k, v, q = to_dev(st.k_new), to_dev(st.v_new), to_dev(st.q)
    cu, cx = dev_i32(st.cu_new), dev_i32(st.ctx_lens)
    total = q.shape[0]
    for use_chunk_step in (False, True):
        g = GpuRunner(w)
        g.append(fill)
        out = torch.full_like(q, float("nan"))
        for lo, hi in ((2, 5), (0, 2)):
            mq, mkv = int(st.new_lens[lo:hi].max()), int(st.seq_lens[lo:hi].max())
            sp.sp_debug_validate_hints(cu[lo:hi + 1], cx[lo:hi], total, mq, mkv)
            if use_chunk_step:
                sp.sp_chunk_step(g.cache, k, v, q, out, cu[lo:hi + 1], cx[lo:hi], g.bt[lo:hi], mq, mkv, float(w.scale))
            else:
                sp.sp_kv_append(g.cache, k, v, cu[lo:hi + 1], cx[lo:hi], g.bt[lo:hi])
            if (lo, hi) == (2, 5):   # after the first call the other range's rows are still canaries
                gk, _ = g.cache_bits()
                assert (gk[w.block_table[1, 0]] == W.CANARY).all()
        torch.cuda.synchronize()
        gk, gv = g.cache_bits()
        assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp), "cache image differs from the oracle's"
        if use_chunk_step:
            assert report_err("chunk step on sub-ranges", bits_of(out), want) <= TOL


def test_fused_append_paths_skip_out_of_range_pages():
    """sp_decode_step and sp_chunk_step (short-chunk path) with a block-table entry outside the pool,
    and with a position past the end of the block-table row: like sp_kv_append, the fused kernels
    must skip those rows — no store into page 0, the last pool page or the sequence's last table
    page.  Every page except the ones that legitimately receive a row stays canary-filled."""
    import torch
    import paper_2507_11830_amd as sp

    for fused in ("decode", "chunk"):
        nq = 1 if fused == "decode" else 3
        lens = np.array([40, 33, 64 + nq, 20])          # sequence 2: its new rows start a page the table row lacks
        w = custom_workload(f"fused-bad-{fused}", lens, lens - nq, 8, 1, 128, "decode" if nq == 1 else "prefill", seed=111)
        fill, st = list(w.steps())
        bt = w.block_table[:, :4].copy()                # 4 pages per row: positions >= 64 are past the row
        bad_page = w.num_pages + 7
        target1 = bt[1, 2]                              # sequence 1's new rows go to its page 2 ...
        bt[1, 2] = bad_page                             # ... which the table names outside the pool
        cache = sp.KVCache.empty(w.num_pages, 1, 128, fill_bits=W.CANARY)
        btd = dev_i32(bt)
        sp.sp_kv_append(cache, to_dev(fill.k_new), to_dev(fill.v_new), dev_i32(fill.cu_new), dev_i32(fill.ctx_lens), btd)
        torch.cuda.synchronize()
        before_k, before_v = bits_of(cache.k_pages).copy(), bits_of(cache.v_pages).copy()
        with pytest.raises(sp.SpError):
            sp.sp_debug_validate_metadata(cache, dev_i32(st.seq_lens), btd)
        q = to_dev(st.q)
        out = torch.empty_like(q)
        mx = int(st.seq_lens.max())
        if fused == "decode":
            ws = torch.empty(sp.sp_attn_decode_workspace_size(4, mx, 8, 128), dtype=torch.uint8, device="cuda")
            sp.sp_decode_step(cache, to_dev(st.k_new), to_dev(st.v_new), q, out, dev_i32(st.seq_lens), btd, mx, float(w.scale), ws)
        else:
            need = sp.sp_attn_prefill_workspace_size(4, q.shape[0], nq, mx, 8, 1, 128)
            assert need > 0
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            sp.sp_chunk_step(cache, to_dev(st.k_new), to_dev(st.v_new), q, out, dev_i32(st.cu_new), dev_i32(st.ctx_lens), btd,
                             nq, mx, float(w.scale), workspace=ws)
        torch.cuda.synchronize()
        after_k, after_v = bits_of(cache.k_pages), bits_of(cache.v_pages)
        changed = np.nonzero((after_k != before_k).any(axis=(1, 2, 3)) | (after_v != before_v).any(axis=(1, 2, 3)))[0]
        legit = set()                                   # pages that sp_kv_append would write with this metadata
        for s_ in range(4):
            for pos in range(int(lens[s_]) - nq, int(lens[s_])):
                if pos // 16 < bt.shape[1] and 0 <= bt[s_, pos // 16] < w.num_pages:
                    legit.add(int(bt[s_, pos // 16]))
        assert set(changed.tolist()) == legit, (fused, changed, legit)
        assert (after_k[target1] == before_k[target1]).all() and (after_k[w.block_table[2, 4]] == W.CANARY).all()
        # sequences with good metadata got their rows, bit for bit
        for s_, L in ((0, 40), (3, 20)):
            for t in range(nq):
                pos = L - nq + t
                row = after_k[bt[s_, pos // 16], 0, pos % 16]
                assert np.array_equal(row, st.k_new[st.cu_new[s_] + t, 0])


# ------------------------------------------------------------------ small shapes, every element
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (2, 1, 64), (32, 8, 128), (4, 4, 64), (6, 2, 128), (1, 1, 128)])
def test_prefill_small_ragged(Hq, Hkv, d):
    lens = [1, 17, 63, 64, 65, 300, 0, 130]
    ctx = [0, 5, 0, 31, 64, 111, 0, 129]
    run_full_compare(custom_workload(f"prefill-{Hq}-{Hkv}-{d}", lens, ctx, Hq, Hkv, d, "prefill", seed=21))


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (2, 1, 64), (32, 8, 128), (6, 2, 128), (40, 1, 64)])
def test_decode_small_ragged(Hq, Hkv, d):
    lens = np.array([1, 15, 16, 17, 127, 128, 129, 255, 256, 257, 1000, 2049])
    run_full_compare(custom_workload(f"decode-{Hq}-{Hkv}-{d}", lens, lens - 1, Hq, Hkv, d, "decode", seed=31))


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (2, 1, 64), (6, 2, 128)])
def test_prefill_both_wave_group_modes(mode, Hq, Hkv, d):
    """The prefill kernel divides a workgroup's work over its two wave groups either by query
    columns or by key tiles (chosen by grid size); both must meet the oracle on the same ragged
    batch, including sequences whose second key-tile stream is empty or fully masked."""
    lens = [1, 17, 63, 64, 65, 127, 128, 129, 300, 0, 130, 1000]
    ctx = [0, 5, 0, 31, 64, 0, 0, 100, 111, 0, 129, 489]
    import paper_2507_11830_amd as sp

    sp.sp_debug_set_tuning("prefill_split", mode)
    try:
        run_full_compare(custom_workload(f"modes-{mode}-{Hq}-{Hkv}-{d}", lens, ctx, Hq, Hkv, d, "prefill", seed=61))
    finally:
        sp.sp_debug_set_tuning("prefill_split", 0)


@pytest.mark.parametrize("pieces", [2, 3, 16])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (4, 2, 64)])
def test_prefill_key_range_cut_into_pieces(pieces, Hq, Hkv, d):
    """With a workspace sp_attn_prefill may cut key ranges into pieces merged by the combine pass;
    forced here for every piece count class (more pieces than tiles included, so empty pieces and
    pieces whose keys are all masked for some rows occur).  Such launches always divide a
    workgroup's work over its wave groups by key tiles."""
    import paper_2507_11830_amd as sp

    lens = [1, 17, 64, 65, 129, 300, 0, 700, 1500]
    ctx = [0, 5, 31, 64, 100, 111, 0, 689, 1490]
    sp.sp_debug_set_tuning("prefill_kv_splits", pieces)
    try:
        run_full_compare(custom_workload(f"pieces-{pieces}-{Hq}-{Hkv}-{d}", lens, ctx, Hq, Hkv, d, "prefill", seed=71))
    finally:
        sp.sp_debug_set_tuning("prefill_kv_splits", 0)


@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("mode,pieces", [(1, 0), (2, 0), (1, 3), (2, 5)])
def test_prefill_dispatch_orders(order, mode, pieces):
    """Work items by launch index (1) and heaviest first (2: every workgroup finds the item of its
    rank by itself), on ragged chunks over ragged prefixes: sequences without new tokens, without
    prefix, chunks of one token, equal weights, more than 64 sequences (two per lane)."""
    import paper_2507_11830_amd as sp

    rng = np.random.default_rng(71)
    new = np.concatenate([[0, 1, 300, 64, 64, 17, 0, 129], rng.integers(0, 40, 70)])
    ctx = np.concatenate([[50, 0, 1000, 2048, 2048, 3000, 0, 511], rng.integers(0, 600, 70)])
    sp.sp_debug_set_tuning("prefill_order", order)
    sp.sp_debug_set_tuning("prefill_split", mode)
    sp.sp_debug_set_tuning("prefill_kv_splits", pieces)
    sp.sp_debug_set_tuning("prefill_short_chunk", 1)
    try:
        run_full_compare(custom_workload(f"order-{order}-{mode}-{pieces}", ctx + new, ctx, 8, 1, 128, "prefill", seed=72))
        run_full_compare(custom_workload(f"order-kv2-{order}-{mode}-{pieces}", (ctx + new)[:9], ctx[:9], 8, 2, 64,
                                         "prefill", seed=73))
    finally:
        for key in ("prefill_order", "prefill_split", "prefill_kv_splits", "prefill_short_chunk"):
            sp.sp_debug_set_tuning(key, 0)


@pytest.mark.parametrize("batch", [256, 257])
def test_prefill_heaviest_first_at_its_batch_limit(batch):
    """256 sequences fill every lane slot of the in-kernel ranking; one more and the launch goes
    back to the static order."""
    rng = np.random.default_rng(75)
    new = rng.integers(0, 20, batch)
    ctx = rng.integers(0, 200, batch)
    new[rng.integers(0, batch)] = 150
    run_full_compare(custom_workload(f"rank-limit-{batch}", ctx + new, ctx, 4, 1, 128, "prefill", seed=76))


def test_prefill_dispatch_orders_agree_bitwise():
    """The order in which workgroups pick their items changes nothing in any item's arithmetic."""
    import paper_2507_11830_amd as sp

    new = np.array([100, 256, 31, 256, 0, 5])
    ctx = np.array([900, 0, 4000, 256, 77, 1300])
    outs = []
    for order in (1, 2):
        sp.sp_debug_set_tuning("prefill_order", order)
        try:
            wl = custom_workload("order-bits", ctx + new, ctx, 8, 1, 128, "prefill", seed=74)
            g = GpuRunner(wl)
            for st in wl.steps():
                g.append(st)
            outs.append(g.attend(st))
        finally:
            sp.sp_debug_set_tuning("prefill_order", 0)
    assert np.array_equal(outs[0], outs[1])


def test_prefill_without_workspace_matches_with_workspace():
    """The workspace is optional: without it the same call computes every key range in one piece."""
    w = custom_workload("no-ws", [600, 40, 2100], [580, 0, 2000], 8, 1, 128, "prefill", seed=72)
    outs = []
    for use_ws in (True, False):
        g = GpuRunner(w)
        g.prefill_workspace = use_ws
        for st in w.steps():
            g.append(st)
            if st.kind == "prefill":
                outs.append(W.bf16_bits_to_f64(g.attend(st)))
    o = OracleRunner(w)
    for st in w.steps():
        o.append(st)
        if st.kind == "prefill":
            want = o.attend(st)
    assert np.abs(outs[0] - want).max() <= TOL and np.abs(outs[1] - want).max() <= TOL


def run_fused_steps(w):
    """Decode steps through sp_decode_step (append fused into the attention launch) against the
    oracle's append + decode; the cache image must come out bit-identical as well."""
    g, o = GpuRunner(w), OracleRunner(w)
    worst = 0.0
    for i, st in enumerate(w.steps()):
        o.append(st)
        if st.kind == "decode":
            worst = max(worst, report_err(f"{w.name} fused step {i}", g.decode_step(st), o.attend(st)))
        else:
            g.append(st)
            if st.kind == "prefill":
                worst = max(worst, report_err(f"{w.name} step {i} prefill", g.attend(st), o.attend(st)))
    gk, gv = g.cache_bits()
    assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp), "cache image differs from the oracle's"
    assert worst <= TOL


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (2, 1, 64), (32, 8, 128), (6, 2, 128), (40, 1, 64)])
def test_fused_decode_step_small_ragged(Hq, Hkv, d):
    """New token on every position class: first row of a page, last row, page interior, first token
    of a sequence (length 1), block boundaries, split boundaries (lengths 1025 / 2049)."""
    lens = np.array([1, 15, 16, 17, 32, 33, 127, 128, 129, 255, 256, 257, 1000, 1024, 1025, 2049])
    run_fused_steps(custom_workload(f"fused-{Hq}-{Hkv}-{d}", lens, lens - 1, Hq, Hkv, d, "decode", seed=81))


def test_fused_decode_steps_c1_and_repeated():
    """C1's 16 consecutive decode steps on one growing sequence, every step fused: each step reads
    the rows the previous fused steps wrote."""
    run_fused_steps(W.c1_tiny())


def test_fused_decode_step_c3_full():
    run_fused_steps(W.c3_decode())


@pytest.mark.parametrize("form", [1, 2])
def test_combine_kernel_forms(form):
    """Both work divisions of the combine kernel (a wave per 32-channel slice, a wave per whole
    row) behind a decode batch (32 and 64 splits per row), a short-chunk batch and a prefill whose
    key ranges are cut into pieces, head_dim 128 and 64."""
    import paper_2507_11830_amd as sp

    sp.sp_debug_set_tuning("combine_form", form)
    sp.sp_debug_set_tuning("decode_fuse", 1)      # keep the combine a kernel of its own
    sp.sp_debug_set_tuning("decode_chunk", 128)
    sp.sp_debug_set_tuning("prefill_kv_splits", 5)
    try:
        lens = np.array([4000, 1, 130, 2049, 0, 777])
        dec = np.where(lens > 0, lens, 1)
        run_full_compare(custom_workload(f"comb-d-{form}", dec, dec - 1, 8, 1, 128, "decode", seed=85), check_cache=False)
        run_full_compare(custom_workload(f"comb-d64-{form}", 2 * dec, 2 * dec - 1, 4, 2, 64, "decode", seed=86), check_cache=False)
        run_full_compare(custom_workload(f"comb-s-{form}", lens + 3, lens, 8, 1, 128, "prefill", seed=87), check_cache=False)
        run_full_compare(custom_workload(f"comb-p-{form}", lens + 40, lens, 8, 1, 128, "prefill", seed=88), check_cache=False)
    finally:
        for key in ("combine_form", "decode_fuse", "decode_chunk", "prefill_kv_splits"):
            sp.sp_debug_set_tuning(key, 0)


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 1, 128), (32, 8, 128), (64, 1, 128), (40, 1, 64), (6, 2, 64)])
def test_decode_combine_inside_and_outside_the_split_kernel(Hq, Hkv, d):
    """Up to 32 splits per sequence the last-arriving wave of a (sequence, head group) merges the
    partials inside the split kernel (one launch); the tuning key forces the separate combine
    kernel.  Both against the oracle, on sequences with 1 .. 32 splits, empty sequences and every
    head-tile shape (8, 4, 32 and 1 heads per wave; a group of 6 split 3 + 3), through
    sp_attn_decode and sp_decode_step; the fused result is bitwise reproducible, and the arrival
    counters are left clean (the second and third call reuse them)."""
    import torch
    import paper_2507_11830_amd as sp

    lens = np.array([4096, 1, 130, 2049, 0, 777, 33, 3967, 128, 129])
    dec = np.where(lens > 0, lens, 1)
    sp.sp_debug_set_tuning("decode_chunk", 128)
    try:
        outs = {}
        for fuse in (2, 1, 2):
            sp.sp_debug_set_tuning("decode_fuse", fuse)
            w = custom_workload(f"fuse-{Hq}-{Hkv}-{d}", dec, dec - 1, Hq, Hkv, d, "decode", seed=131)
            g, o = GpuRunner(w), OracleRunner(w)
            for st in w.steps():
                o.append(st)
                if st.kind == "fill":
                    g.append(st)
            want = o.attend(st)
            got_step = g.decode_step(st)                    # appends inside the kernel
            got = g.attend(st)                              # same cache, plain decode
            assert report_err(f"{w.name} fuse={fuse} step", got_step, want) <= TOL
            assert report_err(f"{w.name} fuse={fuse}", got, want) <= TOL
            outs.setdefault(fuse, []).append(got)
        assert np.array_equal(outs[2][0], outs[2][1])
        a, b = W.bf16_bits_to_f64(outs[2][0]), W.bf16_bits_to_f64(outs[1][0])
        assert np.abs(a - b).max() <= 2.0 ** -7 * max(1.0, np.abs(b).max())   # same partials, other summation order
        # with empty sequences in the batch (length 0: an all-zero row, no partial with keys)
        sp.sp_debug_set_tuning("decode_fuse", 2)
        q = to_dev(st.q)
        out = torch.full_like(q, 7.0)
        sl = st.seq_lens.copy()
        sl[[1, 4]] = 0
        mx = int(sl.max())
        ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, Hq, d), dtype=torch.uint8, device="cuda")
        sp.sp_attn_decode(g.cache, q, out, dev_i32(sl), g.bt, mx, float(w.scale), ws)
        got = bits_of(out)
        assert (got[1] == 0).all() and (got[4] == 0).all()
        want0 = o.o.attn_decode(o.kp, o.vp, st.q, sl, w.block_table, w.scale)
        assert report_err(f"{w.name} with empty sequences", got, want0) <= TOL
    finally:
        sp.sp_debug_set_tuning("decode_chunk", 0)
        sp.sp_debug_set_tuning("decode_fuse", 0)


@pytest.mark.parametrize("ring", [1, 2, 3, 4])
def test_decode_lds_ring_forms(ring):
    """Every LDS staging form of the split kernel (ring of 2..4 K/V block pairs; 1 = two K blocks
    and a single V block) on lengths around every block, page and split boundary."""
    import paper_2507_11830_amd as sp

    lens = np.array([1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 128, 129, 255, 256, 257, 300, 1025, 2000])
    sp.sp_debug_set_tuning("decode_ring", ring)
    sp.sp_debug_set_tuning("decode_chunk", 128)
    try:
        run_full_compare(custom_workload(f"ring-{ring}", lens, lens - 1, 8, 1, 128, "decode", seed=81), check_cache=False)
        run_full_compare(custom_workload(f"ring64-{ring}", lens[::2], lens[::2] - 1, 4, 2, 64, "decode", seed=82), check_cache=False)
    finally:
        sp.sp_debug_set_tuning("decode_ring", 0)
        sp.sp_debug_set_tuning("decode_chunk", 0)


@pytest.mark.parametrize("length", [5000, 12000, 20000])
def test_decode_single_long_sequence_many_splits(length):
    """One long sequence: 40, 94 resp. 157 splits per row, so the combine pass runs its forms with
    8, 16 resp. 32 load instructions per batch (the 4-instruction form serves every short case, the
    100 000-token test several batches)."""
    lens = np.array([length])
    run_full_compare(custom_workload(f"decode-long-{length}", lens, lens - 1, 8, 1, 128, "decode", seed=73), check_cache=False)


@pytest.mark.parametrize("Hq,Hkv", [(16, 2), (32, 4), (64, 8)])
def test_other_shard_shapes_of_the_sp_tp_family(Hq, Hkv):
    """Shards of an SP x TP = P factorisation with fewer GPUs hold several KV heads each; the same
    cache layout and kernels serve them (prefill with prefix, then a decode step)."""
    lens = np.array([200, 77, 513])
    run_full_compare(custom_workload(f"shape-p-{Hq}-{Hkv}", lens, [64, 0, 300], Hq, Hkv, 128, "prefill", seed=51))
    run_full_compare(custom_workload(f"shape-d-{Hq}-{Hkv}", lens, lens - 1, Hq, Hkv, 128, "decode", seed=52))


@pytest.mark.parametrize("Hq,Hkv,d", [(16, 2, 128), (32, 4, 128), (64, 8, 128), (32, 8, 128), (16, 2, 64)])
def test_other_shard_shapes_at_scale(Hq, Hkv, d):
    """The same shapes with sequences of several thousand tokens, so that the launches take the
    forms they take at full scale: 256-column workgroups with shared key tiles, a multiple of 8
    (sequence, head group) streams pinned to XCDs, many query tiles per stream, cached prefixes;
    then a decode step with several splits per sequence.  Every element against the oracle."""
    new = np.array([3000, 1100, 2049, 0, 4096 if Hq <= 32 else 1500])
    ctx = np.array([1000, 0, 300, 77, 0])
    run_full_compare(custom_workload(f"scale-p-{Hq}-{Hkv}-{d}", ctx + new, ctx, Hq, Hkv, d, "prefill", seed=151), check_cache=False)
    lens = np.array([5000, 2049, 777, 1, 4096, 3001, 129, 6000])
    run_full_compare(custom_workload(f"scale-d-{Hq}-{Hkv}-{d}", lens, lens - 1, Hq, Hkv, d, "decode", seed=152), check_cache=False)


def test_tolerance_margin_on_rows_of_moderate_length():
    """Where the 1e-2 bound is tightest: rows with few enough keys that the bf16 rounding of the
    weights does not average out, and outputs of magnitude >= 2, whose own bf16 rounding is up to
    0.0078.  Rows of up to 256 keys take their weights as hi + lo, so their error must stay at
    the output's half ulp; rows of 257..1024 keys must keep 15 % headroom under the bound.  Many
    short sequences, so that thousands of such rows (and a few hundred elements >= 2) occur."""
    rng = np.random.default_rng(161)
    new = rng.integers(200, 1025, size=24)
    ctx = np.where(rng.random(24) < 0.5, 0, rng.integers(0, 300, size=24))
    w = custom_workload("margin", ctx + new, ctx, 8, 1, 128, "prefill", seed=162)
    g, o = GpuRunner(w), OracleRunner(w)
    for st in w.steps():
        g.append(st)
        o.append(st)
    got, want = W.bf16_bits_to_f64(g.attend(st)), o.attend(st)
    err = np.abs(got - want)
    keys = np.concatenate([np.arange(c + 1, c + n + 1) for c, n in zip(st.ctx_lens, st.new_lens)])   # visible keys per token row
    half_ulp = 2.0 ** -8 * 2.0 ** np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -126)))   # bf16: 8 significant bits
    short, mid = keys <= 256, (keys > 256) & (keys <= 1024)
    big = np.abs(want) >= 2.0
    print(f"[margin] rows <= 256 keys: {short.sum()}, elements >= 2 there: {(big & short[:, None, None]).sum()}, "
          f"max err {err[short].max():.5f}; rows 257..1024: {mid.sum()}, elements >= 2: {(big & mid[:, None, None]).sum()}, "
          f"max err {err[mid].max():.5f}", flush=True)
    assert (big & short[:, None, None]).sum() > 0
    # hi + lo rows: the output's own rounding plus fp32 accumulation noise
    assert (err[short] <= half_ulp[short] * 1.02 + 2e-4).all()
    assert err[mid].max() <= 0.85e-2 and err.max() <= TOL


def test_short_query_chunks_on_long_prefixes():
    """Speculative-verification shape: 2-8 query tokens per sequence against a long cached prefix,
    causal inside the chunk, served by sp_attn_prefill on the same cache."""
    new = np.array([4, 8, 2, 5, 1, 3])
    ctx = np.array([1000, 37, 4095, 512, 16, 0])
    run_full_compare(custom_workload("spec-verify", ctx + new, ctx, 8, 1, 128, "prefill", seed=53))


SHORT_CHUNK_CASES = {
    # name: (Hq, Hkv, d, new tokens per sequence, cached tokens per sequence)
    # 8 heads per KV head: 4 tokens fill the 32-column tile
    "g8": (8, 1, 128, [4, 4, 2, 3, 1, 3, 0, 4], [1000, 37, 4095, 512, 16, 0, 99, 2300]),
    # the chunk straddles a split boundary (multiples of 128): columns whose causal limit lies
    # before the split's first key see no key at all in it
    "g8-straddle": (8, 1, 128, [4, 4, 4, 4, 3, 2], [126, 127, 125, 253, 1022, 511]),
    "g4-8b": (32, 8, 128, [8, 3, 6, 1], [700, 2049, 64, 130]),
    "g8x2": (16, 2, 128, [4, 2, 3], [513, 300, 77]),
    "g1": (4, 4, 128, [32, 9, 1], [200, 1500, 33]),
    "g5": (5, 1, 128, [6, 1, 5], [400, 129, 1000]),      # 6 tokens x 5 heads = 30 of 32 columns
    "d64": (8, 2, 64, [8, 5, 2], [333, 1025, 0]),
    "fresh": (8, 1, 128, [4, 3, 1], [0, 0, 0]),          # nothing cached: a prefill of a few tokens
    # chunks of up to twice that: two column tiles per wave on one read of the keys
    "g8-2t": (8, 1, 128, [8, 5, 7, 1, 0, 6, 8, 4], [1000, 37, 4095, 512, 16, 0, 99, 2300]),
    "g8-2t-straddle": (8, 1, 128, [8, 8, 8, 6, 7, 5], [121, 124, 127, 250, 1020, 509]),
    "g4-2t": (32, 8, 128, [16, 9, 12, 1], [700, 2049, 64, 130]),
    "g1-2t": (4, 4, 128, [64, 33, 1], [200, 1500, 33]),
    "g5-2t": (5, 1, 128, [12, 7, 5], [400, 129, 1000]),
    "d64-2t": (8, 2, 64, [16, 9, 2], [333, 1025, 0]),
    "fresh-2t": (8, 1, 128, [8, 3, 5], [0, 0, 0]),
}


@pytest.mark.parametrize("short_path", [0, 1])
@pytest.mark.parametrize("case", sorted(SHORT_CHUNK_CASES))
def test_short_chunks_on_both_kernel_paths(case, short_path):
    """Batches of a few query tokens per sequence (speculative-decoding verification): by default
    the decode kernels serve them when tokens x heads of a KV head fit the 32 tile columns
    (per-column causal limit, split-K + combine); the tuning key forces the general prefill kernel.
    Both against the oracle."""
    import paper_2507_11830_amd as sp

    Hq, Hkv, d, new, ctx = SHORT_CHUNK_CASES[case]
    new, ctx = np.array(new), np.array(ctx)
    sp.sp_debug_set_tuning("prefill_short_chunk", short_path)
    try:
        run_full_compare(custom_workload(f"short-{case}-{short_path}", ctx + new, ctx, Hq, Hkv, d, "prefill", seed=61))
    finally:
        sp.sp_debug_set_tuning("prefill_short_chunk", 0)


def run_chunk_steps(w):
    """Every non-fill step through sp_chunk_step (append fused where the library can); outputs and
    the final cache image against the oracle."""
    g, o = GpuRunner(w), OracleRunner(w)
    worst = 0.0
    for i, st in enumerate(w.steps()):
        o.append(st)
        if st.kind == "fill":
            g.append(st)
        else:
            worst = max(worst, report_err(f"{w.name} chunk step {i}", g.chunk_step(st), o.attend(st)))
    gk, gv = g.cache_bits()
    assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp), "cache image differs from the oracle's"
    assert worst <= TOL


@pytest.mark.parametrize("case", sorted(SHORT_CHUNK_CASES))
def test_fused_chunk_step_short_chunks(case):
    """sp_chunk_step on the short-chunk shapes: the attention kernel itself appends the chunk's
    rows (chunks straddling block, page and split boundaries, one and two column tiles, empty
    chunks, empty prefixes); output and cache image incl. canaries against the oracle."""
    Hq, Hkv, d, new, ctx = SHORT_CHUNK_CASES[case]
    new, ctx = np.array(new), np.array(ctx)
    run_chunk_steps(custom_workload(f"chunkstep-{case}", ctx + new, ctx, Hq, Hkv, d, "prefill", seed=64))


@pytest.mark.parametrize("seed", range(8))
def test_fused_chunk_step_random_batches(seed):
    """Seeded random batches (head configuration, head_dim, prefixes, chunks of 0 .. 2 x 32/G
    tokens, now and then a chunk too long for the fused path) through sp_chunk_step: outputs and
    cache image against the oracle."""
    rng = np.random.default_rng(7000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 8, 16]))
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 12))
    ctx = rng.integers(0, int(rng.choice([40, 300, 1500, 5000])) + 1, size=B)
    two_tiles = 2 * max(32 // min(G, 32), 1)
    new = rng.integers(0, two_tiles + 1, size=B)
    if rng.random() < 0.25:
        new[rng.integers(0, B)] = int(rng.integers(two_tiles + 1, 200))
    if new.max() == 0:
        new[0] = 1
    print(f"[shape] seed {seed}: Hq {Hkv * G} Hkv {Hkv} d {d} new {new.tolist()} ctx {ctx.tolist()}", flush=True)
    run_chunk_steps(custom_workload(f"rand-chunk-{seed}", ctx + new, ctx, Hkv * G, Hkv, d, "prefill", seed=8000 + seed))


def test_fused_chunk_step_small_splits_and_general_chunks():
    import paper_2507_11830_amd as sp

    new = np.array([4, 4, 4, 4, 4, 4, 4, 4])
    ctx = np.array([124, 125, 126, 127, 128, 129, 380, 1])
    sp.sp_debug_set_tuning("decode_chunk", 128)
    try:
        run_chunk_steps(custom_workload("chunkstep-128", ctx + new, ctx, 8, 1, 128, "prefill", seed=65))
        run_chunk_steps(custom_workload("chunkstep-128-2t", ctx + 2 * new - 1, ctx, 8, 1, 128, "prefill", seed=66))
    finally:
        sp.sp_debug_set_tuning("decode_chunk", 0)
    # chunks too long for the short-chunk path: the call is sp_kv_append + sp_attn_prefill
    run_chunk_steps(custom_workload("chunkstep-long", [300, 45, 1000], [100, 0, 990], 8, 1, 128, "prefill", seed=67))
    run_chunk_steps(W.spec_verify())


def test_spec_verify_bench_shape_full_size():
    """The 64-sequence, 4-token verification batch bench.py times, every output element."""
    run_full_compare(W.spec_verify(), check_cache=False)


def test_short_chunks_with_small_splits():
    """128-key splits put a split boundary inside or next to every chunk."""
    import paper_2507_11830_amd as sp

    new = np.array([4, 4, 4, 4, 4, 4, 4, 4])
    ctx = np.array([124, 125, 126, 127, 128, 129, 380, 1])
    sp.sp_debug_set_tuning("decode_chunk", 128)
    try:
        run_full_compare(custom_workload("short-128", ctx + new, ctx, 8, 1, 128, "prefill", seed=62))
        run_full_compare(custom_workload("short-128-2t", ctx + 2 * new - 1, ctx, 8, 1, 128, "prefill", seed=63))
    finally:
        sp.sp_debug_set_tuning("decode_chunk", 0)


def test_decode_with_empty_sequences():
    import torch
    import paper_2507_11830_amd as sp

    w = custom_workload("decode-empty", [40, 7], [39, 6], 8, 1, 128, "decode", seed=32)
    g, o = GpuRunner(w), OracleRunner(w)
    for st in w.steps():
        g.append(st)
        o.append(st)
    seq_lens = np.array([40, 0], np.int32)
    q = to_dev(st.q)
    out = torch.full_like(q, 7.0)
    ws = torch.empty(sp.sp_attn_decode_workspace_size(2, 40, 8, 128), dtype=torch.uint8, device="cuda")
    sp.sp_attn_decode(g.cache, q, out, dev_i32(seq_lens), g.bt, 40, float(w.scale), ws)
    got = bits_of(out)
    want = o.o.attn_decode(o.kp, o.vp, st.q, seq_lens, w.block_table, w.scale)
    assert (got[1] == 0).all()
    assert report_err("decode-empty", got, want) <= TOL
    # all sequences empty: max_seq_len = 0, no workspace needed
    out2 = torch.full_like(q, 7.0)
    sp.sp_attn_decode(g.cache, q, out2, dev_i32([0, 0]), g.bt, 0, float(w.scale), None)
    assert (bits_of(out2) == 0).all()


def test_decode_equals_prefill_row_on_gpu():
    """The two modes read the same cache and agree: decode at length t vs prefill row t-1."""
    import torch
    import paper_2507_11830_amd as sp

    w = W.c2_prefill(batch=2, seqlen=700)
    g = GpuRunner(w)
    st = next(w.steps())
    g.append(st)
    full = W.bf16_bits_to_f64(g.attend(st))
    ws = torch.empty(sp.sp_attn_decode_workspace_size(2, 700, w.Hq, w.d), dtype=torch.uint8, device="cuda")
    for t in (1, 16, 333, 700):
        qd = np.stack([st.q[st.cu_new[s] + t - 1] for s in range(2)])
        out = torch.empty((2, w.Hq, w.d), dtype=torch.bfloat16, device="cuda")
        sp.sp_attn_decode(g.cache, to_dev(qd), out, dev_i32([t, t]), g.bt, t, float(w.scale), ws)
        dec = W.bf16_bits_to_f64(bits_of(out))
        ref = np.stack([full[st.cu_new[s] + t - 1] for s in range(2)])
        assert np.abs(dec - ref).max() <= TOL


def test_results_are_bitwise_reproducible():
    w = custom_workload("repro", [777, 300], [100, 0], 8, 1, 128, "prefill", seed=41)
    g = GpuRunner(w)
    last = None
    for st in w.steps():
        g.append(st)
        last = st
    a, b = g.attend(last), g.attend(last)
    assert np.array_equal(a, b)
    w2 = custom_workload("repro-d", [3000, 900], [2999, 899], 8, 1, 128, "decode", seed=42)
    g2 = GpuRunner(w2)
    for st in w2.steps():
        g2.append(st)
        last = st
    assert np.array_equal(g2.attend(last), g2.attend(last))


# ------------------------------------------------------------------ the five configurations
def test_c1_tiny_gqa_every_step():
    run_full_compare(W.c1_tiny())


def test_c2_70b_prefill_full():
    run_full_compare(W.c2_prefill())


def test_c3_70b_decode_full():
    run_full_compare(W.c3_decode())


def test_c4_mixed_chunked_scaled_full():
    """Same recipe at 1/4 of the lengths: every element of every chunk step compared."""
    run_full_compare(W.c4_chunked(batch=12, median=375.0, lo=16, hi=2048, chunk=128))


def test_c4_mixed_chunked_full_size():
    """C4 at its stated size (32 lognormal sequences, half cached, the rest in 512-token chunk
    steps): every element of every step's output, and the final cache image."""
    run_full_compare(W.c4_chunked())


@pytest.fixture(scope="module")
def c5_long_run():
    """C5a on the GPU, once per module: append + one 32768-token causal prefill in the launch shape
    bench.py times.  The oracle side of the comparison is cut into row ranges by the tests below so
    that no single test runs for minutes."""
    w = W.c5_long(decode_steps=256)
    g, o = GpuRunner(w), OracleRunner(w)
    steps = w.steps()
    st = next(steps)
    g.append(st)
    o.append(st)
    out = g.attend(st)
    return {"w": w, "g": g, "o": o, "steps": steps, "prefill": st, "out": out}


@pytest.mark.parametrize("part", range(6))
def test_c5a_long_prefill_every_row(c5_long_run, part):
    """Every one of the 32768 x 8 output rows of C5a against the oracle, in six row ranges of equal
    oracle work (a range is a chunk on a cached prefix for the oracle: the same rows, by the
    chunked == monolithic property its pins establish)."""
    import oracle

    r = c5_long_run
    w, st, o = r["w"], r["prefill"], r["o"]
    T = int(st.new_lens[0])
    edges = [int(round(T * np.sqrt(k / 6.0) / 16)) * 16 for k in range(7)]   # equal areas under the causal triangle
    lo, hi = edges[part], edges[part + 1]
    want = oracle.attn_prefill(o.kp, o.vp, st.q[lo:hi], np.array([0, hi - lo], np.int32), np.array([lo], np.int32),
                               w.block_table, w.scale)
    assert report_err(f"C5a rows {lo}..{hi - 1}", r["out"][lo:hi], want) <= TOL


def test_c5b_all_decode_steps_on_the_prefilled_cache(c5_long_run):
    """All 256 decode steps on the SAME cache and block table the 32768-token prefill filled: every
    step against the oracle; the pages written by the prefill are byte-identical before and after
    the decode phase, and the final cache image equals the oracle's."""
    r = c5_long_run
    w, g, o = r["w"], r["g"], r["o"]
    full_pages = w.block_table[0, : 32768 // 16]
    gk, gv = g.cache_bits()
    h0 = hashlib.sha256(gk[full_pages].tobytes() + gv[full_pages].tobytes()).hexdigest()
    worst, n = 0.0, 0
    for i, st in enumerate(r["steps"]):
        g.append(st)
        o.append(st)
        got, want = W.bf16_bits_to_f64(g.attend(st)), o.attend(st)
        assert np.isfinite(got).all()
        worst = max(worst, float(np.abs(got - want).max()))
        n += 1
    assert n == 256
    print(f"[parity] C5b: 256 decode steps, max abs err {worst:.5f}", flush=True)
    gk, gv = g.cache_bits()
    assert hashlib.sha256(gk[full_pages].tobytes() + gv[full_pages].tobytes()).hexdigest() == h0
    assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp)
    assert worst <= TOL


def test_c5c_8b_shape_decode_batch():
    run_full_compare(W.c5c_decode_8b(batch=32), check_cache=False)


@pytest.mark.parametrize("kind", ["prefill", "decode"])
def test_large_score_magnitudes(kind):
    """Queries scaled by 16 (exact in bf16): scores of standard deviation ~16, so the softmax is
    nearly one-hot, the running max moves by tens of units between tiles and most weights
    underflow — the lazy-rescale threshold and the exp2 range at work.  On such rows the bf16
    rounding of the one dominant weight (relative 2^-8 at worst) no longer averages out, so the
    bound is elementwise: 2^-8 * sum_j w_j |v_j| (from a second oracle run on |V|), plus the
    output's own half ulp, plus accumulation slack."""
    lens = np.array([700, 65, 2100, 1])
    ctx = np.array([100, 0, 1500, 0]) if kind == "prefill" else lens - 1
    w = custom_workload(f"peaky-{kind}", lens, ctx, 8, 1, 128, kind, seed=97)
    inner = w.make_steps

    def gen():
        for st in inner():
            if st.q is not None:
                nz = (st.q & 0x7FFF) != 0
                st.q = np.where(nz, st.q + np.uint16(4 << 7), st.q).astype(np.uint16)   # exponent + 4: x 16
            yield st

    w.make_steps = gen
    g, o, oabs = GpuRunner(w), OracleRunner(w), OracleRunner(w)
    for st in w.steps():
        g.append(st)
        o.append(st)
        v_signed = st.v_new
        st.v_new = (v_signed & np.uint16(0x7FFF)).astype(np.uint16)   # second oracle run on |V|: sum_j w_j |v_j|
        oabs.append(st)
        st.v_new = v_signed
        if st.kind == "fill":
            continue
        got, want, wabs = W.bf16_bits_to_f64(g.attend(st)), o.attend(st), oabs.attend(st)
        assert np.isfinite(got).all()
        half_ulp = 2.0 ** -8 * 2.0 ** np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -7)))
        bound = 2.0 ** -8 * wabs + half_ulp + 1e-3
        err = np.abs(got - want)
        print(f"[parity] {w.name}: max abs err {err.max():.5f}, max err/bound {(err / bound).max():.3f}", flush=True)
        assert (err <= bound).all()


def test_decode_step_in_a_hip_graph():
    """The library only enqueues work (no allocation, no synchronisation), so a decode step can be
    captured in a HIP graph: capture sp_decode_step once, replay it several times on fresh inputs
    with ordinary eager work and synchronisations in between, and compare every replay with the
    eager call and the oracle."""
    import torch
    import paper_2507_11830_amd as sp

    lens = np.array([700, 33, 1, 2049, 513])
    w = custom_workload("graph-step", lens, lens - 1, 8, 1, 128, "decode", seed=95)
    g, o = GpuRunner(w), OracleRunner(w)
    steps = list(w.steps())
    fill, dec = steps[0], steps[1]
    g.append(fill)
    o.append(fill)
    o.append(dec)
    want = o.attend(dec)
    k_new, v_new, q = to_dev(dec.k_new), to_dev(dec.v_new), to_dev(dec.q)
    sl = dev_i32(dec.seq_lens)
    mx = int(dec.seq_lens.max())
    ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, w.Hq, w.d), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)
    # eager call first: also performs the one-time kernel attribute set-up outside the capture
    sp.sp_decode_step(g.cache, k_new, v_new, q, out, sl, g.bt, mx, float(w.scale), ws)
    torch.cuda.synchronize()
    eager = bits_of(out).copy()
    assert np.abs(W.bf16_bits_to_f64(eager) - want).max() <= TOL
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sp.sp_decode_step(g.cache, k_new, v_new, q, out, sl, g.bt, mx, float(w.scale), ws)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        out.zero_()
        ws.random_(0, 255)                       # stale workspace contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(out), eager), f"replay {rep} differs from the eager result"
    gk, gv = g.cache_bits()
    assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp)


def test_mixed_batch_split_into_two_calls():
    """A batch of single-token sequences followed by prefill chunks, attended in two calls on
    sub-ranges of the same metadata arrays (offset pointers; q / out and the token offsets in
    cu_seqlens_q stay global): the decode-like part takes the short-chunk path, the chunks the
    prefill kernel.  Same result as the oracle's one pass over the whole batch."""
    import torch
    import paper_2507_11830_amd as sp

    new = np.array([1, 1, 1, 1, 1, 1, 300, 64])
    ctx = np.array([700, 33, 4000, 2049, 15, 0, 100, 1500])
    n = 6
    w = custom_workload("mixed-split", ctx + new, ctx, 8, 1, 128, "prefill", seed=97)
    g, o = GpuRunner(w), OracleRunner(w)
    for st in w.steps():
        g.append(st)
        o.append(st)
    want = o.attend(st)
    q = to_dev(st.q)
    out = torch.full_like(q, float("nan"))
    cu, cx = dev_i32(st.cu_new), dev_i32(st.ctx_lens)
    total = q.shape[0]
    for lo, hi in ((n, len(new)), (0, n)):   # in either order: a call writes its own sequences' rows only
        mq, mkv = int(st.new_lens[lo:hi].max()), int(st.seq_lens[lo:hi].max())
        need = sp.sp_attn_prefill_workspace_size(hi - lo, total, mq, mkv, w.Hq, w.Hkv, w.d)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        sp.sp_attn_prefill(g.cache, q, out, cu[lo:hi + 1], cx[lo:hi], g.bt[lo:hi], mq, mkv, float(w.scale), workspace=ws)
    torch.cuda.synchronize()
    assert report_err("mixed batch in two calls", bits_of(out), want) <= TOL


MIXED_CASES = {
    # name: (Hq, Hkv, d, new tokens per sequence, cached tokens per sequence)
    # single-token sequences and chunks in one batch; 4 tokens still fit the split kernel's column
    # tile at 8 heads per KV head, 5 do not
    "decodes+chunk": (8, 1, 128, [1, 1, 1, 1, 1, 1, 300, 1], [700, 33, 4000, 2049, 15, 0, 100, 1500]),
    "cap-boundary": (8, 1, 128, [4, 5, 1, 0, 4, 600, 2, 3], [1000, 1000, 77, 50, 0, 0, 3333, 4095]),
    "two-chunks": (8, 1, 128, [1, 257, 1, 1, 1, 512, 1, 1, 1, 1], [5000, 300, 129, 64, 8191, 1024, 1, 2, 3, 4]),
    "g4-8b": (32, 8, 128, [8, 1, 9, 400, 2], [700, 2049, 64, 130, 999]),
    "d64": (8, 2, 64, [1, 1, 130, 1], [333, 1025, 200, 0]),
    "chunk-first": (8, 1, 128, [700, 1, 1, 1], [0, 900, 901, 902]),
}


@pytest.mark.parametrize("case", sorted(MIXED_CASES))
def test_mixed_batch_in_one_call(case):
    """A continuous-batching step — sequences with a few query tokens next to sequences with long
    chunks — in ONE sp_attn_prefill call: with a workspace the library serves the short sequences
    on the split kernel and the others on the prefill kernel.  Every output row against the oracle;
    the same through sp_chunk_step (cache image too); rows of `out` outside the batch untouched."""
    import torch
    import paper_2507_11830_amd as sp

    Hq, Hkv, d, new, ctx = MIXED_CASES[case]
    new, ctx = np.array(new), np.array(ctx)
    w = custom_workload(f"mixed-{case}", ctx + new, ctx, Hq, Hkv, d, "prefill", seed=141)
    total, mq, mkv = int(new.sum()), int(new.max()), int((ctx + new).max())
    need = sp.sp_attn_prefill_workspace_size(len(new), total, mq, mkv, Hq, Hkv, d)
    assert need > 0                                  # the hints identify the batch as mixed
    run_full_compare(w)
    run_chunk_steps(w)
    # a too small workspace only changes the launch shape, not the result
    g, o = GpuRunner(w), OracleRunner(w)
    g.prefill_workspace = False
    for st in w.steps():
        g.append(st)
        o.append(st)
    assert report_err(f"{w.name} without workspace", g.attend(st), o.attend(st)) <= TOL


def test_chunk_step_in_a_hip_graph():
    """The same for sp_chunk_step on a verification batch (append fused into the attention launch):
    captured once, replayed with stale workspace and output contents, every replay equal to the
    eager result, cache image equal to the oracle's."""
    import torch
    import paper_2507_11830_amd as sp

    new = np.array([4, 2, 3, 4, 1])
    ctx = np.array([700, 33, 0, 2049, 510])
    w = custom_workload("graph-chunk", ctx + new, ctx, 8, 1, 128, "prefill", seed=96)
    g, o = GpuRunner(w), OracleRunner(w)
    fill, st = list(w.steps())
    g.append(fill)
    o.append(fill)
    o.append(st)
    want = o.attend(st)
    k_new, v_new, q = to_dev(st.k_new), to_dev(st.v_new), to_dev(st.q)
    cu, cx = dev_i32(st.cu_new), dev_i32(st.ctx_lens)
    mq, mkv = int(st.new_lens.max()), int(st.seq_lens.max())
    ws = torch.empty(sp.sp_attn_prefill_workspace_size(w.batch, q.shape[0], mq, mkv, w.Hq, w.Hkv, w.d),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)
    call = lambda: sp.sp_chunk_step(g.cache, k_new, v_new, q, out, cu, cx, g.bt, mq, mkv, float(w.scale), workspace=ws)
    call()   # eager first: also the one-time kernel attribute set-up, outside the capture
    torch.cuda.synchronize()
    eager = bits_of(out).copy()
    assert np.abs(W.bf16_bits_to_f64(eager) - want).max() <= TOL
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        out.zero_()
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(out), eager), f"replay {rep} differs from the eager result"
    gk, gv = g.cache_bits()
    assert np.array_equal(gk, o.kp) and np.array_equal(gv, o.vp)


def test_c5c_full_size_every_sequence():
    """C5c at full size in the configuration bench.py times (128 sequences U{1024..16384}, 32q/8kv,
    about 4.7 GB of K/V drawn by torch's seeded GPU generator, the library's own launch shape):
    every output row of every sequence against the oracle, which reads each sequence's pages
    copied back from the device (one copy-back per sequence)."""
    import oracle
    import torch
    import paper_2507_11830_amd as sp

    w = W.c5c_decode_8b()
    lens = w.total_lens
    cache = sp.KVCache.empty(w.num_pages, 8, 128)
    g = torch.Generator(device="cuda").manual_seed(66)
    for pool in (cache.k_pages, cache.v_pages):
        flat = pool.view(-1)
        slab = 1 << 28
        for a in range(0, flat.numel(), slab):
            n = min(slab, flat.numel() - a)
            flat[a:a + n] = torch.randn(n, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((w.batch, 32, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    bt, sl = dev_i32(w.block_table), dev_i32(lens)
    mx = int(lens.max())
    sp.sp_debug_validate_hints(None, sl, 0, 0, mx)
    ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, 32, 128), dtype=torch.uint8, device="cuda")
    sp.sp_attn_decode(cache, q, out, sl, bt, mx, float(w.scale), ws)
    torch.cuda.synchronize()
    got = W.bf16_bits_to_f64(bits_of(out))
    assert np.isfinite(got).all()
    qb = bits_of(q)
    worst, at = 0.0, -1
    for s_ in range(w.batch):
        npages = (int(lens[s_]) + 15) // 16
        pages = torch.from_numpy(w.block_table[s_, :npages].astype(np.int64)).cuda()
        kp, vp = bits_of(cache.k_pages[pages]), bits_of(cache.v_pages[pages])        # [npages, 8, 16, 128]
        bt_local = np.arange(npages, dtype=np.int32)[None, :]
        want = oracle.attn_decode(kp, vp, qb[s_:s_ + 1], np.array([lens[s_]], np.int32), bt_local, w.scale)
        err = float(np.abs(got[s_] - want[0]).max())
        if err > worst:
            worst, at = err, s_
    print(f"[parity] C5c full size, 128 sequences: max abs err {worst:.5f} (sequence {at}, length {int(lens[at])})", flush=True)
    assert worst <= TOL


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_against_oracle(seed):
    """Seeded random batches (head configuration, head_dim, lengths, cached prefixes, empty
    sequences) through prefill, separate decode and the fused decode step, launch shapes left to
    the library's own heuristics."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 8, 16]))
    d = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 9))
    hi = int(rng.choice([40, 300, 1500, 5000]))
    total = rng.integers(1, hi + 1, size=B)
    total[rng.random(B) < 0.15] = 0
    if total.max() == 0:
        total[0] = 7
    ctx = (total * rng.random(B) * (rng.random(B) < 0.7)).astype(np.int64)
    ctx = np.minimum(ctx, np.maximum(total - 1, 0))
    print(f"[shape] seed {seed}: Hq {Hkv * G} Hkv {Hkv} d {d} total {total.tolist()} ctx {ctx.tolist()}", flush=True)
    run_full_compare(custom_workload(f"rand-p-{seed}", total, ctx, Hkv * G, Hkv, d, "prefill", seed=2000 + seed))
    # the same sequences with a chunk of at most 2 * 32 / G tokens each: the short-chunk path
    short = np.minimum(rng.integers(0, 2 * max(32 // min(G, 32), 1) + 1, size=B), total)
    if short.max() > 0:
        run_full_compare(custom_workload(f"rand-s-{seed}", total, total - short, Hkv * G, Hkv, d, "prefill", seed=5000 + seed))
    dec = np.where(total > 0, total, 1)
    run_full_compare(custom_workload(f"rand-d-{seed}", dec, dec - 1, Hkv * G, Hkv, d, "decode", seed=3000 + seed))
    run_fused_steps(custom_workload(f"rand-f-{seed}", dec, dec - 1, Hkv * G, Hkv, d, "decode", seed=4000 + seed))


def test_very_long_context_chunk_and_decode():
    """A 100 000-token cached prefix (1.6 k key tiles, 6 k pages): a 48-token chunk prefilled on it
    (key range cut into the maximum number of pieces) and a fused decode step after it (782 splits,
    combine in four batches), both against the oracle."""
    lens = np.array([100048])
    w = custom_workload("long-100k", lens, lens - 48, 8, 1, 128, "prefill", seed=91)
    run_full_compare(w)
    lens = np.array([100001, 70000])
    run_fused_steps(custom_workload("long-100k-decode", lens, lens - 1, 8, 1, 128, "decode", seed=92))


# ------------------------------------------------------------------ head exchange permutations
@pytest.mark.parametrize("T,H,d,P", [(1000, 64, 128, 8), (777, 8, 128, 8), (513, 8, 64, 2), (1, 6, 128, 3), (300, 32, 128, 1)])
def test_ulysses_pack_unpack_bit_exact(T, H, d, P):
    """The local halves of the SP-mode head exchange: bit-exact against the oracle's index-by-index
    permutation, canaries around the destination untouched, unpack(pack(x)) == x on the GPU."""
    import oracle
    import torch
    import paper_2507_11830_amd as sp

    rng = np.random.default_rng(90 + T)
    x = rng.integers(0, 65536, size=(T, H, d)).astype(np.uint16)
    want = oracle.ulysses_pack(x, P)
    xd = to_dev(x)
    guard = 64
    buf = torch.full((P * T * (H // P) * d + 2 * guard,), W.CANARY, dtype=torch.int16, device="cuda")
    send = buf[guard:-guard].view(torch.bfloat16).view(P, T, H // P, d)
    sp.sp_ulysses_pack(xd, send, P)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(send), want)
    edges = buf.cpu().numpy().view(np.uint16)
    assert (edges[:guard] == 0x7FC0).all() and (edges[-guard:] == 0x7FC0).all()
    y = torch.empty_like(xd)
    sp.sp_ulysses_unpack(send, y)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y), x)
    assert np.array_equal(bits_of(y), oracle.ulysses_unpack(want))
