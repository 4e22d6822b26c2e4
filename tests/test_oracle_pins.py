"""Pins for the fp64 oracle: each test fixes it to something other than itself — a dense
numpy brute force written independently, torch's fp64 SDPA, closed forms and invariants of
softmax attention.  A dropped term, wrong sign, transposed operand, off-by-one in the causal
bound, wrong GQA map or wrong slot formula fails at least one of them."""
import numpy as np
import pytest

import workloads as W

PAGE = 16


def rng_for(tag):
    return np.random.default_rng(sum((i + 1) * ord(c) for i, c in enumerate(tag)))


def bits(rng, shape, scale=1.0):
    return W.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def f64(b):
    return W.bf16_bits_to_f64(b)


def dense_attention(q, k, v, ctx, scale):
    """Independent brute force: full score matrix, tril mask, exp, divide, matmul.
    q: [n, Hq, d] (positions ctx..ctx+n-1), k, v: [L, Hkv, d] floats, L >= ctx+n."""
    n, Hq, d = q.shape
    L, Hkv, _ = k.shape
    G = Hq // Hkv
    out = np.zeros((n, Hq, d))
    for h in range(Hq):
        S = scale * (q[:, h, :] @ k[:, h // G, :].T)           # [n, L]
        visible = np.tril(np.ones((n, L), dtype=bool), k=ctx)   # j <= ctx + i
        S = np.where(visible, S, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        out[:, h, :] = (E / E.sum(axis=1, keepdims=True)) @ v[:, h // G, :]
    return out


def paged_setup(oracle, rng, lens, Hkv, d, k_bits=None, v_bits=None, pool_factor=1.25):
    """Build a cache image holding sequences of the given lengths.  Returns
    (k_pages, v_pages, block_table, k_list, v_list) where k_list[s] is [L_s, Hkv, d] bits."""
    lens = np.asarray(lens, dtype=np.int32)
    bt, pool = W.make_block_table(rng, lens, pool_factor)
    kp = np.full((pool, Hkv, PAGE, d), W.CANARY, np.uint16)
    vp = np.full((pool, Hkv, PAGE, d), W.CANARY, np.uint16)
    T = int(lens.sum())
    k_new = bits(rng, (T, Hkv, d)) if k_bits is None else k_bits
    v_new = bits(rng, (T, Hkv, d)) if v_bits is None else v_bits
    cu = np.zeros(len(lens) + 1, np.int32)
    cu[1:] = np.cumsum(lens)
    oracle.kv_append(kp, vp, k_new, v_new, cu, np.zeros(len(lens), np.int32), bt)
    ks = [k_new[cu[s]:cu[s + 1]] for s in range(len(lens))]
    vs = [v_new[cu[s]:cu[s + 1]] for s in range(len(lens))]
    return kp, vp, bt, ks, vs, cu


# ------------------------------------------------------------------ P1 brute force
@pytest.mark.parametrize("L,Hq,Hkv,d", [(1, 1, 1, 4), (7, 2, 1, 4), (33, 4, 2, 64), (64, 8, 1, 64), (50, 6, 3, 8)])
def test_p1_dense_bruteforce(oracle, L, Hq, Hkv, d):
    rng = rng_for(f"p1-{L}-{Hq}-{Hkv}-{d}")
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q = bits(rng, (L, Hq, d))
    scale = np.float32(1.0 / np.sqrt(d))
    got = oracle.attn_prefill(kp, vp, q, cu, [0], bt, scale)
    want = dense_attention(f64(q), f64(ks[0]), f64(vs[0]), 0, float(scale))
    assert np.abs(got - want).max() <= 1e-12


def test_p1_dense_bruteforce_with_prefix(oracle):
    """Query chunk at positions ctx..ctx+n-1 sees the prefix plus causal within the chunk."""
    rng = rng_for("p1-prefix")
    L, ctx, Hq, Hkv, d = 45, 19, 4, 2, 16
    kp, vp, bt, ks, vs, _ = paged_setup(oracle, rng, [L], Hkv, d)
    n = L - ctx
    q = bits(rng, (n, Hq, d))
    got = oracle.attn_prefill(kp, vp, q, [0, n], [ctx], bt, 0.25)
    want = dense_attention(f64(q), f64(ks[0]), f64(vs[0]), ctx, 0.25)
    assert np.abs(got - want).max() <= 1e-12


# ------------------------------------------------------------------ P2 library routine
@pytest.mark.parametrize("L,Hq,Hkv,d", [(40, 8, 1, 128), (29, 4, 4, 64), (64, 32, 8, 32)])
def test_p2_torch_sdpa_fp64(oracle, L, Hq, Hkv, d):
    import torch

    rng = rng_for(f"p2-{L}-{Hq}")
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q = bits(rng, (L, Hq, d))
    scale = np.float32(1.0 / np.sqrt(d))
    got = oracle.attn_prefill(kp, vp, q, cu, [0], bt, scale)
    G = Hq // Hkv
    tq = torch.from_numpy(f64(q)).permute(1, 0, 2)[None]
    tk = torch.from_numpy(f64(ks[0])).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    tv = torch.from_numpy(f64(vs[0])).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=float(scale))
    want = want[0].permute(1, 0, 2).numpy()
    assert np.abs(got - want).max() <= 1e-10


# ------------------------------------------------------------------ P3 normalisation
def test_p3_weights_sum_to_one(oracle):
    rng = rng_for("p3")
    L, Hkv, d = 70, 1, 32
    ones = np.full((L, Hkv, d), W.f32_to_bf16_bits(np.float32([1.0]))[0], np.uint16)
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d, v_bits=ones)
    q = bits(rng, (L, 2, d))
    out = oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.3)
    assert np.abs(out - 1.0).max() <= 1e-14
    for p in (0, 1, 15, 16, 69):
        _, _, w = oracle.attn_row_paged(kp, vp, bt[0], p, q[p, 1], 0, 0.3)
        assert w.shape == (p + 1,) and (w >= 0).all()
        assert abs(w.sum() - 1.0) <= 1e-14


def test_p3_constant_value_vector(oracle):
    rng = rng_for("p3c")
    L, Hkv, d = 37, 2, 8
    c = bits(rng, (1, Hkv, d))
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d, v_bits=np.repeat(c, L, axis=0))
    q = bits(rng, (L, 4, d))
    out = oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.5)
    want = np.repeat(f64(c)[0], 2, axis=0)[None]          # head h reads kv head h // 2
    assert np.abs(out - want).max() <= 1e-14


# ------------------------------------------------------------------ P4 causal invariance
def test_p4_future_tokens_do_not_matter(oracle):
    rng = rng_for("p4")
    n, extra, Hq, Hkv, d = 41, 23, 4, 2, 16
    k_all, v_all, q_all = bits(rng, (n + extra, Hkv, d)), bits(rng, (n + extra, Hkv, d)), bits(rng, (n + extra, Hq, d))
    bt = np.arange(8, dtype=np.int32)[None, ::-1].copy()
    outs = []
    for L in (n, n + extra):
        kp = np.full((8, Hkv, PAGE, d), W.CANARY, np.uint16)
        vp = kp.copy()
        oracle.kv_append(kp, vp, k_all[:L], v_all[:L], [0, L], [0], bt)
        outs.append(oracle.attn_prefill(kp, vp, q_all[:L], [0, L], [0], bt, 0.25))
    assert np.array_equal(outs[0], outs[1][:n])


# ------------------------------------------------------------------ P5 closed forms
def test_p5_row0_and_running_mean(oracle):
    rng = rng_for("p5")
    L, Hq, Hkv, d = 50, 2, 1, 16
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q = bits(rng, (L, Hq, d))
    out = oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.25)
    assert np.array_equal(out[0, 0], f64(vs[0])[0, 0])        # row 0 sees only itself
    zero_q = np.zeros((L, Hq, d), np.uint16)
    out0 = oracle.attn_prefill(kp, vp, zero_q, cu, [0], bt, 0.25)
    v = f64(vs[0])[:, 0, :]
    mean = np.cumsum(v, axis=0) / np.arange(1, L + 1)[:, None]
    assert np.abs(out0[:, 0, :] - mean).max() <= 1e-13
    assert np.abs(out0[:, 1, :] - mean).max() <= 1e-13


# ------------------------------------------------------------------ P6 chunked == monolithic
def test_p6_chunked_equals_monolithic(oracle):
    rng = rng_for("p6")
    L, Hq, Hkv, d = 77, 4, 1, 32
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q = bits(rng, (L, Hq, d))
    mono = oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.2)
    parts, at = [], 0
    for n in (5, 16, 31, 25):
        parts.append(oracle.attn_prefill(kp, vp, q[at:at + n], [0, n], [at], bt, 0.2))
        at += n
    assert at == L
    assert np.array_equal(mono, np.concatenate(parts, axis=0))


# ------------------------------------------------------------------ P7 decode == prefill row
def test_p7_decode_equals_prefill_row(oracle):
    rng = rng_for("p7")
    lens = [33, 1, 64, 17]
    Hq, Hkv, d = 4, 2, 16
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, lens, Hkv, d)
    q = bits(rng, (int(sum(lens)), Hq, d))
    full = oracle.attn_prefill(kp, vp, q, cu, np.zeros(4), bt, 0.25)
    for t in (1, 8, 17):
        sel = [s for s in range(4) if lens[s] >= t]
        qd = np.stack([q[cu[s] + t - 1] for s in sel])
        dec = oracle.attn_decode(kp, vp, qd, [t] * len(sel), bt[sel], 0.25)
        for i, s in enumerate(sel):
            assert np.array_equal(dec[i], full[cu[s] + t - 1])
    qd = np.stack([q[cu[s + 1] - 1] for s in range(4)])
    dec = oracle.attn_decode(kp, vp, qd, lens, bt, 0.25)
    for s in range(4):
        assert np.array_equal(dec[s], full[cu[s + 1] - 1])


# ------------------------------------------------------------------ P8 / P9 paging
@pytest.mark.parametrize("pool_factor", [1.0, 1.25, 3.0])
def test_p8_paged_equals_contiguous(oracle, pool_factor):
    rng = rng_for(f"p8-{pool_factor}")
    lens = [45, 16, 3, 70]                       # partial last pages, an exact page, a tiny one
    Hq, Hkv, d = 4, 2, 8
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, lens, Hkv, d, pool_factor=pool_factor)
    q = bits(rng, (int(sum(lens)), Hq, d))
    paged = oracle.attn_prefill(kp, vp, q, cu, np.zeros(4), bt, 0.35)
    for s, L in enumerate(lens):
        for p in range(L):
            for h in range(Hq):
                o, lse, w = oracle.attn_row_contig(ks[s], vs[s], p, q[cu[s] + p, h], h // 2, 0.35)
                assert np.array_equal(o, paged[cu[s] + p, h])


def test_p9_slot_formula_and_canaries(oracle):
    rng = rng_for("p9")
    lens = np.array([21, 40, 16], np.int32)
    Hkv, d = 2, 8
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, lens, Hkv, d, pool_factor=2.0)
    touched = np.zeros(kp.shape[0] * PAGE, bool)
    kflat = kp.transpose(0, 2, 1, 3).reshape(-1, Hkv, d)   # [slot, Hkv, d]
    vflat = vp.transpose(0, 2, 1, 3).reshape(-1, Hkv, d)
    for s, L in enumerate(lens):
        for j in range(L):
            slot = bt[s, j // PAGE] * PAGE + j % PAGE
            assert not touched[slot]
            touched[slot] = True
            assert np.array_equal(kflat[slot], ks[s][j])
            assert np.array_equal(vflat[slot], vs[s][j])
    assert (kflat[~touched] == W.CANARY).all() and (vflat[~touched] == W.CANARY).all()
    assert touched.sum() == lens.sum()


def test_p9_append_with_prefix_lands_after_it(oracle):
    rng = rng_for("p9b")
    Hkv, d = 1, 4
    bt = np.array([[3, 0, 2]], np.int32)
    kp = np.full((4, Hkv, PAGE, d), W.CANARY, np.uint16)
    vp = kp.copy()
    a, b = bits(rng, (20, Hkv, d)), bits(rng, (9, Hkv, d))
    va, vb = bits(rng, (20, Hkv, d)), bits(rng, (9, Hkv, d))
    oracle.kv_append(kp, vp, a, va, [0, 20], [0], bt)
    before = kp.copy()
    oracle.kv_append(kp, vp, b, vb, [0, 9], [20], bt)
    # tokens 0..15 -> page 3, 16..28 -> page 0 rows 0..12; page 2 and 1 untouched
    assert np.array_equal(kp[3, 0], a[:16, 0]) and np.array_equal(kp[0, 0, :4], a[16:, 0])
    assert np.array_equal(kp[0, 0, 4:13], b[:, 0]) and np.array_equal(vp[0, 0, 4:13], vb[:, 0])
    assert (kp[0, 0, 13:] == W.CANARY).all() and (kp[1] == W.CANARY).all() and (kp[2] == W.CANARY).all()
    assert np.array_equal(kp[3], before[3])
    with pytest.raises(ValueError):
        oracle.kv_append(kp, vp, b, vb, [0, 9], [20], np.array([[3, 9, 2]], np.int32))


# ------------------------------------------------------------------ P10 GQA map
def test_p10_gqa_head_map(oracle):
    rng = rng_for("p10")
    L, Hq, Hkv, d = 30, 8, 4, 8           # groups of 2
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q1 = bits(rng, (L, 1, d))
    q = np.repeat(q1, Hq, axis=1)
    out = oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.3)
    for g in range(Hkv):
        assert np.array_equal(out[:, 2 * g], out[:, 2 * g + 1])
    assert not np.array_equal(out[:, 0], out[:, 2])
    # swapping the contents of KV heads 1 and 2 swaps the outputs of groups 1 and 2
    kp2, vp2 = kp.copy(), vp.copy()
    kp2[:, [1, 2]] = kp[:, [2, 1]]
    vp2[:, [1, 2]] = vp[:, [2, 1]]
    out2 = oracle.attn_prefill(kp2, vp2, q, cu, [0], bt, 0.3)
    perm = [0, 1, 4, 5, 2, 3, 6, 7]
    assert np.array_equal(out2, out[:, perm])


# ------------------------------------------------------------------ P11 split / combine identity
def test_p11_lse_split_combine(oracle):
    rng = rng_for("p11")
    L, Hkv, d = 200, 1, 16
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d)
    q = bits(rng, (1, d))[0]
    p = L - 1
    o, lse, w = oracle.attn_row_paged(kp, vp, bt[0], p, q, 0, 0.25)
    # lse against its definition from independently computed scores
    s = 0.25 * (f64(ks[0])[:, 0, :] @ f64(q))
    assert abs(lse - (s.max() + np.log(np.exp(s - s.max()).sum()))) <= 1e-12
    for trial in range(5):
        nparts = int(rng.integers(2, 6))
        label = rng.integers(0, nparts, size=L)
        label[:nparts] = np.arange(nparts)                  # every part non-empty
        parts = [oracle.attn_row_subset(kp, vp, bt[0], p, label == a, q, 0, 0.25) for a in range(nparts)]
        M = max(l for _, l in parts)
        den = sum(np.exp(l - M) for _, l in parts)
        num = sum(np.exp(l - M) * oa for oa, l in parts)
        assert np.abs(num / den - o).max() <= 1e-12
        assert abs(M + np.log(den) - lse) <= 1e-12


# ------------------------------------------------------------------ P12 stability
def test_p12_shift_invariance_and_large_scores(oracle):
    rng = rng_for("p12")
    L, Hkv, d = 60, 1, 16
    k = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    u = rng.standard_normal((1, 1, d)).astype(np.float32)
    # pick values exactly representable after the shift: quantise both to multiples of 1/8
    k8, u8 = np.round(k * 8) / 8, np.round(u * 8) / 8
    kb, kb_shift = W.f32_to_bf16_bits(k8), W.f32_to_bf16_bits(k8 + u8)
    assert np.array_equal(W.bf16_bits_to_f32(kb_shift), (k8 + u8).astype(np.float32))
    v = bits(rng, (L, Hkv, d))
    q = bits(rng, (L, 2, d))
    outs = []
    for kk in (kb, kb_shift):
        kp, vp, bt, _, _, cu = paged_setup(oracle, np.random.default_rng(5), [L], Hkv, d, k_bits=kk, v_bits=v)
        outs.append(oracle.attn_prefill(kp, vp, q, cu, [0], bt, 0.25))
    assert np.abs(outs[0] - outs[1]).max() <= 1e-12
    # very large scores: no inf / nan, weights still sum to one
    ones = np.full((L, Hkv, d), 0x3F80, np.uint16)
    qbig = W.f32_to_bf16_bits(W.bf16_bits_to_f32(q) * np.float32(30.0))
    kp, vp, bt, _, _, cu = paged_setup(oracle, np.random.default_rng(5), [L], Hkv, d, k_bits=kb, v_bits=ones)
    out, lse = oracle.attn_prefill(kp, vp, qbig, cu, [0], bt, 1.0, return_lse=True)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert np.abs(lse).max() > 80.0
    assert np.abs(out - 1.0).max() <= 1e-14


# ------------------------------------------------------------------ P13 dominating key
def test_p13_dominating_key_selects_its_value(oracle):
    rng = rng_for("p13")
    L, Hkv, d, jstar = 40, 1, 16, 11
    qf = np.zeros(d, np.float32)
    qf[3] = 4.0                                              # |q| = 4, exactly representable
    kf = (rng.standard_normal((L, Hkv, d)) * 0.25).astype(np.float32)
    kf[:, 0, 3] = 0.0                                        # other keys orthogonal to q: score 0
    kf[jstar, 0, :] = 20.0 * qf / 4.0                        # score(j*) = scale * 4 * 20 = 80*scale
    kb = W.f32_to_bf16_bits(kf)
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [L], Hkv, d, k_bits=kb)
    o, lse, w = oracle.attn_row_paged(kp, vp, bt[0], L - 1, W.f32_to_bf16_bits(qf), 0, 0.5)
    gap = 40.0
    assert abs(w[jstar] - 1.0) <= L * np.exp(-gap)
    assert np.abs(o - f64(vs[0])[jstar, 0]).max() <= 10 * L * np.exp(-gap)
    # a row that cannot see j* yet is NOT dominated
    o2, _, w2 = oracle.attn_row_paged(kp, vp, bt[0], jstar - 1, W.f32_to_bf16_bits(qf), 0, 0.5)
    assert np.abs(w2 - 1.0 / jstar).max() <= 1e-15


# ------------------------------------------------------------------ sampled-row driver
def test_sampled_rows_match_full_prefill(oracle):
    rng = rng_for("rows")
    lens = [30, 50]
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, lens, 1, 16)
    ctx = np.array([10, 20], np.int32)
    n = np.array([20, 30], np.int32)
    cuq = np.array([0, 20, 50], np.int32)
    q = bits(rng, (50, 2, 16))
    full = oracle.attn_prefill(kp, vp, q, cuq, ctx, bt, 0.25)
    rs, rt, rh = [0, 0, 1, 1], [0, 19, 5, 29], [0, 1, 1, 0]
    got = oracle.attn_prefill_rows(kp, vp, q, cuq, ctx, bt, 0.25, rs, rt, rh)
    for i in range(4):
        assert np.array_equal(got[i], full[cuq[rs[i]] + rt[i], rh[i]])


@pytest.mark.parametrize("Hq,Hkv", [(6, 2), (8, 4), (12, 3)])
def test_sampled_rows_gqa_head_map(oracle, Hq, Hkv):
    """The sampled-row driver with several KV heads and several query heads per KV head (Hkv >= 2,
    G >= 2): query head h must read KV head h // G, as in the full driver (pinned by P1/P2/P10) and
    as in an independent dense computation of the same rows.  A contiguous-versus-strided head map
    (h % Hkv) gives a different KV head for some sampled head at every shape here."""
    rng = rng_for(f"rows-gqa-{Hq}-{Hkv}")
    G, d = Hq // Hkv, 8
    lens = [23, 41, 17]
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, lens, Hkv, d)
    ctx = np.array([5, 0, 16], np.int32)
    n = np.array(lens, np.int32) - ctx
    cuq = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    q = bits(rng, (int(n.sum()), Hq, d))
    full = oracle.attn_prefill(kp, vp, q, cuq, ctx, bt, 0.4)
    rs, rt, rh = [], [], []
    for s in range(3):                      # every head on a first, a middle and a last row
        for t in (0, int(n[s]) // 2, int(n[s]) - 1):
            for h in range(Hq):
                rs.append(s), rt.append(t), rh.append(h)
    got = oracle.attn_prefill_rows(kp, vp, q, cuq, ctx, bt, 0.4, rs, rt, rh)
    assert any(h // G != h % Hkv for h in rh)
    for i, (s, t, h) in enumerate(zip(rs, rt, rh)):
        assert np.array_equal(got[i], full[cuq[s] + t, h])
        # independent of both drivers: dense softmax over the contiguous K/V of KV head h // G
        p = int(ctx[s]) + t
        kk, vv = f64(ks[s])[: p + 1, h // G], f64(vs[s])[: p + 1, h // G]
        sc = 0.4 * kk @ f64(q[cuq[s] + t, h])
        w = np.exp(sc - sc.max())
        assert np.abs(got[i] - (w / w.sum()) @ vv).max() <= 1e-12


def test_zero_length_sequences_are_noops(oracle):
    rng = rng_for("zero")
    kp, vp, bt, ks, vs, cu = paged_setup(oracle, rng, [20, 0, 5], 1, 8)
    q = bits(rng, (25, 2, 8))
    out = oracle.attn_prefill(kp, vp, q, cu, [0, 0, 0], bt, 0.3)
    a = oracle.attn_prefill(kp, vp, q[:20], [0, 20], [0], bt[:1], 0.3)
    b = oracle.attn_prefill(kp, vp, q[20:], [0, 5], [0], bt[2:], 0.3)
    assert np.array_equal(out, np.concatenate([a, b]))
    qd = np.stack([q[19], q[0], q[24]])
    dec = oracle.attn_decode(kp, vp, qd, [20, 0, 5], bt, 0.3)
    assert (dec[1] == 0).all()
    assert np.array_equal(dec[0], a[19]) and np.array_equal(dec[2], b[4])


def test_two_key_row_is_a_sigmoid(oracle):
    """With two visible keys the weights are (1 - sig, sig), sig = logistic(s_1 - s_0)."""
    import math

    d, Hkv = 1, 1
    vals = np.float32([[0.5], [-1.25]])           # k_0, k_1 (exact in bf16)
    vv = np.float32([[2.0], [-3.0]])
    kb, vb = W.f32_to_bf16_bits(vals).reshape(2, 1, 1), W.f32_to_bf16_bits(vv).reshape(2, 1, 1)
    kp = np.full((1, Hkv, PAGE, d), W.CANARY, np.uint16)
    vp = kp.copy()
    bt = np.zeros((1, 1), np.int32)
    oracle.kv_append(kp, vp, kb, vb, [0, 2], [0], bt)
    qb = W.f32_to_bf16_bits(np.float32([1.5]))
    o, lse, w = oracle.attn_row_paged(kp, vp, bt[0], 1, qb, 0, 0.75)
    x = 0.75 * 1.5 * (-1.25 - 0.5)
    sig = 1.0 / (1.0 + math.exp(-x))
    assert abs(w[1] - sig) <= 1e-15 and abs(w[0] - (1 - sig)) <= 1e-15
    assert abs(o[0] - (2.0 * (1 - sig) - 3.0 * sig)) <= 1e-14
    assert abs(lse - (0.75 * 1.5 * 0.5 + math.log1p(math.exp(x)))) <= 1e-14


# ------------------------------------------------------------------ head exchange permutations
def _tagged(T, H, d):
    """Element (t, h, c) carries its own coordinates: t in the high bits, h and c below."""
    t, h, c = np.meshgrid(np.arange(T), np.arange(H), np.arange(d), indexing="ij")
    return (t * 1024 + h * 32 + c).astype(np.uint16)


@pytest.mark.parametrize("T,H,d,P", [(5, 8, 16, 2), (3, 8, 8, 8), (7, 6, 24, 3), (4, 4, 8, 1)])
def test_p14_ulysses_pack_is_the_head_slice_view(oracle, T, H, d, P):
    """Pack against the library transpose (block j = heads [j*H/P, (j+1)*H/P) of every token),
    against the coordinates each element carries, and unpack as its inverse."""
    x = _tagged(T, H, d)
    send = oracle.ulysses_pack(x, P)
    assert send.shape == (P, T, H // P, d)
    assert np.array_equal(send, x.reshape(T, P, H // P, d).transpose(1, 0, 2, 3))
    for j in range(P):
        for hl in range(H // P):
            blk = send[j, :, hl, :]
            assert ((blk >> 10) == np.arange(T)[:, None]).all()          # token stays in place
            assert (((blk >> 5) & 31) == j * (H // P) + hl).all()          # head slice j, local head hl
            assert ((blk & 31) == np.arange(d)[None, :]).all()            # channels untouched
    assert np.array_equal(oracle.ulysses_unpack(send), x)


def test_p14_ulysses_exchange_end_to_end(oracle):
    """P simulated ranks: pack on every rank, exchange block j of rank i with block i of rank j,
    and the received buffer of rank j read as [T][H/P][d] is the head slice j of the full
    sequence, tokens in rank order; unpack on the way back restores every rank's rows."""
    rng = np.random.default_rng(14)
    P, T_loc, H, d = 4, 6, 8, 16
    full = rng.integers(0, 65536, size=(P * T_loc, H, d)).astype(np.uint16)
    sends = [oracle.ulysses_pack(full[r * T_loc:(r + 1) * T_loc], P) for r in range(P)]
    for j in range(P):
        recv = np.stack([sends[i][j] for i in range(P)])                   # the all-to-all
        assert np.array_equal(recv.reshape(P * T_loc, H // P, d), full[:, j * (H // P):(j + 1) * (H // P), :])
    # the way back: rank j returns to rank i the block of rank i's tokens
    for i in range(P):
        back = np.stack([full[i * T_loc:(i + 1) * T_loc, j * (H // P):(j + 1) * (H // P), :] for j in range(P)])
        assert np.array_equal(oracle.ulysses_unpack(back), full[i * T_loc:(i + 1) * T_loc])


def test_golden_file_still_matches_the_oracle(oracle):
    """tests/golden/c1_oracle_outputs.txt (written by tests/golden/make_golden.py from the oracle
    alone) is a change detector: an edit to the oracle's arithmetic or to the seeded inputs must
    show up here and be justified.  Probe values to 1e-13, cache image by hash."""
    import importlib.util
    import os

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    now = mg.render().splitlines()
    stored = open(os.path.join(here, "c1_oracle_outputs.txt")).read().splitlines()
    assert len(now) == len(stored)
    assert now[1] == stored[1], "cache image changed"
    for a, b in zip(now[2:], stored[2:]):
        fa, fb = a.split(), b.split()
        assert fa[:4] == fb[:4]
        pa, pb = [float(x) for x in fa[5:8]], [float(x) for x in fb[5:8]]
        assert np.allclose(pa, pb, rtol=0, atol=1e-13), (a, b)
