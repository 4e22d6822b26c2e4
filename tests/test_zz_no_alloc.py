"""The allocation-free decode entry point (sp_attn_decode_static: partials in a static device
array of the library) against sp_attn_decode on the same inputs, through the C ABI."""
import ctypes

import numpy as np
import pytest

import workloads as W
from harness import TOL, GpuRunner, OracleRunner, bits_of, dev_i32, to_dev

pytestmark = pytest.mark.gpu


def _decode_batch(lens, seed, Hq=8, Hkv=1, d=128):
    lens = np.asarray(lens, np.int32)
    rng = np.random.default_rng(seed)
    bt, pool = W.make_block_table(rng, lens)

    def gen():
        r = np.random.default_rng(seed + 1)
        yield W._chunk_step(r, "fill", lens - 1, np.zeros_like(lens), Hq, Hkv, d)
        yield W._chunk_step(r, "decode", np.ones_like(lens), lens - 1, Hq, Hkv, d)

    return W.Workload(f"static-{seed}", Hq, Hkv, d, pool, bt, lens, gen)


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    """Two calls in a row, the second on a smaller batch (fewer sequences, shorter contexts, so
    fewer splits: the array still holds the first call's partials where the second writes none):
    each equals sp_attn_decode bit for bit and meets the oracle's tolerance."""
    import torch
    import paper_2507_11830_amd as sp

    L = sp.lib()
    for lens, seed in (([3000, 700, 33, 2049, 513, 1, 4096, 129], 201), ([300, 65, 7], 202)):
        w = _decode_batch(lens, seed)
        g, o = GpuRunner(w), OracleRunner(w)
        for st in w.steps():
            g.append(st)
            o.append(st)
        want = o.attend(st)
        q = to_dev(st.q)
        sl = dev_i32(st.seq_lens)
        mx = int(st.seq_lens.max())
        ws = torch.empty(sp.sp_attn_decode_workspace_size(w.batch, mx, w.Hq, w.d), dtype=torch.uint8, device="cuda")
        ref = torch.full_like(q, float("nan"))
        sp.sp_attn_decode(g.cache, q, ref, sl, g.bt, mx, float(w.scale), ws)
        out = torch.full_like(q, float("nan"))
        rc = L.sp_attn_decode_static(ctypes.byref(g.cache.desc), q.data_ptr(), out.data_ptr(), sl.data_ptr(), g.bt.data_ptr(),
                                     w.batch, g.bt.shape[1], mx, w.Hq, float(w.scale),
                                     torch.cuda.current_stream().cuda_stream)
        assert rc == sp.SP_OK, L.sp_last_error()
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(out), bits_of(ref))
        assert np.abs(W.bf16_bits_to_f64(bits_of(out)) - want).max() <= TOL


def test_static_scratch_decode_refuses_shapes_beyond_its_array():
    import torch
    import paper_2507_11830_amd as sp

    w = _decode_batch([40, 7], 203)
    g = GpuRunner(w)
    assert sp.sp_attn_decode_workspace_size(4096, 16384, 32, 128) > 16 << 20
    q = torch.zeros((4096, 32, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sp.SpError) as e:
        sp.sp_attn_decode_static(g.cache, q, q, dev_i32(np.ones(4096)), dev_i32(np.zeros((4096, 1024))), 16384, 0.1)
    assert e.value.status == sp.SP_ERR_WORKSPACE
