"""rkv_compress_static (the entry point that allocates nothing: its scratch is a fixed array inside the
library) against rkv_compress on the same inputs, through the C ABI: two calls in a row, the second on a
smaller input, every output bit for bit; a shape beyond the fixed scratch is refused with nothing written."""
import numpy as np
import pytest
import torch

from paper_2505_24133_amd import rkv, synth

pytestmark = pytest.mark.gpu


def _dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def _shape(w):
    return rkv.Shape(num_problems=w.num_problems, kv_heads=w.kv_heads, q_heads=w.q_heads, n_tokens=w.n_tokens,
                     budget=w.budget, alpha=w.alpha, pool_w=w.pool_w, beta=w.beta, sim_threshold=w.sim_threshold,
                     lam=w.lam, eps=w.eps)


def test_static_scratch_entry_point_matches_rkv_compress_twice_in_a_row():
    assert torch.cuda.is_available(), "needs the MI355X"
    rkv.load_library()
    big = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=6)        # 48 heads, N = 1152
    small = synth.Workload("small", 2, 2, 8, 203, 120, seed=5, recipe="rowcopy", redundancy=0.3, copy_noise=0.1)
    for w in (big, small):                                                        # the second call is the smaller one
        shp = _shape(w)
        assert rkv.rkv_workspace_size(shp) <= rkv.RKV_STATIC_SCRATCH_BYTES
        q, k, v = synth.make_batch(w)
        qd, kd, vd = _dev(q), _dev(k), _dev(v)
        print(f"[gpu-case] rkv_compress_static vs rkv_compress: {w.name} P={w.num_problems} N={w.n_tokens}", flush=True)
        st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kd, vd, want_idx=True, want_score=True)
        ko2, vo2 = torch.zeros_like(ko), torch.zeros_like(vo)
        idx2, score2 = torch.zeros_like(idx), torch.zeros_like(score)
        st2 = rkv.rkv_compress_static(shp, qd, kd, vd, ko2, vo2, idx2, score2)
        torch.cuda.synchronize()
        assert st == st2 == rkv.RKV_OK
        assert torch.equal(idx, idx2) and torch.equal(score, score2), f"{w.name}: indices or scores differ"
        assert torch.equal(ko, ko2) and torch.equal(vo, vo2), f"{w.name}: compacted rows differ"
    # too large for the fixed scratch: refused, outputs untouched
    huge = synth.scaled(synth.CONFIGS["cfg3_llama8b_b4096"], num_problems=32)
    shp = _shape(huge)
    assert rkv.rkv_workspace_size(shp) > rkv.RKV_STATIC_SCRATCH_BYTES
    one = torch.zeros((1,), dtype=torch.bfloat16, device="cuda")                  # never dereferenced
    prm = shp.params()
    import ctypes
    s = rkv.load_library().rkv_compress_static(ctypes.byref(prm), one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                               one.data_ptr(), one.data_ptr(), None, None, None)
    assert s == rkv.RKV_ERR_WORKSPACE
    # not triggered: nothing to do, nothing looked up
    calm = rkv.Shape(num_problems=1, kv_heads=2, q_heads=8, n_tokens=256, budget=256)
    prm = calm.params()
    s = rkv.load_library().rkv_compress_static(ctypes.byref(prm), one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                               one.data_ptr(), one.data_ptr(), None, None, None)
    assert s == rkv.RKV_NOT_TRIGGERED
