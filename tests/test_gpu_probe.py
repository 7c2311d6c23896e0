"""The matrix-pipe probe (measurement aid): it must really multiply the caller's data, or the rate bench.py
reports from it would mean nothing.  Checked against a float64 evaluation of what its MFMAs add up to."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


def test_probe_multiplies_the_operands_it_is_given():
    from paper_2505_24133_amd import rkv
    g = torch.Generator().manual_seed(5)
    host = torch.randn(rkv.RKV_PROBE_OPERAND_BYTES // 2, generator=g).bfloat16()
    ops = host.cuda()
    sink = torch.full((rkv.RKV_PROBE_SINK_BYTES // 4,), float("nan"), device="cuda")
    chains = 3
    flops = rkv.rkv_probe_mfma(ops, sink, chains)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    blocks = 2 * cus
    assert flops == blocks * 4 * chains * 8 * 2 * 32 * 32 * 16
    out = sink.cpu().numpy().astype(np.float64)
    assert np.isfinite(out[: blocks * 256]).all() and np.isnan(out[blocks * 256:]).all()
    # Sum of a wave's 64 outputs = sum of all 32 x 32 accumulator elements
    #   = chains * sum_kk  colsum(A_kk) . colsum(B_kk),  lane l holding row l % 32, columns 8 (l / 32) .. + 7
    frag = host.float().numpy().astype(np.float64).reshape(4096, 8)
    for block in (0, 1, blocks - 1):
        for wave in range(4):
            t = wave * 64 + np.arange(64)
            want = 0.0
            for i in range(8):
                fa = (t * 5 + i * 37 + block * 11) & 4095
                fb = (t * 7 + i * 53 + block * 3 + 2048) & 4095
                a, b = frag[fa], frag[fb]                          # [64 lanes, 8]
                ca = np.concatenate([a[:32].sum(0), a[32:].sum(0)])   # column sums over the 32 rows, 16 columns
                cb = np.concatenate([b[:32].sum(0), b[32:].sum(0)])
                want += float(ca @ cb)
            want *= chains
            got = out[block * 256 + wave * 64: block * 256 + wave * 64 + 64].sum()
            scale = chains * 8 * 32 * 32 * 4.0                     # sum of |terms| is of this order
            assert abs(got - want) <= 1e-5 * scale, (block, wave, got, want)
    # a second launch gives the same bits
    sink2 = torch.zeros_like(sink)
    rkv.rkv_probe_mfma(ops, sink2, chains)
    torch.cuda.synchronize()
    assert torch.equal(sink[: blocks * 256], sink2[: blocks * 256])
