"""The two diagnostic libraries on the GPU: the instrumented kernels of libqnn_timeline.so must give the product
library's results bit for bit (which the parity tests pin to the oracle) and leave ordered timestamps; the
operand-fed MFMA loop of libqnn_probe.so must compute what its operands say."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, pack_levels, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import probe, qnn  # noqa: E402


@pytest.mark.parametrize("fp4", [False, True])
@pytest.mark.parametrize("shape", [(300, 260, 200), (513, 257, 1000)])
def test_timeline_level_gemm_equals_product_and_oracle(fp4, shape):
    rows, cols, n = shape
    bits = 2
    gen = np.random.default_rng(rows + n + fp4)
    a, w = levels(gen, (rows, n), bits), levels(gen, (cols, n), bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    plane_sum = qnn.qnn_plane_sum_fp4 if fp4 else qnn.qnn_plane_sum_i8
    gemm = qnn.qnn_level_gemm_fp4 if fp4 else qnn.qnn_level_gemm_i8
    al, wl_ = plane_sum(pack_levels(a, bits), n), plane_sum(pack_levels(w, bits), n)
    sc = dev(s)
    ref_acc, ref_out = gemm(al, wl_, n, scale=sc)
    acc, out = torch.zeros_like(ref_acc), torch.zeros_like(ref_out)
    blocks = ((rows + 255) // 256) * ((cols + 255) // 256)
    buf = torch.zeros((blocks * 8, 6), dtype=torch.int64, device="cuda")
    probe.qnn_level_gemm_timeline_set(buf)
    try:
        probe.timeline_level_gemm(al, wl_, rows, cols, n, acc, sc, out, fp4=fp4)
        torch.cuda.synchronize()
    finally:
        probe.qnn_level_gemm_timeline_set(None)
    assert torch.equal(acc, ref_acc) and torch.equal(out, ref_out)
    assert np.array_equal(acc.cpu().numpy(), oracle.gemm(a, w))
    t = buf.cpu().numpy()
    assert (t[:, 0] > 0).all()
    assert (t[:, 0] <= t[:, 1]).all() and (t[:, 1] <= t[:, 2]).all() and (t[:, 2] <= t[:, 3]).all()
    assert (t[:, 4] >= 0).all() and (t[:, 4] <= t[:, 5]).all()
    # a launch after recording was switched off leaves the buffer alone
    before = buf.clone()
    probe.timeline_level_gemm(al, wl_, rows, cols, n, acc, sc, out, fp4=fp4)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)


def test_timeline_conv_equals_product():
    gen = torch.Generator(device="cuda").manual_seed(7)
    B, HW, cin, cout, bits = 3, 17, 64, 96, 2
    ap = torch.randint(-2**31, 2**31 - 1, (bits, B * HW * HW, cin // 32), dtype=torch.int32, device="cuda", generator=gen)
    wp = torch.randint(-2**31, 2**31 - 1, (bits, cout, 3, 3, cin // 32), dtype=torch.int32, device="cuda", generator=gen)
    sc = torch.rand(cout, device="cuda", generator=gen) * 0.01 + 0.001
    ref_acc, ref_out, _ = qnn.qnn_conv2d(ap, wp, (B, HW, HW), cin, 1, 1, scale=sc, want_out=True)
    acc, out = torch.zeros_like(ref_acc), torch.zeros_like(ref_out)
    d = qnn.qnn_conv_desc(B, HW, HW, cin, cout, 3, 3, 1, 1, bits, bits)
    for hint in (True, False):
        buf = torch.zeros((512 * 8, 5), dtype=torch.int64, device="cuda")
        probe.qnn_timeline_set(buf, pair_hint=hint)
        try:
            probe.timeline_conv2d(d, ap, wp, sc, acc, out, None, 0.0, 0)
            torch.cuda.synchronize()
        finally:
            probe.qnn_timeline_set(None)
        assert torch.equal(acc, ref_acc) and torch.equal(out, ref_out)
        t = buf.cpu().numpy()
        t = t[t[:, 0] > 0]
        assert len(t) > 0 and (t[:, 0] <= t[:, 1]).all() and (t[:, 1] <= t[:, 2]).all() and (t[:, 4] > 0).all()
        acc.zero_(), out.zero_()


@pytest.mark.parametrize("mode, byte, per_mfma", [(0, 0x01, 32), (1, 0x22, 64)])
def test_mfma_operand_probe_computes_its_operands(mode, byte, per_mfma):
    # all-ones operands (int8 1, or fp4 1.0 in both nibbles): every MFMA adds k = 32 (64) to each of a lane's
    # 16 accumulator registers; 4 accumulators x 4 MFMAs each per iteration
    wgs, iters = 3, 5
    out = torch.zeros(wgs * 256, dtype=torch.int32, device="cuda")
    clocks = torch.zeros((wgs * 4, 2), dtype=torch.int64, device="cuda")
    ones = torch.full((256 * 8 * 16,), byte, dtype=torch.uint8, device="cuda")
    probe.qnn_probe_mfma_operands(mode, wgs, iters, ones, out, clocks)
    torch.cuda.synchronize()
    assert (out == 4 * 16 * 4 * iters * per_mfma).all()
    assert (clocks > 0).all()
    probe.qnn_probe_mfma_operands(mode, wgs, iters, torch.zeros_like(ones), out)
    torch.cuda.synchronize()
    assert (out == 0).all()
    with pytest.raises(ValueError):
        probe.qnn_probe_mfma_operands(mode, wgs, iters, ones[:100], out)
