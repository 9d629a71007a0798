"""GPU parity of the decoded-level route on the matrix cores (qnn_encode_levels_i8 +
qnn_level_conv2d_i8) against the CPU oracle: identical int32 accumulators, identical levels after
every layer of a fused chain."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, levels, oracle_full_batch

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

RTOL = 1e-5


def _lv(codes_levels):
    return codes_levels.astype(np.int8)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("count", [1, 15, 16, 17, 1000, 4096 * 3 + 5])
def test_encode_levels_matches_oracle(bits, count):
    gen = np.random.default_rng(bits * 1000 + count)
    x = gen.normal(0, 1, size=count).astype(np.float32)
    x[: min(count, 4)] = np.array([0.0, 5.0, -5.0, 1.5], np.float32)[: min(count, 4)]
    clip = 1.5
    got = qnn.qnn_encode_levels_i8(dev(x), clip, bits)
    torch.cuda.synchronize()
    want, _ = oracle.quantize(x, clip, bits)
    assert np.array_equal(got.cpu().numpy(), _lv(want))


def test_encode_levels_bf16():
    gen = np.random.default_rng(5)
    x = torch.from_numpy(gen.normal(0, 1, size=5000).astype(np.float32)).to(torch.bfloat16)
    got = qnn.qnn_encode_levels_i8(x.cuda(), 2.0, 3)
    torch.cuda.synchronize()
    want, _ = oracle.quantize(x.to(torch.float32).numpy(), 2.0, 3)   # bf16 widens exactly
    assert np.array_equal(got.cpu().numpy(), _lv(want))


GEOMS = [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 7, 9, 16, 4, 3, 1, 1),        # one unit per tap, tiny Cout (512 x 64 tile)
    (1, 8, 8, 32, 6, 3, 2, 1),
    (2, 6, 5, 48, 3, 1, 1, 0),        # 1x1: reduction shorter than a stage
    (1, 9, 7, 48, 70, 5, 1, 2),       # 5x5, Cout in the 256 x 128 tile, ragged columns
    (1, 9, 10, 64, 64, 3, 2, 0),
    (3, 4, 4, 16, 5, 3, 1, 2),        # pad 2 with a 3x3 kernel: windows mostly in the padding
    (2, 14, 14, 128, 130, 3, 1, 1),   # 256 x 256 tile, ragged columns, 9 whole stages
    (1, 12, 12, 160, 32, 3, 1, 1),
    (5, 13, 13, 64, 64, 3, 1, 1),     # several row tiles, ragged tail
    (1, 20, 20, 64, 200, 3, 1, 1),    # two row tiles x one column tile of 256
    (2, 24, 24, 32, 300, 3, 1, 1),    # two column tiles of 256, reduction tail of 32 bytes
    (1, 7, 7, 512, 512, 3, 1, 1),     # long reduction (36 stages)
]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (1, 1), (7, 5)])
def test_level_conv_acc_and_out(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    w_bits, a_bits = bits
    if k * k * Cin * ((1 << w_bits) - 1) * ((1 << a_bits) - 1) >= 2 ** 31:
        pytest.skip("int32 range")
    gen = np.random.default_rng(sum(geom) * 10 + w_bits + a_bits)
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    s = gen.uniform(0.01, 0.1, size=Cout).astype(np.float32)
    acc, out, _ = qnn.qnn_level_conv2d_i8(dev(a), dev(w), stride, pad, a_bits, w_bits, scale=dev(s), want_out=True)
    torch.cuda.synchronize()
    want = oracle.conv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=RTOL, atol=0)


@pytest.mark.parametrize("geom", [(2, 9, 9, 64, 64, 3, 1, 1), (1, 10, 10, 32, 100, 3, 2, 1),
                                  (2, 8, 8, 128, 144, 3, 1, 1), (1, 6, 6, 16, 37, 3, 1, 1)])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_level_conv_fused_next_levels(geom, bits):
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(sum(geom) + bits)
    a, w = levels(gen, (B, H, W, Cin), bits), levels(gen, (Cout, k, k, Cin), bits)
    var = (4.0 ** bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var * var)).astype(np.float32)
    acc, out, nxt = qnn.qnn_level_conv2d_i8(dev(a), dev(w), stride, pad, bits, bits, scale=dev(s), want_out=True,
                                            next_clip=2.5, next_bits=bits)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d(a, w, stride, pad)
    lv, _ = oracle.quantize(oracle.scale(want_acc, s), 2.5, bits)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    assert np.array_equal(nxt.cpu().numpy(), _lv(lv))
    # levels only (no acc / out leaves the chip)
    _, _, nxt2 = qnn.qnn_level_conv2d_i8(dev(a), dev(w), stride, pad, bits, bits, scale=dev(s), want_acc=False,
                                         next_clip=2.5, next_bits=bits)
    torch.cuda.synchronize()
    assert np.array_equal(nxt2.cpu().numpy(), _lv(lv))


def test_level_conv_matches_binary_conv():
    # the two machine routes give the same accumulators on the same levels
    from gpu_util import pack_levels
    gen = np.random.default_rng(77)
    a, w = levels(gen, (2, 11, 11, 64, ), 3), levels(gen, (96, 3, 3, 64), 3)
    acc_m, _, _ = qnn.qnn_level_conv2d_i8(dev(a), dev(w), 1, 1, 3, 3)
    acc_b, _, _ = qnn.qnn_conv2d(pack_levels(a, 3), pack_levels(w, 3).view(3, 96, 3, 3, -1), (2, 11, 11), 64, 1, 1)
    torch.cuda.synchronize()
    assert torch.equal(acc_m, acc_b)


def _run_stack_levels(x, layers, keep_acc):
    lv = qnn.qnn_encode_levels_i8(dev(x), layers[0]["clip"], layers[0]["a_bits"])
    trace = []
    for li, L in enumerate(layers):
        last = li + 1 == len(layers)
        acc, out, nxt = qnn.qnn_level_conv2d_i8(
            lv, dev(L["w"]), L["stride"], L["pad"], L["a_bits"], L["w_bits"], scale=dev(L["scale"]),
            want_acc=keep_acc, want_out=last, next_clip=None if last else layers[li + 1]["clip"],
            next_bits=0 if last else layers[li + 1]["a_bits"])
        trace.append({"levels": lv, "acc": acc, "out": out})
        lv = nxt
    torch.cuda.synchronize()
    return trace


def test_config4_resnet18_stack_levels_small_batch():
    c = wl.resnet18_stack(batch=2)
    trace = _run_stack_levels(c["x"], c["layers"], keep_acc=True)
    want = oracle.conv_stack(c["x"], c["layers"])
    for li, (g, o) in enumerate(zip(trace, want)):
        assert np.array_equal(g["levels"].cpu().numpy(), _lv(o["levels"])), li
        assert np.array_equal(g["acc"].cpu().numpy(), o["acc"]), li
    np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want[-1]["out"], rtol=RTOL, atol=0)
    # fused only: nothing but levels between layers
    trace2 = _run_stack_levels(c["x"], c["layers"], keep_acc=False)
    for li, (g, o) in enumerate(zip(trace2, want)):
        assert np.array_equal(g["levels"].cpu().numpy(), _lv(o["levels"])), li


def test_config5_vgg_ssd_stack_levels_small_batch():
    groups = wl.vgg_ssd_stack(batch=1)
    for g in groups:
        trace = _run_stack_levels(g["x"], g["layers"], keep_acc=True)
        want = oracle.conv_stack(g["x"], g["layers"])
        for li, (t, o) in enumerate(zip(trace, want)):
            assert np.array_equal(t["levels"].cpu().numpy(), _lv(o["levels"])), li
            assert np.array_equal(t["acc"].cpu().numpy(), o["acc"]), li


def test_level_conv_argument_errors():
    a = torch.zeros((1, 4, 4, 24), dtype=torch.int8, device="cuda")
    w = torch.zeros((8, 3, 3, 24), dtype=torch.int8, device="cuda")
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_level_conv2d_i8(a, w, 1, 1, 2, 2)
    assert e.value.code == -2          # Cin not a multiple of 16
    a = torch.zeros((1, 8, 8, 16), dtype=torch.int8, device="cuda")
    w = torch.zeros((8, 7, 7, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_level_conv2d_i8(a, w, 1, 3, 2, 2)
    assert e.value.code == -2          # 49 taps


def test_config4_full_batch_levels_every_image():
    # batch 256 as bench.py times the matrix-core route, against the oracle's chain over the whole batch
    c = wl.resnet18_stack()
    trace = _run_stack_levels(c["x"], c["layers"], keep_acc=False)
    (want_levels, want_out), = oracle_full_batch("stack4")
    for li, (g, lv) in enumerate(zip(trace, want_levels)):
        assert np.array_equal(g["levels"].cpu().numpy(), lv), li
    np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want_out, rtol=RTOL, atol=0)


def test_config5_full_batch_levels_every_image():
    for g, (want_levels, want_out) in zip(wl.vgg_ssd_stack(), oracle_full_batch("stack5")):
        trace = _run_stack_levels(g["x"], g["layers"], keep_acc=False)
        for li, (t, lv) in enumerate(zip(trace, want_levels)):
            assert np.array_equal(t["levels"].cpu().numpy(), lv), li
        np.testing.assert_allclose(trace[-1]["out"].cpu().numpy(), want_out, rtol=RTOL, atol=0)
        del trace
        torch.cuda.empty_cache()
