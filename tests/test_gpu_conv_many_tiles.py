"""Binary convolutions with more row tiles than the chip holds workgroups at one time (512 tiles of 64
output pixels), at small channel counts so that the oracle stays fast: every persistent workgroup then
walks two or more row tiles, the last ones ragged.  The cases cover one-stage and multi-stage reductions,
strides, ragged channel counts, several column tiles, the fused next-layer planes, and the residual-block
epilogue, whose shortcut prefetch follows the same walk."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, pack_levels, planes_to_numpy, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402

CASES = [
    # B, H, W, Cin, Cout, k, stride, pad, w_bits, a_bits
    (3, 112, 112, 32, 64, 3, 1, 1, 2, 2),    # 37632 rows = 588 row tiles: 76 workgroups walk two
    (3, 112, 112, 128, 64, 3, 1, 1, 2, 2),   # 36 reduction words: two stages per tile
    (1, 190, 190, 32, 32, 3, 1, 1, 1, 1),    # 36100 rows, last tile ragged
    (1, 193, 191, 40, 70, 3, 1, 1, 1, 3),    # ragged words and channels, rectangular lane tile side
    (2, 300, 290, 64, 33, 3, 2, 1, 3, 1),    # stride 2: 150 x 145 outputs per image
    (5, 100, 100, 96, 64, 1, 1, 0, 2, 1),    # 1x1 kernel, 50000 rows
    (2, 160, 150, 64, 128, 3, 1, 1, 2, 2),   # two column tiles: 256 workgroups per column
    # one-stage reductions with 4 planes in all and ten or more 64-row tiles per resident workgroup: the taller
    # 2 x 4 lane tile is chosen (5120 tiles of 64 rows on a chip that holds 512 workgroups)
    (7, 230, 210, 32, 64, 3, 1, 1, 2, 2),    # 338100 rows, ragged last tile
    (6, 250, 230, 64, 40, 3, 1, 1, 1, 3),    # 345000 rows, ragged channels
    (3, 250, 230, 32, 128, 3, 1, 1, 3, 1),   # two column tiles make up the count
    # one-stage reductions whose waves take their rows from the workgroup's counter, with more tiles than workgroups
    (3, 120, 120, 32, 64, 3, 1, 1, 3, 3),    # 6 planes: 1024-lane workgroups, 338 tiles of 128 rows on 256 of them
    (2, 140, 130, 64, 40, 3, 1, 1, 4, 4),    # 8 planes: 1138 tiles of 32 rows, ragged channels
    (2, 150, 131, 32, 64, 3, 2, 1, 2, 3),    # 5 planes, stride 2, ragged last tile
]


def _setup(case):
    B, H, W, Cin, Cout, k, stride, pad, w_bits, a_bits = case
    gen = np.random.default_rng(sum(case))
    a, w = levels(gen, (B, H, W, Cin), a_bits), levels(gen, (Cout, k, k, Cin), w_bits)
    var = (4.0 ** w_bits - 1) / 3 * (4.0 ** a_bits - 1) / 3
    s = (gen.uniform(0.5, 1.5, size=Cout) / np.sqrt(k * k * Cin * var)).astype(np.float32)
    wp = pack_levels(w, w_bits).view(w_bits, Cout, k, k, -1)
    return gen, a, w, s, wp


@pytest.mark.parametrize("case", CASES)
def test_many_row_tiles_plain(case):
    B, H, W, Cin, Cout, k, stride, pad, w_bits, a_bits = case
    gen, a, w, s, wp = _setup(case)
    acc, out, nxt = qnn.qnn_conv2d(pack_levels(a, a_bits), wp, (B, H, W), Cin, stride, pad, scale=dev(s),
                                   want_out=True, next_clip=2.0, next_bits=2)
    torch.cuda.synchronize()
    want = oracle.conv2d(a, w, stride, pad)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)
    lv, _ = oracle.quantize(oracle.scale(want, s), 2.0, 2)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 2))


@pytest.mark.parametrize("case", CASES[:2] + CASES[3:5])
def test_many_row_tiles_block_terms(case):
    B, H, W, Cin, Cout, k, stride, pad, w_bits, a_bits = case
    gen, a, w, s, wp = _setup(case)
    want_acc = oracle.conv2d(a, w, stride, pad)
    bias = gen.uniform(-1, 1, size=Cout).astype(np.float32)
    res_lv = levels(gen, want_acc.shape, 2)
    res_f = gen.normal(0, 1, size=want_acc.shape).astype(np.float32)
    acc, out, nxt = qnn.qnn_conv2d_block(pack_levels(a, a_bits), wp, (B, H, W), Cin, stride, pad, dev(s), bias=dev(bias),
                                         res_planes=pack_levels(res_lv.reshape(-1, Cout), 2), res_scale=0.37,
                                         res_f32=dev(res_f), want_out=True, next_clip=2.5, next_bits=3)
    torch.cuda.synchronize()
    want = oracle.block_epilogue(want_acc, s, bias, res_lv, np.float32(0.37), res_f)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=1e-5, atol=0)
    lv, _ = oracle.quantize(want, 2.5, 3)
    assert np.array_equal(planes_to_numpy(nxt), oracle.pack_planes(lv.reshape(-1, Cout), 3))
