"""GPU parity of the bit-plane-sum variant (qnn_plane_sum_i8 + qnn_level_gemm_i8) against the CPU
oracle and against the xor + bitcount path: identical int32 accumulators."""
import numpy as np
import pytest
import torch

import oracle
import qnn_workloads as wl
from gpu_util import dev, pack_levels, levels

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("shape", [(3, 1), (5, 31), (4, 64), (7, 100), (9, 1000), (130, 4096)])
def test_plane_sum_gives_levels(bits, shape):
    gen = np.random.default_rng(bits * 31 + shape[1])
    lv = levels(gen, shape, bits)
    got = qnn.qnn_plane_sum_i8(pack_levels(lv, bits), shape[1])
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    nk = qnn.qnn_level_row_bytes(shape[1])
    assert got.shape == (shape[0], nk) and nk % 64 == 0 and nk >= shape[1]
    # levels are the decode of the planes (oracle.unpack_planes of oracle.pack_planes is the identity)
    assert np.array_equal(oracle.unpack_planes(oracle.pack_planes(lv.astype(np.int16), bits), shape[1]), lv)
    assert np.array_equal(got[:, :shape[1]], lv)
    assert not got[:, shape[1]:].any()


@pytest.mark.parametrize("bits", [(2, 2), (1, 1), (4, 4), (3, 2), (7, 5)])
@pytest.mark.parametrize("shape", [(1, 1, 1), (130, 70, 100), (257, 300, 1000), (512, 256, 2080), (300, 64, 33)])
def test_level_gemm_matches_oracle_and_binary_path(bits, shape):
    w_bits, a_bits = bits
    rows, cols, n = shape
    gen = np.random.default_rng(w_bits * 100 + a_bits * 10 + rows)
    a, w = levels(gen, (rows, n), a_bits), levels(gen, (cols, n), w_bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    ap, wp = pack_levels(a, a_bits), pack_levels(w, w_bits)
    a8, w8 = qnn.qnn_plane_sum_i8(ap, n), qnn.qnn_plane_sum_i8(wp, n)
    acc, out = qnn.qnn_level_gemm_i8(a8, w8, n, scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)
    if max(bits) <= 4:
        acc2, _ = qnn.qnn_binary_gemm(ap, wp, n)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc2)


def test_level_gemm_full_size_equals_binary_path():
    c = wl.gemm_square(2, 2, 4096)
    ap, wp = pack_levels(c["a"], 2), pack_levels(c["w"], 2)
    acc, _ = qnn.qnn_level_gemm_i8(qnn.qnn_plane_sum_i8(ap, 4096), qnn.qnn_plane_sum_i8(wp, 4096), 4096)
    acc2, _ = qnn.qnn_binary_gemm(ap, wp, 4096)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2)
    rsel = [0, 1234, 4095]
    assert np.array_equal(acc.cpu().numpy()[rsel], oracle.gemm(c["a"][rsel], c["w"]))


# fp4 (E2M1) values by nibble, sign in bit 3: the published OCP microscaling element format
FP4_VALUE = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.0, -0.5, -1, -1.5, -2, -3, -4, -6])


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("shape", [(3, 1), (5, 31), (4, 64), (7, 100), (9, 1000), (130, 4096)])
def test_plane_sum_fp4_gives_levels(bits, shape):
    gen = np.random.default_rng(bits * 37 + shape[1])
    lv = levels(gen, shape, bits)
    got = qnn.qnn_plane_sum_fp4(pack_levels(lv, bits), shape[1])
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    nb = qnn.qnn_fp4_row_bytes(shape[1])
    assert got.shape == (shape[0], nb) and nb % 128 == 0 and 2 * nb >= shape[1]
    nib = np.stack([got & 15, got >> 4], axis=-1).reshape(shape[0], 2 * nb)   # element 2i = low nibble
    dec = FP4_VALUE[nib]
    assert np.array_equal(dec[:, :shape[1]], lv.astype(np.float64))
    assert not nib[:, shape[1]:].any()


@pytest.mark.parametrize("bits", [(2, 2), (1, 1), (2, 1), (1, 2)])
@pytest.mark.parametrize("shape", [(1, 1, 1), (130, 70, 100), (257, 300, 1000), (512, 256, 2080), (300, 64, 33),
                                   (64, 64, 65536)])
def test_level_gemm_fp4_matches_oracle(bits, shape):
    w_bits, a_bits = bits
    rows, cols, n = shape
    gen = np.random.default_rng(w_bits * 100 + a_bits * 10 + rows + 1)
    a, w = levels(gen, (rows, n), a_bits), levels(gen, (cols, n), w_bits)
    s = gen.uniform(0.01, 0.1, size=cols).astype(np.float32)
    a4 = qnn.qnn_plane_sum_fp4(pack_levels(a, a_bits), n)
    w4 = qnn.qnn_plane_sum_fp4(pack_levels(w, w_bits), n)
    acc, out = qnn.qnn_level_gemm_fp4(a4, w4, n, scale=dev(s))
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert np.array_equal(acc.cpu().numpy(), want)
    np.testing.assert_allclose(out.cpu().numpy(), oracle.scale(want, s), rtol=1e-5, atol=0)


def test_level_gemm_fp4_exact_at_the_accumulator_limit():
    # all-maximum 2-bit operands: every product is 9 and acc = 9 n climbs to just below 2^24, the
    # largest magnitude the fp32 accumulators of the instruction hold exactly; mixed signs beside it
    n = (1 << 24) // 9
    a = np.full((3, n), 3, np.int8)
    w = np.full((2, n), 3, np.int8)
    a[1] = -3
    a[2, ::2] = -1
    w[1, 1::3] = 1
    a4 = qnn.qnn_plane_sum_fp4(pack_levels(a, 2), n)
    w4 = qnn.qnn_plane_sum_fp4(pack_levels(w, 2), n)
    acc, _ = qnn.qnn_level_gemm_fp4(a4, w4, n)
    torch.cuda.synchronize()
    want = a.astype(np.int64) @ w.astype(np.int64).T
    assert want[0, 0] == 9 * n and 9 * n < (1 << 24)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.array_equal(oracle.gemm(a, w), want)
    with pytest.raises(qnn.QnnError) as e:
        qnn.qnn_level_gemm_fp4(a4, w4, n + 50)      # same row bytes, 9 n >= 2^24
    assert e.value.code == -4


def test_fp4_full_size_matches_int8_route():
    c = wl.gemm_square(2, 2, 4096)
    ap, wp = pack_levels(c["a"], 2), pack_levels(c["w"], 2)
    acc4, out4 = qnn.qnn_level_gemm_fp4(qnn.qnn_plane_sum_fp4(ap, 4096), qnn.qnn_plane_sum_fp4(wp, 4096), 4096,
                                        scale=dev(c["scale"]))
    acc8, out8 = qnn.qnn_level_gemm_i8(qnn.qnn_plane_sum_i8(ap, 4096), qnn.qnn_plane_sum_i8(wp, 4096), 4096,
                                       scale=dev(c["scale"]))
    torch.cuda.synchronize()
    assert torch.equal(acc4, acc8) and torch.equal(out4, out8)
    rows = [0, 1, 2047, 4095]
    assert np.array_equal(acc4[rows].cpu().numpy(), oracle.gemm(c["a"][rows], c["w"]))


def test_level_gemm_i8_longest_reduction():
    # 7-bit levels at the largest n the int32 accumulator allows: 127^2 n < 2^31
    n = (2 ** 31 - 1) // (127 * 127)
    gen = np.random.default_rng(1)
    a, w = levels(gen, (3, n), 7), levels(gen, (4, n), 7)
    a[0], w[0], w[1] = 127, 127, -127
    a8 = qnn.qnn_plane_sum_i8(pack_levels(a, 7), n)
    w8 = qnn.qnn_plane_sum_i8(pack_levels(w, 7), n)
    acc, _ = qnn.qnn_level_gemm_i8(a8, w8, n)
    torch.cuda.synchronize()
    want = oracle.gemm(a, w)
    assert want[0, 0] == n * 127 * 127 and want[0, 1] == -n * 127 * 127
    assert np.array_equal(acc.cpu().numpy(), want)
