"""Pins for the oracle's binary dot, multi-branch product, GEMM, convolution and scale
(CPU only).  Brute force on tiny inputs, numpy int64 matmul, torch float64 conv2d, closed
forms and the paper's printed 1/9 scale."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def _levels(gen, shape, bits, dtype=np.int16):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(dtype)


def _bits_to_words(bits_pm1):
    n = len(bits_pm1)
    words = np.zeros((n + 31) // 32, dtype=np.uint32)
    for t, b in enumerate(bits_pm1):
        if b > 0:
            words[t // 32] |= np.uint32(1 << (t % 32))
    return words


def test_xnor_bitcount_dot_exhaustive_small():
    # every pair of {-1,+1}^n vectors for n <= 5 against the plain +-1 dot product
    for n in range(1, 6):
        vecs = list(itertools.product((-1, 1), repeat=n))
        words = [_bits_to_words(v) for v in vecs]
        for va, wa in zip(vecs, words):
            for vb, wb in zip(vecs, words):
                assert oracle.xnor_bitcount_dot(wa, wb, n) == sum(x * y for x, y in zip(va, vb))


@pytest.mark.parametrize("n", [1, 31, 32, 33, 63, 64, 65, 100])
def test_xnor_bitcount_dot_random_lengths(n):
    gen = np.random.default_rng(n)
    for _ in range(20):
        a = gen.choice((-1, 1), size=n)
        b = gen.choice((-1, 1), size=n)
        assert oracle.xnor_bitcount_dot(_bits_to_words(a), _bits_to_words(b), n) == int(a @ b)


def test_worked_two_bit_example():
    # Derived by hand from Eq. 9 / Eq. 10: a = [3, -1], w = [1, -3].
    # planes: a_hi = [+,-], a_lo = [+,+], w_hi = [+,-], w_lo = [-,-]
    # y_hh = 2, y_hl = 0 (w_hi.a_lo), y_lh = 0 (w_lo.a_hi), y_ll = -2 -> 4*2 + 0 + 0 - 2 = 6
    a = np.array([[3, -1]], dtype=np.int16)
    w = np.array([[1, -3]], dtype=np.int16)
    acc, br = oracle.multibranch_gemm(oracle.pack_planes(a, 2), oracle.pack_planes(w, 2), 2,
                                      want_branches=True)
    assert acc[0, 0] == 6 == 3 * 1 + (-1) * (-3)
    # br[r][c][i (w bit)][j (a bit)]
    assert br[0, 0].tolist() == [[-2, 0], [0, 2]]
    assert oracle.gemm(a, w)[0, 0] == 6
    # in quantized reals: 1 * 1/3 + (-1/3)(-1) = 2/3 = 6/9
    assert Fraction(6, 9) == Fraction(1) * Fraction(1, 3) + Fraction(-1, 3) * Fraction(-1)


@pytest.mark.parametrize("w_bits", range(1, 9))
@pytest.mark.parametrize("a_bits", range(1, 9))
def test_multibranch_equals_integer_matmul(w_bits, a_bits):
    # Eq. 7-9 with Eq. 10: the M x K branch sum is the integer matmul of the decoded levels
    gen = np.random.default_rng(1000 + 10 * w_bits + a_bits)
    rows, cols, n = 5, 4, 45
    a = _levels(gen, (rows, n), a_bits)
    w = _levels(gen, (cols, n), w_bits)
    want = a.astype(np.int64) @ w.astype(np.int64).T
    got = oracle.multibranch_gemm(oracle.pack_planes(a, a_bits), oracle.pack_planes(w, w_bits), n)
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.gemm(a, w), want)


def test_one_bit_case_is_bnn():
    # M = K = 1 reduces to the binarized network: one branch, acc = 2 popcount(xnor) - n
    gen = np.random.default_rng(7)
    n = 77
    a = _levels(gen, (3, n), 1)
    w = _levels(gen, (2, n), 1)
    ap, wp = oracle.pack_planes(a, 1), oracle.pack_planes(w, 1)
    acc, br = oracle.multibranch_gemm(ap, wp, n, want_branches=True)
    for r in range(3):
        for c in range(2):
            x = ~(ap[0, r] ^ wp[0, c])
            # count only the n valid bits
            pop = sum(bin(int(word)).count("1") for word in x) - (32 * len(x) - n)
            assert acc[r, c] == 2 * pop - n == br[r, c, 0, 0]


@pytest.mark.parametrize("shape", [(17, 9, 130), (64, 256, 512), (33, 65, 1000)])
@pytest.mark.parametrize("bits", [(2, 2), (4, 3), (7, 7), (8, 8)])
def test_gemm_against_numpy_int64(shape, bits):
    rows, cols, n = shape
    w_bits, a_bits = bits
    gen = np.random.default_rng(rows + cols + n + w_bits)
    a = _levels(gen, (rows, n), a_bits)
    w = _levels(gen, (cols, n), w_bits)
    want = a.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(oracle.gemm(a, w), want)
    if max(w_bits, a_bits) <= 7:
        assert np.array_equal(oracle.gemm(a.astype(np.int8), w.astype(np.int8)), want)
        assert oracle.gemm_one(a[3].astype(np.int8), w[5].astype(np.int8)) == want[3, 5]


def test_gemm_is_not_transposed():
    # a single non-trivial entry pins the operand order / index convention
    a = np.ones((2, 3), dtype=np.int16)
    w = np.ones((4, 3), dtype=np.int16)
    a[1, 2] = -3
    w[3, 2] = 3
    acc = oracle.gemm(a, w)
    assert acc.shape == (2, 4)
    assert acc[1, 3] == 1 + 1 - 9 and acc[0, 3] == 1 + 1 + 3 and acc[1, 0] == 1 + 1 - 3
    assert acc[0, 0] == 3


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_recombination_closed_form_and_invariants(bits):
    # acc = n (2^M-1)(2^K-1) - 2 sum_s 2^s P_s with P_ij = popcount(w_i xor a_j);
    # acc == n (mod 2); |acc| <= n (2^M-1)(2^K-1) with equality for all-max inputs;
    # complementing the weight planes negates acc.
    gen = np.random.default_rng(bits)
    n = 83
    top = (1 << bits) - 1
    a = _levels(gen, (4, n), bits)
    w = _levels(gen, (3, n), bits)
    ap, wp = oracle.pack_planes(a, bits), oracle.pack_planes(w, bits)
    acc = oracle.gemm(a, w)
    for r in range(4):
        for c in range(3):
            tot = 0
            for i in range(bits):
                for j in range(bits):
                    x = wp[i, c] ^ ap[j, r]
                    tot += (1 << (i + j)) * sum(bin(int(v)).count("1") for v in x)
            assert acc[r, c] == n * top * top - 2 * tot
    assert np.all((acc - n) % 2 == 0)
    assert np.all(np.abs(acc) <= n * top * top)
    hi = np.full((1, n), top, dtype=np.int16)
    assert oracle.gemm(hi, hi)[0, 0] == n * top * top
    assert oracle.gemm(hi, -hi)[0, 0] == -n * top * top
    mask = np.uint32(0xFFFFFFFF)
    wneg = oracle.unpack_planes((wp ^ mask), n)
    # complementing sets the pad bits too; unpack only reads the n valid ones
    assert np.array_equal(wneg, -w)
    assert np.array_equal(oracle.gemm(a, wneg), -acc)


def test_zero_one_route_identity():
    # Eq. 16-17: with x_q = 2 x01/(2^M-1) - 1 the same real product follows from the {0,1}
    # integers through a four-term polynomial; Eq. 18 gives it from the {-1,+1} integers
    # with one factor.  Checked exactly with fractions.
    gen = np.random.default_rng(17)
    M, K = 3, 2
    n = 40
    ux = gen.integers(0, 1 << M, size=n)
    uw = gen.integers(0, 1 << K, size=n)
    tx, tw = (1 << M) - 1, (1 << K) - 1
    poly = sum(Fraction(4, tx * tw) * int(x) * int(w) - Fraction(2, tx) * int(x)
               - Fraction(2, tw) * int(w) + 1 for x, w in zip(ux, uw))
    a = (2 * ux - tx).astype(np.int16).reshape(1, n)
    w = (2 * uw - tw).astype(np.int16).reshape(1, n)
    assert Fraction(int(oracle.gemm(a, w)[0, 0]), tx * tw) == poly


# ----------------------------------------------------------------------------- conv
def _torch_conv(a, w, stride, pad, dilation=1):
    ta = torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2)
    tw = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    out = torch.nn.functional.conv2d(ta, tw, stride=stride, padding=pad, dilation=dilation)
    return out.permute(0, 2, 3, 1).numpy().round().astype(np.int64)


@pytest.mark.parametrize("geom", [
    # B, H, W, Cin, Cout, k, stride, pad
    (2, 7, 9, 5, 4, 3, 1, 1),
    (1, 8, 8, 32, 6, 3, 2, 1),
    (2, 6, 5, 3, 3, 1, 1, 0),
    (1, 9, 7, 4, 2, 5, 1, 2),
    (1, 9, 10, 4, 2, 3, 2, 0),
    (3, 4, 4, 7, 5, 3, 1, 2),
])
def test_conv_against_torch_float64(geom):
    B, H, W, Cin, Cout, k, stride, pad = geom
    gen = np.random.default_rng(sum(geom))
    a = _levels(gen, (B, H, W, Cin), 3, np.int8)
    w = _levels(gen, (Cout, k, k, Cin), 2, np.int8)
    assert np.array_equal(oracle.conv2d(a, w, stride, pad), _torch_conv(a, w, stride, pad))


@pytest.mark.parametrize("geom", [
    # B, H, W, Cin, Cout, kh, kw, stride, pad, dilation
    (1, 19, 19, 6, 4, 3, 3, 1, 6, 6),     # the detection network's layer: 3x3, dilation 6, pad 6, same size
    (2, 9, 11, 5, 3, 3, 3, 1, 2, 2),
    (1, 10, 9, 4, 2, 3, 2, 2, 1, 3),      # rectangular kernel, stride 2
    (1, 7, 7, 3, 2, 2, 2, 1, 0, 4),       # no padding: the output shrinks by dilation (k - 1)
    (2, 5, 5, 8, 3, 3, 3, 1, 4, 4),       # whole rows of taps outside the image
    (1, 6, 6, 4, 2, 1, 1, 1, 0, 5),       # 1x1: dilation has no effect
])
def test_dilated_conv_against_torch_float64(geom):
    B, H, W, Cin, Cout, kh, kw, stride, pad, dil = geom
    gen = np.random.default_rng(sum(geom))
    a = _levels(gen, (B, H, W, Cin), 3, np.int8)
    w = _levels(gen, (Cout, kh, kw, Cin), 2, np.int8)
    got = oracle.conv2d(a, w, stride, pad, dil)
    assert np.array_equal(got, _torch_conv(a, w, stride, pad, dil))
    if kh == 1 and kw == 1:
        assert np.array_equal(got, oracle.conv2d(a, w, stride, pad))


def test_dilated_conv_is_the_conv_of_a_kernel_with_zeros_between_its_taps():
    # brute force through the undilated definition: spread the taps d apart with zero weights between them
    gen = np.random.default_rng(61)
    a = _levels(gen, (2, 8, 9, 4), 2, np.int8)
    w = _levels(gen, (3, 3, 3, 4), 3, np.int8)
    for d in (2, 3):
        wide = np.zeros((3, 2 * d + 1, 2 * d + 1, 4), dtype=np.int8)
        wide[:, ::d, ::d, :] = w
        assert np.array_equal(oracle.conv2d(a, w, 1, d, d), oracle.conv2d(a, wide, 1, d))


def test_conv_rectangular_kernel_and_orientation():
    # kh != kw and an asymmetric weight pin the (kh, kw) index order and the absence of a flip
    gen = np.random.default_rng(3)
    a = _levels(gen, (1, 6, 7, 2), 2, np.int8)
    w = _levels(gen, (3, 2, 3, 2), 2, np.int8)
    assert np.array_equal(oracle.conv2d(a, w, 1, 0), _torch_conv(a, w, 1, 0))


def test_conv_1x1_is_gemm_and_pad0_is_im2col_gemm():
    gen = np.random.default_rng(5)
    a = _levels(gen, (2, 5, 6, 8), 2, np.int8)
    w1 = _levels(gen, (7, 1, 1, 8), 2, np.int8)
    assert np.array_equal(oracle.conv2d(a, w1, 1, 0).reshape(-1, 7),
                          oracle.gemm(a.reshape(-1, 8), w1.reshape(7, 8)))
    w3 = _levels(gen, (7, 3, 3, 8), 2, np.int8)
    cols = []
    for b in range(2):
        for ho in range(3):
            for wo in range(4):
                cols.append(a[b, ho:ho + 3, wo:wo + 3, :].reshape(-1))
    im2col = np.stack(cols)
    assert np.array_equal(oracle.conv2d(a, w3, 1, 0).reshape(-1, 7),
                          oracle.gemm(im2col, w3.reshape(7, -1)))


# ----------------------------------------------------------------------------- scale
def test_fig1_fixed_scale(golden_dir):
    # Fig. 1 / Eq. 18: with scale 1/9 the 2-bit layer output equals the dot product of the
    # quantized reals {-1, -1/3, 1/3, 1} of Table 2
    with open(os.path.join(golden_dir, "fig1_scale.txt")) as f:
        row = [l for l in f if l.strip() and not l.startswith("#")][0].split()
    xb, wb, num, den = map(int, row)
    assert (xb, wb) == (2, 2) and den == ((1 << xb) - 1) * ((1 << wb) - 1)
    gen = np.random.default_rng(11)
    n = 50
    a = _levels(gen, (6, n), 2)
    w = _levels(gen, (5, n), 2)
    acc = oracle.gemm(a, w)
    out = oracle.scale(acc, np.full(5, num / den, dtype=np.float32))
    real = (a.astype(np.float64) / 3.0) @ (w.astype(np.float64) / 3.0).T
    assert np.allclose(out, real, rtol=1e-6, atol=1e-6)


def test_scale_is_one_fp32_multiply():
    gen = np.random.default_rng(13)
    acc = gen.integers(-(1 << 23), 1 << 23, size=(9, 11)).astype(np.int32)
    s = gen.uniform(0.01, 0.1, size=11).astype(np.float32)
    want = acc.astype(np.float32) * s[None, :]
    assert np.array_equal(oracle.scale(acc, s), want)
    # per-column, not per-row
    s2 = np.zeros(11, dtype=np.float32)
    s2[4] = 2.0
    out = oracle.scale(acc, s2)
    assert np.array_equal(out[:, 4], acc[:, 4].astype(np.float32) * 2) and not out[:, :4].any()


def test_conv_stack_chain_small():
    # layer chaining: every layer's levels must be the quantizer applied to the previous
    # layer's scaled output, and with unit-variance scaling every level occurs
    gen = np.random.default_rng(19)
    x = gen.standard_normal((2, 12, 12, 32), dtype=np.float32)
    bits = 3
    var_w = (4.0 ** bits - 1) / 3          # uniform odd levels
    var_a = (7 / 3.0) ** 2 + 1 / 3.0       # unit Gaussian through the 3-bit ladder, clip 3
    layers = []
    for cin, cout, stride in ((32, 32, 1), (32, 64, 2)):
        w = _levels(gen, (cout, 3, 3, cin), bits, np.int8)
        layers.append({"w": w, "scale": np.full(cout, 1.0 / np.sqrt(9 * cin * var_w * var_a), np.float32),
                       "clip": 3.0, "a_bits": bits, "stride": stride, "pad": 1})
    trace = oracle.conv_stack(x, layers)
    assert trace[0]["acc"].shape == (2, 12, 12, 32) and trace[1]["acc"].shape == (2, 6, 6, 64)
    lv1, _ = oracle.quantize(trace[0]["out"], 3.0, bits)
    assert np.array_equal(lv1, trace[1]["levels"])
    assert set(np.unique(trace[1]["levels"]).tolist()) == set(range(-7, 8, 2))
    assert np.array_equal(trace[1]["acc"],
                          _torch_conv(trace[1]["levels"].astype(np.int8), layers[1]["w"], 2, 1))
