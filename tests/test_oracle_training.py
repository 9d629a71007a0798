"""Pins of the training-side gradients in the oracle (quantize_ste_backward, encoder_backward): the
values Eq. 12-13 print for the 2-bit encoders, central differences of the sines they differentiate,
the link between those sines and the quantizer's planes, and the straight-through rule."""
import numpy as np

import oracle


def _planes(t, bits):
    """plane values in {-1,+1} of the oracle's quantizer, [bits][n], index m - 1 (m = 1 lowest)."""
    _, code = oracle.quantize(t.astype(np.float32), 1.0, bits)
    return np.stack([2.0 * ((code >> j) & 1) - 1.0 for j in range(bits)])


def _sines(t, bits):
    K = (1 << bits) - 1
    return np.stack([(1.0 if m == bits else -1.0) * np.sin(np.pi * K * t / (1 << m)) for m in range(1, bits + 1)])


def test_two_bit_values_of_eq_12_13():
    x = np.array([0.0, 1.0, -1.0, 0.5, 1.5, -1.0001], np.float32)
    one, zero = np.ones_like(x, dtype=np.float64), np.zeros_like(x, dtype=np.float64)
    hi = oracle.encoder_backward(x, np.stack([zero, one]), 1.0, 2)     # d phi_2^2 / dx
    lo = oracle.encoder_backward(x, np.stack([one, zero]), 1.0, 2)     # d phi_2^1 / dx
    a, b = 0.75 * np.pi, 1.5 * np.pi
    np.testing.assert_allclose(hi, [a, a * np.cos(a), a * np.cos(a), a * np.cos(a / 2), 0, 0], atol=1e-12)
    np.testing.assert_allclose(lo, [-b, -b * np.cos(b), -b * np.cos(b), -b * np.cos(b / 2), 0, 0], atol=1e-12)


def test_encoder_gradient_is_the_derivative_of_the_sines():
    gen = np.random.default_rng(0)
    for bits in range(1, 9):
        t = gen.uniform(-0.999, 0.999, size=2000)
        t32 = t.astype(np.float32).astype(np.float64)
        h = 1e-6
        num = (_sines(t32 + h, bits) - _sines(t32 - h, bits)) / (2 * h)       # [bits][n]
        g = gen.normal(size=(bits, t.size))
        got = oracle.encoder_backward(t32.astype(np.float32), g, 1.0, bits)
        np.testing.assert_allclose(got, (g * num).sum(0), rtol=1e-6, atol=1e-4 * (1 << bits))
        # one plane at a time, so a swapped or mis-signed plane shows
        for m in range(bits):
            e = np.zeros((bits, t.size)); e[m] = 1.0
            np.testing.assert_allclose(oracle.encoder_backward(t32.astype(np.float32), e, 1.0, bits), num[m],
                                       rtol=1e-6, atol=1e-4 * (1 << bits))


def test_sines_are_the_encoders_of_the_quantizer():
    # the sign of each differentiated sine is the plane the quantizer emits (away from the thresholds)
    for bits in range(1, 9):
        K = (1 << bits) - 1
        t = np.linspace(-1, 1, 20001)
        v = K * (t + 1) / 2
        clear = np.abs(v + 0.5 - np.round(v + 0.5)) > 1e-3
        s = np.sign(_sines(t, bits))
        p = _planes(t, bits)
        assert clear.mean() > 0.7
        assert np.array_equal(s[:, clear], p[:, clear]), bits


def test_clip_scales_and_limits_both_gradients():
    gen = np.random.default_rng(1)
    x = gen.uniform(-4, 4, size=3000).astype(np.float32)
    g = gen.normal(size=x.size)
    clip = 2.5
    inside = np.abs(x.astype(np.float64)) <= clip
    ste = oracle.quantize_ste_backward(x, g, clip)
    inv = np.float64(np.float32(1.0) / np.float32(clip))
    np.testing.assert_allclose(ste, np.where(inside, g * inv, 0.0), rtol=1e-12)
    # central difference of the range limit itself, away from the corners
    h = 1e-4
    lim = lambda z: np.clip(z / clip, -1, 1)
    far = np.abs(np.abs(x) - clip) > 1e-2
    num = (lim(x.astype(np.float64) + h) - lim(x.astype(np.float64) - h)) / (2 * h)
    np.testing.assert_allclose(ste[far], (g * num)[far], rtol=1e-5, atol=1e-9)
    # the encoder gradient with clip equals the unit-range one at x / clip, times 1 / clip
    gp = gen.normal(size=(3, x.size))
    a = oracle.encoder_backward(x, gp, clip, 3)
    t = (x * (np.float32(1.0) / np.float32(clip))).astype(np.float32)
    b = oracle.encoder_backward(t, gp, 1.0, 3) * inv
    np.testing.assert_allclose(a[far], b[far], rtol=1e-6, atol=1e-6)
    # the ends of the range belong to it (Eq. 12-13: -1 <= x <= 1)
    ends = oracle.quantize_ste_backward(np.array([-1, 1, np.nextafter(np.float32(1), np.float32(2))], np.float32),
                                        np.ones(3), 1.0)
    assert ends.tolist() == [1.0, 1.0, 0.0]


def test_binarize_is_the_one_bit_encoder_and_shares_the_ste():
    # Eq. 14: Binarize(x) = sign(HTanh(x)); sign(0) = +1 as for the encoders
    x = np.array([-3, -1, -0.2, 0.0, 0.3, 1, 7], np.float32)
    lv, _ = oracle.quantize(x, 1.0, 1)
    assert lv.tolist() == [-1, -1, -1, 1, 1, 1, 1]
    for clip in (0.5, 1.0, 4.0):
        assert np.array_equal(oracle.quantize(x, clip, 1)[0], lv)
    assert oracle.quantize_ste_backward(x, np.full(7, 2.0), 1.0).tolist() == [0, 2, 2, 2, 2, 2, 0]
