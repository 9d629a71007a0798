"""The values the paper prints, through the HIP path itself: Table 2's four 2-bit reals and their
{high, low} states out of qnn_encode_pack, and Fig. 1's fixed decoder scale 1/9 out of
qnn_binary_gemm (the scaled binary product equals the product of the quantized reals)."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from gpu_util import dev, planes_to_numpy

pytestmark = pytest.mark.gpu

from paper_1905_13389_amd import qnn  # noqa: E402


def _table2(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "table2_encoded_states.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                q, hi, lo = line.split()
                rows.append((Fraction(q), int(hi), int(lo)))
    return rows


def test_table2_states_from_the_device_encoder(golden_dir):
    rows = _table2(golden_dir)
    x = np.array([float(q) for q, _, _ in rows], dtype=np.float32).reshape(1, -1)
    planes = planes_to_numpy(qnn.qnn_encode_pack(dev(x), 1.0, 2))          # [2][1][1]
    for t, (q, hi, lo) in enumerate(rows):
        assert (1 if (planes[1, 0, 0] >> t) & 1 else -1) == hi             # plane 1 = high bit x2
        assert (1 if (planes[0, 0, 0] >> t) & 1 else -1) == lo             # plane 0 = low bit x1
    assert planes[0, 0, 0] >> 4 == 0 and planes[1, 0, 0] >> 4 == 0          # pad bits are 0


def test_fig1_scale_from_the_device_product(golden_dir):
    with open(os.path.join(golden_dir, "fig1_scale.txt")) as f:
        xb, wb, num, den = [int(v) for v in [l for l in f if l.strip() and not l.startswith("#")][0].split()]
    assert (xb, wb) == (2, 2)
    reals = np.array([float(q) for q, _, _ in _table2(golden_dir)])
    gen = np.random.default_rng(9)
    x = gen.choice(reals, size=(5, 100)).astype(np.float32)
    w = gen.choice(reals, size=(7, 100)).astype(np.float32)
    scale = np.full(7, num / den, np.float32)
    _, out = qnn.qnn_binary_gemm(qnn.qnn_encode_pack(dev(x), 1.0, 2), qnn.qnn_encode_pack(dev(w), 1.0, 2), 100,
                                 want_acc=False, scale=dev(scale))
    torch.cuda.synchronize()
    want = x.astype(np.float64) @ w.astype(np.float64).T                  # product of the quantized reals
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=1e-5, atol=1e-6)
