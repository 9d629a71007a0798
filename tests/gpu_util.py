"""Helpers for the GPU parity tests: numpy <-> device tensors and level packing through the
library's own qnn_encode_pack (int8 level path)."""
import numpy as np
import torch

from paper_1905_13389_amd import qnn


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def planes_to_numpy(p):
    torch.cuda.synchronize()
    return p.cpu().numpy().view(np.uint32)


def pack_levels(levels_np, bits):
    """int8 levels [..., n] -> device planes via qnn_encode_pack(dtype = int8 levels)."""
    return qnn.qnn_encode_pack(dev(levels_np.astype(np.int8)), 1.0, bits)


def levels(gen, shape, bits):
    top = (1 << bits) - 1
    return (2 * gen.integers(0, top + 1, size=shape) - top).astype(np.int8)
