"""ctypes binding of libqnn_probe.so (include/qnn_probe.h): register-only issue-rate loops that the benchmark
uses to state what the vector ALUs and the matrix cores sustain on the device at hand.  Measurement aids, kept
out of the product library; nothing on the hot path calls them."""
import ctypes
import os

import torch

from . import build as _build

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqnn_probe.so")
EXPORTS = ("qnn_probe_valu", "qnn_probe_mfma", "qnn_probe_last_error")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int
        L.qnn_probe_valu.argtypes = [i32, i32, i32, vp, vp, vp]
        L.qnn_probe_valu.restype = i32
        L.qnn_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
        L.qnn_probe_mfma.restype = i32
        L.qnn_probe_last_error.argtypes = []
        L.qnn_probe_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise RuntimeError("libqnn_probe error %d: %s" % (rc, lib().qnn_probe_last_error().decode()))


def _buf(name, t, numel):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype in (torch.int32, torch.uint32)
            and t.numel() >= numel):
        raise ValueError("%s: a contiguous CUDA int32 tensor of at least %d elements is needed" % (name, numel))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def qnn_probe_valu(mode, workgroups, iters, out, clocks=None):
    """Launch one issue-rate loop; out: int32 [workgroups * 256]; clocks: int64 [workgroups * 4][2] or None
    (per wave: ticks of the shader's cycle counter and of the constant-rate counter across the loop)."""
    cp = None
    if clocks is not None:
        if not (clocks.is_cuda and clocks.is_contiguous() and clocks.dtype == torch.int64
                and clocks.numel() >= workgroups * 8):
            raise ValueError("clocks: a contiguous CUDA int64 tensor of at least %d elements is needed" % (workgroups * 8))
        cp = ctypes.c_void_p(clocks.data_ptr())
    _check(lib().qnn_probe_valu(int(mode), int(workgroups), int(iters), _buf("out", out, workgroups * 256), cp, _stream()))


def qnn_probe_mfma(mode, workgroups, iters, out):
    """Launch one register-only MFMA loop; out: int32 [workgroups * 256]."""
    _check(lib().qnn_probe_mfma(int(mode), int(workgroups), int(iters), _buf("out", out, workgroups * 256), _stream()))
