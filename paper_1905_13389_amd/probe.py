"""ctypes binding of libqnn_probe.so and libqnn_timeline.so (include/qnn_probe.h): register-only issue-rate loops that
the benchmark uses to state what the vector ALUs and the matrix cores sustain on the device at hand, and the
convolution kernels compiled with wave timestamps.  Measurement aids, kept out of the product library; nothing on the
hot path calls them."""
import ctypes
import os

import torch

from . import build as _build

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqnn_probe.so")
EXPORTS = ("qnn_probe_valu", "qnn_probe_mfma", "qnn_probe_mfma_operands", "qnn_probe_last_error")
TIMELINE_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqnn_timeline.so")
TIMELINE_EXPORTS = ("qnn_timeline_set", "qnn_conv2d", "qnn_conv2d_block", "qnn_deconv2d", "qnn_last_error",
                    "qnn_level_gemm_timeline_set", "qnn_level_gemm_i8", "qnn_level_gemm_fp4")
_lib = None
_timeline_lib = None


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
        L.qnn_probe_mfma_operands.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        L.qnn_probe_mfma_operands.restype = i32
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


def qnn_probe_mfma_operands(mode, workgroups, iters, operands, out, clocks=None):
    """The MFMA loop on caller-supplied operands; operands: 32 KiB (uint8 [256][8][16]); out: int32 [workgroups * 256];
    clocks: int64 [workgroups * 4][2] or None."""
    if not (operands.is_cuda and operands.is_contiguous() and operands.dtype in (torch.uint8, torch.int8)
            and operands.numel() == 256 * 8 * 16):
        raise ValueError("operands: a contiguous CUDA byte tensor of 32768 elements is needed")
    cp = None
    if clocks is not None:
        if not (clocks.is_cuda and clocks.is_contiguous() and clocks.dtype == torch.int64
                and clocks.numel() >= workgroups * 8):
            raise ValueError("clocks: a contiguous CUDA int64 tensor of at least %d elements is needed" % (workgroups * 8))
        cp = ctypes.c_void_p(clocks.data_ptr())
    _check(lib().qnn_probe_mfma_operands(int(mode), int(workgroups), int(iters), ctypes.c_void_p(operands.data_ptr()),
                                         _buf("out", out, workgroups * 256), cp, _stream()))


def timeline_lib():
    global _timeline_lib
    if _timeline_lib is None:
        if not os.path.exists(TIMELINE_LIB_PATH):
            _build.build()
        from .qnn import qnn_conv_desc
        L = ctypes.CDLL(TIMELINE_LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.qnn_timeline_set.argtypes = [vp, i32, i32]
        L.qnn_timeline_set.restype = i32
        L.qnn_conv2d.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d.restype = i32
        L.qnn_last_error.argtypes = []
        L.qnn_last_error.restype = ctypes.c_char_p
        L.qnn_level_gemm_timeline_set.argtypes = [vp, i32]
        L.qnn_level_gemm_timeline_set.restype = i32
        i64 = ctypes.c_int64
        for fn in (L.qnn_level_gemm_i8, L.qnn_level_gemm_fp4):
            fn.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp]
            fn.restype = i32
        _timeline_lib = L
    return _timeline_lib


def qnn_timeline_set(buffer, pair_hint=True):
    """buffer: int64 CUDA tensor [waves][5] (or None: stop recording); see include/qnn_probe.h."""
    L = timeline_lib()
    if buffer is None:
        rc = L.qnn_timeline_set(None, 0, int(bool(pair_hint)))
    else:
        if not (buffer.is_cuda and buffer.is_contiguous() and buffer.dtype == torch.int64 and buffer.dim() == 2
                and buffer.shape[1] == 5):
            raise ValueError("buffer: a contiguous CUDA int64 tensor [waves][5] is needed")
        rc = L.qnn_timeline_set(ctypes.c_void_p(buffer.data_ptr()), int(buffer.shape[0]), int(bool(pair_hint)))
    if rc != 0:
        raise RuntimeError("libqnn_timeline error %d: %s" % (rc, L.qnn_last_error().decode()))


def timeline_conv2d(desc, a_planes, w_planes, scale, acc, out, next_planes, next_clip, next_bits):
    """qnn_conv2d of libqnn_timeline.so on tensors the caller has checked (the benchmark builds them with the
    product binding first); None for outputs that are not wanted."""
    ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())  # noqa: E731
    L = timeline_lib()
    rc = L.qnn_conv2d(ctypes.byref(desc), ptr(a_planes), ptr(w_planes), ptr(scale), ptr(acc), ptr(out), ptr(next_planes),
                      float(next_clip), int(next_bits), _stream())
    if rc != 0:
        raise RuntimeError("libqnn_timeline error %d: %s" % (rc, L.qnn_last_error().decode()))


def qnn_level_gemm_timeline_set(buffer):
    """buffer: int64 CUDA tensor [waves][6] (or None: stop recording); see include/qnn_probe.h."""
    L = timeline_lib()
    if buffer is None:
        rc = L.qnn_level_gemm_timeline_set(None, 0)
    else:
        if not (buffer.is_cuda and buffer.is_contiguous() and buffer.dtype == torch.int64 and buffer.dim() == 2
                and buffer.shape[1] == 6):
            raise ValueError("buffer: a contiguous CUDA int64 tensor [waves][6] is needed")
        rc = L.qnn_level_gemm_timeline_set(ctypes.c_void_p(buffer.data_ptr()), int(buffer.shape[0]))
    if rc != 0:
        raise RuntimeError("libqnn_timeline error %d: %s" % (rc, L.qnn_last_error().decode()))


def timeline_level_gemm(a_levels, w_levels, rows, cols, n, acc, scale, out, fp4=False):
    """qnn_level_gemm_i8 / _fp4 of libqnn_timeline.so on tensors the caller has checked (level rows padded as
    qnn_level_row_bytes / qnn_fp4_row_bytes say); None for an output that is not wanted."""
    ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())  # noqa: E731
    L = timeline_lib()
    fn = L.qnn_level_gemm_fp4 if fp4 else L.qnn_level_gemm_i8
    rc = fn(ptr(a_levels), ptr(w_levels), int(rows), int(cols), int(n), ptr(acc), ptr(scale), ptr(out), _stream())
    if rc != 0:
        raise RuntimeError("libqnn_timeline error %d: %s" % (rc, L.qnn_last_error().decode()))
