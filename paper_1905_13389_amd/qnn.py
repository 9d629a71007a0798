"""ctypes binding of libqnn.so: same names and argument order as include/qnn.h.

Marshalling only.  Tensors are torch CUDA tensors used as device-memory handles; the stream is
torch's current stream.  There is no CPU fallback: a missing library or a failing call raises.
"""
import ctypes
import os

import torch  # loads the HIP runtime that libqnn.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
# QNN_LIB_PATH selects another build of the same library (e.g. a tuning variant)
LIB_PATH = os.environ.get("QNN_LIB_PATH") or os.path.join(_HERE, "libqnn.so")

QNN_OK = 0
QNN_ERR_INVALID_ARG = -1
QNN_ERR_UNSUPPORTED = -2
QNN_ERR_ALIGNMENT = -3
QNN_ERR_RANGE = -4
QNN_ERR_LAUNCH = -5

QNN_DTYPE_F32 = 0
QNN_DTYPE_BF16 = 1
QNN_DTYPE_I8 = 2

EXPORTS = ("qnn_encode_pack", "qnn_binary_gemm", "qnn_dequant_scale", "qnn_conv2d", "qnn_conv2d_block",
           "qnn_level_conv2d_block_i8", "qnn_deconv_phase_words", "qnn_deconv_pack_weights", "qnn_deconv2d",
           "qnn_quantize_ste_backward", "qnn_encoder_backward",
           "qnn_probe_valu", "qnn_probe_mfma", "qnn_level_row_bytes", "qnn_plane_sum_i8", "qnn_level_gemm_i8",
           "qnn_encode_levels_i8", "qnn_level_conv2d_i8",
           "qnn_fp4_row_bytes", "qnn_plane_sum_fp4", "qnn_level_gemm_fp4",
           "qnn_encode_levels_fp4", "qnn_levels_to_fp4", "qnn_level_conv2d_fp4", "qnn_level_conv2d_block_fp4", "qnn_maxpool_levels_fp4",
           "qnn_pool_out_size", "qnn_maxpool_planes", "qnn_maxpool_levels_i8",
           "qnn_dense_conv2d_f32", "qnn_dense_conv2d_f32_levels", "qnn_global_avgpool_f32", "qnn_dense_fc_f32", "qnn_fc_fused",
           "qnn_last_error", "qnn_version")


class QnnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("libqnn error %d: %s" % (code, message))
        self.code = code


class qnn_conv_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Cin", ctypes.c_int64), ("Cout", ctypes.c_int64),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("pad", ctypes.c_int32), ("a_bits", ctypes.c_int32), ("w_bits", ctypes.c_int32)]


class qnn_dense_conv_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Cin", ctypes.c_int64), ("Cout", ctypes.c_int64),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


class qnn_block_epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("res_q", ctypes.c_void_p), ("res_bits", ctypes.c_int32),
                ("res_scale", ctypes.c_float), ("res_f32", ctypes.c_void_p), ("relu", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded C-ABI library.  Built in-tree beforehand; if the file is missing it is compiled
    once (hipcc cross-compiles without a GPU); any failure raises."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        L.qnn_encode_pack.argtypes = [vp, i32, i64, i64, i64, f32, i32, vp, vp]
        L.qnn_encode_pack.restype = i32
        L.qnn_binary_gemm.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_binary_gemm.restype = i32
        L.qnn_dequant_scale.argtypes = [vp, vp, i64, i64, vp, vp]
        L.qnn_dequant_scale.restype = i32
        L.qnn_conv2d.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d.restype = i32
        L.qnn_conv2d_block.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, ctypes.POINTER(qnn_block_epilogue),
                                       vp, vp, vp, f32, i32, vp]
        L.qnn_conv2d_block.restype = i32
        L.qnn_level_conv2d_block_i8.argtypes = L.qnn_conv2d_block.argtypes
        L.qnn_level_conv2d_block_i8.restype = i32
        L.qnn_dense_conv2d_f32.argtypes = [ctypes.POINTER(qnn_dense_conv_desc), vp, vp, vp, vp, i32, vp, vp, f32, i32, vp]
        L.qnn_dense_conv2d_f32.restype = i32
        L.qnn_dense_conv2d_f32_levels.argtypes = L.qnn_dense_conv2d_f32.argtypes
        L.qnn_dense_conv2d_f32_levels.restype = i32
        L.qnn_global_avgpool_f32.argtypes = [vp, i64, i64, i64, vp, vp]
        L.qnn_global_avgpool_f32.restype = i32
        L.qnn_dense_fc_f32.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        L.qnn_dense_fc_f32.restype = i32
        L.qnn_fc_fused.argtypes = [vp, i32, i64, i64, i64, f32, i32, vp, i32, i64, vp, vp, vp, vp]
        L.qnn_fc_fused.restype = i32
        L.qnn_probe_valu.argtypes = [i32, i32, i32, vp, vp]
        L.qnn_probe_valu.restype = i32
        L.qnn_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
        L.qnn_probe_mfma.restype = i32
        L.qnn_level_row_bytes.argtypes = [i64]
        L.qnn_level_row_bytes.restype = i64
        L.qnn_plane_sum_i8.argtypes = [vp, i32, i64, i64, vp, vp]
        L.qnn_plane_sum_i8.restype = i32
        L.qnn_level_gemm_i8.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_level_gemm_i8.restype = i32
        L.qnn_pool_out_size.argtypes = [i64, i32, i32, i32, i32]
        L.qnn_pool_out_size.restype = i64
        L.qnn_maxpool_planes.argtypes = [vp, i32, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_planes.restype = i32
        L.qnn_maxpool_levels_i8.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_levels_i8.restype = i32
        L.qnn_fp4_row_bytes.argtypes = [i64]
        L.qnn_fp4_row_bytes.restype = i64
        L.qnn_plane_sum_fp4.argtypes = [vp, i32, i64, i64, vp, vp]
        L.qnn_plane_sum_fp4.restype = i32
        L.qnn_level_gemm_fp4.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp]
        L.qnn_level_gemm_fp4.restype = i32
        L.qnn_encode_levels_i8.argtypes = [vp, i32, i64, f32, i32, vp, vp]
        L.qnn_encode_levels_i8.restype = i32
        L.qnn_level_conv2d_i8.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_level_conv2d_i8.restype = i32
        L.qnn_deconv_phase_words.argtypes = [i32, i64, i32, i32, i64, i32]
        L.qnn_deconv_phase_words.restype = i64
        L.qnn_deconv_pack_weights.argtypes = [vp, i32, i64, i32, i32, i64, i32, vp, vp]
        L.qnn_deconv_pack_weights.restype = i32
        L.qnn_deconv2d.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_deconv2d.restype = i32
        L.qnn_quantize_ste_backward.argtypes = [vp, vp, i64, f32, vp, vp]
        L.qnn_quantize_ste_backward.restype = i32
        L.qnn_encoder_backward.argtypes = [vp, vp, i64, f32, i32, vp, vp]
        L.qnn_encoder_backward.restype = i32
        L.qnn_encode_levels_fp4.argtypes = [vp, i32, i64, f32, i32, vp, vp]
        L.qnn_encode_levels_fp4.restype = i32
        L.qnn_levels_to_fp4.argtypes = [vp, i64, vp, vp]
        L.qnn_levels_to_fp4.restype = i32
        L.qnn_level_conv2d_fp4.argtypes = [ctypes.POINTER(qnn_conv_desc), vp, vp, vp, vp, vp, vp, f32, i32, vp]
        L.qnn_level_conv2d_fp4.restype = i32
        L.qnn_level_conv2d_block_fp4.argtypes = L.qnn_conv2d_block.argtypes
        L.qnn_level_conv2d_block_fp4.restype = i32
        L.qnn_maxpool_levels_fp4.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, i32, vp, vp]
        L.qnn_maxpool_levels_fp4.restype = i32
        L.qnn_last_error.argtypes = []
        L.qnn_last_error.restype = ctypes.c_char_p
        L.qnn_version.argtypes = []
        L.qnn_version.restype = i32
        _lib = L
    return _lib


def _check(rc):
    if rc != QNN_OK:
        raise QnnError(rc, lib().qnn_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_DTYPES = {torch.float32: QNN_DTYPE_F32, torch.bfloat16: QNN_DTYPE_BF16, torch.int8: QNN_DTYPE_I8}


def qnn_version():
    return lib().qnn_version()


def qnn_encode_pack(src, clip, bits, planes=None):
    """src: CUDA tensor [..., n] (fp32 / bf16 values, or int8 levels), contiguous.  Returns planes
    uint32-as-int32 [bits][rows][ceil(n/32)] with rows = product of the leading dimensions."""
    assert src.is_cuda and src.is_contiguous() and src.dtype in _DTYPES
    n = src.shape[-1]
    rows = src.numel() // n if n else 0
    nw = (n + 31) // 32
    if planes is None:
        planes = torch.empty((bits, rows, nw), dtype=torch.int32, device=src.device)
    _check(lib().qnn_encode_pack(_ptr(src), _DTYPES[src.dtype], rows, n, n, float(clip), int(bits),
                                 _ptr(planes), _stream()))
    return planes


def qnn_fc_fused(src, clip, a_bits, w_planes, want_acc=True, scale=None, acc=None, out=None):
    """src [rows][n] (fp32 / bf16 values or int8 levels, contiguous), w_planes [w_bits][cols][nw] ->
    (acc int32 [rows][cols] or None, out fp32 [rows][cols] or None): qnn_encode_pack + qnn_binary_gemm in one launch."""
    assert src.is_cuda and src.is_contiguous() and src.dtype in _DTYPES and src.dim() == 2
    rows, n = src.shape
    w_bits, cols, nw = w_planes.shape
    assert nw == (n + 31) // 32
    if want_acc and acc is None:
        acc = torch.empty((rows, cols), dtype=torch.int32, device=src.device)
    if scale is not None and out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=src.device)
    _check(lib().qnn_fc_fused(_ptr(src), _DTYPES[src.dtype], rows, n, n, float(clip), int(a_bits), _ptr(w_planes), w_bits,
                              cols, _ptr(scale), _ptr(acc), _ptr(out), _stream()))
    return acc, out


def qnn_binary_gemm(a_planes, w_planes, n, want_acc=True, scale=None, acc=None, out=None):
    """a_planes [a_bits][rows][nw], w_planes [w_bits][cols][nw] -> (acc int32 [rows][cols] or None,
    out fp32 [rows][cols] or None)."""
    a_bits, rows, nw = a_planes.shape
    w_bits, cols, nw2 = w_planes.shape
    assert nw == nw2 == (n + 31) // 32
    dev = a_planes.device
    if want_acc and acc is None:
        acc = torch.empty((rows, cols), dtype=torch.int32, device=dev)
    if scale is not None and out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    _check(lib().qnn_binary_gemm(_ptr(a_planes), a_bits, _ptr(w_planes), w_bits, rows, cols, n,
                                 _ptr(acc), _ptr(scale), _ptr(out), _stream()))
    return acc, out


def qnn_level_row_bytes(n):
    return lib().qnn_level_row_bytes(int(n))


def qnn_plane_sum_i8(planes, n, levels=None):
    """planes [bits][rows][nw] -> int8 levels [rows][qnn_level_row_bytes(n)] (bit-plane-sum variant)."""
    bits, rows, nw = planes.shape
    assert nw == (n + 31) // 32
    if levels is None:
        levels = torch.empty((rows, qnn_level_row_bytes(n)), dtype=torch.int8, device=planes.device)
    _check(lib().qnn_plane_sum_i8(_ptr(planes), bits, rows, n, _ptr(levels), _stream()))
    return levels


def qnn_level_gemm_i8(a_levels, w_levels, n, want_acc=True, scale=None, acc=None, out=None):
    """int8 MFMA GEMM on levels as written by qnn_plane_sum_i8 -> (acc int32 or None, out fp32 or None)."""
    rows, cols = a_levels.shape[0], w_levels.shape[0]
    assert a_levels.shape[1] == w_levels.shape[1] == qnn_level_row_bytes(n)
    dev = a_levels.device
    if want_acc and acc is None:
        acc = torch.empty((rows, cols), dtype=torch.int32, device=dev)
    if scale is not None and out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    _check(lib().qnn_level_gemm_i8(_ptr(a_levels), _ptr(w_levels), rows, cols, n, _ptr(acc), _ptr(scale),
                                   _ptr(out), _stream()))
    return acc, out


def qnn_pool_out_size(size, k, stride, pad=0, ceil_mode=False):
    return int(lib().qnn_pool_out_size(int(size), int(k), int(stride), int(pad), int(bool(ceil_mode))))


def qnn_maxpool_planes(planes, shape, channels, k, stride, pad=0, ceil_mode=False, out=None):
    """planes [bits][B*H*W][cw] of an NHWC tensor of shape=(B, H, W) -> planes [bits][B*Ho*Wo][cw]."""
    B, H, W = shape
    bits, rows, cw = planes.shape
    assert rows == B * H * W and cw == (channels + 31) // 32
    ho, wo = qnn_pool_out_size(H, k, stride, pad, ceil_mode), qnn_pool_out_size(W, k, stride, pad, ceil_mode)
    if out is None:
        out = torch.empty((bits, B * max(ho, 0) * max(wo, 0), cw), dtype=torch.int32, device=planes.device)
    _check(lib().qnn_maxpool_planes(_ptr(planes), bits, B, H, W, channels, int(k), int(stride), int(pad),
                                    int(bool(ceil_mode)), _ptr(out), _stream()))
    return out


def qnn_maxpool_levels_i8(levels, k, stride, pad=0, ceil_mode=False, out=None):
    """int8 levels [B][H][W][C] -> [B][Ho][Wo][C]."""
    B, H, W, C = levels.shape
    ho, wo = qnn_pool_out_size(H, k, stride, pad, ceil_mode), qnn_pool_out_size(W, k, stride, pad, ceil_mode)
    if out is None:
        out = torch.empty((B, max(ho, 0), max(wo, 0), C), dtype=torch.int8, device=levels.device)
    _check(lib().qnn_maxpool_levels_i8(_ptr(levels), B, H, W, C, int(k), int(stride), int(pad),
                                       int(bool(ceil_mode)), _ptr(out), _stream()))
    return out


def qnn_fp4_row_bytes(n):
    return int(lib().qnn_fp4_row_bytes(int(n)))


def qnn_plane_sum_fp4(planes, n, levels=None):
    """planes [bits][rows][nw], bits <= 2 -> fp4 levels, two per byte, uint8 [rows][qnn_fp4_row_bytes(n)]."""
    bits, rows, nw = planes.shape
    assert nw == (n + 31) // 32
    if levels is None:
        levels = torch.empty((rows, qnn_fp4_row_bytes(n)), dtype=torch.uint8, device=planes.device)
    _check(lib().qnn_plane_sum_fp4(_ptr(planes), bits, rows, n, _ptr(levels), _stream()))
    return levels


def qnn_level_gemm_fp4(a_levels, w_levels, n, want_acc=True, scale=None, acc=None, out=None):
    """fp4 MFMA GEMM on levels as written by qnn_plane_sum_fp4 -> (acc int32 or None, out fp32 or None)."""
    rows, cols = a_levels.shape[0], w_levels.shape[0]
    assert a_levels.shape[1] == w_levels.shape[1] == qnn_fp4_row_bytes(n)
    dev = a_levels.device
    if want_acc and acc is None:
        acc = torch.empty((rows, cols), dtype=torch.int32, device=dev)
    if scale is not None and out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    _check(lib().qnn_level_gemm_fp4(_ptr(a_levels), _ptr(w_levels), rows, cols, n, _ptr(acc), _ptr(scale),
                                    _ptr(out), _stream()))
    return acc, out


def qnn_encode_levels_i8(src, clip, bits, levels=None):
    """src: CUDA fp32 / bf16 tensor, contiguous -> int8 levels of the same shape."""
    assert src.is_cuda and src.is_contiguous() and src.dtype in (torch.float32, torch.bfloat16)
    if levels is None:
        levels = torch.empty(src.shape, dtype=torch.int8, device=src.device)
    _check(lib().qnn_encode_levels_i8(_ptr(src), _DTYPES[src.dtype], src.numel(), float(clip), int(bits),
                                      _ptr(levels), _stream()))
    return levels


def _block_epilogue(bias, res_q, res_bits, res_scale, res_f32, relu=False):
    return qnn_block_epilogue(_ptr(bias), _ptr(res_q), int(res_bits), float(res_scale), _ptr(res_f32), int(bool(relu)))


def _level_conv(entry, epi, a_levels, w_levels, stride, pad, a_bits, w_bits, scale, want_acc, want_out, next_clip,
                next_bits, acc, out, next_levels):
    B, H, W, cin = a_levels.shape
    cout, kh, kw, cin2 = w_levels.shape
    assert cin == cin2 and a_levels.dtype == torch.int8 and w_levels.dtype == torch.int8
    assert a_levels.is_contiguous() and w_levels.is_contiguous()
    ho = (H + 2 * pad - kh) // stride + 1
    wo = (W + 2 * pad - kw) // stride + 1
    dev = a_levels.device
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    if want_acc and acc is None:
        acc = torch.empty((B, ho, wo, cout), dtype=torch.int32, device=dev)
    if want_out and out is None:
        out = torch.empty((B, ho, wo, cout), dtype=torch.float32, device=dev)
    if next_clip is not None and next_levels is None:
        next_levels = torch.empty((B, ho, wo, cout), dtype=torch.int8, device=dev)
    head = (ctypes.byref(d), _ptr(a_levels), _ptr(w_levels), _ptr(scale))
    tail = (_ptr(acc), _ptr(out), _ptr(next_levels), float(next_clip) if next_clip is not None else 0.0,
            int(next_bits), _stream())
    _check(entry(*head, *tail) if epi is None else entry(*head, ctypes.byref(epi), *tail))
    return acc, out, next_levels


def qnn_level_conv2d_i8(a_levels, w_levels, stride, pad, a_bits, w_bits, scale=None, want_acc=True,
                        want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """a_levels int8 [B][H][W][Cin], w_levels int8 [Cout][kh][kw][Cin].  Returns (acc, out, next_levels);
    entries not requested are None."""
    return _level_conv(lib().qnn_level_conv2d_i8, None, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                       want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_level_conv2d_block_i8(a_levels, w_levels, stride, pad, a_bits, w_bits, scale, bias=None, res_levels=None,
                              res_bits=0, res_scale=0.0, res_f32=None, want_acc=True, want_out=False,
                              next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, relu=False):
    """qnn_level_conv2d_i8 with the residual-block terms: bias fp32 [Cout], res_levels int8 [B][Ho][Wo][Cout]
    with its factor res_scale, res_f32 fp32 [B][Ho][Wo][Cout], relu (max(y, 0) after them)."""
    epi = _block_epilogue(bias, res_levels, res_bits, res_scale, res_f32, relu)
    return _level_conv(lib().qnn_level_conv2d_block_i8, epi, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                       want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_deconv_pack_weights(w_planes, cin, stride, phase_planes=None):
    """w_planes [w_bits][Cout][kh][kw][cw] -> the phase-ordered sub-kernel planes qnn_deconv2d reads (1-D int32)."""
    w_bits, cout, kh, kw, cw = w_planes.shape
    assert cw == (cin + 31) // 32 and w_planes.is_contiguous()
    words = lib().qnn_deconv_phase_words(w_bits, cout, kh, kw, cin, stride)
    if words < 0:
        raise QnnError(QNN_ERR_INVALID_ARG, "qnn_deconv_phase_words: bad geometry")
    if phase_planes is None:
        phase_planes = torch.zeros((words,), dtype=torch.int32, device=w_planes.device)
    assert phase_planes.numel() >= words
    _check(lib().qnn_deconv_pack_weights(_ptr(w_planes), w_bits, cout, kh, kw, cin, stride, _ptr(phase_planes), _stream()))
    return phase_planes


def qnn_deconv2d(a_planes, phase_planes, shape, cin, cout, kh, kw, stride, pad, w_bits, scale=None, bias=None,
                 want_acc=True, want_out=False, next_clip=None, next_bits=0, acc=None, out=None, next_planes=None):
    """Transposed convolution of a_planes [a_bits][B*H*W][cw], shape = (B, H, W), with weights from
    qnn_deconv_pack_weights.  Returns (acc, out, next_planes) on the [B][Ho][Wo][Cout] output."""
    B, H, W = shape
    a_bits = a_planes.shape[0]
    ho, wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
    dev = a_planes.device
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    if want_acc and acc is None:
        acc = torch.empty((B, ho, wo, cout), dtype=torch.int32, device=dev)
    if want_out and out is None:
        out = torch.empty((B, ho, wo, cout), dtype=torch.float32, device=dev)
    if next_clip is not None and next_planes is None:
        next_planes = torch.empty((next_bits, B * ho * wo, (cout + 31) // 32), dtype=torch.int32, device=dev)
    _check(lib().qnn_deconv2d(ctypes.byref(d), _ptr(a_planes), _ptr(phase_planes), _ptr(scale), _ptr(bias), _ptr(acc),
                              _ptr(out), _ptr(next_planes), float(next_clip) if next_clip is not None else 0.0,
                              int(next_bits), _stream()))
    return acc, out, next_planes


def qnn_quantize_ste_backward(x, grad_q, clip, grad_x=None):
    """x, grad_q fp32 of one shape -> grad_x fp32 (straight-through gradient of the ladder behind the range limit)."""
    assert x.dtype == torch.float32 and grad_q.dtype == torch.float32 and x.shape == grad_q.shape
    if grad_x is None:
        grad_x = torch.empty_like(x)
    _check(lib().qnn_quantize_ste_backward(_ptr(x), _ptr(grad_q), x.numel(), float(clip), _ptr(grad_x), _stream()))
    return grad_x


def qnn_encoder_backward(x, grad_planes, clip, grad_x=None):
    """x fp32 [...], grad_planes fp32 [bits][...] -> grad_x fp32 (surrogate gradient of the encoder)."""
    bits = grad_planes.shape[0]
    assert x.dtype == torch.float32 and grad_planes.dtype == torch.float32 and grad_planes.shape[1:] == x.shape
    assert grad_planes.is_contiguous() and x.is_contiguous()
    if grad_x is None:
        grad_x = torch.empty_like(x)
    _check(lib().qnn_encoder_backward(_ptr(x), _ptr(grad_planes), x.numel(), float(clip), bits, _ptr(grad_x), _stream()))
    return grad_x


def qnn_encode_levels_fp4(src, clip, bits, levels=None):
    """fp32 / bf16 [..., C] (C even) -> fp4 levels uint8 [..., C / 2], two channels per byte."""
    dtype = {torch.float32: QNN_DTYPE_F32, torch.bfloat16: QNN_DTYPE_BF16}[src.dtype]
    assert src.is_contiguous() and src.shape[-1] % 2 == 0
    if levels is None:
        levels = torch.empty(src.shape[:-1] + (src.shape[-1] // 2,), dtype=torch.uint8, device=src.device)
    _check(lib().qnn_encode_levels_fp4(_ptr(src), dtype, src.numel(), float(clip), int(bits), _ptr(levels), _stream()))
    return levels


def qnn_levels_to_fp4(levels, out=None):
    """int8 levels [..., C] (C even, |level| <= 3) -> fp4 levels uint8 [..., C / 2]."""
    assert levels.dtype == torch.int8 and levels.is_contiguous() and levels.shape[-1] % 2 == 0
    if out is None:
        out = torch.empty(levels.shape[:-1] + (levels.shape[-1] // 2,), dtype=torch.uint8, device=levels.device)
    _check(lib().qnn_levels_to_fp4(_ptr(levels), levels.numel(), _ptr(out), _stream()))
    return out


def _level_conv_fp4(entry, epi, a_levels, w_levels, stride, pad, a_bits, w_bits, scale, want_acc, want_out, next_clip,
                    next_bits, acc, out, next_levels):
    B, H, W, cinb = a_levels.shape
    cout, kh, kw, cinb2 = w_levels.shape
    assert cinb == cinb2 and a_levels.dtype == torch.uint8 and w_levels.dtype == torch.uint8
    assert a_levels.is_contiguous() and w_levels.is_contiguous()
    ho = (H + 2 * pad - kh) // stride + 1
    wo = (W + 2 * pad - kw) // stride + 1
    dev = a_levels.device
    d = qnn_conv_desc(B, H, W, 2 * cinb, cout, kh, kw, stride, pad, a_bits, w_bits)
    if want_acc and acc is None:
        acc = torch.empty((B, ho, wo, cout), dtype=torch.int32, device=dev)
    if want_out and out is None:
        out = torch.empty((B, ho, wo, cout), dtype=torch.float32, device=dev)
    if next_clip is not None and next_levels is None:
        next_levels = torch.empty((B, ho, wo, cout // 2), dtype=torch.uint8, device=dev)
    head = (ctypes.byref(d), _ptr(a_levels), _ptr(w_levels), _ptr(scale))
    tail = (_ptr(acc), _ptr(out), _ptr(next_levels), float(next_clip) if next_clip is not None else 0.0,
            int(next_bits), _stream())
    _check(entry(*head, *tail) if epi is None else entry(*head, ctypes.byref(epi), *tail))
    return acc, out, next_levels


def qnn_level_conv2d_fp4(a_levels, w_levels, stride, pad, a_bits, w_bits, scale=None, want_acc=True, want_out=False,
                         next_clip=None, next_bits=0, acc=None, out=None, next_levels=None):
    """a_levels uint8 [B][H][W][Cin/2], w_levels uint8 [Cout][kh][kw][Cin/2] (fp4, two channels per byte).
    Returns (acc, out, next_levels [B][Ho][Wo][Cout/2]); entries not requested are None."""
    return _level_conv_fp4(lib().qnn_level_conv2d_fp4, None, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                           want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_level_conv2d_block_fp4(a_levels, w_levels, stride, pad, a_bits, w_bits, scale, bias=None, res_levels=None,
                               res_bits=0, res_scale=0.0, res_f32=None, want_acc=True, want_out=False,
                               next_clip=None, next_bits=0, acc=None, out=None, next_levels=None, relu=False):
    """qnn_level_conv2d_fp4 with the residual-block terms; res_levels uint8 fp4 [B][Ho][Wo][Cout/2]."""
    epi = _block_epilogue(bias, res_levels, res_bits, res_scale, res_f32, relu)
    return _level_conv_fp4(lib().qnn_level_conv2d_block_fp4, epi, a_levels, w_levels, stride, pad, a_bits, w_bits, scale,
                           want_acc, want_out, next_clip, next_bits, acc, out, next_levels)


def qnn_maxpool_levels_fp4(levels, k, stride, pad=0, ceil_mode=False, out=None):
    """levels uint8 [B][H][W][C/2] (fp4) -> pooled uint8 [B][Ho][Wo][C/2]."""
    B, H, W, cb = levels.shape
    ho, wo = qnn_pool_out_size(H, k, stride, pad, ceil_mode), qnn_pool_out_size(W, k, stride, pad, ceil_mode)
    if out is None:
        out = torch.empty((B, max(ho, 0), max(wo, 0), cb), dtype=torch.uint8, device=levels.device)
    _check(lib().qnn_maxpool_levels_fp4(_ptr(levels), B, H, W, 2 * cb, k, stride, pad, int(ceil_mode), _ptr(out), _stream()))
    return out


def qnn_dense_conv2d_f32(x, w, stride, pad, scale=None, shift=None, relu=False, want_out=True, next_clip=None,
                         next_bits=0, out=None, next_planes=None):
    """x fp32 [B][H][W][Cin], w fp32 [Cout][kh][kw][Cin] -> (out fp32 [B][Ho][Wo][Cout] or None,
    next planes int32 [next_bits][B*Ho*Wo][ceil(Cout/32)] or None)."""
    B, H, W, cin = x.shape
    cout, kh, kw, cin2 = w.shape
    assert cin == cin2
    ho, wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    if want_out and out is None:
        out = torch.empty((B, max(ho, 0), max(wo, 0), cout), dtype=torch.float32, device=x.device)
    if next_bits and next_planes is None:
        next_planes = torch.empty((next_bits, B * max(ho, 0) * max(wo, 0), (cout + 31) // 32), dtype=torch.int32,
                                  device=x.device)
    d = qnn_dense_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad)
    _check(lib().qnn_dense_conv2d_f32(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(scale), _ptr(shift), int(bool(relu)),
                                      _ptr(out), _ptr(next_planes), float(next_clip or 0.0), int(next_bits), _stream()))
    return out, next_planes


def qnn_dense_conv2d_f32_levels(x, w, stride, pad, next_clip, next_bits, scale=None, shift=None, relu=False, want_out=False,
                                out=None, next_levels=None):
    """As qnn_dense_conv2d_f32 with the quantized output as int8 levels [B][Ho][Wo][Cout]: (out or None, levels)."""
    B, H, W, cin = x.shape
    cout, kh, kw, cin2 = w.shape
    assert cin == cin2
    ho, wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    if want_out and out is None:
        out = torch.empty((B, max(ho, 0), max(wo, 0), cout), dtype=torch.float32, device=x.device)
    if next_levels is None:
        next_levels = torch.empty((B, max(ho, 0), max(wo, 0), cout), dtype=torch.int8, device=x.device)
    d = qnn_dense_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad)
    _check(lib().qnn_dense_conv2d_f32_levels(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(scale), _ptr(shift), int(bool(relu)),
                                             _ptr(out), _ptr(next_levels), float(next_clip), int(next_bits), _stream()))
    return out, next_levels


def qnn_global_avgpool_f32(x, out=None):
    """x fp32 [B][H][W][C] (or [B][hw][C]) -> fp32 [B][C]."""
    B, C = x.shape[0], x.shape[-1]
    hw = 1
    for extent in x.shape[1:-1]:
        hw *= extent
    if out is None:
        out = torch.empty((B, C), dtype=torch.float32, device=x.device)
    _check(lib().qnn_global_avgpool_f32(_ptr(x), B, hw, C, _ptr(out), _stream()))
    return out


def qnn_dense_fc_f32(x, w, bias=None, out=None):
    """x fp32 [rows][n], w fp32 [cols][n], bias fp32 [cols] or None -> fp32 [rows][cols]."""
    rows, n = x.shape
    cols = w.shape[0]
    assert w.shape[1] == n
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=x.device)
    _check(lib().qnn_dense_fc_f32(_ptr(x), _ptr(w), _ptr(bias), rows, cols, n, _ptr(out), _stream()))
    return out


def qnn_probe_valu(mode, workgroups, iters, out):
    """Launch the register-only issue-rate loop (see include/qnn.h); out: int32 [workgroups*256]."""
    assert out.numel() >= workgroups * 256
    _check(lib().qnn_probe_valu(int(mode), int(workgroups), int(iters), _ptr(out), _stream()))


def qnn_probe_mfma(mode, workgroups, iters, out):
    """Launch the register-only MFMA loop (see include/qnn.h); out: int32 [workgroups*256]."""
    assert out.numel() >= workgroups * 256
    _check(lib().qnn_probe_mfma(int(mode), int(workgroups), int(iters), _ptr(out), _stream()))


def qnn_dequant_scale(acc, scale, out=None):
    rows, cols = acc.shape[:-1].numel(), acc.shape[-1]
    if out is None:
        out = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    _check(lib().qnn_dequant_scale(_ptr(acc), _ptr(scale), rows, cols, _ptr(out), _stream()))
    return out


def _conv(entry, epi, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out, next_clip, next_bits,
          acc, out, next_planes):
    B, H, W = shape
    a_bits = a_planes.shape[0]
    w_bits, cout, kh, kw, cw = w_planes.shape
    assert cw == (cin + 31) // 32 and a_planes.numel() == a_bits * B * H * W * cw
    ho = (H + 2 * pad - kh) // stride + 1
    wo = (W + 2 * pad - kw) // stride + 1
    dev = a_planes.device
    d = qnn_conv_desc(B, H, W, cin, cout, kh, kw, stride, pad, a_bits, w_bits)
    if want_acc and acc is None:
        acc = torch.empty((B, ho, wo, cout), dtype=torch.int32, device=dev)
    if want_out and out is None:
        out = torch.empty((B, ho, wo, cout), dtype=torch.float32, device=dev)
    if next_clip is not None and next_planes is None:
        next_planes = torch.empty((next_bits, B * ho * wo, (cout + 31) // 32), dtype=torch.int32, device=dev)
    head = (ctypes.byref(d), _ptr(a_planes), _ptr(w_planes), _ptr(scale))
    tail = (_ptr(acc), _ptr(out), _ptr(next_planes), float(next_clip) if next_clip is not None else 0.0,
            int(next_bits), _stream())
    _check(entry(*head, *tail) if epi is None else entry(*head, ctypes.byref(epi), *tail))
    return acc, out, next_planes


def qnn_conv2d(a_planes, w_planes, shape, cin, stride, pad, scale=None, want_acc=True, want_out=False,
               next_clip=None, next_bits=0, acc=None, out=None, next_planes=None):
    """a_planes [a_bits][B*H*W][cw] for an NHWC tensor of shape=(B, H, W); w_planes
    [w_bits][Cout][kh][kw][cw].  Returns (acc, out, next_planes); entries not requested are None."""
    return _conv(lib().qnn_conv2d, None, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out,
                 next_clip, next_bits, acc, out, next_planes)


def qnn_conv2d_block(a_planes, w_planes, shape, cin, stride, pad, scale, bias=None, res_planes=None, res_scale=0.0,
                     res_f32=None, want_acc=True, want_out=False, next_clip=None, next_bits=0, acc=None, out=None,
                     next_planes=None, relu=False):
    """qnn_conv2d with the residual-block terms: bias fp32 [Cout], res_planes [res_bits][B*Ho*Wo][ceil(Cout/32)]
    with its factor res_scale, res_f32 fp32 [B][Ho][Wo][Cout], relu (max(y, 0) after them)."""
    res_bits = res_planes.shape[0] if res_planes is not None else 0
    epi = _block_epilogue(bias, res_planes, res_bits, res_scale, res_f32, relu)
    return _conv(lib().qnn_conv2d_block, epi, a_planes, w_planes, shape, cin, stride, pad, scale, want_acc, want_out,
                 next_clip, next_bits, acc, out, next_planes)
