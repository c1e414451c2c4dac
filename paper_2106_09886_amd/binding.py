"""Thin Python binding of libqnn (see include/qnn.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device
pointers to the C entry point of the same name on torch's current stream, and returns the
output tensors it allocated.  No step of the method runs in Python or in torch ops.  If the
HIP library has not been built the import of :func:`lib` raises; there is no fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqnn.so")

QNN_OK, QNN_EINVAL, QNN_EALIGN, QNN_EUNSUPPORTED, QNN_EWORKSPACE, QNN_EHIP = range(6)
QNN_PACK_VALIDATE = 1
QNN_TUNE_WAVES_PER_SIMD, QNN_TUNE_ROWS_PER_WAVE, QNN_TUNE_GENERAL_ONLY, QNN_TUNE_BLOCK_ORDER, QNN_TUNE_LDS_PARTIALS = 1, 2, 3, 4, 5
QNN_TUNE_SPLIT_CHANNELS = 6

EXPORTS = (
    "qnn_status_string", "qnn_last_hip_error", "qnn_version", "qnn_device_info", "qnn_tune", "qnn_set_wave_trace",
    "qnn_encode_pack",
    "qnn_branch_gemm", "qnn_conv2d_im2col_workspace_bytes", "qnn_conv2d_im2col", "qnn_conv2d_im2col_static",
    "qnn_conv2d_packed", "qnn_requant_pack", "qnn_scale_epilogue",
    "qnn_requant_workspace_bytes", "qnn_branch_gemm_requant", "qnn_conv2d_packed_requant",
    "qnn_conv2d_im2col_requant_workspace_bytes", "qnn_conv2d_im2col_requant", "qnn_maxpool2x2_planes",
    "qnn_encode_real", "qnn_encoder_backward", "qnn_binarize", "qnn_binarize_backward", "qnn_quantize_k",
    "qnn_quantize_k_backward", "qnn_branch_gemm_backward_input", "qnn_branch_gemm_backward_weight", "qnn_update_sgd", "qnn_update_adam",
    "qnn_conv2d_backward_input", "qnn_conv2d_backward_weight_workspace_bytes", "qnn_conv2d_backward_weight",
    "qnn_compare_mfma_arranged_bytes", "qnn_compare_mfma_arrange", "qnn_compare_mfma_gemm",
    "qnn_compare_dot4_gemm",
    "qnn_conv2d_general_output_size", "qnn_conv2d_general_workspace_bytes", "qnn_conv2d_general",
)


class ConvGeometry(ctypes.Structure):
    """qnn_conv_geometry of include/qnn.h."""
    _fields_ = [(n, ctypes.c_int) for n in ("kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w",
                                            "transposed", "out_pad_h", "out_pad_w", "dense_rows")]


def _pair(v):
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def conv_geometry(kh, kw, stride=1, pad=0, dilation=1, transposed=False, output_padding=0, dense_rows=False):
    (sh, sw), (ph, pw), (dh, dw), (oh, ow) = _pair(stride), _pair(pad), _pair(dilation), _pair(output_padding)
    return ConvGeometry(kh, kw, sh, sw, ph, pw, dh, dw, 1 if transposed else 0, oh, ow, 1 if dense_rows else 0)


class QnnError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = lib().qnn_status_string(status).decode()
        if status == QNN_EHIP:
            msg += " (hipError %d)" % lib().qnn_last_hip_error()
        super().__init__("%s: %s" % (what, msg))


_lib = None


def lib():
    """The loaded C library with argument types set.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libqnn.so is not built (%s); run `python -m paper_2106_09886_amd.build`" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, u32, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint, ctypes.c_size_t
    L.qnn_status_string.argtypes = [i32]
    L.qnn_status_string.restype = ctypes.c_char_p
    L.qnn_last_hip_error.argtypes = []
    L.qnn_last_hip_error.restype = i32
    L.qnn_version.argtypes = []
    L.qnn_version.restype = i32
    L.qnn_device_info.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.qnn_device_info.restype = i32
    L.qnn_tune.argtypes = [i32, i32]
    L.qnn_tune.restype = i32
    L.qnn_set_wave_trace.argtypes = [vp, sz]
    L.qnn_set_wave_trace.restype = i32
    L.qnn_encode_pack.argtypes = [vp, i32, i64, i64, i32, vp, vp, u32, vp]
    L.qnn_encode_pack.restype = i32
    L.qnn_branch_gemm.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, vp, vp, vp]
    L.qnn_branch_gemm.restype = i32
    L.qnn_conv2d_im2col_workspace_bytes.argtypes = [i64, i64, i64, i64, i32]
    L.qnn_conv2d_im2col_workspace_bytes.restype = sz
    L.qnn_conv2d_im2col.argtypes = [vp, i32, i32, vp, i32, i64, i64, i64, i64, i64, vp, vp, vp, vp, sz, vp]
    L.qnn_conv2d_im2col.restype = i32
    L.qnn_conv2d_im2col_static.argtypes = [vp, i32, i32, vp, i32, i64, i64, i64, i64, i64, vp, vp, vp, vp]
    L.qnn_conv2d_im2col_static.restype = i32
    L.qnn_conv2d_packed.argtypes = [vp, i32, vp, i32, i64, i64, i64, i64, i64, vp, vp, vp, vp]
    L.qnn_conv2d_packed.restype = i32
    L.qnn_requant_pack.argtypes = [vp, i64, i64, i64, i64, i32, i32, vp, vp, vp]
    L.qnn_requant_pack.restype = i32
    L.qnn_scale_epilogue.argtypes = [vp, i64, i64, vp, vp, vp]
    L.qnn_scale_epilogue.restype = i32
    L.qnn_requant_workspace_bytes.argtypes = [i64, i64]
    L.qnn_requant_workspace_bytes.restype = sz
    L.qnn_branch_gemm_requant.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, i32, vp, vp, vp, vp, sz, vp]
    L.qnn_branch_gemm_requant.restype = i32
    L.qnn_conv2d_packed_requant.argtypes = [vp, i32, vp, i32, i64, i64, i64, i64, i64, vp, i32, vp, vp, vp, vp,
                                            sz, vp]
    L.qnn_conv2d_packed_requant.restype = i32
    L.qnn_conv2d_im2col_requant_workspace_bytes.argtypes = [i64, i64, i64, i64, i32, i64]
    L.qnn_conv2d_im2col_requant_workspace_bytes.restype = sz
    L.qnn_conv2d_im2col_requant.argtypes = [vp, i32, i32, vp, i32, i64, i64, i64, i64, i64, vp, i32, vp, vp, vp,
                                            vp, sz, vp]
    L.qnn_conv2d_im2col_requant.restype = i32
    L.qnn_maxpool2x2_planes.argtypes = [vp, i64, i64, i64, i64, i32, vp, vp]
    L.qnn_maxpool2x2_planes.restype = i32
    L.qnn_compare_mfma_arranged_bytes.argtypes = [i64, i64]
    L.qnn_compare_mfma_arranged_bytes.restype = sz
    L.qnn_compare_mfma_arrange.argtypes = [vp, i64, i64, vp, vp]
    L.qnn_compare_mfma_arrange.restype = i32
    L.qnn_compare_mfma_gemm.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    L.qnn_compare_mfma_gemm.restype = i32
    L.qnn_compare_dot4_gemm.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    L.qnn_compare_dot4_gemm.restype = i32
    L.qnn_encode_real.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
    L.qnn_encode_real.restype = i32
    L.qnn_encoder_backward.argtypes = [vp, vp, i64, i32, vp, vp]
    L.qnn_encoder_backward.restype = i32
    L.qnn_binarize.argtypes = [vp, i64, i64, vp, vp, vp]
    L.qnn_binarize.restype = i32
    L.qnn_binarize_backward.argtypes = [vp, vp, i64, vp, vp]
    L.qnn_binarize_backward.restype = i32
    L.qnn_quantize_k.argtypes = [vp, i64, i32, ctypes.c_float, vp, vp, vp]
    L.qnn_quantize_k.restype = i32
    L.qnn_quantize_k_backward.argtypes = [vp, vp, i64, ctypes.c_float, vp, vp]
    L.qnn_quantize_k_backward.restype = i32
    L.qnn_branch_gemm_backward_input.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp, vp]
    L.qnn_branch_gemm_backward_input.restype = i32
    L.qnn_branch_gemm_backward_weight.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp, vp]
    L.qnn_branch_gemm_backward_weight.restype = i32
    L.qnn_update_sgd.argtypes = [vp, vp, i64, ctypes.c_float, vp]
    L.qnn_update_sgd.restype = i32
    L.qnn_conv2d_backward_input.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i64, i32, vp, vp]
    L.qnn_conv2d_backward_input.restype = i32
    L.qnn_conv2d_backward_weight_workspace_bytes.argtypes = [i64, i64, i64, i64, i64]
    L.qnn_conv2d_backward_weight_workspace_bytes.restype = sz
    L.qnn_conv2d_backward_weight.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i64, i32, vp, vp, sz, vp]
    L.qnn_conv2d_backward_weight.restype = i32
    f32 = ctypes.c_float
    L.qnn_update_adam.argtypes = [vp, vp, vp, vp, i64, f32, f32, f32, f32, i32, vp]
    L.qnn_update_adam.restype = i32
    gp = ctypes.POINTER(ConvGeometry)
    L.qnn_conv2d_general_output_size.argtypes = [i64, i64, gp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.qnn_conv2d_general_output_size.restype = i32
    L.qnn_conv2d_general_workspace_bytes.argtypes = [i64, i64, i64, i64, i64, i32, i32, gp]
    L.qnn_conv2d_general_workspace_bytes.restype = sz
    L.qnn_conv2d_general.argtypes = [vp, i32, vp, i32, i64, i64, i64, i64, i64, gp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.qnn_conv2d_general.restype = i32
    _lib = L
    return L


def _check(status, what):
    if status != QNN_OK:
        raise QnnError(status, what)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if t.dtype != dtype:
        raise ValueError("%s must have dtype %s" % (name, dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t


def device_info():
    """(compute units, peak shader clock in kHz) of the current GPU."""
    cus, khz = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().qnn_device_info(ctypes.byref(cus), ctypes.byref(khz)), "qnn_device_info")
    return cus.value, khz.value


def tune(waves_per_simd=None, rows_per_wave=None, general_only=None, block_order=None, lds_partials=None,
         split_channels=None):
    if split_channels is not None:
        _check(lib().qnn_tune(QNN_TUNE_SPLIT_CHANNELS, int(split_channels)), "qnn_tune")
    if lds_partials is not None:
        _check(lib().qnn_tune(QNN_TUNE_LDS_PARTIALS, int(lds_partials)), "qnn_tune")
    if block_order is not None:
        _check(lib().qnn_tune(QNN_TUNE_BLOCK_ORDER, int(block_order)), "qnn_tune")
    if general_only is not None:
        _check(lib().qnn_tune(QNN_TUNE_GENERAL_ONLY, int(general_only)), "qnn_tune")
    if waves_per_simd is not None:
        _check(lib().qnn_tune(QNN_TUNE_WAVES_PER_SIMD, int(waves_per_simd)), "qnn_tune")
    if rows_per_wave is not None:
        _check(lib().qnn_tune(QNN_TUNE_ROWS_PER_WAVE, int(rows_per_wave)), "qnn_tune")


def set_wave_trace(buf):
    """buf: int64 GPU tensor receiving 4 words per wavefront, or None to switch tracing off."""
    if buf is None:
        _check(lib().qnn_set_wave_trace(None, 0), "qnn_set_wave_trace")
    else:
        _dev(buf, torch.int64, "buf")
        _check(lib().qnn_set_wave_trace(_ptr(buf), buf.numel() * 8), "qnn_set_wave_trace")


def encode_pack(codes, bits, validate=False, out=None):
    """codes: int8/int16 GPU tensor [rows][K] -> uint32-as-int32 planes [rows][bits][Kw].

    With validate=True also returns the device int32 counter of invalid entries."""
    if codes.dtype not in (torch.int8, torch.int16):
        raise ValueError("codes must be int8 or int16")
    _dev(codes, codes.dtype, "codes")
    rows, K = codes.shape
    Kw = (K + 31) // 32
    planes = out if out is not None else torch.empty((rows, bits, Kw), dtype=torch.int32, device=codes.device)
    bad = torch.zeros(1, dtype=torch.int32, device=codes.device) if validate else None
    st = lib().qnn_encode_pack(_ptr(codes), codes.element_size(), rows, K, bits, _ptr(planes), _ptr(bad),
                               QNN_PACK_VALIDATE if validate else 0, _stream())
    _check(st, "qnn_encode_pack")
    return (planes, bad) if validate else planes


def _outputs(rows_shape, N, device, scale, want_acc):
    acc = torch.empty(tuple(rows_shape) + (N,), dtype=torch.int32, device=device) if want_acc else None
    out = torch.empty(tuple(rows_shape) + (N,), dtype=torch.float32, device=device) if scale is not None else None
    return acc, out


def branch_gemm(A, ab, Wt, wb, K, scale=None, want_acc=True):
    """A planes [M][ab][Kw], Wt planes [N][wb][Kw] -> (acc int32 [M][N] | None, out fp32 | None)."""
    _dev(A, torch.int32, "A")
    _dev(Wt, torch.int32, "Wt")
    M, N = A.shape[0], Wt.shape[0]
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    acc, out = _outputs((M,), N, A.device, scale, want_acc)
    st = lib().qnn_branch_gemm(_ptr(A), ab, _ptr(Wt), wb, M, N, K, _ptr(acc), _ptr(scale), _ptr(out), _stream())
    _check(st, "qnn_branch_gemm")
    return acc, out


def conv2d_im2col_workspace_bytes(Nb, H, W, C, ab):
    return int(lib().qnn_conv2d_im2col_workspace_bytes(Nb, H, W, C, ab))


def conv2d_im2col(x_codes, ab, Wt, wb, Cout, scale=None, want_acc=True, workspace=None, out=None):
    """x_codes NHWC int8/int16, Wt planes [Cout][9][wb][Cw] -> (acc int32 NHWC | None, out fp32 | None)."""
    _dev(x_codes, x_codes.dtype, "x_codes")
    _dev(Wt, torch.int32, "Wt")
    Nb, H, W, C = x_codes.shape
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    if out is None:
        acc, o32 = _outputs((Nb, H, W), Cout, x_codes.device, scale, want_acc)
    else:
        acc, o32 = out
    need = conv2d_im2col_workspace_bytes(Nb, H, W, C, ab)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x_codes.device)
    st = lib().qnn_conv2d_im2col(_ptr(x_codes), x_codes.element_size(), ab, _ptr(Wt), wb, Nb, H, W, C, Cout,
                                 _ptr(acc), _ptr(scale), _ptr(o32), _ptr(workspace), workspace.numel(),
                                 _stream())
    _check(st, "qnn_conv2d_im2col")
    return acc, o32


QNN_STATIC_SCRATCH_BYTES = 8 << 20


def conv2d_im2col_static(x_codes, ab, Wt, wb, Cout, scale=None, want_acc=True, out=None):
    """qnn_conv2d_im2col without a workspace: the library's own static scratch holds the planes.
    With out=(acc, out_f32) the call itself touches no allocator at all."""
    _dev(x_codes, x_codes.dtype, "x_codes")
    _dev(Wt, torch.int32, "Wt")
    Nb, H, W, C = x_codes.shape
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    if out is None:
        acc, o32 = _outputs((Nb, H, W), Cout, x_codes.device, scale, want_acc)
    else:
        acc, o32 = out
    st = lib().qnn_conv2d_im2col_static(_ptr(x_codes), x_codes.element_size(), ab, _ptr(Wt), wb, Nb, H, W, C, Cout,
                                        _ptr(acc), _ptr(scale), _ptr(o32), _stream())
    _check(st, "qnn_conv2d_im2col_static")
    return acc, o32


def conv2d_packed(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, scale=None, want_acc=True, out=None):
    _dev(x_planes, torch.int32, "x_planes")
    _dev(Wt, torch.int32, "Wt")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    if out is None:
        acc, o32 = _outputs((Nb, H, W), Cout, x_planes.device, scale, want_acc)
    else:
        acc, o32 = out
    st = lib().qnn_conv2d_packed(_ptr(x_planes), ab, _ptr(Wt), wb, Nb, H, W, C, Cout, _ptr(acc), _ptr(scale),
                                 _ptr(o32), _stream())
    _check(st, "qnn_conv2d_packed")
    return acc, o32


def requant_pack(y, bits, pool=False, want_codes=True, want_planes=True):
    """y fp32 NHWC -> (codes int8/int16 NHWC | None, planes int32 [pixels][bits][Cw] | None)."""
    _dev(y, torch.float32, "y")
    Nb, H, W, C = y.shape
    Ho, Wo = (H // 2, W // 2) if pool else (H, W)
    codes = torch.empty((Nb, Ho, Wo, C), dtype=torch.int8 if bits <= 7 else torch.int16,
                        device=y.device) if want_codes else None
    planes = torch.empty((Nb * Ho * Wo, bits, (C + 31) // 32), dtype=torch.int32,
                         device=y.device) if want_planes else None
    st = lib().qnn_requant_pack(_ptr(y), Nb, H, W, C, 1 if pool else 0, bits, _ptr(codes), _ptr(planes), _stream())
    _check(st, "qnn_requant_pack")
    return codes, planes


def scale_epilogue(acc, scale):
    _dev(acc, torch.int32, "acc")
    _dev(scale, torch.float32, "scale")
    N = acc.shape[-1]
    M = acc.numel() // N if N else 0
    out = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    _check(lib().qnn_scale_epilogue(_ptr(acc), M, N, _ptr(scale), _ptr(out), _stream()), "qnn_scale_epilogue")
    return out


def _requant_outputs(rows_shape, N, device, scale, out_bits, want_acc, want_f32):
    rows = 1
    for d in rows_shape:
        rows *= d
    planes = torch.empty((rows, out_bits, (N + 31) // 32), dtype=torch.int32, device=device)
    acc = torch.empty(tuple(rows_shape) + (N,), dtype=torch.int32, device=device) if want_acc else None
    o32 = torch.empty(tuple(rows_shape) + (N,), dtype=torch.float32, device=device) if want_f32 else None
    if want_f32 and scale is None:
        raise ValueError("the fp32 output needs a scale")
    return planes, acc, o32, rows


def branch_gemm_requant(A, ab, Wt, wb, K, out_bits, scale=None, want_acc=False, want_f32=False):
    """GEMM + scale + re-encode: -> (planes int32 [M][out_bits][Nw], acc | None, out fp32 | None)."""
    _dev(A, torch.int32, "A")
    _dev(Wt, torch.int32, "Wt")
    M, N = A.shape[0], Wt.shape[0]
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    planes, acc, o32, rows = _requant_outputs((M,), N, A.device, scale, out_bits, want_acc, want_f32)
    ws = None
    if acc is None and o32 is None:
        ws = torch.empty(max(16, int(lib().qnn_requant_workspace_bytes(rows, N))), dtype=torch.uint8, device=A.device)
    st = lib().qnn_branch_gemm_requant(_ptr(A), ab, _ptr(Wt), wb, M, N, K, _ptr(scale), out_bits, _ptr(planes),
                                       _ptr(acc), _ptr(o32), _ptr(ws), 0 if ws is None else ws.numel(), _stream())
    _check(st, "qnn_branch_gemm_requant")
    return planes, acc, o32


def conv2d_packed_requant(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, out_bits, scale=None, want_acc=False,
                          want_f32=False):
    """3x3 conv from packed planes + scale + re-encode -> (planes [Nb*H*W][out_bits][CoutW], acc, out)."""
    _dev(x_planes, torch.int32, "x_planes")
    _dev(Wt, torch.int32, "Wt")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    planes, acc, o32, rows = _requant_outputs((Nb, H, W), Cout, x_planes.device, scale, out_bits, want_acc, want_f32)
    ws = None
    if acc is None and o32 is None:
        ws = torch.empty(max(16, int(lib().qnn_requant_workspace_bytes(rows, Cout))), dtype=torch.uint8,
                         device=x_planes.device)
    st = lib().qnn_conv2d_packed_requant(_ptr(x_planes), ab, _ptr(Wt), wb, Nb, H, W, C, Cout, _ptr(scale), out_bits,
                                         _ptr(planes), _ptr(acc), _ptr(o32), _ptr(ws),
                                         0 if ws is None else ws.numel(), _stream())
    _check(st, "qnn_conv2d_packed_requant")
    return planes, acc, o32


def conv2d_im2col_requant(x_codes, ab, Wt, wb, Cout, out_bits, scale=None, want_acc=False, want_f32=False):
    """3x3 conv from codes + scale + re-encode -> (planes [Nb*H*W][out_bits][CoutW], acc, out)."""
    _dev(x_codes, x_codes.dtype, "x_codes")
    _dev(Wt, torch.int32, "Wt")
    Nb, H, W, C = x_codes.shape
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    planes, acc, o32, rows = _requant_outputs((Nb, H, W), Cout, x_codes.device, scale, out_bits, want_acc, want_f32)
    need = int(lib().qnn_conv2d_im2col_requant_workspace_bytes(Nb, H, W, C, ab, Cout))
    ws = torch.empty(max(16, need), dtype=torch.uint8, device=x_codes.device)
    st = lib().qnn_conv2d_im2col_requant(_ptr(x_codes), x_codes.element_size(), ab, _ptr(Wt), wb, Nb, H, W, C, Cout,
                                         _ptr(scale), out_bits, _ptr(planes), _ptr(acc), _ptr(o32), _ptr(ws),
                                         ws.numel(), _stream())
    _check(st, "qnn_conv2d_im2col_requant")
    return planes, acc, o32


def maxpool2x2_planes(planes, Nb, H, W, C, bits):
    """planes int32 [Nb*H*W][bits][Cw] -> [Nb*(H/2)*(W/2)][bits][Cw]."""
    _dev(planes, torch.int32, "planes")
    out = torch.empty((Nb * (H // 2) * (W // 2), bits, (C + 31) // 32), dtype=torch.int32, device=planes.device)
    st = lib().qnn_maxpool2x2_planes(_ptr(planes), Nb, H, W, C, bits, _ptr(out), _stream())
    _check(st, "qnn_maxpool2x2_planes")
    return out


def conv2d_general_output_size(H, W, geo):
    ho, wo = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().qnn_conv2d_general_output_size(H, W, ctypes.byref(geo), ctypes.byref(ho), ctypes.byref(wo)),
           "qnn_conv2d_general_output_size")
    return ho.value, wo.value


def conv2d_general(x_planes, ab, Wt, wb, Nb, H, W, C, Cout, geo, scale=None, want_acc=True, out_bits=0,
                   workspace=True):
    """Any-geometry convolution from packed planes -> (acc | None, out fp32 | None, planes | None).
    workspace=False withholds the scratch that enables the packed-window path."""
    _dev(x_planes, torch.int32, "x_planes")
    _dev(Wt, torch.int32, "Wt")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    Ho, Wo = conv2d_general_output_size(H, W, geo)
    acc, o32 = _outputs((Nb, Ho, Wo), Cout, x_planes.device, scale, want_acc)
    planes = ws = None
    if out_bits:
        planes = torch.empty((Nb * Ho * Wo, out_bits, (Cout + 31) // 32), dtype=torch.int32, device=x_planes.device)
    if workspace:
        ws = torch.empty(max(16, int(lib().qnn_conv2d_general_workspace_bytes(Nb, H, W, C, Cout, ab, wb,
                                                                              ctypes.byref(geo)))),
                         dtype=torch.uint8, device=x_planes.device)
    elif out_bits and acc is None and o32 is None:
        ws = torch.empty(max(16, int(lib().qnn_requant_workspace_bytes(Nb * Ho * Wo, Cout))), dtype=torch.uint8,
                         device=x_planes.device)
    st = lib().qnn_conv2d_general(_ptr(x_planes), ab, _ptr(Wt), wb, Nb, H, W, C, Cout, ctypes.byref(geo), _ptr(acc),
                                  _ptr(scale), _ptr(o32), out_bits, _ptr(planes), _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream())
    _check(st, "qnn_conv2d_general")
    return acc, o32, planes


CLIPS = {"htanh": 0, "hrelu": 1, "tanh": 2, "sigmoid": 3}


def encode_real(x, bits, hrelu=False, want_codes=True, want_planes=True, clip=None):
    """x fp32 [rows][K] -> (codes int8/int16 | None, planes int32 [rows][bits][Kw] | None).
    clip: "htanh" (default), "hrelu", "tanh" or "sigmoid" (Table 1); hrelu=True is "hrelu"."""
    _dev(x, torch.float32, "x")
    rows, K = x.shape
    mode = CLIPS[clip] if clip is not None else (1 if hrelu else 0)
    codes = torch.empty((rows, K), dtype=torch.int8 if bits <= 7 else torch.int16, device=x.device) if want_codes else None
    planes = torch.empty((rows, bits, (K + 31) // 32), dtype=torch.int32, device=x.device) if want_planes else None
    st = lib().qnn_encode_real(_ptr(x), rows, K, bits, mode, _ptr(codes), _ptr(planes), _stream())
    _check(st, "qnn_encode_real")
    return codes, planes


def encoder_backward(x, g_bits):
    """x fp32 [n], g_bits fp32 [bits][n] -> g_x fp32 [n] (Eq. (12))."""
    _dev(x, torch.float32, "x")
    _dev(g_bits, torch.float32, "g_bits")
    out = torch.empty_like(x)
    _check(lib().qnn_encoder_backward(_ptr(x), _ptr(g_bits), x.numel(), g_bits.shape[0], _ptr(out), _stream()),
           "qnn_encoder_backward")
    return out


def binarize(w, want_codes=True, want_planes=True):
    """w fp32 [rows][K] -> (codes int8 +-1 | None, planes int32 [rows][1][Kw] | None) (Eq. (14))."""
    _dev(w, torch.float32, "w")
    rows, K = w.shape
    codes = torch.empty((rows, K), dtype=torch.int8, device=w.device) if want_codes else None
    planes = torch.empty((rows, 1, (K + 31) // 32), dtype=torch.int32, device=w.device) if want_planes else None
    _check(lib().qnn_binarize(_ptr(w), rows, K, _ptr(codes), _ptr(planes), _stream()), "qnn_binarize")
    return codes, planes


def binarize_backward(w, g_wb):
    _dev(w, torch.float32, "w")
    _dev(g_wb, torch.float32, "g_wb")
    out = torch.empty_like(w)
    _check(lib().qnn_binarize_backward(_ptr(w), _ptr(g_wb), w.numel(), _ptr(out), _stream()), "qnn_binarize_backward")
    return out


def quantize_k(x, bits, t):
    """-> (q fp32, levels int32) of Eq. (15)."""
    _dev(x, torch.float32, "x")
    q = torch.empty_like(x)
    lv = torch.empty(x.shape, dtype=torch.int32, device=x.device)
    _check(lib().qnn_quantize_k(_ptr(x), x.numel(), bits, ctypes.c_float(t), _ptr(q), _ptr(lv), _stream()),
           "qnn_quantize_k")
    return q, lv


def quantize_k_backward(x, g_q, t):
    _dev(x, torch.float32, "x")
    _dev(g_q, torch.float32, "g_q")
    out = torch.empty_like(x)
    _check(lib().qnn_quantize_k_backward(_ptr(x), _ptr(g_q), x.numel(), ctypes.c_float(t), _ptr(out), _stream()),
           "qnn_quantize_k_backward")
    return out


def branch_gemm_backward_input(g_out, Wt, wb, K, ab, scale=None):
    """Alg. 1 backward towards the activations: g_out fp32 [M][N], Wt planes [N][wb][Kw] -> fp32 [ab][M][K]."""
    _dev(g_out, torch.float32, "g_out")
    _dev(Wt, torch.int32, "Wt")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    M, N = g_out.shape
    out = torch.empty((ab, M, K), dtype=torch.float32, device=g_out.device)
    _check(lib().qnn_branch_gemm_backward_input(_ptr(g_out), _ptr(scale), _ptr(Wt), wb, M, N, K, ab, _ptr(out), _stream()),
           "qnn_branch_gemm_backward_input")
    return out


def branch_gemm_backward_weight(g_out, A, ab, K, wb, scale=None):
    """Alg. 1 backward towards the binary weights: g_out fp32 [M][N], A planes [M][ab][Kw] -> fp32 [wb][N][K]."""
    _dev(g_out, torch.float32, "g_out")
    _dev(A, torch.int32, "A")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    M, N = g_out.shape
    out = torch.empty((wb, N, K), dtype=torch.float32, device=g_out.device)
    _check(lib().qnn_branch_gemm_backward_weight(_ptr(g_out), _ptr(scale), _ptr(A), ab, M, N, K, wb, _ptr(out), _stream()),
           "qnn_branch_gemm_backward_weight")
    return out


def update_sgd(w, g, lr):
    """In place: w <- w - lr * g."""
    _dev(w, torch.float32, "w")
    _dev(g, torch.float32, "g")
    _check(lib().qnn_update_sgd(_ptr(w), _ptr(g), w.numel(), ctypes.c_float(lr), _stream()), "qnn_update_sgd")
    return w


def conv2d_backward_input(g_out, Wt, wb, C, ab, scale=None):
    """Alg. 1 backward through the 3x3 convolution, towards the activations: g_out fp32 [Nb][H][W][Cout],
    Wt planes [Cout][9][wb][Cw] -> fp32 [ab][Nb][H][W][C]."""
    _dev(g_out, torch.float32, "g_out")
    _dev(Wt, torch.int32, "Wt")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    Nb, H, W, Cout = g_out.shape
    out = torch.empty((ab, Nb, H, W, C), dtype=torch.float32, device=g_out.device)
    _check(lib().qnn_conv2d_backward_input(_ptr(g_out), _ptr(scale), _ptr(Wt), wb, Nb, H, W, C, Cout, ab, _ptr(out), _stream()),
           "qnn_conv2d_backward_input")
    return out


def conv2d_backward_weight(g_out, x_planes, ab, C, wb, scale=None, workspace=None):
    """... towards the binary weights: x_planes [Nb*H*W][ab][Cw] -> fp32 [wb][Cout][3][3][C]."""
    _dev(g_out, torch.float32, "g_out")
    _dev(x_planes, torch.int32, "x_planes")
    if scale is not None:
        _dev(scale, torch.float32, "scale")
    Nb, H, W, Cout = g_out.shape
    out = torch.empty((wb, Cout, 3, 3, C), dtype=torch.float32, device=g_out.device)
    need = int(lib().qnn_conv2d_backward_weight_workspace_bytes(Nb, H, W, C, Cout))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=g_out.device)
    _check(lib().qnn_conv2d_backward_weight(_ptr(g_out), _ptr(scale), _ptr(x_planes), ab, Nb, H, W, C, Cout, wb, _ptr(out),
                                            _ptr(workspace), workspace.numel(), _stream()), "qnn_conv2d_backward_weight")
    return out


def update_adam(w, g, m, v, lr, beta1, beta2, eps, step):
    """In place: one Adam step on (w, m, v)."""
    for t, name in ((w, "w"), (g, "g"), (m, "m"), (v, "v")):
        _dev(t, torch.float32, name)
    _check(lib().qnn_update_adam(_ptr(w), _ptr(g), _ptr(m), _ptr(v), w.numel(), ctypes.c_float(lr), ctypes.c_float(beta1),
                                 ctypes.c_float(beta2), ctypes.c_float(eps), int(step), _stream()), "qnn_update_adam")
    return w


def compare_mfma_arrange(codes):
    """Comparison line: int8 codes [rows][K] -> opaque matrix-core operand buffer."""
    _dev(codes, torch.int8, "codes")
    rows, K = codes.shape
    out = torch.empty(max(16, int(lib().qnn_compare_mfma_arranged_bytes(rows, K))), dtype=torch.uint8, device=codes.device)
    _check(lib().qnn_compare_mfma_arrange(_ptr(codes), rows, K, _ptr(out), _stream()), "qnn_compare_mfma_arrange")
    return out


def compare_mfma_gemm(A_arranged, Wt_arranged, M, N, K, out=None):
    """Comparison line: acc int32 [M][N] of the decoded product on the int8 matrix cores."""
    acc = out if out is not None else torch.empty((M, N), dtype=torch.int32, device=A_arranged.device)
    _check(lib().qnn_compare_mfma_gemm(_ptr(A_arranged), _ptr(Wt_arranged), M, N, K, _ptr(acc), _stream()),
           "qnn_compare_mfma_gemm")
    return acc


def compare_dot4_gemm(A_codes, Wt_codes, out=None):
    """Comparison line: acc int32 [M][N] of the decoded product with the packed int8 dot product.
    A_codes int8 [M][K], Wt_codes int8 [N][K], K a multiple of 4."""
    _dev(A_codes, torch.int8, "A_codes")
    _dev(Wt_codes, torch.int8, "Wt_codes")
    M, K = A_codes.shape
    N, K2 = Wt_codes.shape
    if K != K2:
        raise ValueError("A_codes and Wt_codes disagree on K")
    acc = out if out is not None else torch.empty((M, N), dtype=torch.int32, device=A_codes.device)
    _check(lib().qnn_compare_dot4_gemm(_ptr(A_codes), _ptr(Wt_codes), M, N, K, _ptr(acc), _stream()),
           "qnn_compare_dot4_gemm")
    return acc
