"""ctypes loader and numpy marshalling for the C oracle (``qnn_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this module; the product path must not.

Every function here only converts arrays and calls the C routine of the same
name; the arithmetic, with its citations of the paper, is in the C file.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qnn_oracle.c")
_LIB = os.path.join(_HERE, "libqnn_oracle.so")

__all__ = [
    "build", "threads", "encode", "decode", "pack_planes", "gemm", "gemm_wt", "conv3x3",
    "conv2d", "conv2d_transposed", "conv_out_size", "encode_real",
    "branch_dot", "scale_f64", "scale_f32", "maxpool2x2", "round_odd", "requant",
    "encode_smooth", "encoder_backward", "binarize", "binarize_backward", "quantize_k", "quantize_k_backward",
    "branch_backward_input", "branch_backward_weight", "update_sgd", "update_adam",
    "conv3x3_backward_input", "conv3x3_backward_weight",
]


def build(force=True):
    """Compile the oracle with gcc (-O2, no fast-math, no FMA contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-Wall", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.qnn_oracle_encode.argtypes = [i64, i32, vp]
        lib.qnn_oracle_encode.restype = i32
        lib.qnn_oracle_decode.argtypes = [vp, i32]
        lib.qnn_oracle_decode.restype = i64
        lib.qnn_oracle_pack_planes.argtypes = [vp, i64, i64, i32, vp]
        lib.qnn_oracle_pack_planes.restype = i64
        lib.qnn_oracle_gemm.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.qnn_oracle_gemm.restype = None
        lib.qnn_oracle_gemm_wt.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.qnn_oracle_gemm_wt.restype = None
        lib.qnn_oracle_conv3x3.argtypes = [vp, vp, i64, i64, i64, i64, i64, vp]
        lib.qnn_oracle_conv3x3.restype = None
        conv_args = [vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32, i32, i64, i64, vp]
        lib.qnn_oracle_conv2d.argtypes = conv_args
        lib.qnn_oracle_conv2d.restype = None
        lib.qnn_oracle_conv2d_transposed.argtypes = conv_args
        lib.qnn_oracle_conv2d_transposed.restype = None
        lib.qnn_oracle_branch_dot.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        lib.qnn_oracle_branch_dot.restype = i64
        lib.qnn_oracle_scale_f64.argtypes = [vp, i64, i64, vp, vp]
        lib.qnn_oracle_scale_f64.restype = None
        lib.qnn_oracle_scale_f32.argtypes = [vp, i64, i64, vp, vp]
        lib.qnn_oracle_scale_f32.restype = None
        lib.qnn_oracle_encode_real.argtypes = [vp, i64, i32, i32, vp]
        lib.qnn_oracle_encode_real.restype = None
        lib.qnn_oracle_encode_smooth.argtypes = [vp, i64, i32, i32, vp, vp]
        lib.qnn_oracle_encode_smooth.restype = None
        lib.qnn_oracle_encoder_backward.argtypes = [vp, vp, i64, i32, vp]
        lib.qnn_oracle_encoder_backward.restype = None
        lib.qnn_oracle_binarize.argtypes = [vp, i64, vp]
        lib.qnn_oracle_binarize.restype = None
        lib.qnn_oracle_binarize_backward.argtypes = [vp, vp, i64, vp]
        lib.qnn_oracle_binarize_backward.restype = None
        lib.qnn_oracle_quantize_k.argtypes = [vp, i64, i32, ctypes.c_float, vp, vp]
        lib.qnn_oracle_quantize_k.restype = None
        lib.qnn_oracle_quantize_k_backward.argtypes = [vp, vp, i64, ctypes.c_float, vp]
        lib.qnn_oracle_quantize_k_backward.restype = None
        lib.qnn_oracle_branch_backward_input.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        lib.qnn_oracle_branch_backward_input.restype = None
        lib.qnn_oracle_branch_backward_weight.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        lib.qnn_oracle_branch_backward_weight.restype = None
        lib.qnn_oracle_update_sgd.argtypes = [vp, vp, i64, ctypes.c_float]
        lib.qnn_oracle_update_sgd.restype = None
        cb_args = [vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, vp]
        lib.qnn_oracle_conv3x3_backward_input.argtypes = cb_args
        lib.qnn_oracle_conv3x3_backward_input.restype = None
        lib.qnn_oracle_conv3x3_backward_weight.argtypes = cb_args
        lib.qnn_oracle_conv3x3_backward_weight.restype = None
        f32 = ctypes.c_float
        lib.qnn_oracle_update_adam.argtypes = [vp, vp, vp, vp, i64, f32, f32, f32, f32, i32]
        lib.qnn_oracle_update_adam.restype = None
        lib.qnn_oracle_maxpool2x2.argtypes = [vp, i64, i64, i64, i64, vp]
        lib.qnn_oracle_maxpool2x2.restype = None
        lib.qnn_oracle_round_odd.argtypes = [ctypes.c_float, i32]
        lib.qnn_oracle_round_odd.restype = ctypes.c_int16
        lib.qnn_oracle_requant.argtypes = [vp, i64, i32, vp]
        lib.qnn_oracle_requant.restype = None
        _lib = lib
    return _lib


def threads():
    """Number of OpenMP threads the oracle's parallel loops use."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _codes(a):
    return np.ascontiguousarray(a, dtype=np.int16)


def encode(v, bits):
    """Elements [c_1..c_bits] in {-1,+1} of one odd code; ValueError if not a code."""
    c = np.zeros(8, dtype=np.int8)
    if _L().qnn_oracle_encode(int(v), int(bits), _p(c)) != 0:
        raise ValueError("%r is not a %d-bit {-1,+1} code" % (v, bits))
    return c[:bits].copy()


def decode(c):
    c = np.ascontiguousarray(c, dtype=np.int8)
    return int(_L().qnn_oracle_decode(_p(c), int(c.size)))


def pack_planes(codes, bits):
    """codes[rows][K] -> (planes uint32 [rows][bits][ceil(K/32)], bad_count)."""
    a = _codes(codes)
    rows, K = a.shape
    out = np.zeros((rows, bits, (K + 31) // 32), dtype=np.uint32)
    bad = _L().qnn_oracle_pack_planes(_p(a), rows, K, int(bits), _p(out))
    return out, int(bad)


def gemm(A, W):
    """A[M][K] . W[K][N] -> int64 [M][N]."""
    A, W = _codes(A), _codes(W)
    M, K = A.shape
    K2, N = W.shape
    assert K == K2
    C = np.zeros((M, N), dtype=np.int64)
    _L().qnn_oracle_gemm(_p(A), _p(W), M, N, K, _p(C))
    return C


def gemm_wt(A, Wt):
    """A[M][K] . Wt[N][K]^T -> int64 [M][N]."""
    A, Wt = _codes(A), _codes(Wt)
    M, K = A.shape
    N, K2 = Wt.shape
    assert K == K2
    C = np.zeros((M, N), dtype=np.int64)
    _L().qnn_oracle_gemm_wt(_p(A), _p(Wt), M, N, K, _p(C))
    return C


def conv3x3(X, Wt):
    """X NHWC [Nb][H][W][C], Wt [Cout][3][3][C] -> int64 NHWC [Nb][H][W][Cout]."""
    X, Wt = _codes(X), _codes(Wt)
    Nb, H, W, C = X.shape
    Cout, kh, kw, C2 = Wt.shape
    assert (kh, kw, C2) == (3, 3, C)
    O = np.zeros((Nb, H, W, Cout), dtype=np.int64)
    _L().qnn_oracle_conv3x3(_p(X), _p(Wt), Nb, H, W, C, Cout, _p(O))
    return O


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def conv_out_size(H, K, stride, pad, dil):
    return (H + 2 * pad - dil * (K - 1) - 1) // stride + 1


def conv2d(X, Wt, stride=1, pad=0, dilation=1):
    """X NHWC, Wt [Cout][KH][KW][C] -> int64 NHWC [Nb][Ho][Wo][Cout]; zero padding, no kernel flip."""
    X, Wt = _codes(X), _codes(Wt)
    Nb, H, W, C = X.shape
    Cout, KH, KW, C2 = Wt.shape
    assert C2 == C
    (sh, sw), (ph, pw), (dh, dw) = _pair(stride), _pair(pad), _pair(dilation)
    Ho, Wo = conv_out_size(H, KH, sh, ph, dh), conv_out_size(W, KW, sw, pw, dw)
    assert Ho > 0 and Wo > 0
    O = np.zeros((Nb, Ho, Wo, Cout), dtype=np.int64)
    _L().qnn_oracle_conv2d(_p(X), _p(Wt), Nb, H, W, C, Cout, KH, KW, sh, sw, ph, pw, dh, dw, Ho, Wo, _p(O))
    return O


def conv2d_transposed(X, Wt, stride=1, pad=0, dilation=1, output_padding=0):
    """Transposed convolution: X NHWC, Wt [Cout][KH][KW][C] -> int64 NHWC [Nb][Ho][Wo][Cout],
    Ho = (H-1)*sh - 2*ph + dh*(KH-1) + output_padding + 1."""
    X, Wt = _codes(X), _codes(Wt)
    Nb, H, W, C = X.shape
    Cout, KH, KW, C2 = Wt.shape
    assert C2 == C
    (sh, sw), (ph, pw), (dh, dw), (oph, opw) = _pair(stride), _pair(pad), _pair(dilation), _pair(output_padding)
    Ho = (H - 1) * sh - 2 * ph + dh * (KH - 1) + oph + 1
    Wo = (W - 1) * sw - 2 * pw + dw * (KW - 1) + opw + 1
    assert Ho > 0 and Wo > 0
    O = np.zeros((Nb, Ho, Wo, Cout), dtype=np.int64)
    _L().qnn_oracle_conv2d_transposed(_p(X), _p(Wt), Nb, H, W, C, Cout, KH, KW, sh, sw, ph, pw, dh, dw, Ho, Wo,
                                      _p(O))
    return O


def branch_dot(x, w, xb, wb):
    """x.w through the literal multi-branch sum of +-1 vectors."""
    x, w = _codes(x).ravel(), _codes(w).ravel()
    assert x.size == w.size
    n = x.size
    cm = np.zeros(max(n, 1), dtype=np.int8)
    dk = np.zeros(max(n, 1), dtype=np.int8)
    r = _L().qnn_oracle_branch_dot(_p(x), _p(w), n, int(xb), int(wb), _p(cm), _p(dk))
    if r == -(1 << 63):
        raise ValueError("input holds a value that is not a code")
    return int(r)


def _acc2d(acc):
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    cols = acc.shape[-1]
    return acc, acc.size // cols if cols else 0, cols


def scale_f64(acc, s):
    acc, rows, cols = _acc2d(acc)
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.size == cols
    y = np.zeros(acc.shape, dtype=np.float64)
    _L().qnn_oracle_scale_f64(_p(acc), rows, cols, _p(s), _p(y))
    return y


def scale_f32(acc, s):
    acc, rows, cols = _acc2d(acc)
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.size == cols
    y = np.zeros(acc.shape, dtype=np.float32)
    _L().qnn_oracle_scale_f32(_p(acc), rows, cols, _p(s), _p(y))
    return y


def maxpool2x2(y):
    y = np.ascontiguousarray(y, dtype=np.float32)
    Nb, H, W, C = y.shape
    assert H % 2 == 0 and W % 2 == 0
    o = np.zeros((Nb, H // 2, W // 2, C), dtype=np.float32)
    _L().qnn_oracle_maxpool2x2(_p(y), Nb, H, W, C, _p(o))
    return o


def round_odd(y, bits):
    return int(_L().qnn_oracle_round_odd(float(np.float32(y)), int(bits)))


def requant(y, bits):
    y = np.ascontiguousarray(y, dtype=np.float32)
    codes = np.zeros(y.shape, dtype=np.int16)
    _L().qnn_oracle_requant(_p(y), y.size, int(bits), _p(codes))
    return codes


def encode_real(x, bits, hrelu=False):
    """Real values (nominally in [-1,1], or [0,1] after HReLU) -> odd codes int16, same shape."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.zeros(x.shape, dtype=np.int16)
    _L().qnn_oracle_encode_real(_p(x), x.size, int(bits), 1 if hrelu else 0, _p(codes))
    return codes



def encode_smooth(x, bits, clip):
    """Tanh ("tanh") or Sigmoid ("sigmoid") of Table 1, then the encoder -> (codes int16, limited fp32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.zeros(x.shape, dtype=np.int16)
    limited = np.zeros(x.shape, dtype=np.float32)
    _L().qnn_oracle_encode_smooth(_p(x), x.size, int(bits), {"tanh": 2, "sigmoid": 3}[clip], _p(codes), _p(limited))
    return codes, limited


def encoder_backward(x, g):
    """x fp32 [n], g fp32 [M][n] (gradients of the M encoded bits, low bit first) -> g_x float64 [n]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    M = g.shape[0]
    assert g.shape[1:] == x.shape
    out = np.zeros(x.shape, dtype=np.float64)
    _L().qnn_oracle_encoder_backward(_p(x), _p(g), x.size, int(M), _p(out))
    return out


def binarize(w):
    w = np.ascontiguousarray(w, dtype=np.float32)
    out = np.zeros(w.shape, dtype=np.int8)
    _L().qnn_oracle_binarize(_p(w), w.size, _p(out))
    return out


def binarize_backward(w, g_wb):
    w = np.ascontiguousarray(w, dtype=np.float32)
    g_wb = np.ascontiguousarray(g_wb, dtype=np.float32)
    out = np.zeros(w.shape, dtype=np.float32)
    _L().qnn_oracle_binarize_backward(_p(w), _p(g_wb), w.size, _p(out))
    return out


def quantize_k(x, K, t):
    """-> (quantized fp32, integer levels int32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.zeros(x.shape, dtype=np.float32)
    lv = np.zeros(x.shape, dtype=np.int32)
    _L().qnn_oracle_quantize_k(_p(x), x.size, int(K), ctypes.c_float(t), _p(q), _p(lv))
    return q, lv


def quantize_k_backward(x, g_q, t):
    x = np.ascontiguousarray(x, dtype=np.float32)
    g_q = np.ascontiguousarray(g_q, dtype=np.float32)
    out = np.zeros(x.shape, dtype=np.float32)
    _L().qnn_oracle_quantize_k_backward(_p(x), _p(g_q), x.size, ctypes.c_float(t), _p(out))
    return out


def branch_backward_input(g_a, s, W, xb, wb):
    """Alg. 1 backward through the product, towards the activations.  g_a fp32 [M][N], s fp32 [N] or
    None, W codes [N][K] of wb bits -> float64 [xb][M][K] (gradient of every encoded element, low first)."""
    g_a = np.ascontiguousarray(g_a, dtype=np.float32)
    W = _codes(W)
    M, N = g_a.shape
    K = W.shape[1]
    assert W.shape[0] == N
    sp = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    out = np.zeros((xb, M, K), dtype=np.float64)
    _L().qnn_oracle_branch_backward_input(_p(g_a), None if sp is None else _p(sp), _p(W), M, N, K, int(xb), int(wb), _p(out))
    return out


def branch_backward_weight(g_a, s, A, xb, wb):
    """Alg. 1 backward through the product, towards the binary weights.  g_a fp32 [M][N], s fp32 [N] or
    None, A codes [M][K] of xb bits -> float64 [wb][N][K]."""
    g_a = np.ascontiguousarray(g_a, dtype=np.float32)
    A = _codes(A)
    M, N = g_a.shape
    K = A.shape[1]
    assert A.shape[0] == M
    sp = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    out = np.zeros((wb, N, K), dtype=np.float64)
    _L().qnn_oracle_branch_backward_weight(_p(g_a), None if sp is None else _p(sp), _p(A), M, N, K, int(xb), int(wb), _p(out))
    return out


def update_sgd(w, g, eta):
    w = np.array(w, dtype=np.float32, order="C", copy=True)
    g = np.ascontiguousarray(g, dtype=np.float32)
    _L().qnn_oracle_update_sgd(_p(w), _p(g), w.size, ctypes.c_float(eta))
    return w


def update_adam(w, g, m, v, eta, b1, b2, eps, t):
    """-> (w, m, v) after one Adam step (copies; binary32 throughout)."""
    w, m, v = (np.array(a, dtype=np.float32, order="C", copy=True) for a in (w, m, v))
    g = np.ascontiguousarray(g, dtype=np.float32)
    _L().qnn_oracle_update_adam(_p(w), _p(g), _p(m), _p(v), w.size, ctypes.c_float(eta), ctypes.c_float(b1),
                                ctypes.c_float(b2), ctypes.c_float(eps), int(t))
    return w, m, v


def conv3x3_backward_input(g_a, s, Wt, xb, wb):
    """Alg. 1 backward through a 3x3 / stride 1 / pad 1 convolution, towards the activations.
    g_a fp32 [Nb][H][W][O], s fp32 [O] or None, Wt codes [O][3][3][C] -> float64 [xb][Nb][H][W][C]."""
    g_a = np.ascontiguousarray(g_a, dtype=np.float32)
    Wt = _codes(Wt)
    Nb, H, W, O = g_a.shape
    C = Wt.shape[3]
    assert Wt.shape[:3] == (O, 3, 3)
    sp = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    out = np.zeros((xb, Nb, H, W, C), dtype=np.float64)
    _L().qnn_oracle_conv3x3_backward_input(_p(g_a), None if sp is None else _p(sp), _p(Wt), Nb, H, W, C, O, int(xb), int(wb), _p(out))
    return out


def conv3x3_backward_weight(g_a, s, X, xb, wb):
    """... towards the binary weights.  X codes [Nb][H][W][C] -> float64 [wb][O][3][3][C]."""
    g_a = np.ascontiguousarray(g_a, dtype=np.float32)
    X = _codes(X)
    Nb, H, W, O = g_a.shape
    C = X.shape[3]
    assert X.shape[:3] == (Nb, H, W)
    sp = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    out = np.zeros((wb, O, 3, 3, C), dtype=np.float64)
    _L().qnn_oracle_conv3x3_backward_weight(_p(g_a), None if sp is None else _p(sp), _p(X), Nb, H, W, C, O, int(xb), int(wb), _p(out))
    return out
