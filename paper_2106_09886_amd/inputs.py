"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws numbers: odd integer codes with the value ranges and
distributions of the workloads, and per-channel fp32 scales.  It holds none of
the method's arithmetic and imports neither the HIP binding nor the oracle, so
that both can be fed the same bytes.

Random source: a counter-based generator.  Element ``i`` of stream ``seed`` is
``mix(seed * 0x9E3779B97F4A7C15 + i)`` with the 64-bit finalizer ``mix`` below
(xor-shift / multiply rounds), so any element can be reproduced on its own.
"""
from collections import namedtuple
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z):
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z += np.uint64(0x9E3779B97F4A7C15)
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return z


def raw_u64(seed, n, offset=0):
    """n 64-bit words of stream ``seed`` starting at element ``offset``."""
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * np.uint64(0x9E3779B97F4A7C15)
        idx = np.arange(offset, offset + n, dtype=np.uint64)
        return _mix(_mix(base + idx) ^ np.uint64(seed))


def _dtype_for(bits):
    return np.int8 if bits <= 7 else np.int16


def uniform_codes(seed, shape, bits):
    """Odd integers uniform over [-(2^bits-1), 2^bits-1]; int8 (bits<=7) or int16."""
    n = int(np.prod(shape))
    r = raw_u64(seed, n) >> np.uint64(40)
    k = (r % np.uint64(1 << bits)).astype(np.int64)
    v = 2 * k - ((1 << bits) - 1)
    return v.astype(_dtype_for(bits)).reshape(shape)


def relu_like_codes(seed, shape, bits):
    """Half of the entries at the lowest code, the rest uniform over the others."""
    n = int(np.prod(shape))
    r = raw_u64(seed, n)
    low = ((r >> np.uint64(63)) == np.uint64(0))
    k = 1 + ((r >> np.uint64(20)) % np.uint64((1 << bits) - 1)).astype(np.int64)
    k[low] = 0
    v = 2 * k - ((1 << bits) - 1)
    return v.astype(_dtype_for(bits)).reshape(shape)


def uniform_f32(seed, n, lo, hi):
    """fp32 values lo + (hi-lo)*U[0,1) from 24 random bits each."""
    r = (raw_u64(seed, n) >> np.uint64(40)).astype(np.float32)
    u = r * np.float32(1.0 / (1 << 24))
    return (np.float32(lo) + np.float32(hi - lo) * u).astype(np.float32)


# ---------------------------------------------------------------------------
# Workloads.  GEMM: C[M][N] = A[M][K] . W[K][N]; conv: NHWC input, 3x3, stride 1,
# pad 1, weights [Cout][3][3][C].  ``ab``/``wb`` = activation / weight bits.
# ---------------------------------------------------------------------------
Gemm = namedtuple("Gemm", "name M N K ab wb act_dist scale_lo scale_hi beta seeds")
Conv = namedtuple("Conv", "name Nb H W C Cout ab wb act_dist scale_lo scale_hi beta seeds")

WORKLOADS = {
    # small single GEMM, no scaling
    "gemm64": Gemm("gemm64", 64, 64, 256, 2, 2, "uniform", None, None, None, (1001, 2001, 3001)),
    # fully connected layer, batch 256, 4096 -> 4096
    "fc4096": Gemm("fc4096", 256, 4096, 4096, 2, 2, "uniform", 0.01, 0.1, 0.05, (1002, 2002, 3002)),
    # ResNet-18 stage-1 shaped 3x3 conv
    "resnet18_s1": Conv("resnet18_s1", 32, 56, 56, 64, 64, 2, 2, "relu", 0.01, 0.1, 1.0,
                        (1003, 2003, 3003)),
    # ResNet-50 stage-3 shaped 3x3 conv, 4-bit activations, 3-bit weights
    "resnet50_s3": Conv("resnet50_s3", 64, 14, 14, 256, 256, 4, 3, "uniform", None, None, None,
                        (1004, 2004, 3004)),
    # the matrix product of the paper's efficiency experiment (Sec. 5.4): 8192 x 8192 x 8192
    "gemm8192": Gemm("gemm8192", 8192, 8192, 8192, 2, 2, "uniform", None, None, None, (1006, 2006, 3006)),
}


def with_bits(w, bits):
    """The same GEMM workload with `bits`-bit activations and weights."""
    return w._replace(ab=bits, wb=bits, name="%s_w%da%d" % (w.name, bits, bits))


def make_gemm(w, M=None):
    """(A codes [M][K], W codes [K][N], scale fp32 [N] or None)."""
    M = w.M if M is None else M
    sa, sw, ss = w.seeds
    A = uniform_codes(sa, (M, w.K), w.ab)
    W = uniform_codes(sw, (w.K, w.N), w.wb)
    s = None
    if w.scale_lo is not None:
        alpha = uniform_f32(ss, w.N, w.scale_lo, w.scale_hi)
        s = (alpha * np.float32(w.beta)).astype(np.float32)
    return A, W, s


def make_conv(w, Nb=None):
    """(X codes NHWC, Wt codes [Cout][3][3][C], scale fp32 [Cout] or None)."""
    Nb = w.Nb if Nb is None else Nb
    sa, sw, ss = w.seeds
    gen = relu_like_codes if w.act_dist == "relu" else uniform_codes
    X = gen(sa, (Nb, w.H, w.W, w.C), w.ab)
    Wt = uniform_codes(sw, (w.Cout, 3, 3, w.C), w.wb)
    s = None
    if w.scale_lo is not None:
        alpha = uniform_f32(ss, w.Cout, w.scale_lo, w.scale_hi)
        s = (alpha * np.float32(w.beta)).astype(np.float32)
    return X, Wt, s


# ---------------------------------------------------------------------------
# VGG-16-shaped stack of 13 3x3 convolutions (stride 1, pad 1) with a 2x2 max-pool after each
# block.  First layer: 3 input channels of 8-bit codes; every other layer 4-bit activation
# codes; 2-bit weights throughout.  Per-output-channel scales keep the re-encoded activations
# spread over the 16 levels: with uniform codes var(w) = 5, var(a8) = 21845, var(a4) = 85, so
#   layer 1:  s = U(0.8, 1.2) * 8 / sqrt(27 * 5 * 21845),   others:  s = U(0.8, 1.2) / sqrt(5 * 9 * Cin).
# ---------------------------------------------------------------------------
Stack = namedtuple("Stack", "name Nb H W C0 widths pool_after wb ab_first ab seeds")

VGG16 = Stack("vgg16_stack", 16, 224, 224, 3,
              (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512),
              (2, 4, 7, 10, 13), 2, 8, 4, (1005, 2005, 3005))


def make_stack(w=VGG16, Nb=None, H=None, W=None):
    """(X0 int16 codes NHWC, [(Wt int8 [Cout][3][3][Cin], scale fp32 [Cout], pool_after), ...])."""
    Nb = w.Nb if Nb is None else Nb
    H = w.H if H is None else H
    W = w.W if W is None else W
    sa, sw, ss = w.seeds
    X0 = uniform_codes(sa, (Nb, H, W, w.C0), w.ab_first)
    layers = []
    cin = w.C0
    for l, cout in enumerate(w.widths, start=1):
        Wt = uniform_codes(sw + l, (cout, 3, 3, cin), w.wb)
        jitter = uniform_f32(ss + l, cout, 0.8, 1.2)
        if l == 1:
            base = np.float32(8.0 / np.sqrt(27.0 * 5.0 * 21845.0))
        else:
            base = np.float32(1.0 / np.sqrt(5.0 * 9.0 * cin))
        layers.append((Wt, (jitter * base).astype(np.float32), l in w.pool_after))
        cin = cout
    return X0, layers
