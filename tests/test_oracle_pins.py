"""Pins of the CPU oracle against what the paper and plain mathematics fix.

None of these tests touches the GPU library.  Each names the passage it checks.
Python integers / Fractions, numpy float64 matmul and torch's CPU conv2d are
the independent references; no expected value comes from the HIP path.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def all_codes(bits):
    m = (1 << bits) - 1
    return list(range(-m, m + 1, 2))


def rng(seed):
    return np.random.default_rng(seed)


def rand_codes(r, shape, bits):
    m = (1 << bits) - 1
    return (2 * r.integers(0, 1 << bits, size=shape) - m).astype(np.int16)


# ------------------------------------------------------------------ Eq. (7)
@pytest.mark.parametrize("bits", range(1, 9))
def test_encoding_round_trip_and_state_count(oracle, bits):
    """Eq. (7): every odd code in [-(2^M-1), 2^M-1] has exactly one +-1 expansion."""
    seen = set()
    for v in all_codes(bits):
        c = oracle.encode(v, bits)
        assert set(np.unique(c)).issubset({-1, 1})
        assert sum((1 << m) * int(c[m]) for m in range(bits)) == v   # Eq. (7) in Python ints
        assert oracle.decode(c) == v
        seen.add(tuple(c))
    assert len(seen) == 1 << bits                                    # 2^M states
    # every +-1 vector decodes to a code of the space (bijection)
    for c in itertools.product((-1, 1), repeat=bits):
        assert oracle.decode(c) in all_codes(bits)


@pytest.mark.parametrize("bits", range(1, 9))
def test_non_codes_are_rejected(oracle, bits):
    m = (1 << bits) - 1
    for v in (0, 2, -2, m + 1, m + 2, -m - 2):
        with pytest.raises(ValueError):
            oracle.encode(v, bits)


def _table2():
    rows = []
    with open(os.path.join(GOLDEN, "table2_states.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            lo, loc, hi, hic, q, a, b = line.split()
            rows.append((Fraction(lo), int(loc), Fraction(hi), int(hic), Fraction(q), int(a), int(b)))
    return rows


def test_table2_states(oracle):
    """Table 2: the four printed 2-bit states, printed as {high, low}; alpha = 3."""
    rows = _table2()
    assert len(rows) == 4
    for _, _, _, _, q, high, low in rows:
        v = q * 3
        assert v.denominator == 1
        c = oracle.encode(int(v), 2)
        assert (int(c[1]), int(c[0])) == (high, low)
        assert low + 2 * high == int(v)            # Sec. 3.2: x = x_1 + 2 x_2


@pytest.mark.parametrize("bits", range(1, 7))
def test_trigonometric_encoder_agrees(oracle, bits):
    """Eq. (10)/(11): sign(+-sin((2^M-1)/2^m pi x)) at the quantized points x = v/(2^M-1)."""
    M = bits
    for v in all_codes(M):
        x = v / ((1 << M) - 1)
        c = oracle.encode(v, M)
        for m in range(1, M + 1):
            s = math.sin(((1 << M) - 1) / (1 << m) * math.pi * x)
            if m != M:
                s = -s
            assert abs(s) > 1e-9
            assert (1 if s > 0 else -1) == int(c[m - 1]), (M, m, v)


@pytest.mark.parametrize("bits", range(1, 9))
def test_zero_one_index_identity_and_bit_convention(oracle, bits):
    """Eq. (17): x^q = 2u/(2^M-1) - 1 with u the {0,1} fixed-point integer, so the
    code is v = 2u-(2^M-1) and stored plane p must be binary digit p of u."""
    codes = np.array([all_codes(bits)], dtype=np.int16)       # one row, K = 2^bits
    planes, bad = oracle.pack_planes(codes, bits)
    assert bad == 0
    K = codes.shape[1]
    for k in range(K):
        v = int(codes[0, k])
        u = (v + (1 << bits) - 1) // 2
        assert Fraction(2 * u, (1 << bits) - 1) - 1 == Fraction(v, (1 << bits) - 1)
        for p in range(bits):
            bit = (int(planes[0, p, k // 32]) >> (k % 32)) & 1
            assert bit == (u >> p) & 1


# ---------------------------------------------------------- bit-plane store
def test_pack_layout_tail_and_position(oracle):
    """Element k lands in bit k%32 of word k//32 of every plane; tail bits are zero."""
    for bits in (1, 2, 3, 8):
        m = (1 << bits) - 1
        for K in (1, 27, 31, 32, 33, 64, 65, 100):
            for k in (0, K // 2, K - 1):
                codes = np.full((3, K), -m, dtype=np.int16)
                codes[1, k] = m
                planes, bad = oracle.pack_planes(codes, bits)
                assert bad == 0 and planes.shape == (3, bits, (K + 31) // 32)
                assert not planes[0].any() and not planes[2].any()
                want = np.zeros((bits, (K + 31) // 32), dtype=np.uint32)
                want[:, k // 32] = np.uint32(1) << np.uint32(k % 32)
                assert (planes[1] == want).all()
            allp = np.full((1, K), m, dtype=np.int16)
            planes, _ = oracle.pack_planes(allp, bits)
            total = sum(bin(int(x)).count("1") for x in planes.ravel())
            assert total == bits * K                           # nothing set past K


def test_pack_counts_invalid_codes(oracle):
    codes = np.array([[1, 0, 3, 5, -3, 2]], dtype=np.int16)
    planes, bad = oracle.pack_planes(codes, 2)
    assert bad == 3                                            # 0, 5, 2
    good, _ = oracle.pack_planes(np.array([[1, -3, 3, -3, -3, -3]], dtype=np.int16), 2)
    assert (planes == good).all()                              # invalid entries pack as zeros


# ----------------------------------------------------- XnorPopcount, Eq. (8)
def test_xnor_popcount_identity_brute_force(oracle):
    """1-bit x 1-bit: c.d = 2*popcount(xnor) - L = L - 2*popcount(xor), all vectors L<=6."""
    for L in range(1, 7):
        vecs = list(itertools.product((-1, 1), repeat=L))
        for c in vecs:
            pc = sum(1 << i for i in range(L) if c[i] == 1)
            for d in vecs:
                pd = sum(1 << i for i in range(L) if d[i] == 1)
                dot = sum(a * b for a, b in zip(c, d))
                assert oracle.branch_dot(c, d, 1, 1) == dot
                xnor = ~(pc ^ pd) & ((1 << L) - 1)
                assert 2 * bin(xnor).count("1") - L == dot
                assert L - 2 * bin(pc ^ pd).count("1") == dot


@pytest.mark.parametrize("L", [1, 27, 31, 32, 33, 63, 64, 65, 576])
def test_xor_popcount_on_packed_planes(oracle, L):
    """The stored planes reproduce every branch dot product as L - 2 popcount(xor),
    with the zero tail bits contributing nothing."""
    r = rng(100 + L)
    for xb, wb in ((1, 1), (2, 2), (4, 3), (8, 2)):
        x = rand_codes(r, (1, L), xb)
        w = rand_codes(r, (1, L), wb)
        px, _ = oracle.pack_planes(x, xb)
        pw, _ = oracle.pack_planes(w, wb)
        total = 0
        for m in range(xb):
            for k in range(wb):
                pop = sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(px[0, m], pw[0, k]))
                total += (1 << (m + k)) * (L - 2 * pop)
        assert total == int(np.dot(x[0].astype(np.int64), w[0].astype(np.int64)))


@pytest.mark.parametrize("xb", range(1, 9))
@pytest.mark.parametrize("wb", range(1, 9))
def test_branch_sum_equals_integer_dot(oracle, xb, wb):
    """Eq. (8) = Eq. (1) for every bit-width pair (M x K branches)."""
    r = rng(1000 + 8 * xb + wb)
    for n in (1, 2, 7, 40):
        x = rand_codes(r, (n,), xb)
        w = rand_codes(r, (n,), wb)
        want = sum(int(a) * int(b) for a, b in zip(x, w))
        assert oracle.branch_dot(x, w, xb, wb) == want
        assert int(oracle.gemm(x[None, :], w[:, None])[0, 0]) == want


def test_two_bit_fc_example(oracle):
    """Sec. 3.2 / Fig. 1: x = x1 + 2 x2, w = w1 + 2 w2, four branch products with
    weights 1, 2, 2, 4 and the final factor 1/9 on values in {-1,-1/3,1/3,1}."""
    consts = {}
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                k, v = line.split()
                consts[k] = v
    scale = Fraction(consts["fc_2bit_scale"])
    assert scale == Fraction(1, (2 ** 2 - 1) * (2 ** 2 - 1))          # Eq. (9), r = 1
    r = rng(7)
    n = 12
    x = rand_codes(r, (n,), 2)
    w = rand_codes(r, (n,), 2)
    x1 = [int(oracle.encode(v, 2)[0]) for v in x]
    x2 = [int(oracle.encode(v, 2)[1]) for v in x]
    w1 = [int(oracle.encode(v, 2)[0]) for v in w]
    w2 = [int(oracle.encode(v, 2)[1]) for v in w]
    dot = lambda a, b: sum(p * q for p, q in zip(a, b))
    y = [dot(x1, w1), dot(x2, w1), dot(x1, w2), dot(x2, w2)]
    assert len(y) == int(consts["fc_2bit_branches"])
    enc = y[0] + 2 * y[1] + 2 * y[2] + 4 * y[3]
    assert enc == oracle.branch_dot(x, w, 2, 2) == int(oracle.gemm(x[None], w[:, None])[0, 0])
    real = sum(Fraction(int(a), 3) * Fraction(int(b), 3) for a, b in zip(x, w))   # Eq. (19)
    assert real == scale * enc
    y64 = oracle.scale_f64(np.array([[enc]]), np.array([1.0 / 9.0], dtype=np.float32))
    assert abs(y64[0, 0] - float(real)) <= 1e-6 * max(1.0, abs(float(real)))


# ------------------------------------------------------------- Eq. (1) GEMM
@pytest.mark.parametrize("ab,wb", [(1, 1), (2, 2), (4, 3), (8, 2), (8, 8)])
def test_gemm_against_float64_matmul(oracle, ab, wb):
    r = rng(ab * 10 + wb)
    M, N, K = 13, 9, 77
    A = rand_codes(r, (M, K), ab)
    W = rand_codes(r, (K, N), wb)
    want = np.matmul(A.astype(np.float64), W.astype(np.float64))     # exact: |values| << 2^53
    got = oracle.gemm(A, W)
    assert got.dtype == np.int64 and (got == want.astype(np.int64)).all()
    assert (oracle.gemm_wt(A, np.ascontiguousarray(W.T)) == got).all()
    # a transposed operand would change the result
    A2 = rand_codes(r, (K, K), ab)
    W2 = rand_codes(r, (K, K), wb)
    assert not (oracle.gemm(A2, W2) == oracle.gemm(A2, np.ascontiguousarray(W2.T))).all()


def test_gemm_closed_forms(oracle):
    for ab, wb, K in ((2, 2, 256), (4, 3, 2304), (8, 8, 33), (1, 1, 5)):
        ma, mw = (1 << ab) - 1, (1 << wb) - 1
        A = np.full((2, K), ma, dtype=np.int16)
        W = np.full((K, 3), mw, dtype=np.int16)
        assert (oracle.gemm(A, W) == K * ma * mw).all()              # all agree: S = 0
        assert (oracle.gemm(-A, W) == -K * ma * mw).all()
        r = rng(K)
        A = rand_codes(r, (5, K), ab)
        W = rand_codes(r, (K, 4), wb)
        C = oracle.gemm(A, W)
        assert (oracle.gemm(-A, W) == -C).all()
        assert ((C - K) % 2 == 0).all()                              # odd*odd summed K times
        assert (np.abs(C) <= K * ma * mw).all()
    alt = np.array([[1, -1] * 8], dtype=np.int16)
    assert oracle.gemm(alt, np.ones((16, 1), dtype=np.int16))[0, 0] == 0


def test_one_bit_case_is_binary_network(oracle):
    """M = K = 1 reduces to a +-1 (binary network) product."""
    r = rng(3)
    A = rand_codes(r, (6, 50), 1)
    W = rand_codes(r, (50, 7), 1)
    assert set(np.unique(A)) <= {-1, 1}
    agree = (A[:, :, None] == W[None, :, :]).sum(axis=1)
    assert (oracle.gemm(A, W) == 2 * agree - 50).all()


# --------------------------------------------------------------- convolution
@pytest.mark.parametrize("shape", [(2, 1, 1, 3, 2), (1, 2, 2, 5, 3), (2, 3, 4, 7, 5), (1, 6, 5, 33, 4)])
def test_conv_against_torch(oracle, shape):
    import torch
    Nb, H, W, C, Cout = shape
    r = rng(sum(shape))
    X = rand_codes(r, (Nb, H, W, C), 4)
    Wt = rand_codes(r, (Cout, 3, 3, C), 3)
    got = oracle.conv3x3(X, Wt)
    x = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2)
    w = torch.from_numpy(Wt.astype(np.float64)).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(x, w, stride=1, padding=1).permute(0, 2, 3, 1).numpy()
    assert (got == want.astype(np.int64)).all()


def test_conv_equals_explicit_im2col_gemm(oracle):
    """3x3/pad 1 conv = GEMM on the explicit patch matrix with K ordered (kh, kw, c)."""
    r = rng(11)
    Nb, H, W, C, Cout = 2, 4, 5, 6, 3
    X = rand_codes(r, (Nb, H, W, C), 2)
    Wt = rand_codes(r, (Cout, 3, 3, C), 2)
    Xp = np.zeros((Nb, H + 2, W + 2, C), dtype=np.int16)
    Xp[:, 1:-1, 1:-1] = X
    rows = []
    for n in range(Nb):
        for oh in range(H):
            for ow in range(W):
                rows.append(Xp[n, oh:oh + 3, ow:ow + 3, :].reshape(-1))
    patches = np.stack(rows)
    # zero padding is not a code, so use float64 matmul rather than the code GEMM
    want = patches.astype(np.float64) @ Wt.reshape(Cout, -1).T.astype(np.float64)
    assert (oracle.conv3x3(X, Wt).reshape(-1, Cout) == want.astype(np.int64)).all()


def test_conv_special_cases(oracle):
    r = rng(5)
    Nb, H, W, C = 1, 5, 6, 4
    X = rand_codes(r, (Nb, H, W, C), 3)
    # all-ones image and kernel: counts the valid taps (4 / 6 / 9) times C
    ones = np.ones((Nb, H, W, C), dtype=np.int16)
    k1 = np.ones((1, 3, 3, C), dtype=np.int16)
    O = oracle.conv3x3(ones, k1)[0, :, :, 0]
    taps = np.array([[(3 - (oh == 0) - (oh == H - 1)) * (3 - (ow == 0) - (ow == W - 1))
                      for ow in range(W)] for oh in range(H)])
    assert (O == taps * C).all()
    # parity: sum of (valid taps * C) odd products
    Wt = rand_codes(r, (2, 3, 3, C), 2)
    O = oracle.conv3x3(X, Wt)
    assert (((O[0] - (taps * C)[:, :, None]) % 2) == 0).all()
    # no kernel flip: a kernel with a single +1-vs-(-1) asymmetry at (kh=0,kw=0) looks up-left
    Xs = np.ones((1, 3, 3, 1), dtype=np.int16)
    Xs[0, 0, 0, 0] = 3
    K = np.ones((1, 3, 3, 1), dtype=np.int16)
    K[0, 0, 0, 0] = 3
    O = oracle.conv3x3(Xs, K)
    assert O[0, 1, 1, 0] == 8 + 9                                   # x[0,0]*k[0,0] aligned
    K2 = np.ones((1, 3, 3, 1), dtype=np.int16)
    K2[0, 2, 2, 0] = 3
    assert oracle.conv3x3(Xs, K2)[0, 1, 1, 0] == 3 + 7 + 3           # x[0,0]*1 + 7 + x[2,2]*3


# ------------------------------------------------------------ Eq. (9) scale
def test_scale_epilogue(oracle):
    r = rng(9)
    acc = r.integers(-(1 << 23), 1 << 23, size=(50, 17)).astype(np.int64)
    s = r.uniform(0.0005, 0.005, size=17).astype(np.float32)
    y64 = oracle.scale_f64(acc, s)
    assert (y64 == acc.astype(np.float64) * s.astype(np.float64)[None, :]).all()
    y32 = oracle.scale_f32(acc, s)
    assert y32.dtype == np.float32
    assert (y32 == (acc.astype(np.float32) * s[None, :])).all()       # one binary32 multiply
    rel = np.abs(y32.astype(np.float64) - y64) / np.maximum(np.abs(y64), 1e-30)
    assert rel.max() <= 2.0 ** -24 * 1.0001
    # column j uses s[j], not s[i]
    acc1 = np.ones((3, 17), dtype=np.int64)
    assert (oracle.scale_f64(acc1, s)[2] == s.astype(np.float64)).all()


# ------------------------------------------------- re-encoding between layers
def test_round_odd_reproduces_table2_intervals(oracle):
    """Table 2 scaled by alpha = 3: closures of the four intervals, endpoints included."""
    for lo, loc, hi, hic, q, _, _ in _table2():
        code = int(q * 3)
        lo3, hi3 = float(lo * 3), float(hi * 3)
        pts = [lo3 + (hi3 - lo3) * t for t in (0.001, 0.25, 0.5, 0.75, 0.999)]
        if loc:
            pts.append(lo3)
        if hic:
            pts.append(hi3)
        for y in pts:
            assert oracle.round_odd(y, 2) == code, (y, code)
        if not loc:
            assert oracle.round_odd(lo3, 2) != code
        if not hic:
            assert oracle.round_odd(hi3, 2) != code


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_round_odd_properties(oracle, bits):
    m = (1 << bits) - 1
    ys = np.linspace(-m - 3.0, m + 3.0, 2001).astype(np.float32)
    codes = oracle.requant(ys, bits)
    assert (np.diff(codes.astype(np.int64)) >= 0).all()               # monotone
    assert set(np.unique(codes)) == set(all_codes(bits))              # onto the code space
    assert (np.abs(codes) <= m).all()
    for v in all_codes(bits):                                         # codes are fixed points
        assert oracle.round_odd(float(v), bits) == v
    assert oracle.round_odd(0.0, bits) == -1 and oracle.round_odd(-0.0, bits) == -1
    assert oracle.round_odd(1e30, bits) == m and oracle.round_odd(-1e30, bits) == -m


def test_maxpool_and_requant_commute(oracle):
    r = rng(21)
    y = r.normal(0, 6, size=(2, 4, 6, 5)).astype(np.float32)
    p = oracle.maxpool2x2(y)
    want = y.reshape(2, 2, 2, 3, 2, 5).max(axis=(2, 4))
    assert (p == want).all()
    a = oracle.requant(p, 4)
    b = oracle.maxpool2x2(oracle.requant(y, 4).astype(np.float32)).astype(np.int16)
    assert (a == b).all()


# ------------------------------------------------- general and transposed convolution
GEOMETRIES = [
    # KH, KW, stride, pad, dilation
    (1, 1, 1, 0, 1), (1, 1, 2, 0, 1), (3, 3, 2, 1, 1), (7, 7, 2, 3, 1), (5, 5, 1, 0, 1), (3, 3, 1, 2, 2),
    (3, 1, (1, 2), (1, 0), 1), (2, 4, (2, 1), (0, 2), (1, 2)),
]


@pytest.mark.parametrize("geo", GEOMETRIES)
def test_general_conv_against_torch(oracle, geo):
    """Library cross-check (float64 is exact at these magnitudes): strides, paddings, dilations and
    kernel sizes of the networks of Sec. 5, NHWC vs torch's NCHW."""
    import torch
    KH, KW, stride, pad, dil = geo
    rng = np.random.default_rng(KH * 100 + KW)
    X = (2 * rng.integers(0, 16, size=(2, 9, 11, 5)) - 15).astype(np.int16)
    Wt = (2 * rng.integers(0, 4, size=(6, KH, KW, 5)) - 3).astype(np.int16)
    got = oracle.conv2d(X, Wt, stride=stride, pad=pad, dilation=dil)
    x = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2)
    w = torch.from_numpy(Wt.astype(np.float64)).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad, dilation=dil).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape and (got == want.astype(np.int64)).all()


def test_general_conv_reduces_to_the_3x3_case_and_to_gemm(oracle):
    rng = np.random.default_rng(3)
    X = (2 * rng.integers(0, 4, size=(2, 6, 7, 8)) - 3).astype(np.int16)
    Wt = (2 * rng.integers(0, 4, size=(5, 3, 3, 8)) - 3).astype(np.int16)
    assert (oracle.conv2d(X, Wt, stride=1, pad=1) == oracle.conv3x3(X, Wt)).all()
    W1 = (2 * rng.integers(0, 4, size=(5, 1, 1, 8)) - 3).astype(np.int16)
    assert (oracle.conv2d(X, W1).reshape(-1, 5) == oracle.gemm(X.reshape(-1, 8), W1.reshape(5, 8).T.copy())).all()


def test_general_conv_single_tap_positions(oracle):
    """A kernel with a single 1 at (kh, kw) shifts the image by (kh*d - p, kw*d - p) and samples
    every s-th pixel: fixes the roles of stride, pad and dilation and the absence of a flip."""
    X = np.arange(1, 1 + 7 * 8, dtype=np.int16).reshape(1, 7, 8, 1)
    for KH, KW, s, p, d in [(3, 3, 2, 1, 1), (3, 3, 1, 2, 2), (2, 2, 1, 0, 1)]:
        for kh in range(KH):
            for kw in range(KW):
                K = np.zeros((1, KH, KW, 1), dtype=np.int16)
                K[0, kh, kw, 0] = 1
                O = oracle.conv2d(X, K, stride=s, pad=p, dilation=d)[0, :, :, 0]
                for oh in range(O.shape[0]):
                    for ow in range(O.shape[1]):
                        ih, iw = oh * s - p + kh * d, ow * s - p + kw * d
                        want = X[0, ih, iw, 0] if 0 <= ih < 7 and 0 <= iw < 8 else 0
                        assert O[oh, ow] == want


@pytest.mark.parametrize("geo", [(2, 2, 2, 0, 1, 0), (3, 3, 2, 1, 1, 1), (4, 4, 2, 1, 1, 0), (3, 3, 1, 1, 1, 0),
                                 (3, 2, (2, 3), (1, 0), (1, 2), (1, 2))])
def test_transposed_conv_against_torch(oracle, geo):
    import torch
    KH, KW, stride, pad, dil, opad = geo
    rng = np.random.default_rng(KH * 10 + KW)
    X = (2 * rng.integers(0, 16, size=(2, 5, 6, 4)) - 15).astype(np.int16)
    Wt = (2 * rng.integers(0, 4, size=(3, KH, KW, 4)) - 3).astype(np.int16)
    got = oracle.conv2d_transposed(X, Wt, stride=stride, pad=pad, dilation=dil, output_padding=opad)
    x = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2)
    w = torch.from_numpy(Wt.astype(np.float64)).permute(3, 0, 1, 2)          # torch: [Cin][Cout][KH][KW]
    want = torch.nn.functional.conv_transpose2d(x, w, stride=stride, padding=pad, dilation=dil,
                                                output_padding=opad).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape and (got == want.astype(np.int64)).all()


def test_transposed_conv_is_the_adjoint_of_conv(oracle):
    """<conv(x), y> = <x, conv_transposed(y)> with input and output channels swapped: the defining
    property of the transposed operation, independent of any library."""
    rng = np.random.default_rng(11)
    for (KH, KW, s, p, d) in [(3, 3, 2, 1, 1), (2, 2, 2, 0, 1), (3, 3, 1, 1, 2)]:
        X = (2 * rng.integers(0, 8, size=(1, 7, 7, 3)) - 7).astype(np.int16)
        Wt = (2 * rng.integers(0, 4, size=(4, KH, KW, 3)) - 3).astype(np.int16)      # [Cout=4][KH][KW][C=3]
        Y0 = oracle.conv2d(X, Wt, stride=s, pad=p, dilation=d)
        Y = (2 * rng.integers(0, 8, size=Y0.shape) - 7).astype(np.int16)
        WtT = np.ascontiguousarray(Wt.transpose(3, 1, 2, 0))                          # [C=3][KH][KW][Cout=4]
        Ho = (Y.shape[1] - 1) * s - 2 * p + d * (KH - 1) + 1
        opad = 7 - Ho
        Xb = oracle.conv2d_transposed(Y, WtT, stride=s, pad=p, dilation=d, output_padding=opad)
        assert Xb.shape == X.shape
        assert int((Y0 * Y.astype(np.int64)).sum()) == int((X.astype(np.int64) * Xb).sum())


# ------------------------------------------------------------------ real-valued front end
def test_encode_real_reproduces_table2(oracle):
    """Table 2 on the unscaled number space [-1,1] with its printed closures (2 bits, alpha = 3)."""
    x = np.array([-1.0, -0.9, -2.0 / 3.0, -0.6666, -0.3, -1e-30, 0.0, 1e-30, 0.3, 0.6666, 2.0 / 3.0, 0.9, 1.0],
                 dtype=np.float32)
    want = np.array([-3, -3, -3, -1, -1, -1, -1, 1, 1, 1, 3, 3, 3])
    assert (oracle.encode_real(x, 2) == want).all()
    # Table 1: HTanh clips to [-1,1] (beyond it the extreme states), HReLU to [0,1] (nothing below the state of 0)
    big = np.array([-7.5, -1.0001, 1.0001, 40.0, np.inf, -np.inf], dtype=np.float32)
    assert (oracle.encode_real(big, 2) == np.array([-3, -3, 3, 3, 3, -3])).all()
    neg = np.array([-5.0, -0.5, -0.0, 0.0, 0.2, 0.7, 3.0, np.nan], dtype=np.float32)
    assert (oracle.encode_real(neg, 2, hrelu=True) == np.array([-1, -1, -1, -1, 1, 3, 3, -1])).all()


@pytest.mark.parametrize("bits", range(1, 7))
def test_encode_real_agrees_with_the_trigonometric_encoder(oracle, bits):
    """Eq. (10) at generic points of (-1,1): element m of the code is sign(+-sin((2^M-1)/2^m pi x)).
    Points within 1e-4 of an interval boundary 2j/(2^M-1) are left out (the sine vanishes there)."""
    M, alpha = bits, (1 << bits) - 1
    rng = np.random.default_rng(M)
    x = rng.uniform(-1, 1, 4000).astype(np.float32)
    pos = x.astype(np.float64) * alpha / 2.0
    x = x[np.abs(pos - np.round(pos)) > 1e-4 * alpha]
    codes = oracle.encode_real(x, M)
    for xi, v in zip(x.tolist(), codes.tolist()):
        c = oracle.encode(int(v), M)
        for m in range(1, M + 1):
            s = math.sin(alpha / (1 << m) * math.pi * xi)
            if m != M:
                s = -s
            assert (1 if s > 0 else -1) == int(c[m - 1]), (M, m, xi, v)


def test_encode_real_is_the_scaled_reencoder(oracle):
    """encode_real(x) = requant(x * alpha) with the product formed in binary32; quantised points
    v/alpha come back as v for every bit width (round trip through the number space)."""
    for bits in range(1, 9):
        alpha = (1 << bits) - 1
        v = np.array(all_codes(bits), dtype=np.int16)
        x = (v.astype(np.float64) / alpha).astype(np.float32)
        assert (oracle.encode_real(x, bits) == v).all(), bits
        y = np.random.default_rng(bits).normal(0, 0.7, 500).astype(np.float32)
        assert (oracle.encode_real(y, bits) == oracle.requant(y * np.float32(alpha), bits)).all()


# ------------------------------------------------------------------ front end: Tanh / Sigmoid of Table 1
def _consts():
    out = {}
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                k, v = line.split()
                out[k] = v
    return out


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_encode_smooth_against_numpy(oracle, bits):
    """Tanh / Sigmoid of Table 1 followed by the Table 2 rule: away from the interval boundaries the
    codes equal the rule applied to numpy's float64 tanh / logistic; Sigmoid only reaches the
    positive codes (its range is (0,1), like HReLU's); Tanh is odd."""
    r = rng(60 + bits)
    x = r.uniform(-4, 4, 20000).astype(np.float32)
    alpha = (1 << bits) - 1
    for clip, fn in (("tanh", np.tanh), ("sigmoid", lambda v: 1.0 / (1.0 + np.exp(-v)))):
        codes, limited = oracle.encode_smooth(x, bits, clip)
        y = fn(x.astype(np.float64)) * alpha
        assert np.abs(limited.astype(np.float64) - fn(x.astype(np.float64))).max() < 1e-7
        clear = np.abs(y - 2 * np.round(y / 2)) > 1e-4            # not within 1e-4 of an interval boundary
        mag = np.minimum(2 * np.floor(np.abs(y) / 2) + 1, alpha)
        want = np.where(y > 0, mag, -mag)
        assert clear.mean() > 0.99
        assert (codes[clear] == want[clear]).all()
        if clip == "sigmoid":
            assert (codes >= 1).all()
        else:
            back, _ = oracle.encode_smooth(-x, bits, clip)
            assert (back[clear] == -codes[clear]).all()
    # saturation: far out the limiters reach the extreme states
    far = np.array([-30.0, 30.0], dtype=np.float32)
    assert (oracle.encode_smooth(far, bits, "tanh")[0] == np.array([-alpha, alpha])).all()
    assert oracle.encode_smooth(far, bits, "sigmoid")[0][1] == alpha


# ------------------------------------------------------------------ training-side pieces (Sec. 4)
def test_encoder_backward_printed_two_bit_case(oracle):
    """Eq. (13): at x = 0 the high bit's derivative is (3/4) pi and the low bit's -(3/2) pi; outside
    [-1, 1] both vanish."""
    c = _consts()
    hi, lo = float(Fraction(c["enc2_dhigh_at0_over_pi"])), float(Fraction(c["enc2_dlow_at0_over_pi"]))
    x = np.array([0.0, 0.0, 1.5, -1.0001], dtype=np.float32)
    only_low = np.array([[1, 0, 1, 1], [0, 0, 0, 0]], dtype=np.float32)
    only_high = np.array([[0, 0, 0, 0], [1, 1, 1, 1]], dtype=np.float32)
    assert np.allclose(oracle.encoder_backward(x, only_low), [lo * np.pi, 0, 0, 0], rtol=1e-12, atol=0)
    assert np.allclose(oracle.encoder_backward(x, only_high), [hi * np.pi, hi * np.pi, 0, 0], rtol=1e-12, atol=0)


@pytest.mark.parametrize("M", [1, 2, 3, 5, 8])
def test_encoder_backward_is_the_slope_of_the_trigonometric_encoder(oracle, M):
    """Eq. (12) is the derivative of the function under the sign in Eq. (10): central differences of
    +-sin((2^M - 1) / 2^m pi x) in float64 reproduce every bit's term, and the terms add up linearly."""
    r = rng(70 + M)
    x = r.uniform(-1, 1, 500).astype(np.float32)
    g = r.normal(size=(M, x.size)).astype(np.float32)
    xd = x.astype(np.float64)
    h = 1e-6
    want = np.zeros_like(xd)
    for m in range(1, M + 1):
        c = (2 ** M - 1) / 2 ** m * np.pi
        f = (lambda v: np.sin(c * v)) if m == M else (lambda v: -np.sin(c * v))
        want += g[m - 1] * (f(xd + h) - f(xd - h)) / (2 * h)
    got = oracle.encoder_backward(x, g)
    assert np.abs(got - want).max() <= 1e-4 * (1 + np.abs(want).max())
    assert (oracle.encoder_backward(np.array([1.01, -7.0, 2.0], dtype=np.float32), np.ones((M, 3), np.float32)) == 0).all()
    # the ends of the interval belong to it
    assert (oracle.encoder_backward(np.array([1.0, -1.0], dtype=np.float32), np.ones((M, 2), np.float32)) != 0).all()


def test_binarize_and_its_gradient(oracle):
    """Eq. (14): sign(HTanh(w)), values in {-1,+1}, zero on the + side; the gradient passes exactly
    where HTanh is the identity."""
    w = np.array([-3.0, -1.0, -0.2, -0.0, 0.0, 1e-30, 0.7, 1.0, 1.0001, 5.0], dtype=np.float32)
    wb = oracle.binarize(w)
    assert (wb == np.array([-1, -1, -1, 1, 1, 1, 1, 1, 1, 1])).all()
    htanh = np.clip(w, -1, 1)
    nz = htanh != 0
    assert (wb[nz] == np.sign(htanh[nz])).all()
    g = np.arange(1, 11, dtype=np.float32)
    assert (oracle.binarize_backward(w, g) == np.array([0, 2, 3, 4, 5, 6, 7, 8, 0, 0], dtype=np.float32)).all()
    # with one bit the code of a non-zero weight is the Eq. (7) code of its sign
    r = rng(81)
    v = r.normal(size=1000).astype(np.float32)
    assert (oracle.binarize(v) == np.where(v >= 0, 1, -1)).all()


@pytest.mark.parametrize("K", [2, 3, 4, 8])
def test_quantize_k_properties(oracle, K):
    """Eq. (15): 2^K - 1 equally spaced states k * d with |k| <= 2^(K-1) - 1 and d = t / (2^(K-1) - 1);
    within the clamp the error is at most d / 2; the map is monotone and idempotent; the ends are
    +-t; midpoints go to the even state (the reading of `round`); numpy's float32 arithmetic with
    rint gives the same values."""
    r = rng(90 + K)
    t = np.float32(0.75)
    n = 2 ** (K - 1) - 1
    d = np.float32(t / np.float32(n))
    x = np.sort(r.uniform(-1.5, 1.5, 5000).astype(np.float32))
    q, lv = oracle.quantize_k(x, K, t)
    assert set(np.unique(lv)) == set(range(-n, n + 1))
    assert (q == lv.astype(np.float32) * d).all()
    inside = np.abs(x) <= t
    assert (np.abs(q[inside].astype(np.float64) - x[inside]) <= float(d) / 2 * (1 + 1e-6)).all()
    assert (np.diff(q) >= 0).all()
    assert (oracle.quantize_k(q, K, t)[0] == q).all()
    assert (oracle.quantize_k(np.array([t, -t, 9.0, -9.0], dtype=np.float32), K, t)[0] == np.array([t, -t, t, -t])).all()
    want = np.rint(np.clip(x / t, np.float32(-1), np.float32(1)) * np.float32(n)).astype(np.float32) * d
    assert (q == want).all()
    if n >= 2:
        half = np.array([0.5, 1.5, -0.5, -1.5], dtype=np.float32) / np.float32(n)      # x/t*n exactly at midpoints (t = 1)
        assert (oracle.quantize_k(half, K, 1.0)[1] == np.array([0, 2, 0, -2])).all()
    g = np.ones_like(x)
    assert (oracle.quantize_k_backward(x, g, t) == (np.abs(x / t) <= 1).astype(np.float32)).all()


def _elements(codes, bits):
    """{-1,+1} elements of odd codes, low element first, by the binary expansion of (v + 2^bits - 1) / 2
    (Eq. (7) written with Python integers; independent of the oracle's greedy encoder)."""
    u = (codes.astype(np.int64) + (1 << bits) - 1) // 2
    return [(2 * ((u >> p) & 1) - 1).astype(np.float64) for p in range(bits)]


def _forward_from_elements(a_el, w_el, s):
    """Forward lines of Alg. 1 on real-valued element matrices: sum_m sum_k 2^(m+k-2) a_m W_k^T, then the scale."""
    a_hat = sum(2.0 ** (m + k) * (a_el[m] @ w_el[k].T) for m in range(len(a_el)) for k in range(len(w_el)))
    return a_hat * s[None, :]


@pytest.mark.parametrize("xb,wb", [(1, 1), (2, 2), (3, 2), (2, 4)])
def test_branch_backward_is_the_slope_of_the_forward_lines(oracle, xb, wb):
    """Alg. 1: the forward lines are linear in every element a^{mb}[i][c] and W^{kb}[n][c], so with the cost
    C = sum g_a * a the gradient of an element is exactly C(element + 1) - C(element).  Every element of a
    small layer, one at a time (brute force): catches a wrong factor 2^(m+k-2), a dropped scale, a
    transposed operand, a wrong index order of the outputs."""
    r = rng(900 + 10 * xb + wb)
    M, N, K = 3, 4, 5
    A, W = rand_codes(r, (M, K), xb), rand_codes(r, (N, K), wb)
    g = r.normal(size=(M, N)).astype(np.float32)
    s = r.uniform(0.5, 2.0, N).astype(np.float32)
    a_el, w_el = _elements(A, xb), _elements(W, wb)
    cost = lambda ae, we: float((g.astype(np.float64) * _forward_from_elements(ae, we, s.astype(np.float64))).sum())
    base = cost(a_el, w_el)
    gi = oracle.branch_backward_input(g, s, W, xb, wb)
    gw = oracle.branch_backward_weight(g, s, A, xb, wb)
    assert gi.shape == (xb, M, K) and gw.shape == (wb, N, K)
    for m in range(xb):
        for i in range(M):
            for c in range(K):
                bumped = [e.copy() for e in a_el]
                bumped[m][i, c] += 1.0
                assert abs((cost(bumped, w_el) - base) - gi[m, i, c]) <= 1e-9 * (1 + abs(gi[m, i, c]))
    for k in range(wb):
        for n in range(N):
            for c in range(K):
                bumped = [e.copy() for e in w_el]
                bumped[k][n, c] += 1.0
                assert abs((cost(a_el, bumped) - base) - gw[k, n, c]) <= 1e-9 * (1 + abs(gw[k, n, c]))


@pytest.mark.parametrize("xb,wb", [(1, 1), (2, 2), (4, 3), (8, 8)])
def test_branch_backward_closed_form_on_codes(oracle, xb, wb):
    """Summing the branches of Alg. 1's backward lines (Eq. (7) read backwards): element m of the activation
    gradient is 2^(m-1) * (s g_a) @ W_codes, element k of the weight gradient 2^(k-1) * (s g_a)^T @ A_codes
    -- numpy float64 products of the decoded codes; with one bit each it is the textbook gradient of a
    matrix product.  Without a scale the scale is one."""
    r = rng(950 + xb + wb)
    M, N, K = 9, 11, 37
    A, W = rand_codes(r, (M, K), xb), rand_codes(r, (N, K), wb)
    g = r.normal(size=(M, N)).astype(np.float32)
    for s in (None, r.uniform(0.25, 4.0, N).astype(np.float32)):
        gs = g.astype(np.float64) * (1.0 if s is None else s.astype(np.float64)[None, :])
        gi = oracle.branch_backward_input(g, s, W, xb, wb)
        gw = oracle.branch_backward_weight(g, s, A, xb, wb)
        base_i, base_w = gs @ W.astype(np.float64), gs.T @ A.astype(np.float64)
        for m in range(xb):
            assert np.abs(gi[m] - 2.0 ** m * base_i).max() <= 1e-9 * (1 + np.abs(base_i).max() * 2.0 ** m)
        for k in range(wb):
            assert np.abs(gw[k] - 2.0 ** k * base_w).max() <= 1e-9 * (1 + np.abs(base_w).max() * 2.0 ** k)


@pytest.mark.parametrize("xb,wb", [(1, 1), (2, 2), (4, 3)])
def test_conv_backward_against_torch_autograd_and_transposed_convolution(oracle, xb, wb):
    """Alg. 1's backward lines through a 3x3 convolution.  Summed over the other operand's elements they are
    2^(m-1) * d/dx and 2^(k-1) * d/dW of sum(g_a * s * conv(x, W)) on the decoded codes: torch's float64
    autograd through its own conv2d gives both (a library routine, independent of the oracle's loops), and
    the first is also the transposed convolution of s * g_a with the weights (conv_transpose2d)."""
    import torch
    import torch.nn.functional as F
    r = rng(970 + xb * 8 + wb)
    Nb, H, W, C, O = 2, 5, 4, 6, 7
    X, Wt = rand_codes(r, (Nb, H, W, C), xb), rand_codes(r, (O, 3, 3, C), wb)
    g = r.normal(size=(Nb, H, W, O)).astype(np.float32)
    s = r.uniform(0.5, 2.0, O).astype(np.float32)
    x = torch.tensor(X.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)          # NCHW
    wt = torch.tensor(Wt.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)        # [O][C][3][3]
    gs = torch.tensor(g.astype(np.float64) * s.astype(np.float64)).permute(0, 3, 1, 2)
    (F.conv2d(x, wt, padding=1) * gs).sum().backward()
    dx = x.grad.permute(0, 2, 3, 1).numpy()
    dw = wt.grad.permute(0, 2, 3, 1).numpy()
    gi = oracle.conv3x3_backward_input(g, s, Wt, xb, wb)
    gw = oracle.conv3x3_backward_weight(g, s, X, xb, wb)
    assert gi.shape == (xb, Nb, H, W, C) and gw.shape == (wb, O, 3, 3, C)
    for m in range(xb):
        assert np.abs(gi[m] - 2.0 ** m * dx).max() <= 1e-9 * (1 + 2.0 ** m * np.abs(dx).max())
    for k in range(wb):
        assert np.abs(gw[k] - 2.0 ** k * dw).max() <= 1e-9 * (1 + 2.0 ** k * np.abs(dw).max())
    tr = F.conv_transpose2d(gs, wt.detach(), padding=1).permute(0, 2, 3, 1).numpy()
    assert np.abs(gi[0] - tr).max() <= 1e-9 * (1 + np.abs(tr).max())
    # without a scale the scale is one; a single pixel in the corner touches four taps only
    g1 = np.zeros((1, 3, 3, 2), np.float32)
    g1[0, 0, 0, 1] = 1.0
    W1 = rand_codes(r, (2, 3, 3, 1), 1)
    one = oracle.conv3x3_backward_input(g1, None, W1, 1, 1)[0, 0, :, :, 0]
    want = np.zeros((3, 3))
    want[0:2, 0:2] = W1[1, 1:3, 1:3, 0]                  # input (h, w) feeds output (0, 0) through tap (h + 1, w + 1)
    assert (one == want).all()


def test_update_sgd_is_one_multiply_and_one_subtraction(oracle):
    """Update() of Alg. 1 / Alg. 2 as plain gradient descent: w - eta * g with both steps rounded to binary32
    (numpy float32 arithmetic does exactly that), not a fused multiply-add."""
    r = rng(990)
    w, g = r.normal(size=4000).astype(np.float32), r.normal(size=4000).astype(np.float32)
    eta = np.float32(0.0371)
    want = w - (eta * g).astype(np.float32)
    got = oracle.update_sgd(w, g, float(eta))
    assert got.dtype == np.float32 and (got == want).all()
    fused = (w.astype(np.float64) - float(eta) * g.astype(np.float64)).astype(np.float32)
    assert (fused != want).any()            # the two readings differ on this input, so the pin separates them


def test_update_adam_against_the_textbook_rule(oracle):
    """Adam as the text's other choice for Update(): the float64 evaluation of the published rule (numpy)
    within a few binary32 roundings, for several steps run one after the other; the first step from zero
    moments moves every weight by eta against the sign of its gradient (|g| >> eps); a zero gradient with zero
    moments moves nothing."""
    r = rng(991)
    n = 3000
    w0 = r.normal(size=n).astype(np.float32)
    eta, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    w, m, v = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    wd, md, vd = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        g = r.normal(size=n).astype(np.float32)
        w, m, v = oracle.update_adam(w, g, m, v, eta, b1, b2, eps, t)
        gd = g.astype(np.float64)
        md = np.float32(b1) * md + (1 - np.float64(np.float32(b1))) * gd
        vd = np.float32(b2) * vd + (1 - np.float64(np.float32(b2))) * gd * gd
        wd = wd - np.float32(eta) * (md / (1 - np.float64(np.float32(b1)) ** t)) / (np.sqrt(vd / (1 - np.float64(np.float32(b2)) ** t)) + np.float32(eps))
        assert np.abs(w - wd).max() <= 1e-5 * eta * t + 4e-7 * np.abs(wd).max()
        assert np.abs(m - md).max() <= 1e-6 * (1 + np.abs(md).max()) and np.abs(v - vd).max() <= 1e-6 * (1 + np.abs(vd).max())
    g = r.normal(size=n).astype(np.float32)
    g[np.abs(g) < 1e-3] = 1.0
    w1, _, _ = oracle.update_adam(w0, g, np.zeros(n, np.float32), np.zeros(n, np.float32), eta, b1, b2, eps, 1)
    assert np.abs((w1.astype(np.float64) - w0) + eta * np.sign(g)).max() <= 1e-6
    w2, m2, v2 = oracle.update_adam(w0, np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32), eta, b1, b2, eps, 3)
    assert (w2 == w0).all() and (m2 == 0).all() and (v2 == 0).all()


def test_speedup_model_reading(oracle):
    """Eq. (16) with the constants of Sec. 5.4 (gamma = 1.91, L = 64, beta = gamma / 2) at N = 8192
    reproduces the printed 2-bit figure; this is the reading quoted as context beside the measured
    8192^3 sweep."""
    c = _consts()
    gamma, L = float(c["gamma"]), int(c["register_bits"])
    beta = gamma / 2
    S = lambda M, K, N: N * gamma / (M * K * (gamma + 2 * -(-N // L)) + (M * K - 1) * beta)
    assert abs(S(2, 2, 8192) - float(c["speedup_2bit"])) < 0.01          # 15.125 against the printed ~15.13
    assert S(1, 1, 8192) > S(2, 2, 8192) > S(3, 3, 8192) > S(6, 6, 8192) > 1.0
