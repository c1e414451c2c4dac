"""GPU parity of the smooth range limiters of the front end (Table 1: Tanh, Sigmoid) and of the
element-wise training-side pieces (Eq. (12), (14), (15)) against the CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from gpu_util import dev, host, planes_u32, say  # noqa: E402


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "no GPU visible"
    from paper_2106_09886_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("clip", ["tanh", "sigmoid"])
@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("shape", [(7, 100), (64, 256), (3, 64)])
def test_encode_real_smooth_limiters(q, oracle, clip, bits, shape):
    """The limiter is a transcendental function taken in binary32 on the GPU and in float64 (rounded
    once) by the oracle, so the limited values may differ by a few units of the last place.  Where the
    oracle's value is further than 1e-5 (in code units) from an interval boundary the codes must be
    equal; the few elements inside that band may sit in either neighbouring state, nothing else."""
    say("encode_real", clip, bits, shape)
    rng = np.random.default_rng(bits * 31 + shape[0] + (5 if clip == "tanh" else 0))
    x = rng.uniform(-4, 4, shape).astype(np.float32)
    x[0, :4] = [0.0, -0.0, 30.0, -30.0]
    want, limited = oracle.encode_smooth(x, bits, clip)
    codes, planes = q.encode_real(dev(x), bits, clip=clip)
    got = host(codes).astype(np.int64)
    alpha = (1 << bits) - 1
    y = limited.astype(np.float64) * alpha
    near = np.abs(y - 2 * np.round(y / 2)) <= 1e-5 * max(1.0, alpha / 3.0)
    assert (got[~near] == want[~near]).all()
    assert (np.abs(got[near] - want[near]) <= 2).all()
    assert near.sum() <= 4 + 0.01 * near.size            # the four planted values sit on boundaries
    # the planes are the packed form of the codes the GPU itself chose
    pw, bad = oracle.pack_planes(got.astype(np.int16), bits)
    assert bad == 0 and (planes_u32(planes) == pw).all()


@pytest.mark.parametrize("bits", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("n", [1, 1000, 70001])
def test_encoder_backward(q, oracle, bits, n):
    """fp32 result against the float64 oracle: the kernel sums in double precision and rounds once, so
    the error is one binary32 rounding of the result plus the cancellation of the terms; the bound
    used is 2^-22 of the sum of the terms' magnitudes."""
    say("encoder_backward", bits, n)
    rng = np.random.default_rng(bits * 7 + n)
    x = rng.uniform(-1.3, 1.3, n).astype(np.float32)
    x[:1] = 1.0
    g = rng.normal(size=(bits, n)).astype(np.float32)
    want = oracle.encoder_backward(x, g)
    got = host(q.encoder_backward(dev(x), dev(g))).astype(np.float64)
    scale = sum(np.abs(g[m - 1].astype(np.float64)) * ((2 ** bits - 1) / 2 ** m) * np.pi for m in range(1, bits + 1))
    assert (np.abs(got - want) <= 2.0 ** -22 * scale + 1e-30).all()
    assert (got[np.abs(x) > 1] == 0).all()


@pytest.mark.parametrize("shape", [(1, 1), (5, 31), (4, 64), (3, 65), (9, 200), (128, 576)])
def test_binarize(q, oracle, shape):
    say("binarize", shape)
    rng = np.random.default_rng(shape[0] * 3 + shape[1])
    w = rng.normal(size=shape).astype(np.float32) * 1.5
    w.flat[: min(4, w.size)] = np.array([0.0, -0.0, 1.0, -1.0], dtype=np.float32)[: min(4, w.size)]
    want = oracle.binarize(w)
    codes, planes = q.binarize(dev(w))
    assert (host(codes) == want).all()
    pw, bad = oracle.pack_planes(want.astype(np.int16), 1)
    assert bad == 0 and (planes_u32(planes) == pw).all()
    g = rng.normal(size=shape).astype(np.float32)
    assert (host(q.binarize_backward(dev(w), dev(g))) == oracle.binarize_backward(w, g)).all()


def test_binarized_weights_feed_the_branch_gemm(q, oracle):
    """Alg. 1 forward with one bit: the planes qnn_binarize writes are the weight operand of the product."""
    rng = np.random.default_rng(12)
    M, N, K = 33, 70, 300
    w = rng.normal(size=(N, K)).astype(np.float32)
    a = (2 * rng.integers(0, 4, size=(M, K)) - 3).astype(np.int8)
    _, wp = q.binarize(dev(w), want_codes=False)
    ap = q.encode_pack(dev(a), 2)
    acc, _ = q.branch_gemm(ap, 2, wp, 1, K)
    want = oracle.gemm(a, oracle.binarize(w).T.copy())
    assert (host(acc).astype(np.int64) == want).all()


@pytest.mark.parametrize("bits", [2, 3, 4, 8, 16])
@pytest.mark.parametrize("t", [1.0, 0.75, 3.3])
def test_quantize_k(q, oracle, bits, t):
    """Every step is one binary32 operation on both sides: bit-equal values, equal integer states."""
    say("quantize_k", bits, t)
    rng = np.random.default_rng(bits * 13 + int(t * 10))
    x = rng.uniform(-1.5 * t, 1.5 * t, 50001).astype(np.float32)
    n = 2 ** (bits - 1) - 1
    x[:6] = np.array([t, -t, 0.0, 0.5 * t / n, 1.5 * t / n, np.inf], dtype=np.float32)
    want_q, want_l = oracle.quantize_k(x, bits, t)
    gq, gl = q.quantize_k(dev(x), bits, t)
    assert (host(gl) == want_l).all()
    assert (host(gq).view(np.uint32) == want_q.view(np.uint32)).all()
    g = rng.normal(size=x.shape).astype(np.float32)
    assert (host(q.quantize_k_backward(dev(x), dev(g), t)) == oracle.quantize_k_backward(x, g, t)).all()


# ------------------------------------------------------------------ Alg. 1, backward through the product
def _backward_case(q, oracle, M, N, K, ab, wb, with_scale, seed):
    from gpu_util import rand_codes
    rng = np.random.default_rng(seed)
    A, W = rand_codes(rng, (M, K), ab), rand_codes(rng, (N, K), wb)
    g = rng.normal(size=(M, N)).astype(np.float32)
    s = rng.uniform(0.25, 4.0, N).astype(np.float32) if with_scale else None
    Ap = q.encode_pack(dev(A), ab) if M and K else None
    Wp = q.encode_pack(dev(W), wb) if N and K else None
    return A, W, g, s, Ap, Wp


def _bound(g, s, codes_abs_sum_matrix, J):
    """(J + 2) * 2^-24 * sum_j |g_ahat| |code|: binary32 accumulation of J terms in any order, one rounding
    of the scale product, exact codes and exact powers of two (the tolerance the header states)."""
    return (J + 2) * 2.0 ** -24 * codes_abs_sum_matrix


BACKWARD_CASES = [
    # (M, N, K, ab, wb, with_scale): several 32-row / 128-column tiles with ragged tails in every
    # direction, reduction lengths that are and are not multiples of 8 (vector and scalar load paths),
    # every code width, single rows and columns
    (70, 100, 130, 2, 2, True), (33, 64, 257, 4, 3, False), (128, 256, 128, 2, 2, True), (1, 1, 1, 1, 1, False),
    (5, 8, 32, 8, 8, True), (200, 24, 40, 3, 5, True), (257, 40, 129, 1, 4, False), (64, 7, 64, 6, 1, True),
    (96, 136, 300, 7, 2, False), (40, 264, 96, 2, 6, True), (300, 16, 33, 5, 7, False),
]


@pytest.mark.parametrize("case", BACKWARD_CASES, ids=lambda c: "M%d-N%d-K%d-A%dW%d%s" % (c[0], c[1], c[2], c[3], c[4], "-s" if c[5] else ""))
def test_branch_gemm_backward(q, oracle, case):
    """Both gradients of Alg. 1's backward lines against the float64 oracle, element by element, within the
    binary32 accumulation bound; the 2^(m-1) / 2^(k-1) copies are exact multiples of the first."""
    M, N, K, ab, wb, with_scale = case
    say("branch_gemm_backward", case)
    A, W, g, s, Ap, Wp = _backward_case(q, oracle, M, N, K, ab, wb, with_scale, 7 * M + 3 * N + K + ab + wb)
    gs = np.abs(g.astype(np.float64)) * (1.0 if s is None else s.astype(np.float64)[None, :])
    want_i = oracle.branch_backward_input(g, s, W, ab, wb)
    got_i = host(q.branch_gemm_backward_input(dev(g), Wp, wb, K, ab, scale=None if s is None else dev(s))).astype(np.float64)
    assert got_i.shape == want_i.shape == (ab, M, K)
    bound_i = _bound(g, s, gs @ np.abs(W.astype(np.float64)), N)
    for m in range(ab):
        assert (np.abs(got_i[m] - want_i[m]) <= 2.0 ** m * bound_i).all()
        assert (got_i[m] == 2.0 ** m * got_i[0]).all()
    want_w = oracle.branch_backward_weight(g, s, A, ab, wb)
    got_w = host(q.branch_gemm_backward_weight(dev(g), Ap, ab, K, wb, scale=None if s is None else dev(s))).astype(np.float64)
    assert got_w.shape == want_w.shape == (wb, N, K)
    bound_w = _bound(g, s, gs.T @ np.abs(A.astype(np.float64)), M)
    for k in range(wb):
        assert (np.abs(got_w[k] - want_w[k]) <= 2.0 ** k * bound_w).all()
        assert (got_w[k] == 2.0 ** k * got_w[0]).all()
    # not vacuous: the results are far from zero compared with the bound
    assert np.abs(want_i[0]).mean() > 100 * bound_i.mean() and np.abs(want_w[0]).mean() > 100 * bound_w.mean()


def test_branch_gemm_backward_exact_on_small_integers(q, oracle):
    """Integer-valued gradients of small magnitude: every product and partial sum is an integer below 2^24,
    so binary32 accumulation is exact in any order and the result must equal the oracle's bit for bit."""
    from gpu_util import rand_codes
    rng = np.random.default_rng(5)
    M, N, K, ab, wb = 100, 72, 200, 3, 4
    A, W = rand_codes(rng, (M, K), ab), rand_codes(rng, (N, K), wb)
    g = rng.integers(-8, 9, size=(M, N)).astype(np.float32)
    s = (2.0 ** rng.integers(-1, 3, size=N)).astype(np.float32)
    Ap, Wp = q.encode_pack(dev(A), ab), q.encode_pack(dev(W), wb)
    assert (host(q.branch_gemm_backward_input(dev(g), Wp, wb, K, ab, scale=dev(s))).astype(np.float64)
            == oracle.branch_backward_input(g, s, W, ab, wb)).all()
    assert (host(q.branch_gemm_backward_weight(dev(g), Ap, ab, K, wb, scale=dev(s))).astype(np.float64)
            == oracle.branch_backward_weight(g, s, A, ab, wb)).all()


def test_branch_gemm_backward_degenerate_sizes(q, oracle):
    """An empty sum writes zeros; an empty output launches nothing."""
    import torch
    from gpu_util import rand_codes
    rng = np.random.default_rng(6)
    g0 = torch.empty((5, 0), dtype=torch.float32, device="cuda")
    Wp0 = torch.empty((0, 2, 2), dtype=torch.int32, device="cuda")
    out = q.branch_gemm_backward_input(g0, Wp0, 2, 40, 3)
    assert tuple(out.shape) == (3, 5, 40) and (host(out) == 0).all()
    gM0 = torch.empty((0, 7), dtype=torch.float32, device="cuda")
    Ap0 = torch.empty((0, 2, 2), dtype=torch.int32, device="cuda")
    out = q.branch_gemm_backward_weight(gM0, Ap0, 2, 40, 3)
    assert tuple(out.shape) == (3, 7, 40) and (host(out) == 0).all()
    assert tuple(q.branch_gemm_backward_input(gM0, q.encode_pack(dev(rand_codes(rng, (7, 40), 2)), 2), 2, 40, 3).shape) == (3, 0, 40)


def test_branch_gemm_backward_at_the_fc_layer_size(q, oracle):
    """The fully connected configuration of the benchmark (256 x 4096 x 4096, W2A2) in the launch shape the
    library picks; sampled rows against the oracle (the oracle computes only those rows / filters)."""
    from gpu_util import rand_codes
    rng = np.random.default_rng(11)
    M, N, K, ab, wb = 256, 4096, 4096, 2, 2
    A, W = rand_codes(rng, (M, K), ab), rand_codes(rng, (N, K), wb)
    g = rng.normal(size=(M, N)).astype(np.float32)
    s = rng.uniform(0.5, 2.0, N).astype(np.float32)
    Ap, Wp = q.encode_pack(dev(A), ab), q.encode_pack(dev(W), wb)
    got_i = host(q.branch_gemm_backward_input(dev(g), Wp, wb, K, ab, scale=dev(s))).astype(np.float64)
    got_w = host(q.branch_gemm_backward_weight(dev(g), Ap, ab, K, wb, scale=dev(s))).astype(np.float64)
    gs = np.abs(g.astype(np.float64)) * s.astype(np.float64)[None, :]
    rows = np.array([0, 31, 32, 127, 128, 255])
    want = oracle.branch_backward_input(g[rows], s, W, ab, wb)
    bound = _bound(g, s, gs[rows] @ np.abs(W.astype(np.float64)), N)
    for m in range(ab):
        assert (np.abs(got_i[m][rows] - want[m]) <= 2.0 ** m * bound).all()
    filt = np.array([0, 63, 64, 2047, 4095])
    want = oracle.branch_backward_weight(g[:, filt], s[filt], A, ab, wb)
    bound = _bound(g, s, gs[:, filt].T @ np.abs(A.astype(np.float64)), M)
    for k in range(wb):
        assert (np.abs(got_w[k][filt] - want[k]) <= 2.0 ** k * bound).all()


@pytest.mark.parametrize("n", [1, 255, 4096, 100003])
def test_update_sgd(q, oracle, n):
    rng = np.random.default_rng(n)
    w, g = rng.normal(size=n).astype(np.float32), rng.normal(size=n).astype(np.float32)
    want = oracle.update_sgd(w, g, 0.0371)
    wd = dev(w)
    q.update_sgd(wd, dev(g), 0.0371)
    assert (host(wd) == want).all()


@pytest.mark.parametrize("M,N,K,ab,wb", [(2053, 204, 4001, 2, 3), (2050, 203, 4033, 3, 2), (2176, 40, 4096, 8, 8), (2048, 36, 4000, 1, 1)])
def test_branch_gemm_backward_input_many_tiles(q, oracle, M, N, K, ab, wb):
    """Outputs of more than 512 block tiles take the kernel that stages the gradient through LDS: sum
    lengths that are and are not multiples of 4 (16-byte and scalar loads) and of 32 (last tile partly
    empty), ragged last row and column tiles, one to eight code bits.  Sampled rows against the oracle."""
    say("backward_input_many_tiles", M, N, K, ab, wb)
    A, W, g, s, Ap, Wp = _backward_case(q, oracle, M, N, K, ab, wb, True, M + N + K)
    got = host(q.branch_gemm_backward_input(dev(g), Wp, wb, K, ab, scale=dev(s))).astype(np.float64)
    rows = np.array([0, 1, 31, 32, 127, 128, 1000, M - 130, M - 2, M - 1])
    want = oracle.branch_backward_input(g[rows], s, W, ab, wb)
    gs = np.abs(g[rows].astype(np.float64)) * s.astype(np.float64)[None, :]
    bound = _bound(g, s, gs @ np.abs(W.astype(np.float64)), N)
    for m in range(ab):
        assert (np.abs(got[m][rows] - want[m]) <= 2.0 ** m * bound).all()
        assert (got[m] == 2.0 ** m * got[0]).all()
    assert np.abs(want[0]).mean() > 100 * bound.mean()


@pytest.mark.parametrize("M,N,K,ab,wb", [(150, 2052, 4001, 3, 2), (97, 2053, 4033, 2, 3), (64, 2176, 4096, 8, 8), (33, 2048, 4000, 1, 1)])
def test_branch_gemm_backward_weight_many_tiles(q, oracle, M, N, K, ab, wb):
    """The same for the gradient of the weights (the gradient matrix is read along its rows)."""
    say("backward_weight_many_tiles", M, N, K, ab, wb)
    A, W, g, s, Ap, Wp = _backward_case(q, oracle, M, N, K, ab, wb, True, M + N + K + 1)
    got = host(q.branch_gemm_backward_weight(dev(g), Ap, ab, K, wb, scale=dev(s))).astype(np.float64)
    filt = np.array([0, 1, 31, 32, 127, 128, 1000, N - 130, N - 2, N - 1])
    want = oracle.branch_backward_weight(g[:, filt], s[filt], A, ab, wb)
    gs = np.abs(g[:, filt].astype(np.float64)) * s[filt].astype(np.float64)[None, :]
    bound = _bound(g, s, gs.T @ np.abs(A.astype(np.float64)), M)
    for k in range(wb):
        assert (np.abs(got[k][filt] - want[k]) <= 2.0 ** k * bound).all()
        assert (got[k] == 2.0 ** k * got[0]).all()
    assert np.abs(want[0]).mean() > 100 * bound.mean()


@pytest.mark.parametrize("M,N,K", [(2048, 64, 4096), (40, 2048, 4096), (70, 96, 130)])
def test_branch_gemm_backward_unaligned_gradient(q, oracle, M, N, K):
    """A gradient and a scale that are only 4-byte aligned (views one element into a buffer): the kernels
    must fall back to scalar loads; sampled rows / filters against the oracle."""
    import torch
    say("backward unaligned", M, N, K)
    ab = wb = 2
    A, W, g, s, Ap, Wp = _backward_case(q, oracle, M, N, K, ab, wb, True, M * 3 + N)
    gbuf = torch.empty(M * N + 1, dtype=torch.float32, device="cuda")
    gd = gbuf[1:].view(M, N)
    gd.copy_(dev(g))
    sbuf = torch.empty(N + 1, dtype=torch.float32, device="cuda")
    sd = sbuf[1:]
    sd.copy_(dev(s))
    assert gd.data_ptr() % 16 == 4 and sd.data_ptr() % 16 == 4
    gs = np.abs(g.astype(np.float64)) * s.astype(np.float64)[None, :]
    rows = np.unique(np.array([0, 33, M // 2, M - 1]))
    got = host(q.branch_gemm_backward_input(gd, Wp, wb, K, ab, scale=sd)).astype(np.float64)
    want = oracle.branch_backward_input(g[rows], s, W, ab, wb)
    bound = _bound(g, s, gs[rows] @ np.abs(W.astype(np.float64)), N)
    for m in range(ab):
        assert (np.abs(got[m][rows] - want[m]) <= 2.0 ** m * bound).all()
    filt = np.unique(np.array([0, 31, N // 2, N - 1]))
    got = host(q.branch_gemm_backward_weight(gd, Ap, ab, K, wb, scale=sd)).astype(np.float64)
    want = oracle.branch_backward_weight(g[:, filt], s[filt], A, ab, wb)
    bound = _bound(g, s, gs[:, filt].T @ np.abs(A.astype(np.float64)), M)
    for k in range(wb):
        assert (np.abs(got[k][filt] - want[k]) <= 2.0 ** k * bound).all()


@pytest.mark.parametrize("n", [1, 257, 100003])
def test_update_adam(q, oracle, n):
    """Five Adam steps in a row, bit for bit: both sides take the same sequence of correctly rounded binary32
    operations (including a gradient of zero and tiny second moments)."""
    rng = np.random.default_rng(n + 17)
    w = rng.normal(size=n).astype(np.float32)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    wd, md, vd = dev(w), dev(m), dev(v)
    for t in range(1, 6):
        g = (rng.normal(size=n) * 10.0 ** rng.integers(-6, 2)).astype(np.float32)
        g[:: 7] = 0.0
        w, m, v = oracle.update_adam(w, g, m, v, 1e-3, 0.9, 0.999, 1e-8, t)
        q.update_adam(wd, dev(g), md, vd, 1e-3, 0.9, 0.999, 1e-8, t)
        assert (host(md) == m).all() and (host(vd) == v).all() and (host(wd) == w).all()


# ------------------------------------------------------------------ Alg. 1, backward through the 3x3 convolution
CONV_BACKWARD_CASES = [
    # (Nb, H, W, C, Cout, ab, wb, with_scale): images smaller than the window, ragged channel and filter
    # counts, several 128-pixel row blocks, filter counts that are and are not multiples of 4 (16-byte and
    # scalar loads of the weight gradient), several pixel ranges (> 1024 pixels), one to eight bits
    (1, 1, 1, 3, 2, 1, 1, False), (2, 5, 4, 6, 7, 2, 2, True), (1, 9, 11, 70, 33, 4, 3, True), (3, 8, 8, 64, 64, 2, 2, True),
    (2, 14, 14, 130, 40, 3, 2, False), (1, 2, 7, 32, 128, 8, 8, True), (2, 32, 32, 32, 36, 2, 4, True),
    (1, 40, 40, 40, 130, 4, 2, True),
]


@pytest.mark.parametrize("case", CONV_BACKWARD_CASES, ids=lambda c: "%dx%dx%dx%d-O%d-A%dW%d%s" % (c[:7] + ("-s" if c[7] else "",)))
def test_conv2d_backward(q, oracle, case):
    """Both gradients of the backward lines through the 3x3 convolution against the float64 oracle, element by
    element within the binary32 accumulation bound (J = 9*Cout terms towards the activations, Nb*H*W towards
    the weights); the copies per encoded element are exact multiples of the first."""
    from gpu_util import rand_codes
    Nb, H, W, C, Cout, ab, wb, with_scale = case
    say("conv2d_backward", case)
    rng = np.random.default_rng(sum(case[:7]) * 3 + 1)
    X, Wt = rand_codes(rng, (Nb, H, W, C), ab), rand_codes(rng, (Cout, 3, 3, C), wb)
    g = rng.normal(size=(Nb, H, W, Cout)).astype(np.float32)
    s = rng.uniform(0.25, 4.0, Cout).astype(np.float32) if with_scale else None
    sd = None if s is None else dev(s)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    gabs = np.abs(g.astype(np.float32)) * (1.0 if s is None else s[None, None, None, :])
    ones_w = np.abs(Wt.astype(np.int64)).astype(np.int16)
    ones_x = np.abs(X.astype(np.int64)).astype(np.int16)
    # sum of |terms|: the same backward lines on absolute values (one encoded element of weight 1 suffices: use the
    # closed form sum |g_ahat| |code| through the oracle's own routine on 8-bit "codes" is not possible for even
    # values, so take numpy)
    import torch
    import torch.nn.functional as F
    ga = torch.tensor(gabs.astype(np.float64)).permute(0, 3, 1, 2)
    wa = torch.tensor(ones_w.astype(np.float64)).permute(0, 3, 1, 2)
    xa = torch.tensor(ones_x.astype(np.float64)).permute(0, 3, 1, 2)
    abs_i = F.conv_transpose2d(ga, wa, padding=1).permute(0, 2, 3, 1).numpy()
    xa.requires_grad_(False)
    wz = torch.zeros_like(wa, requires_grad=True)
    (F.conv2d(xa, wz, padding=1) * ga).sum().backward()
    abs_w = wz.grad.permute(0, 2, 3, 1).numpy()
    want_i = oracle.conv3x3_backward_input(g, s, Wt, ab, wb)
    got_i = host(q.conv2d_backward_input(dev(g), Wp, wb, C, ab, scale=sd)).astype(np.float64)
    assert got_i.shape == want_i.shape
    bound_i = (9 * Cout + 2) * 2.0 ** -24 * abs_i
    for m in range(ab):
        assert (np.abs(got_i[m] - want_i[m]) <= 2.0 ** m * bound_i + 1e-30).all()
        assert (got_i[m] == 2.0 ** m * got_i[0]).all()
    want_w = oracle.conv3x3_backward_weight(g, s, X, ab, wb)
    got_w = host(q.conv2d_backward_weight(dev(g), Xp, ab, C, wb, scale=sd)).astype(np.float64)
    assert got_w.shape == want_w.shape
    bound_w = (Nb * H * W + 2) * 2.0 ** -24 * abs_w
    for k in range(wb):
        assert (np.abs(got_w[k] - want_w[k]) <= 2.0 ** k * bound_w + 1e-30).all()
        assert (got_w[k] == 2.0 ** k * got_w[0]).all()
    if Nb * H * W >= 64:
        assert np.abs(want_i[0]).mean() > 50 * bound_i.mean() and np.abs(want_w[0]).mean() > 50 * bound_w.mean()


def test_conv2d_backward_exact_on_small_integers(q, oracle):
    """Integer gradients: every partial sum stays below 2^24, so any summation order is exact and both
    gradients must equal the oracle bit for bit (this also pins the fixed-order addition of the pixel ranges)."""
    from gpu_util import rand_codes
    rng = np.random.default_rng(77)
    Nb, H, W, C, Cout, ab, wb = 2, 24, 24, 40, 24, 2, 2
    X, Wt = rand_codes(rng, (Nb, H, W, C), ab), rand_codes(rng, (Cout, 3, 3, C), wb)
    g = rng.integers(-4, 5, size=(Nb, H, W, Cout)).astype(np.float32)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    assert (host(q.conv2d_backward_input(dev(g), Wp, wb, C, ab)).astype(np.float64) == oracle.conv3x3_backward_input(g, None, Wt, ab, wb)).all()
    assert (host(q.conv2d_backward_weight(dev(g), Xp, ab, C, wb)).astype(np.float64) == oracle.conv3x3_backward_weight(g, None, X, ab, wb)).all()


def test_conv2d_backward_at_the_resnet18_layer_size(q, oracle):
    """The headline layer (32 x 56 x 56 x 64 -> 64, W2A2) in the launch shape the library picks; towards the
    activations on the first image against the oracle (its pixels see only that image), towards the weights
    through torch's float64 autograd on the decoded codes (the routine that pins the oracle)."""
    import torch
    import torch.nn.functional as F
    from gpu_util import rand_codes
    rng = np.random.default_rng(18)
    Nb, H, W, C, Cout, ab, wb = 32, 56, 56, 64, 64, 2, 2
    X, Wt = rand_codes(rng, (Nb, H, W, C), ab), rand_codes(rng, (Cout, 3, 3, C), wb)
    g = rng.normal(size=(Nb, H, W, Cout)).astype(np.float32)
    s = rng.uniform(0.5, 2.0, Cout).astype(np.float32)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    got_i = host(q.conv2d_backward_input(dev(g), Wp, wb, C, ab, scale=dev(s))).astype(np.float64)
    want_i = oracle.conv3x3_backward_input(g[:1], s, Wt, ab, wb)
    tol_i = (9 * Cout + 2) * 2.0 ** -24 * 9 * Cout * 3 * np.abs(g).max() * 2.0
    for m in range(ab):
        assert np.abs(got_i[m][:1] - want_i[m]).max() <= 2.0 ** m * tol_i
    got_w = host(q.conv2d_backward_weight(dev(g), Xp, ab, C, wb, scale=dev(s))).astype(np.float64)
    x = torch.tensor(X.astype(np.float64)).permute(0, 3, 1, 2)
    wz = torch.zeros((Cout, C, 3, 3), dtype=torch.float64, requires_grad=True)
    gs = torch.tensor(g.astype(np.float64) * s.astype(np.float64)).permute(0, 3, 1, 2)
    (F.conv2d(x, wz, padding=1) * gs).sum().backward()
    dw = wz.grad.permute(0, 2, 3, 1).numpy()
    tol_w = (Nb * H * W + 2) * 2.0 ** -24 * 3 * np.abs(g).sum(axis=(0, 1, 2)).max() * 2.0
    for k in range(wb):
        assert np.abs(got_w[k] - 2.0 ** k * dw).max() <= 2.0 ** k * tol_w
    assert np.abs(dw).mean() > 100 * tol_w / 1000           # the tolerance is small against the gradient's size
