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
