"""GPU parity of the fused layer kernels (product -> scale -> re-encode -> bit planes in one
launch, Alg. 1 forward) and of the max-pool on bit planes, against the CPU oracle taken step by
step: integer product, one binary32 multiply, Table 2 rule, plane packing.  Everything here is
integer or bit work after the single multiply, so every comparison is exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from gpu_util import dev, host, rand_codes, planes_u32, say  # noqa: E402


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "no GPU visible"
    from paper_2106_09886_amd import binding
    binding.lib()
    return binding


def scales_for(rng, acc, out_bits, n):
    """Per-column scales that spread the products over the whole code range (and beyond it)."""
    rms = float(np.sqrt(np.mean(acc.astype(np.float64) ** 2))) + 1.0
    return (rng.uniform(0.5, 1.5, n) * ((1 << out_bits) / rms)).astype(np.float32)


def want_planes(oracle, acc, s, out_bits):
    y = oracle.scale_f32(acc, s) if s is not None else acc.astype(np.float32)
    codes = oracle.requant(y, out_bits)
    flat = codes.reshape(-1, codes.shape[-1])
    planes, bad = oracle.pack_planes(flat, out_bits)
    assert bad == 0
    return y, planes


CONV_CASES = [
    # Nb, H, W, C, Cout, ab, wb, out_bits
    (1, 1, 1, 32, 1, 2, 2, 2),
    (2, 5, 7, 64, 64, 2, 2, 2),          # pixel pairs, one column tile
    (1, 6, 6, 64, 70, 4, 2, 4),          # ragged second column tile (words 2 and 3 of 3)
    (1, 4, 9, 32, 33, 1, 1, 1),          # pixel groups of four
    (2, 8, 8, 128, 96, 4, 2, 4),         # one chunk of four words
    (1, 7, 5, 256, 40, 4, 2, 3),         # two chunk passes, partial sums in the workspace
    (1, 6, 6, 512, 130, 4, 2, 4),        # four chunk passes, three column tiles
    (1, 5, 6, 96, 64, 3, 3, 5),          # runtime plane stride
    (1, 5, 6, 384, 70, 4, 2, 4),         # runtime plane stride of twelve words: chunks of four
    (1, 4, 4, 40, 20, 6, 2, 8),          # wide activations (unpipelined path), 8-bit result
    (1, 3, 10, 256, 64, 4, 3, 7),        # taps in separate chunks
    (3, 14, 14, 64, 64, 2, 2, 2),        # several wavefronts per image
    (1, 5, 5, 64, 256, 2, 2, 2),         # four column tiles: blocks numbered per XCD
    (2, 4, 6, 256, 260, 4, 2, 4),        # the same with two chunk passes and a ragged fifth tile
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("extra", ["none", "acc", "f32", "both"])
def test_conv_packed_requant(q, oracle, case, extra):
    Nb, H, W, C, Cout, ab, wb, ob = case
    say("conv_packed_requant", case, extra)
    rng = np.random.default_rng(sum(case) * 7 + len(extra))
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
    acc = oracle.conv3x3(X, Wt)
    s = scales_for(rng, acc, ob, Cout)
    if extra == "acc" and Cout % 2 == 0:
        s = None                                     # also the scale-free form: y = (float)acc
    y, planes = want_planes(oracle, acc, s, ob)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    gp, gacc, gy = q.conv2d_packed_requant(Xp, ab, Wp, wb, Nb, H, W, C, Cout, ob,
                                           scale=None if s is None else dev(s),
                                           want_acc=extra in ("acc", "both"),
                                           want_f32=extra in ("f32", "both") and s is not None)
    assert (planes_u32(gp) == planes).all()
    if gacc is not None:
        assert (host(gacc).astype(np.int64) == acc).all()
    if gy is not None:
        assert (host(gy) == y).all()


@pytest.mark.parametrize("case", [(2, 6, 8, 3, 64, 8, 2, 4), (1, 5, 5, 1, 20, 4, 4, 2), (2, 4, 4, 3, 130, 8, 2, 8),
                                  (1, 6, 6, 64, 64, 2, 2, 2), (1, 4, 4, 5, 33, 2, 1, 1)])
def test_conv_im2col_requant(q, oracle, case):
    Nb, H, W, C, Cout, ab, wb, ob = case
    say("conv_im2col_requant", case)
    rng = np.random.default_rng(sum(case) * 11)
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
    acc = oracle.conv3x3(X, Wt)
    s = scales_for(rng, acc, ob, Cout)
    y, planes = want_planes(oracle, acc, s, ob)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    for want_acc, want_f32 in ((False, False), (True, True)):
        gp, gacc, gy = q.conv2d_im2col_requant(dev(X), ab, Wp, wb, Cout, ob, scale=dev(s), want_acc=want_acc,
                                               want_f32=want_f32)
        assert (planes_u32(gp) == planes).all()
        if want_acc:
            assert (host(gacc).astype(np.int64) == acc).all() and (host(gy) == y).all()


GEMM_CASES = [
    # M, N, K, ab, wb, out_bits
    (1, 1, 1, 1, 1, 1),
    (5, 64, 256, 2, 2, 2),
    (33, 70, 100, 4, 2, 4),
    (64, 130, 2500, 2, 2, 3),        # several chunk passes, ragged K and N
    (256, 96, 4096, 2, 2, 4),        # K chunks split over the wavefronts of a block
    (17, 40, 700, 5, 3, 8),
    (300, 64, 64, 3, 4, 6),
]


@pytest.mark.parametrize("case", GEMM_CASES)
@pytest.mark.parametrize("extra", ["none", "both"])
def test_branch_gemm_requant(q, oracle, case, extra):
    M, N, K, ab, wb, ob = case
    say("branch_gemm_requant", case, extra)
    rng = np.random.default_rng(sum(case) * 13)
    A = rand_codes(rng, (M, K), ab)
    Wm = rand_codes(rng, (K, N), wb)
    acc = oracle.gemm(A, Wm)
    s = scales_for(rng, acc, ob, N)
    y, planes = want_planes(oracle, acc, s, ob)
    Ap = q.encode_pack(dev(A), ab)
    Wp = q.encode_pack(dev(np.ascontiguousarray(Wm.T)), wb)
    gp, gacc, gy = q.branch_gemm_requant(Ap, ab, Wp, wb, K, ob, scale=dev(s), want_acc=extra == "both",
                                         want_f32=extra == "both")
    assert (planes_u32(gp) == planes).all()
    if extra == "both":
        assert (host(gacc).astype(np.int64) == acc).all() and (host(gy) == y).all()


def test_gemm_requant_feeds_next_gemm(q, oracle):
    """Two chained fully connected layers: the planes emitted by the first are the second's input."""
    rng = np.random.default_rng(5)
    M, K, N1, N2, ab, wb = 40, 300, 100, 50, 4, 2
    A = rand_codes(rng, (M, K), ab)
    W1, W2 = rand_codes(rng, (K, N1), wb), rand_codes(rng, (N1, N2), wb)
    acc1 = oracle.gemm(A, W1)
    s1 = scales_for(rng, acc1, ab, N1)
    codes1 = oracle.requant(oracle.scale_f32(acc1, s1), ab)
    acc2 = oracle.gemm(codes1.astype(np.int16), W2)
    p1, _, _ = q.branch_gemm_requant(q.encode_pack(dev(A), ab), ab, q.encode_pack(dev(np.ascontiguousarray(W1.T)), wb),
                                     wb, K, ab, scale=dev(s1))
    g2, _ = q.branch_gemm(p1, ab, q.encode_pack(dev(np.ascontiguousarray(W2.T)), wb), wb, N1)
    assert (host(g2).astype(np.int64) == acc2).all()


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("shape", [(1, 2, 2, 1), (2, 4, 6, 33), (1, 8, 2, 64), (3, 6, 10, 130), (2, 16, 16, 256)])
def test_maxpool2x2_planes(q, oracle, bits, shape):
    say("maxpool2x2_planes", bits, shape)
    Nb, H, W, C = shape
    rng = np.random.default_rng(bits * 31 + sum(shape))
    codes = rand_codes(rng, shape, bits)
    pooled = oracle.maxpool2x2(codes.astype(np.float32)).astype(np.int16)       # small integers: exact in fp32
    want, bad = oracle.pack_planes(pooled.reshape(-1, C), bits)
    assert bad == 0
    planes = q.encode_pack(dev(codes.reshape(Nb * H * W, C)), bits)
    got = q.maxpool2x2_planes(planes, Nb, H, W, C, bits)
    assert (planes_u32(got) == want).all()


# ------------------------------------------------------------------------- chains
def run_stack_fused(q, oracle, X0, layers, ab_first, ab, wb, report=False):
    """GPU: one fused kernel per layer (plus the plane max-pool after a block); nothing but bit
    planes travels between layers.  Oracle: the plain chain.  Compared layer by layer."""
    Nb, H, W, C = X0.shape
    codes = X0
    x_planes = None
    for l, (Wt, s, pool) in enumerate(layers, start=1):
        Cout = Wt.shape[0]
        bits_in = ab_first if l == 1 else ab
        Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
        if l == 1:
            x_planes, _, _ = q.conv2d_im2col_requant(dev(X0), bits_in, Wp, wb, Cout, ab, scale=dev(s))
        else:
            x_planes, _, _ = q.conv2d_packed_requant(x_planes, bits_in, Wp, wb, Nb, H, W, C, Cout, ab, scale=dev(s))
        if pool:
            x_planes = q.maxpool2x2_planes(x_planes, Nb, H, W, Cout, ab)
        o_acc = oracle.conv3x3(codes, Wt)
        o_y = oracle.scale_f32(o_acc, s)
        o_codes = oracle.requant(oracle.maxpool2x2(o_y) if pool else o_y, ab)
        want, bad = oracle.pack_planes(o_codes.reshape(-1, Cout), ab)
        assert bad == 0 and (planes_u32(x_planes) == want).all(), "layer %d planes" % l
        if report:
            say("layer %2d: %s -> %d ch, pool=%d ok" % (l, (Nb, H, W, C), Cout, pool))
        codes = o_codes
        C = Cout
        if pool:
            H, W = H // 2, W // 2


def test_stack_small_fused(q, oracle):
    from paper_2106_09886_amd import inputs
    w = inputs.VGG16
    X0, layers = inputs.make_stack(w, Nb=2, H=32, W=32)
    run_stack_fused(q, oracle, X0, layers, w.ab_first, w.ab, w.wb)


def test_stack_odd_sizes_fused(q, oracle):
    rng = np.random.default_rng(78)
    X0 = rand_codes(rng, (2, 12, 20, 5), 8)
    chans = [5, 33, 70, 64, 130]
    layers = []
    for l in range(1, len(chans)):
        Wt = rand_codes(rng, (chans[l], 3, 3, chans[l - 1]), 2)
        s = (rng.uniform(0.8, 1.2, chans[l]) / np.sqrt(45.0 * chans[l - 1] * (300.0 if l == 1 else 1.0))).astype(np.float32)
        layers.append((Wt, s, l in (2, 3)))
    run_stack_fused(q, oracle, X0, layers, 8, 4, 2)


def test_stack_config5_full_fused(q, oracle):
    """VGG-16-shaped stack at full size through the fused kernels."""
    from paper_2106_09886_amd import inputs
    w = inputs.VGG16
    X0, layers = inputs.make_stack(w)
    say("vgg16 stack, fused kernels: oracle + gpu, layer by layer")
    run_stack_fused(q, oracle, X0, layers, w.ab_first, w.ab, w.wb, report=True)


def test_stack_mixed_precision(q, oracle):
    """Per-layer bit widths (Sec. 5: activations at 4 bits with 5/3/2/2/6-bit weights; here also a
    change of the activation width along the chain): every layer's out_bits is the next one's ab."""
    rng = np.random.default_rng(404)
    Nb, H, W = 2, 16, 16
    chans = [3, 32, 64, 64, 96, 40]
    wbs = [5, 3, 2, 2, 6]
    abs_in = [8, 4, 4, 3, 4]          # activation width each layer reads
    ab_out = [4, 4, 3, 4, 2]          # = width the next layer reads (the last one is free)
    pools = [False, True, False, True, False]
    codes = rand_codes(rng, (Nb, H, W, chans[0]), abs_in[0])
    x_planes = None
    C = chans[0]
    for l in range(5):
        Cout, wb, ab, ob, pool = chans[l + 1], wbs[l], abs_in[l], ab_out[l], pools[l]
        Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
        o_acc = oracle.conv3x3(codes, Wt)
        s = scales_for(rng, o_acc, ob, Cout)
        Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
        if l == 0:
            x_planes, _, _ = q.conv2d_im2col_requant(dev(codes), ab, Wp, wb, Cout, ob, scale=dev(s))
        else:
            x_planes, _, _ = q.conv2d_packed_requant(x_planes, ab, Wp, wb, Nb, H, W, C, Cout, ob, scale=dev(s))
        if pool:
            x_planes = q.maxpool2x2_planes(x_planes, Nb, H, W, Cout, ob)
        o_y = oracle.scale_f32(o_acc, s)
        codes = oracle.requant(oracle.maxpool2x2(o_y) if pool else o_y, ob)
        want, bad = oracle.pack_planes(codes.reshape(-1, Cout), ob)
        assert bad == 0 and (planes_u32(x_planes) == want).all(), "layer %d" % (l + 1)
        assert len(np.unique(codes)) > 1
        C = Cout
        if pool:
            H, W = H // 2, W // 2
