"""GPU parity of the any-geometry convolution (strides, paddings, dilations, kernel sizes,
transposed form) against the CPU oracle: int32 results bit-exact, fp32 results bit-equal to the
oracle's single binary32 multiply, emitted planes equal to the oracle's re-encoding."""
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


def run_case(q, oracle, Nb, H, W, C, Cout, ab, wb, KH, KW, stride=1, pad=0, dilation=1, transposed=False,
             output_padding=0, out_bits=0, seed=0, workspace=True, dense_rows=False):
    rng = np.random.default_rng(seed + Nb * 7 + H * 5 + C * 3 + Cout + KH * 11 + KW)
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, KH, KW, C), wb)
    if transposed:
        want = oracle.conv2d_transposed(X, Wt, stride=stride, pad=pad, dilation=dilation, output_padding=output_padding)
    else:
        want = oracle.conv2d(X, Wt, stride=stride, pad=pad, dilation=dilation)
    rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2))) + 1.0
    s = (rng.uniform(0.5, 1.5, Cout) * ((1 << max(out_bits, 2)) / rms)).astype(np.float32)
    geo = q.conv_geometry(KH, KW, stride=stride, pad=pad, dilation=dilation, transposed=transposed,
                          output_padding=output_padding, dense_rows=dense_rows)
    # row-dense: one packed row per image row (bit w*C + c), else one per pixel
    Xp = q.encode_pack(dev(X.reshape(Nb * H, W * C) if dense_rows else X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * KH * KW, C)), wb)
    y_want = oracle.scale_f32(want, s)
    y64 = oracle.scale_f64(want, s)
    # a 3x3 window at stride 1, padding 1 goes to the dedicated 3x3 kernel unless told otherwise:
    # such a case runs both ways
    pair = lambda v: tuple(v) if isinstance(v, (tuple, list)) else (v, v)
    handed_over = (not transposed and not dense_rows and (KH, KW) == (3, 3) and pair(stride) in ((1, 1), (2, 2))
                   and pair(pad) == (1, 1) and pair(dilation) == (1, 1))
    # ... and so does any odd window with "same" padding at stride 1 (atrous 3x3, 5x5, 1x3 ...) from 128 channels on
    d2 = pair(dilation)
    handed_over = handed_over or (not transposed and not dense_rows and KH % 2 == 1 and KW % 2 == 1 and KH * KW > 1
                                  and pair(stride) == (1, 1) and d2[0] == d2[1]
                                  and pair(pad) == ((KH // 2) * d2[0], (KW // 2) * d2[1]))
    for general_only in ((1, 0) if handed_over else (0,)):
        q.tune(general_only=general_only)
        try:
            acc, y, planes = q.conv2d_general(Xp, ab, Wp, wb, Nb, H, W, C, Cout, geo, scale=dev(s),
                                              out_bits=out_bits, workspace=workspace)
        finally:
            q.tune(general_only=0)
        assert tuple(acc.shape) == want.shape
        assert (host(acc).astype(np.int64) == want).all()
        assert (host(y) == y_want).all()
        assert (np.abs(host(y).astype(np.float64) - y64) <= 1e-6 * np.abs(y64)).all()
        if out_bits:
            codes = oracle.requant(y_want, out_bits)
            pw, bad = oracle.pack_planes(codes.reshape(-1, Cout), out_bits)
            assert bad == 0 and (planes_u32(planes) == pw).all()
    return want


CASES = [
    # the geometries of the networks the paper evaluates
    dict(Nb=2, H=20, W=22, C=3, Cout=64, ab=8, wb=2, KH=7, KW=7, stride=2, pad=3),          # ResNet stem
    dict(Nb=2, H=12, W=12, C=64, Cout=128, ab=2, wb=2, KH=3, KW=3, stride=2, pad=1),        # strided 3x3
    dict(Nb=2, H=9, W=9, C=256, Cout=64, ab=4, wb=3, KH=1, KW=1),                           # bottleneck 1x1
    dict(Nb=1, H=10, W=11, C=128, Cout=70, ab=4, wb=2, KH=1, KW=1, stride=2),               # strided 1x1 shortcut
    dict(Nb=2, H=28, W=28, C=1, Cout=20, ab=8, wb=4, KH=5, KW=5),                           # LeNet conv1
    dict(Nb=2, H=12, W=12, C=20, Cout=50, ab=4, wb=4, KH=5, KW=5),                          # LeNet conv2
    dict(Nb=1, H=13, W=13, C=96, Cout=33, ab=3, wb=3, KH=3, KW=3, pad=2, dilation=2),       # atrous conv
    dict(Nb=1, H=17, W=15, C=40, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=4, dilation=4),
    # atrous 3x3 on the 3x3 kernel (one tap per stage: 128 channels and more): interior run and border
    # pixels, images narrower than two dilations, images of fewer rows than the dilation, several
    # wavefronts per image, the channel-split shapes (256 and 512 channels), emitted planes
    dict(Nb=2, H=9, W=11, C=128, Cout=70, ab=2, wb=2, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=2, H=7, W=7, C=256, Cout=64, ab=4, wb=3, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=1, H=5, W=9, C=512, Cout=64, ab=4, wb=2, KH=3, KW=3, pad=4, dilation=4, out_bits=4),
    dict(Nb=2, H=6, W=5, C=128, Cout=64, ab=4, wb=2, KH=3, KW=3, pad=3, dilation=3),
    dict(Nb=3, H=2, W=6, C=256, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=2, H=19, W=17, C=128, Cout=130, ab=3, wb=3, KH=3, KW=3, pad=2, dilation=2, out_bits=3),
    dict(Nb=1, H=3, W=3, C=128, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=1, H=12, W=12, C=192, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=2, dilation=2),
    # other odd windows with "same" padding on the 3x3 kernel: 5x5 (three tap chunks, the last of seven
    # taps), 7x7, 1x3 and 3x1, 5x5 with dilation, 5x3; images smaller than the window; split shapes
    dict(Nb=2, H=9, W=10, C=128, Cout=70, ab=2, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=1, H=8, W=8, C=256, Cout=64, ab=4, wb=2, KH=5, KW=5, pad=2, out_bits=4),
    dict(Nb=1, H=9, W=9, C=128, Cout=64, ab=2, wb=2, KH=7, KW=7, pad=3),
    dict(Nb=2, H=6, W=7, C=256, Cout=64, ab=4, wb=3, KH=1, KW=3, pad=(0, 1)),
    dict(Nb=2, H=6, W=7, C=512, Cout=64, ab=4, wb=2, KH=3, KW=1, pad=(1, 0)),
    dict(Nb=1, H=11, W=12, C=128, Cout=64, ab=3, wb=2, KH=5, KW=5, pad=4, dilation=2),
    dict(Nb=1, H=7, W=9, C=128, Cout=130, ab=2, wb=2, KH=5, KW=3, pad=(2, 1)),
    dict(Nb=2, H=3, W=2, C=128, Cout=64, ab=2, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=3, H=17, W=19, C=128, Cout=64, ab=4, wb=2, KH=5, KW=5, pad=2),
    # ... and on the shapes whose 3x3 kernel holds several taps or pixels per stage (an instantiation of its
    # own for other windows): 128 channels at one and two bits, 256 channels with one-bit weights, 64 channels
    dict(Nb=1, H=10, W=9, C=128, Cout=64, ab=1, wb=1, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=2, H=8, W=9, C=128, Cout=70, ab=2, wb=1, KH=5, KW=5, pad=2, out_bits=2),
    dict(Nb=1, H=9, W=8, C=256, Cout=64, ab=4, wb=1, KH=5, KW=5, pad=2),
    dict(Nb=1, H=7, W=10, C=256, Cout=64, ab=3, wb=1, KH=7, KW=3, pad=(3, 1)),
    dict(Nb=2, H=9, W=10, C=64, Cout=70, ab=2, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=1, H=11, W=9, C=64, Cout=64, ab=4, wb=2, KH=5, KW=5, pad=2, out_bits=2),
    dict(Nb=1, H=8, W=9, C=64, Cout=64, ab=1, wb=1, KH=7, KW=7, pad=3),
    dict(Nb=2, H=7, W=8, C=64, Cout=130, ab=3, wb=4, KH=3, KW=3, pad=3, dilation=3),
    dict(Nb=1, H=6, W=12, C=64, Cout=64, ab=4, wb=4, KH=1, KW=5, pad=(0, 2)),
    dict(Nb=1, H=9, W=14, C=64, Cout=64, ab=2, wb=1, KH=3, KW=1, stride=(1, 2), pad=(1, 0)),
    dict(Nb=2, H=8, W=10, C=100, Cout=130, ab=1, wb=1, KH=2, KW=4, stride=(2, 1), pad=(0, 2), dilation=(1, 2)),
    dict(Nb=1, H=6, W=6, C=64, Cout=64, ab=6, wb=2, KH=3, KW=3, pad=1),                     # wide activations
    dict(Nb=1, H=7, W=7, C=512, Cout=64, ab=4, wb=2, KH=3, KW=3, stride=2, pad=1),          # many channel chunks
    dict(Nb=3, H=16, W=16, C=64, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=1),                   # several wavefronts per image
    # channel counts whose word count is a multiple of 3 (chunks of three words) or odd (one word)
    dict(Nb=2, H=9, W=10, C=96, Cout=64, ab=2, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=1, H=8, W=8, C=192, Cout=70, ab=2, wb=3, KH=3, KW=3, stride=2, pad=1),
    dict(Nb=1, H=7, W=9, C=288, Cout=64, ab=1, wb=1, KH=3, KW=3, pad=1, dilation=1),
    dict(Nb=1, H=7, W=7, C=160, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=1),                    # five words
    dict(Nb=1, H=6, W=6, C=90, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=1, transposed=True, stride=2, output_padding=1),
    # single tap: the GEMM kernels, with strided row selection when there is a stride
    dict(Nb=3, H=7, W=7, C=256, Cout=64, ab=2, wb=2, KH=1, KW=1, stride=2),                 # Ho*stride > H
    dict(Nb=2, H=9, W=8, C=96, Cout=130, ab=1, wb=1, KH=1, KW=1, stride=(2, 3)),
    dict(Nb=2, H=6, W=7, C=1100, Cout=64, ab=2, wb=2, KH=1, KW=1, stride=(3, 2)),           # two chunks, the second ragged
    dict(Nb=5, H=5, W=5, C=40, Cout=64, ab=4, wb=4, KH=1, KW=1, stride=(1, 2), dilation=3),
    dict(Nb=2, H=8, W=8, C=64, Cout=64, ab=6, wb=2, KH=1, KW=1, stride=2),                  # wide activations: general kernel
    dict(Nb=2, H=8, W=8, C=64, Cout=64, ab=2, wb=2, KH=1, KW=1, stride=2, pad=1),           # padded: general kernel
    # transposed
    dict(Nb=2, H=7, W=7, C=64, Cout=32, ab=2, wb=2, KH=2, KW=2, stride=2, transposed=True),
    dict(Nb=1, H=6, W=8, C=128, Cout=64, ab=4, wb=2, KH=4, KW=4, stride=2, pad=1, transposed=True),
    dict(Nb=1, H=5, W=5, C=40, Cout=21, ab=4, wb=4, KH=3, KW=3, stride=2, pad=1, transposed=True, output_padding=1),
    dict(Nb=1, H=6, W=5, C=32, Cout=64, ab=2, wb=2, KH=3, KW=2, stride=(2, 3), pad=(1, 0), dilation=(1, 2),
         transposed=True, output_padding=(1, 2)),
    dict(Nb=1, H=6, W=6, C=64, Cout=64, ab=2, wb=2, KH=3, KW=3, stride=1, pad=1, transposed=True),
    # output phases without any tap (kernel smaller than the stride): their pixels are zero sums
    dict(Nb=2, H=5, W=6, C=64, Cout=32, ab=2, wb=2, KH=1, KW=1, stride=2, transposed=True, output_padding=1),
    dict(Nb=1, H=4, W=5, C=33, Cout=70, ab=3, wb=2, KH=2, KW=2, stride=3, pad=1, transposed=True),
    # dilation above the stride; a phase with more taps than one chunk holds; wavefronts that start inside a row
    dict(Nb=1, H=6, W=7, C=64, Cout=64, ab=2, wb=2, KH=3, KW=3, stride=2, pad=2, dilation=3, transposed=True),
    dict(Nb=1, H=6, W=6, C=96, Cout=64, ab=2, wb=2, KH=5, KW=5, stride=2, pad=2, transposed=True, output_padding=1),
    dict(Nb=3, H=14, W=13, C=64, Cout=130, ab=2, wb=2, KH=4, KW=4, stride=2, pad=1, transposed=True),
    dict(Nb=2, H=9, W=9, C=128, Cout=64, ab=1, wb=1, KH=3, KW=3, stride=(1, 2), pad=(1, 0), transposed=True),
    # phases of at most four taps, one or two activation bits: the four-tap chunk (4 and 8 channel words)
    dict(Nb=2, H=7, W=9, C=128, Cout=70, ab=2, wb=3, KH=4, KW=4, stride=2, pad=1, transposed=True),
    dict(Nb=1, H=6, W=5, C=256, Cout=64, ab=1, wb=2, KH=3, KW=3, stride=2, pad=1, transposed=True, output_padding=1),
    dict(Nb=1, H=5, W=7, C=512, Cout=33, ab=2, wb=1, KH=4, KW=4, stride=2, pad=1, transposed=True),
    dict(Nb=1, H=6, W=6, C=256, Cout=64, ab=2, wb=2, KH=4, KW=4, stride=2, pad=0, transposed=True),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join("%s%s" % (k, v) for k, v in c.items() if k in
                                                               ("H", "C", "Cout", "ab", "wb", "KH", "stride", "transposed")))
def test_conv2d_general(q, oracle, case):
    say("conv2d_general", case)
    run_case(q, oracle, **case)


WINDOW_CASES = [
    # few input channels: the packed-window path (and, without workspace, the general kernel)
    dict(Nb=2, H=20, W=22, C=3, Cout=64, ab=8, wb=2, KH=7, KW=7, stride=2, pad=3),          # 147 bits, 5 words
    dict(Nb=2, H=11, W=9, C=3, Cout=20, ab=8, wb=2, KH=3, KW=3, stride=2, pad=1),           # 27 bits, 1 word
    dict(Nb=1, H=12, W=12, C=6, Cout=70, ab=4, wb=4, KH=5, KW=5, pad=2),                    # 150 bits, 5 words
    dict(Nb=1, H=9, W=10, C=10, Cout=33, ab=2, wb=3, KH=3, KW=3, pad=2, dilation=2),        # 90 bits, 3 words
    dict(Nb=2, H=6, W=6, C=32, Cout=64, ab=2, wb=2, KH=2, KW=2),                            # 128 bits, whole words per tap
    dict(Nb=1, H=8, W=7, C=32, Cout=16, ab=3, wb=1, KH=4, KW=2, pad=1),                     # 256 bits, 8 words
    dict(Nb=1, H=8, W=8, C=7, Cout=130, ab=5, wb=2, KH=3, KW=3, stride=(2, 1), pad=1),      # 63 bits, 2 words
    dict(Nb=3, H=28, W=28, C=1, Cout=20, ab=8, wb=4, KH=5, KW=5),                           # LeNet conv1, 25 bits
    dict(Nb=1, H=5, W=5, C=11, Cout=8, ab=1, wb=1, KH=1, KW=3, pad=(0, 1)),                 # 33 bits: one bit in word 1
    dict(Nb=2, H=20, W=22, C=3, Cout=64, ab=8, wb=8, KH=7, KW=7, stride=2, pad=3),          # 8-bit stem (Table 4's first layer)
    dict(Nb=1, H=9, W=9, C=3, Cout=70, ab=4, wb=6, KH=3, KW=3, pad=1),                      # wide weights, one word
]


@pytest.mark.parametrize("case", WINDOW_CASES, ids=lambda c: "C%d-k%dx%d-ab%d-wb%d" % (c["C"], c["KH"], c["KW"],
                                                                                        c["ab"], c["wb"]))
@pytest.mark.parametrize("workspace", [True, False])
def test_conv2d_few_channels(q, oracle, case, workspace):
    say("conv2d few channels", case, "workspace", workspace)
    run_case(q, oracle, workspace=workspace, **case)
    run_case(q, oracle, workspace=workspace, out_bits=4, seed=5, **case)


# 3x3 at stride 2 with padding 1 on the 3x3 kernel's strided variant: even and odd image sizes (an
# odd width puts the last column's right-hand tap outside), one-pixel images, several images,
# channel counts with one and with several chunk passes, pixel groups of two (W2A2, 64 channels)
STRIDE2_CASES = [(1, 1, 1, 64, 64, 2, 2), (1, 2, 2, 64, 64, 2, 2), (2, 3, 3, 64, 70, 2, 2), (3, 8, 8, 64, 64, 2, 2),
                 (2, 9, 7, 64, 64, 2, 2), (2, 7, 10, 64, 130, 2, 2), (1, 56, 56, 64, 128, 4, 3),
                 (2, 13, 14, 128, 64, 2, 2), (1, 14, 13, 256, 70, 4, 2), (2, 7, 7, 512, 64, 4, 2),
                 (1, 5, 6, 32, 33, 1, 1), (1, 28, 28, 128, 256, 4, 2), (2, 11, 11, 256, 64, 3, 4)]


@pytest.mark.parametrize("case", STRIDE2_CASES, ids=lambda c: "s2-%dx%dx%d-C%d-N%d-a%dw%d" % c)
def test_conv3x3_stride2(q, oracle, case):
    Nb, H, W, C, Cout, ab, wb = case
    say("conv 3x3 stride 2", case)
    run_case(q, oracle, Nb=Nb, H=H, W=W, C=C, Cout=Cout, ab=ab, wb=wb, KH=3, KW=3, stride=2, pad=1)
    run_case(q, oracle, Nb=Nb, H=H, W=W, C=C, Cout=Cout, ab=ab, wb=wb, KH=3, KW=3, stride=2, pad=1, out_bits=4, seed=3)


@pytest.mark.parametrize("rpw", [1, 2, 3, 5, 1000])
def test_conv3x3_stride2_any_rows_per_wave(q, oracle, rpw):
    q.tune(rows_per_wave=rpw)
    try:
        run_case(q, oracle, Nb=2, H=9, W=11, C=64, Cout=64, ab=2, wb=2, KH=3, KW=3, stride=2, pad=1)
        run_case(q, oracle, Nb=2, H=10, W=8, C=256, Cout=70, ab=4, wb=2, KH=3, KW=3, stride=2, pad=1)
    finally:
        q.tune(rows_per_wave=0)


def test_conv3x3_stride2_split_channels(q, oracle):
    """Stride 2 together with the channel-splitting variant, forced on (and an emitted result)."""
    q.tune(split_channels=2)
    try:
        run_case(q, oracle, Nb=2, H=14, W=14, C=256, Cout=70, ab=4, wb=2, KH=3, KW=3, stride=2, pad=1)
        run_case(q, oracle, Nb=1, H=9, W=11, C=512, Cout=64, ab=4, wb=2, KH=3, KW=3, stride=2, pad=1, out_bits=4, seed=2)
        run_case(q, oracle, Nb=2, H=7, W=7, C=512, Cout=128, ab=4, wb=2, KH=3, KW=3, stride=1, pad=1, out_bits=4, seed=4)
    finally:
        q.tune(split_channels=0)


# the layers bench.py times (`--workload conv_geometries`), at their full sizes and in the launch
# configuration the library picks for them; the oracle computes the whole layer
FULL_SIZE_CASES = [
    dict(Nb=32, H=224, W=224, C=3, Cout=64, ab=8, wb=2, KH=7, KW=7, stride=2, pad=3),
    dict(Nb=32, H=224, W=224, C=3, Cout=64, ab=8, wb=2, KH=7, KW=7, stride=2, pad=3, dense_rows=True),
    dict(Nb=32, H=56, W=56, C=128, Cout=128, ab=2, wb=2, KH=3, KW=3, stride=2, pad=1),
    dict(Nb=32, H=56, W=56, C=256, Cout=512, ab=2, wb=2, KH=1, KW=1, stride=2),
    dict(Nb=32, H=56, W=56, C=256, Cout=64, ab=2, wb=2, KH=1, KW=1),
    dict(Nb=32, H=56, W=56, C=64, Cout=64, ab=2, wb=2, KH=3, KW=3, pad=1),
    dict(Nb=16, H=33, W=33, C=256, Cout=256, ab=4, wb=3, KH=3, KW=3, pad=2, dilation=2),
    dict(Nb=16, H=17, W=17, C=512, Cout=512, ab=4, wb=2, KH=3, KW=3, pad=4, dilation=4),
    dict(Nb=32, H=28, W=28, C=128, Cout=128, ab=4, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=16, H=56, W=56, C=64, Cout=64, ab=4, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=32, H=28, W=28, C=96, Cout=96, ab=2, wb=2, KH=5, KW=5, pad=2),
    dict(Nb=16, H=28, W=28, C=256, Cout=128, ab=2, wb=2, KH=4, KW=4, stride=2, pad=1, transposed=True),
]


@pytest.mark.parametrize("case", FULL_SIZE_CASES, ids=lambda c: "full-%dx%d-C%d-k%d-s%s%s%s" % (
    c["H"], c["W"], c["C"], c["KH"], c.get("stride", 1), "-T" if c.get("transposed") else "",
    "-dense" if c.get("dense_rows") else ""))
def test_conv2d_general_full_size(q, oracle, case):
    say("conv2d_general full size", case)
    run_case(q, oracle, **case)


@pytest.mark.parametrize("case", WINDOW_CASES + [
    dict(Nb=2, H=9, W=13, C=3, Cout=64, ab=8, wb=2, KH=7, KW=7, stride=2, pad=3, dilation=(1, 2)),   # dilated along w: tap by tap
    dict(Nb=1, H=5, W=40, C=5, Cout=33, ab=2, wb=2, KH=2, KW=9, pad=(0, 4)),                          # 45 bits per kernel row: two groups
    dict(Nb=2, H=4, W=3, C=32, Cout=64, ab=1, wb=1, KH=2, KW=3, pad=1),                                # whole words per tap
], ids=lambda c: "dense-C%d-k%dx%d-ab%d-wb%d" % (c["C"], c["KH"], c["KW"], c["ab"], c["wb"]))
def test_conv2d_few_channels_dense_rows(q, oracle, case):
    """The packed-window path fed from row-dense planes (one packed row per image row)."""
    say("conv2d few channels, dense rows", case)
    run_case(q, oracle, dense_rows=True, **case)
    run_case(q, oracle, dense_rows=True, out_bits=4, seed=7, **case)


def test_conv2d_dense_rows_rejected_elsewhere(q):
    """Row-dense input is refused where the packed-window path does not apply, or without its workspace."""
    import torch
    x = torch.zeros(4096, dtype=torch.int32, device="cuda")
    w = torch.zeros(4096, dtype=torch.int32, device="cuda")
    for kwargs, C, workspace in ((dict(kh=3, kw=3, pad=1), 64, True), (dict(kh=1, kw=1), 3, True),
                                 (dict(kh=3, kw=3, pad=1, transposed=True), 3, True), (dict(kh=3, kw=3, pad=1), 3, False)):
        geo = q.conv_geometry(kwargs.pop("kh"), kwargs.pop("kw"), dense_rows=True, **kwargs)
        with pytest.raises(q.QnnError):
            q.conv2d_general(x, 2, w, 2, 1, 4, 4, C, 8, geo, workspace=workspace)


@pytest.mark.parametrize("out_bits", [1, 2, 4, 8])
def test_conv2d_general_requant(q, oracle, out_bits):
    say("conv2d_general requant", out_bits)
    run_case(q, oracle, Nb=2, H=12, W=12, C=64, Cout=70, ab=4, wb=2, KH=3, KW=3, stride=2, pad=1, out_bits=out_bits)
    run_case(q, oracle, Nb=1, H=6, W=6, C=256, Cout=64, ab=2, wb=2, KH=2, KW=2, stride=2, transposed=True,
             out_bits=out_bits)
    run_case(q, oracle, Nb=2, H=9, W=9, C=128, Cout=70, ab=2, wb=2, KH=1, KW=1, stride=2, out_bits=out_bits)
    run_case(q, oracle, Nb=2, H=5, W=6, C=128, Cout=64, ab=4, wb=2, KH=1, KW=1, out_bits=out_bits)


def test_conv2d_general_planes_only(q, oracle):
    """No int32 / fp32 result requested: the partial sums live in the workspace."""
    rng = np.random.default_rng(9)
    Nb, H, W, C, Cout, ab, wb, ob = 2, 10, 10, 128, 96, 4, 2, 4
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
    want = oracle.conv2d(X, Wt, stride=2, pad=1)
    s = (rng.uniform(0.5, 1.5, Cout) * 16.0 / (np.sqrt(np.mean(want.astype(np.float64) ** 2)) + 1)).astype(np.float32)
    codes = oracle.requant(oracle.scale_f32(want, s), ob)
    pw, _ = oracle.pack_planes(codes.reshape(-1, Cout), ob)
    geo = q.conv_geometry(3, 3, stride=2, pad=1)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    import torch
    Ho, Wo = q.conv2d_general_output_size(H, W, geo)
    planes = torch.empty((Nb * Ho * Wo, ob, (Cout + 31) // 32), dtype=torch.int32, device="cuda")
    ws = torch.empty(Nb * Ho * Wo * Cout * 4, dtype=torch.uint8, device="cuda")
    import ctypes
    st = q.lib().qnn_conv2d_general(ctypes.c_void_p(Xp.data_ptr()), ab, ctypes.c_void_p(Wp.data_ptr()), wb, Nb, H, W,
                                    C, Cout, ctypes.byref(geo), None, ctypes.c_void_p(dev(s).data_ptr()), None, ob,
                                    ctypes.c_void_p(planes.data_ptr()), ctypes.c_void_p(ws.data_ptr()), ws.numel(),
                                    None)
    assert st == 0
    torch.cuda.synchronize()
    assert (planes_u32(planes) == pw).all()


@pytest.mark.parametrize("stride,C", [(1, 1100), (2, 1100), (2, 256), (3, 40)])
def test_conv2d_single_tap_planes_only(q, oracle, stride, C):
    """1x1 convolutions (the GEMM kernels, with the row walker when strided) with only the next
    layer's planes requested; the workspace is sized by qnn_conv2d_general_workspace_bytes."""
    say("single tap planes only", stride, C)
    import ctypes
    import torch
    rng = np.random.default_rng(stride * 1000 + C)
    Nb, H, W, Cout, ab, wb, ob = 2, 9, 7, 70, 2, 2, 4
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 1, 1, C), wb)
    want = oracle.conv2d(X, Wt, stride=stride)
    s = (rng.uniform(0.5, 1.5, Cout) * 16.0 / (np.sqrt(np.mean(want.astype(np.float64) ** 2)) + 1)).astype(np.float32)
    codes = oracle.requant(oracle.scale_f32(want, s), ob)
    pw, _ = oracle.pack_planes(codes.reshape(-1, Cout), ob)
    geo = q.conv_geometry(1, 1, stride=stride)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout, C)), wb)
    Ho, Wo = q.conv2d_general_output_size(H, W, geo)
    planes = torch.empty((Nb * Ho * Wo, ob, (Cout + 31) // 32), dtype=torch.int32, device="cuda")
    need = int(q.lib().qnn_conv2d_general_workspace_bytes(Nb, H, W, C, Cout, ab, wb, ctypes.byref(geo)))
    ws = torch.empty(max(16, need), dtype=torch.uint8, device="cuda")
    sd = dev(s)
    st = q.lib().qnn_conv2d_general(ctypes.c_void_p(Xp.data_ptr()), ab, ctypes.c_void_p(Wp.data_ptr()), wb, Nb, H, W,
                                    C, Cout, ctypes.byref(geo), None, ctypes.c_void_p(sd.data_ptr()), None, ob,
                                    ctypes.c_void_p(planes.data_ptr()), ctypes.c_void_p(ws.data_ptr()), need, None)
    assert st == 0
    torch.cuda.synchronize()
    assert (planes_u32(planes) == pw).all()


def test_general_equals_the_3x3_kernels(q, oracle):
    """Same product through the dedicated 3x3 kernels and through the general one."""
    rng = np.random.default_rng(21)
    Nb, H, W, C, Cout, ab, wb = 2, 14, 14, 64, 64, 2, 2
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
    Xp = q.encode_pack(dev(X.reshape(Nb * H * W, C)), ab)
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    a1, _ = q.conv2d_packed(Xp, ab, Wp, wb, Nb, H, W, C, Cout)
    a2, _, _ = q.conv2d_general(Xp, ab, Wp, wb, Nb, H, W, C, Cout, q.conv_geometry(3, 3, pad=1))
    assert (host(a1) == host(a2)).all() and (host(a1).astype(np.int64) == oracle.conv3x3(X, Wt)).all()


def random_case(rng):
    """A small random layer: any geometry the entry point accepts, sizes that keep the oracle quick."""
    transposed = bool(rng.integers(0, 3) == 0)
    KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    dilation = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    pad = (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
    H, W = int(rng.integers(1, 12)), int(rng.integers(1, 12))
    C = int(rng.choice([1, 3, 8, 31, 32, 33, 64, 96, 100, 128, 160, 192, 300]))
    Cout = int(rng.choice([1, 5, 32, 63, 64, 65, 100, 130]))
    ab, wb = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    case = dict(Nb=int(rng.integers(1, 4)), H=H, W=W, C=C, Cout=Cout, ab=ab, wb=wb, KH=KH, KW=KW, stride=stride,
                pad=pad, dilation=dilation, transposed=transposed)
    if transposed:
        case["output_padding"] = (int(rng.integers(0, max(stride[0], dilation[0]))),
                                  int(rng.integers(0, max(stride[1], dilation[1]))))
    return case


@pytest.mark.parametrize("idx", [0, 1, 6, 13])
def test_conv2d_general_plain_block_order(q, oracle, idx):
    """These kernels number their blocks per XCD unless told otherwise; the plain numbering gives the same."""
    say("plain block order", CASES[idx])
    q.tune(block_order=1)
    try:
        run_case(q, oracle, **CASES[idx])
    finally:
        q.tune(block_order=0)


def test_conv2d_general_random_geometries(q, oracle):
    """Seeded random geometries, channel counts and bit widths, with and without re-encoding."""
    rng = np.random.default_rng(20240607)
    done = 0
    for i in range(400):
        case = random_case(rng)
        sh, sw = case["stride"]
        dh, dw = case["dilation"]
        ph, pw = case["pad"]
        if case["transposed"]:
            oph, opw = case["output_padding"]
            Ho = (case["H"] - 1) * sh - 2 * ph + dh * (case["KH"] - 1) + oph + 1
            Wo = (case["W"] - 1) * sw - 2 * pw + dw * (case["KW"] - 1) + opw + 1
        else:
            Ho = (case["H"] + 2 * ph - dh * (case["KH"] - 1) - 1) // sh + 1
            Wo = (case["W"] + 2 * pw - dw * (case["KW"] - 1) - 1) // sw + 1
        if Ho < 1 or Wo < 1 or case["KH"] * case["KW"] * case["C"] * 255 * 255 >= 2 ** 31:
            continue
        out_bits = int(rng.choice([0, 0, 1, 3, 4, 8]))
        say("random geometry", i, case, "out_bits", out_bits)
        run_case(q, oracle, out_bits=out_bits, seed=i, workspace=bool(rng.integers(0, 2)), **case)
        done += 1
    assert done >= 200
