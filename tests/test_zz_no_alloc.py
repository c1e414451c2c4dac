"""qnn_conv2d_im2col_static (the entry point for callers that cannot allocate): same results as
qnn_conv2d_im2col, bit for bit, on two calls in a row that share the library's static scratch, the
second one smaller than the first.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from gpu_util import dev, host, rand_codes, say

pytestmark = pytest.mark.gpu


def _layer(rng, Nb, H, W, C, Cout, ab, wb):
    X = rand_codes(rng, (Nb, H, W, C), ab)
    Wt = rand_codes(rng, (Cout, 3, 3, C), wb)
    s = (0.01 + 0.09 * rng.random(Cout)).astype(np.float32)
    return X, Wt, s


def _both(q, X, Wt, s, ab, wb):
    Cout, C = Wt.shape[0], Wt.shape[3]
    Wp = q.encode_pack(dev(Wt.reshape(Cout * 9, C)), wb)
    xd, sd = dev(X), dev(s)
    want_acc, want_out = q.conv2d_im2col(xd, ab, Wp, wb, Cout, scale=sd)
    # outputs allocated here, poisoned, then handed to the call: it allocates nothing itself
    acc = torch.full(tuple(X.shape[:3]) + (Cout,), -7, dtype=torch.int32, device="cuda")
    out = torch.full(tuple(X.shape[:3]) + (Cout,), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    q.conv2d_im2col_static(xd, ab, Wp, wb, Cout, scale=sd, out=(acc, out))
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    return host(want_acc), host(want_out), host(acc), host(out)


def test_static_scratch_two_calls_second_smaller(oracle):
    from paper_2106_09886_amd import binding as q
    rng = np.random.default_rng(77)
    # first call: 64 channels (two words per plane), several wavefronts, ragged filter tile;
    # second call: fewer and smaller images and another bit width, so it reuses only the front of
    # the scratch the first call filled
    cases = [(3, 20, 28, 64, 72, 2, 2), (1, 9, 11, 40, 24, 4, 3), (2, 12, 12, 3, 16, 8, 2)]
    for (Nb, H, W, C, Cout, ab, wb) in cases:
        say("static scratch: Nb=%d H=%d W=%d C=%d Cout=%d A%dW%d" % (Nb, H, W, C, Cout, ab, wb))
        X, Wt, s = _layer(rng, Nb, H, W, C, Cout, ab, wb)
        want_acc, want_out, acc, out = _both(q, X, Wt, s, ab, wb)
        assert (acc == want_acc).all()
        assert (out.view(np.uint32) == want_out.view(np.uint32)).all()
        assert (acc.astype(np.int64) == oracle.conv3x3(X, Wt)).all()


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2106_09886_amd import binding as q
    L = q.lib()
    P = 1 << 20
    limit = q.QNN_STATIC_SCRATCH_BYTES
    # 2 bits x 2 words x 4 bytes per pixel: one pixel more than fits
    pixels = limit // 16 + 1
    assert L.qnn_conv2d_im2col_static(P, 1, 2, P, 2, 1, 1, pixels, 64, 64, P, None, None, None) == q.QNN_EUNSUPPORTED
