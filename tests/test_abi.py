"""The C-ABI library loads, exports every symbol include/qnn.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed, no compute call made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2106_09886_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qnn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    from paper_2106_09886_amd import binding
    names = declared_functions()
    assert {"qnn_encode_pack", "qnn_branch_gemm", "qnn_conv2d_im2col", "qnn_scale_epilogue"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(binding.EXPORTS)


def test_status_strings(L):
    seen = set()
    for st in range(6):
        s = L.qnn_status_string(st)
        assert s and s not in seen
        seen.add(s)
    assert L.qnn_status_string(99) == b"unknown status"
    assert L.qnn_version() >= 100


P = 1 << 20          # a fake, 16-byte aligned, never dereferenced device address


def test_encode_pack_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EUNSUPPORTED
    f = L.qnn_encode_pack
    assert f(P, 1, 4, 64, 0, P, None, 0, None) == QNN_EINVAL          # bits
    assert f(P, 1, 4, 64, 9, P, None, 0, None) == QNN_EINVAL
    assert f(P, 3, 4, 64, 2, P, None, 0, None) == QNN_EINVAL          # code size
    assert f(P, 1, 4, 64, 8, P, None, 0, None) == QNN_EINVAL          # 8 bits need int16
    assert f(P, 1, -1, 64, 2, P, None, 0, None) == QNN_EINVAL
    assert f(P, 1, 4, -5, 2, P, None, 0, None) == QNN_EINVAL
    assert f(P, 1, 4, 64, 2, P, None, 2, None) == QNN_EINVAL          # unknown flag
    assert f(None, 1, 4, 64, 2, P, None, 0, None) == QNN_EINVAL
    assert f(P, 1, 4, 64, 2, None, None, 0, None) == QNN_EINVAL
    assert f(P, 1, 4, 64, 2, P + 4, None, 0, None) == QNN_EALIGN
    assert f(P + 1, 2, 4, 64, 2, P, None, 0, None) == QNN_EALIGN
    assert f(P, 1, 4, 1 << 31, 2, P, None, 0, None) == QNN_EUNSUPPORTED
    assert f(None, 1, 0, 64, 2, None, None, 0, None) == QNN_OK          # empty: nothing launched
    assert f(None, 1, 4, 0, 2, None, None, 0, None) == QNN_OK


def test_branch_gemm_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EUNSUPPORTED
    f = L.qnn_branch_gemm
    assert f(P, 0, P, 2, 4, 4, 64, P, None, None, None) == QNN_EINVAL
    assert f(P, 2, P, 9, 4, 4, 64, P, None, None, None) == QNN_EINVAL
    assert f(P, 2, P, 2, -1, 4, 64, P, None, None, None) == QNN_EINVAL
    assert f(P, 2, P, 2, 4, 4, 64, None, None, None, None) == QNN_EINVAL    # no output at all
    assert f(P, 2, P, 2, 4, 4, 64, P, P, None, None) == QNN_EINVAL          # scale without out
    assert f(P, 2, P, 2, 4, 4, 64, P, None, P, None) == QNN_EINVAL          # out without scale
    assert f(None, 2, P, 2, 4, 4, 64, P, None, None, None) == QNN_EINVAL
    assert f(P + 8, 2, P, 2, 4, 4, 64, P, None, None, None) == QNN_EALIGN
    assert f(P, 2, P + 4, 2, 4, 4, 64, P, None, None, None) == QNN_EALIGN
    assert f(P, 2, P, 2, 4, 4, 64, P + 2, None, None, None) == QNN_EALIGN
    # K (2^8-1)^2 >= 2^31: the int32 result could overflow
    assert f(P, 8, P, 8, 4, 4, 40000, P, None, None, None) == QNN_EUNSUPPORTED
    assert f(P, 2, P, 2, 1 << 31, 4, 64, P, None, None, None) == QNN_EUNSUPPORTED
    assert f(P, 2, P, 2, 0, 4, 64, P, None, None, None) == QNN_OK            # empty
    assert f(P, 2, P, 2, 4, 0, 64, P, None, None, None) == QNN_OK


def test_conv_argument_errors(L):
    from paper_2106_09886_amd.binding import (QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EUNSUPPORTED,
                                              QNN_EWORKSPACE)
    f = L.qnn_conv2d_im2col
    need = L.qnn_conv2d_im2col_workspace_bytes(2, 8, 8, 64, 2)
    assert need == 2 * 8 * 8 * 2 * 2 * 4
    assert L.qnn_conv2d_im2col_workspace_bytes(2, 8, 8, 33, 4) == 2 * 8 * 8 * 4 * 2 * 4
    assert L.qnn_conv2d_im2col_workspace_bytes(0, 8, 8, 64, 2) == 0
    ok = dict(x=P, cb=1, ab=2, wt=P, wb=2, nb=2, h=8, w=8, c=64, co=64, acc=P, sc=None, out=None,
              ws=P, wsb=need)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return f(a["x"], a["cb"], a["ab"], a["wt"], a["wb"], a["nb"], a["h"], a["w"], a["c"], a["co"],
                 a["acc"], a["sc"], a["out"], a["ws"], a["wsb"], None)

    assert call(ab=0) == QNN_EINVAL
    assert call(wb=9) == QNN_EINVAL
    assert call(cb=4) == QNN_EINVAL
    assert call(ab=8, cb=1) == QNN_EINVAL
    assert call(nb=-1) == QNN_EINVAL
    assert call(x=None) == QNN_EINVAL
    assert call(ws=None) == QNN_EINVAL
    assert call(acc=None) == QNN_EINVAL
    assert call(wt=None) == QNN_EINVAL
    assert call(ws=P + 4) == QNN_EALIGN
    assert call(wt=P + 8) == QNN_EALIGN
    assert call(wsb=need - 1) == QNN_EWORKSPACE
    assert call(nb=1 << 20, h=1 << 10, w=1 << 10) == QNN_EUNSUPPORTED
    assert call(ab=8, cb=2, wb=8, c=1 << 16) == QNN_EUNSUPPORTED
    assert call(nb=0) == QNN_OK
    assert call(co=0) == QNN_OK
    g = L.qnn_conv2d_packed
    assert g(P, 2, P, 2, 2, 8, 8, 64, 64, None, None, None, None) == QNN_EINVAL
    assert g(P + 4, 2, P, 2, 2, 8, 8, 64, 64, P, None, None, None) == QNN_EALIGN
    assert g(P, 2, P, 2, 0, 8, 8, 64, 64, P, None, None, None) == QNN_OK


def test_scale_epilogue_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK
    f = L.qnn_scale_epilogue
    assert f(None, 4, 4, P, P, None) == QNN_EINVAL
    assert f(P, 4, 4, None, P, None) == QNN_EINVAL
    assert f(P, 4, 4, P, None, None) == QNN_EINVAL
    assert f(P, -4, 4, P, P, None) == QNN_EINVAL
    assert f(P + 1, 4, 4, P, P, None) == QNN_EALIGN
    assert f(P, 0, 4, P, P, None) == QNN_OK
    assert f(P, 4, 0, P, P, None) == QNN_OK


def test_requant_variants_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EWORKSPACE, QNN_EUNSUPPORTED
    g = L.qnn_branch_gemm_requant
    #  A, ab, Wt, wb, M, N, K, scale, out_bits, out_planes, acc, out_f32, workspace, workspace_bytes, stream
    assert g(P, 2, P, 2, 4, 8, 64, None, 0, P, P, None, None, 0, None) == QNN_EINVAL       # out_bits
    assert g(P, 2, P, 2, 4, 8, 64, None, 9, P, P, None, None, 0, None) == QNN_EINVAL
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, None, P, None, None, 0, None) == QNN_EINVAL    # no planes
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, P + 4, P, None, None, 0, None) == QNN_EALIGN
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, P, None, P, None, 0, None) == QNN_EINVAL       # fp32 out needs a scale
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, P, None, None, None, 0, None) == QNN_EINVAL    # no result, no workspace
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, P, None, None, P, 4 * 8 * 4 - 1, None) == QNN_EWORKSPACE
    assert g(P, 2, P, 2, 4, 8, 64, None, 4, P, None, None, P + 8, 1 << 20, None) == QNN_EALIGN
    assert g(P, 2, P, 2, 0, 8, 64, None, 4, None, None, None, None, 0, None) == QNN_OK     # empty
    assert L.qnn_requant_workspace_bytes(4, 8) == 128 and L.qnn_requant_workspace_bytes(0, 8) == 0
    c = L.qnn_conv2d_packed_requant
    #  x, ab, Wt, wb, Nb, H, W, C, Cout, scale, out_bits, out_planes, acc, out_f32, ws, ws_bytes, stream
    assert c(P, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, None, None, None, 0, None) == QNN_EINVAL
    assert c(P, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, None, None, P, 16 * 64 * 4 - 1, None) == QNN_EWORKSPACE
    assert c(P, 2, P, 2, 1, 4, 4, 64, 64, None, 0, P, P, None, None, 0, None) == QNN_EINVAL
    assert c(P, 2, P, 2, 1, -4, 4, 64, 64, None, 4, P, P, None, None, 0, None) == QNN_EINVAL
    assert c(P, 2, P, 2, 1 << 20, 1 << 10, 1 << 10, 64, 64, None, 4, P, P, None, None, 0, None) == QNN_EUNSUPPORTED
    i = L.qnn_conv2d_im2col_requant
    need = L.qnn_conv2d_im2col_requant_workspace_bytes(1, 4, 4, 64, 2, 64)
    assert need == 16 * 2 * 2 * 4 + 16 * 64 * 4
    #  codes, code_bytes, ab, Wt, wb, Nb, H, W, C, Cout, scale, out_bits, planes, acc, out, ws, ws_bytes, stream
    assert i(P, 1, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, None, None, P, need - 1, None) == QNN_EWORKSPACE
    assert i(P, 1, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, None, None, None, 0, None) == QNN_EINVAL
    assert i(P, 3, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, P, None, P, need, None) == QNN_EINVAL
    assert i(P, 1, 2, P, 2, 1, 4, 4, 64, 64, None, 4, P, P, None, P, 16 * 2 * 2 * 4 - 1, None) == QNN_EWORKSPACE
    m = L.qnn_maxpool2x2_planes
    assert m(P, 1, 3, 4, 64, 4, P, None) == QNN_EINVAL              # odd height
    assert m(P, 1, 4, 4, 64, 0, P, None) == QNN_EINVAL
    assert m(None, 1, 4, 4, 64, 4, P, None) == QNN_EINVAL
    assert m(P, 1, 4, 4, 64, 4, P + 4, None) == QNN_EALIGN
    assert m(P, 0, 4, 4, 64, 4, None, None) == QNN_OK


def test_general_conv_geometry_and_argument_errors(L):
    import ctypes
    from paper_2106_09886_amd.binding import (QNN_EINVAL, QNN_OK, QNN_EUNSUPPORTED, QNN_EWORKSPACE, conv_geometry,
                                              conv2d_general_output_size, QnnError)
    assert conv2d_general_output_size(224, 224, conv_geometry(7, 7, stride=2, pad=3)) == (112, 112)
    assert conv2d_general_output_size(56, 56, conv_geometry(3, 3, stride=2, pad=1)) == (28, 28)
    assert conv2d_general_output_size(56, 57, conv_geometry(1, 1, stride=2)) == (28, 29)
    assert conv2d_general_output_size(33, 33, conv_geometry(3, 3, pad=4, dilation=4)) == (33, 33)
    assert conv2d_general_output_size(28, 28, conv_geometry(5, 5)) == (24, 24)
    assert conv2d_general_output_size(14, 14, conv_geometry(2, 2, stride=2, transposed=True)) == (28, 28)
    assert conv2d_general_output_size(14, 14, conv_geometry(3, 3, stride=2, pad=1, transposed=True,
                                                            output_padding=1)) == (28, 28)
    for bad in (conv_geometry(0, 3), conv_geometry(3, 3, stride=0), conv_geometry(3, 3, dilation=0),
                conv_geometry(3, 3, pad=-1), conv_geometry(3, 3, output_padding=1),
                conv_geometry(3, 3, stride=2, transposed=True, output_padding=2), conv_geometry(9, 9)):
        with pytest.raises(QnnError):
            conv2d_general_output_size(4, 4, bad)
    with pytest.raises(QnnError) as ei:
        conv2d_general_output_size(4, 4, conv_geometry(5000, 1, pad=3000))
    assert ei.value.status == QNN_EUNSUPPORTED
    stem = conv_geometry(7, 7, stride=2, pad=3)
    # the larger of the packed windows (7x7x3 = 147 bits = 5 words per plane, 8 planes + mask) and the partial sums
    assert L.qnn_conv2d_general_workspace_bytes(1, 224, 224, 3, 16, 8, 2, ctypes.byref(stem)) == 112 * 112 * 9 * 5 * 4
    assert L.qnn_conv2d_general_workspace_bytes(1, 224, 224, 3, 64, 8, 2, ctypes.byref(stem)) == 112 * 112 * 64 * 4
    assert L.qnn_conv2d_general_workspace_bytes(1, 224, 224, 64, 64, 2, 2, ctypes.byref(stem)) == 112 * 112 * 64 * 4
    assert L.qnn_conv2d_general_workspace_bytes(1, 224, 224, 3, 64, 9, 2, ctypes.byref(stem)) == 0
    f = L.qnn_conv2d_general
    g = conv_geometry(3, 3, stride=2, pad=1)
    gp = ctypes.byref(g)
    #  x, ab, Wt, wb, Nb, H, W, C, Cout, geo, acc, scale, out, out_bits, planes, ws, ws_bytes, stream
    assert f(P, 2, P, 2, 1, 8, 8, 64, 64, None, P, None, None, 0, None, None, 0, None) == QNN_EINVAL
    assert f(P, 2, P, 2, 1, 8, 8, 64, 64, gp, None, None, None, 0, None, None, 0, None) == QNN_EINVAL
    assert f(None, 2, P, 2, 1, 8, 8, 64, 64, gp, P, None, None, 0, None, None, 0, None) == QNN_EINVAL
    assert f(P, 2, P, 2, 1, 8, 8, 64, 64, gp, P, None, None, 9, P, None, 0, None) == QNN_EINVAL
    assert f(P, 2, P, 2, 1, 8, 8, 64, 64, gp, None, None, None, 4, P, P, 16 * 64 * 4 - 1, None) == QNN_EWORKSPACE
    assert f(P, 2, P, 2, 0, 8, 8, 64, 64, gp, None, None, None, 0, None, None, 0, None) == QNN_OK
    # row-dense input: a flag of 0 or 1, and only where the packed-window path applies, with its workspace
    bad = conv_geometry(3, 3, pad=1)
    bad.dense_rows = 2
    assert f(P, 2, P, 2, 1, 8, 8, 3, 64, ctypes.byref(bad), P, None, None, 0, None, None, 0, None) == QNN_EINVAL
    dense = conv_geometry(3, 3, pad=1, dense_rows=True)
    dp = ctypes.byref(dense)
    assert f(P, 2, P, 2, 1, 8, 8, 64, 64, dp, P, None, None, 0, None, P, 1 << 20, None) == QNN_EUNSUPPORTED   # 64 channels
    assert f(P, 2, P, 2, 1, 8, 8, 3, 64, dp, P, None, None, 0, None, None, 0, None) == QNN_EWORKSPACE
    one = conv_geometry(1, 1, dense_rows=True)
    assert f(P, 2, P, 2, 1, 8, 8, 3, 64, ctypes.byref(one), P, None, None, 0, None, P, 1 << 20, None) == QNN_EUNSUPPORTED


def test_encode_real_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK
    f = L.qnn_encode_real
    assert f(P, 4, 64, 0, 0, P, P, None) == QNN_EINVAL
    assert f(P, 4, 64, 2, 4, P, P, None) == QNN_EINVAL            # clip is one of the four range limiters
    assert f(P, 4, 64, 2, -1, P, P, None) == QNN_EINVAL
    assert f(P, -1, 64, 2, 0, P, P, None) == QNN_EINVAL
    assert f(None, 4, 64, 2, 0, P, P, None) == QNN_EINVAL
    assert f(P, 4, 64, 2, 0, None, None, None) == QNN_EINVAL
    assert f(P + 2, 4, 64, 2, 0, P, P, None) == QNN_EALIGN
    assert f(P, 4, 64, 2, 0, P, P + 4, None) == QNN_EALIGN
    assert f(P, 0, 64, 2, 0, None, None, None) == QNN_OK


def test_compare_dot4_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_EUNSUPPORTED, QNN_OK
    f = L.qnn_compare_dot4_gemm
    assert f(None, P, 4, 4, 8, P, None) == QNN_EINVAL
    assert f(P, P, 4, 4, 8, None, None) == QNN_EINVAL
    assert f(P, P, -1, 4, 8, P, None) == QNN_EINVAL
    assert f(P + 1, P, 4, 4, 8, P, None) == QNN_EALIGN
    assert f(P, P, 4, 4, 6, P, None) == QNN_EUNSUPPORTED          # K not a multiple of 4
    assert f(P, P, 4, 4, 1 << 20, P, None) == QNN_EUNSUPPORTED    # K * 127^2 overflows int32
    assert f(P, P, 0, 4, 8, P, None) == QNN_OK


def test_tune_rejects_unknown_keys(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_OK
    assert L.qnn_tune(1, 4) == QNN_OK and L.qnn_tune(1, 0) == QNN_OK
    assert L.qnn_tune(2, 0) == QNN_OK
    assert L.qnn_tune(3, 1) == QNN_OK and L.qnn_tune(3, 0) == QNN_OK
    assert L.qnn_tune(4, 2) == QNN_OK and L.qnn_tune(4, 1) == QNN_OK and L.qnn_tune(4, 0) == QNN_OK
    assert L.qnn_tune(4, 3) == QNN_EINVAL
    assert L.qnn_tune(5, 2) == QNN_OK and L.qnn_tune(5, 0) == QNN_OK and L.qnn_tune(5, 3) == QNN_EINVAL
    assert L.qnn_tune(99, 1) == QNN_EINVAL
    assert L.qnn_tune(1, -1) == QNN_EINVAL


def test_product_path_has_no_oracle_or_cpu_fallback():
    """Nothing under the package may import the oracle."""
    pkg = os.path.join(ROOT, "paper_2106_09886_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            src = open(os.path.join(pkg, fn)).read()
            assert "import oracle" not in src and "from oracle" not in src, fn


def test_static_scratch_entry_point_checks_on_the_host(L):
    """The entry point without a workspace validates like qnn_conv2d_im2col and refuses planes that
    do not fit its static scratch, all before any GPU call."""
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EUNSUPPORTED, QNN_STATIC_SCRATCH_BYTES
    f = L.qnn_conv2d_im2col_static
    text = open(os.path.join(ROOT, "include", "qnn.h")).read()
    m = re.search(r"#define\s+QNN_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert m and (int(m.group(1)) << int(m.group(2))) == QNN_STATIC_SCRATCH_BYTES
    fits = QNN_STATIC_SCRATCH_BYTES // 16                      # W2A2, 64 channels: 16 bytes of planes per pixel
    assert f(P, 1, 2, P, 2, 1, 1, fits + 1, 64, 64, P, None, None, None) == QNN_EUNSUPPORTED
    assert f(P, 1, 0, P, 2, 1, 4, 4, 64, 64, P, None, None, None) == QNN_EINVAL          # bits
    assert f(P, 3, 2, P, 2, 1, 4, 4, 64, 64, P, None, None, None) == QNN_EINVAL          # code size
    assert f(None, 1, 2, P, 2, 1, 4, 4, 64, 64, P, None, None, None) == QNN_EINVAL
    assert f(P, 1, 2, P, 2, 1, 4, 4, 64, 64, None, None, None, None) == QNN_EINVAL       # no output
    assert f(P, 1, 2, P + 4, 2, 1, 4, 4, 64, 64, P, None, None, None) == QNN_EALIGN
    assert f(None, 1, 2, None, 2, 0, 4, 4, 64, 64, None, None, None, None) == QNN_OK     # empty: nothing launched


def test_training_side_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK
    f = L.qnn_encoder_backward
    assert f(P, P, 16, 0, P, None) == QNN_EINVAL and f(P, P, 16, 9, P, None) == QNN_EINVAL
    assert f(None, P, 16, 2, P, None) == QNN_EINVAL and f(P, None, 16, 2, P, None) == QNN_EINVAL
    assert f(P, P, 16, 2, None, None) == QNN_EINVAL and f(P, P, -1, 2, P, None) == QNN_EINVAL
    assert f(P + 2, P, 16, 2, P, None) == QNN_EALIGN
    assert f(None, None, 0, 2, None, None) == QNN_OK
    f = L.qnn_binarize
    assert f(P, -1, 8, P, P, None) == QNN_EINVAL and f(None, 4, 8, P, P, None) == QNN_EINVAL
    assert f(P, 4, 8, None, None, None) == QNN_EINVAL
    assert f(P, 4, 8, None, P + 4, None) == QNN_EALIGN
    assert f(None, 0, 8, None, None, None) == QNN_OK
    f = L.qnn_binarize_backward
    assert f(P, P, -1, P, None) == QNN_EINVAL and f(P, None, 4, P, None) == QNN_EINVAL
    assert f(None, None, 0, None, None) == QNN_OK
    f = L.qnn_quantize_k
    c = ctypes.c_float
    assert f(P, 16, 1, c(1.0), P, None, None) == QNN_EINVAL          # one bit has no state but 0
    assert f(P, 16, 25, c(1.0), P, None, None) == QNN_EINVAL
    assert f(P, 16, 3, c(0.0), P, None, None) == QNN_EINVAL and f(P, 16, 3, c(-1.0), P, None, None) == QNN_EINVAL
    assert f(P, 16, 3, c(float("nan")), P, None, None) == QNN_EINVAL
    assert f(P, 16, 3, c(1.0), None, None, None) == QNN_EINVAL
    assert f(None, 0, 3, c(1.0), None, None, None) == QNN_OK
    f = L.qnn_quantize_k_backward
    assert f(P, P, 16, c(0.0), P, None) == QNN_EINVAL and f(P, None, 16, c(1.0), P, None) == QNN_EINVAL
    assert f(None, None, 0, c(1.0), None, None) == QNN_OK


def test_backward_product_argument_errors(L):
    from paper_2106_09886_amd.binding import QNN_EINVAL, QNN_EALIGN, QNN_OK, QNN_EUNSUPPORTED, QNN_EWORKSPACE
    for f in (L.qnn_branch_gemm_backward_input, L.qnn_branch_gemm_backward_weight):
        assert f(P, None, P, 0, 4, 4, 32, 2, P, None) == QNN_EINVAL and f(P, None, P, 2, 4, 4, 32, 9, P, None) == QNN_EINVAL
        assert f(P, None, P, 2, -1, 4, 32, 2, P, None) == QNN_EINVAL
        assert f(None, None, P, 2, 4, 4, 32, 2, P, None) == QNN_EINVAL and f(P, None, None, 2, 4, 4, 32, 2, P, None) == QNN_EINVAL
        assert f(P, None, P, 2, 4, 4, 32, 2, None, None) == QNN_EINVAL
        assert f(P + 2, None, P, 2, 4, 4, 32, 2, P, None) == QNN_EALIGN and f(P, None, P + 4, 2, 4, 4, 32, 2, P, None) == QNN_EALIGN
        assert f(P, P + 1, P, 2, 4, 4, 32, 2, P, None) == QNN_EALIGN
        assert f(P, None, P, 2, 1 << 31, 4, 32, 2, P, None) == QNN_EUNSUPPORTED
        assert f(None, None, None, 2, 4, 4, 0, 2, None, None) == QNN_OK          # no columns: empty output
    assert L.qnn_branch_gemm_backward_input(None, None, None, 2, 0, 4, 32, 2, None, None) == QNN_OK
    assert L.qnn_branch_gemm_backward_weight(None, None, None, 2, 4, 0, 32, 2, None, None) == QNN_OK
    f = L.qnn_update_sgd
    assert f(P, P, -1, 0.1, None) == QNN_EINVAL and f(None, P, 4, 0.1, None) == QNN_EINVAL and f(P, None, 4, 0.1, None) == QNN_EINVAL
    assert f(P + 2, P, 4, 0.1, None) == QNN_EALIGN and f(None, None, 0, 0.1, None) == QNN_OK
    f = L.qnn_update_adam
    ok = (0.001, 0.9, 0.999, 1e-8, 1, None)
    assert f(P, P, P, P, -1, *ok) == QNN_EINVAL and f(None, P, P, P, 4, *ok) == QNN_EINVAL and f(P, P, None, P, 4, *ok) == QNN_EINVAL
    assert f(P, P, P, P, 4, 0.001, 0.9, 0.999, 1e-8, 0, None) == QNN_EINVAL           # steps count from one
    assert f(P, P, P, P, 4, 0.001, 1.0, 0.999, 1e-8, 1, None) == QNN_EINVAL and f(P, P, P, P, 4, 0.001, 0.9, -0.1, 1e-8, 1, None) == QNN_EINVAL
    assert f(P, P, P, P, 4, 0.001, 0.9, 0.999, -1.0, 1, None) == QNN_EINVAL
    assert f(P, P, P + 2, P, 4, *ok) == QNN_EALIGN and f(None, None, None, None, 0, *ok) == QNN_OK
    f = L.qnn_conv2d_backward_input
    assert f(P, None, P, 0, 1, 4, 4, 32, 8, 2, P, None) == QNN_EINVAL and f(P, None, P, 2, -1, 4, 4, 32, 8, 2, P, None) == QNN_EINVAL
    assert f(None, None, P, 2, 1, 4, 4, 32, 8, 2, P, None) == QNN_EINVAL and f(P, None, P, 2, 1, 4, 4, 32, 8, 2, None, None) == QNN_EINVAL
    assert f(P, None, P + 4, 2, 1, 4, 4, 32, 8, 2, P, None) == QNN_EALIGN and f(P + 2, None, P, 2, 1, 4, 4, 32, 8, 2, P, None) == QNN_EALIGN
    assert f(P, None, P, 2, 1 << 20, 1 << 10, 1 << 10, 32, 8, 2, P, None) == QNN_EUNSUPPORTED
    assert f(None, None, None, 2, 0, 4, 4, 32, 8, 2, None, None) == QNN_OK
    need = L.qnn_conv2d_backward_weight_workspace_bytes(2, 8, 8, 64, 64)
    assert need >= 64 * 9 * 64 * 4 and need % (64 * 9 * 64 * 4) == 0
    assert L.qnn_conv2d_backward_weight_workspace_bytes(2, 8, 8, 0, 64) == 0
    f = L.qnn_conv2d_backward_weight
    assert f(P, None, P, 2, 2, 8, 8, 64, 64, 2, P, P, need - 1, None) == QNN_EWORKSPACE
    assert f(P, None, P, 2, 2, 8, 8, 64, 64, 2, P, None, need, None) == QNN_EINVAL and f(P, None, P, 2, 2, 8, 8, 64, 64, 9, P, P, need, None) == QNN_EINVAL
    assert f(P, None, P, 2, 2, 8, 8, 64, 64, 2, P, P + 4, need, None) == QNN_EALIGN
    assert f(None, None, None, 2, 2, 8, 8, 64, 0, 2, None, None, 0, None) == QNN_OK
