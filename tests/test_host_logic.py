"""Host-side logic of the library that has no GPU in it, compiled and run on the CPU."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_scalar_division_constants_are_exact():
    """The kernels divide wave-uniform numbers by launch constants with one multiply-high and a shift
    (FastDiv); the constants the host prepares must give the exact quotient for every n < 2^31."""
    tmp = tempfile.mkdtemp(prefix="qnn_host_")
    try:
        exe = os.path.join(tmp, "fast_div")
        subprocess.run([HIPCC, "-O2", "-std=c++17", "-x", "hip", "--cuda-host-only",
                        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2106_09886_amd", "csrc"),
                        os.path.join(ROOT, "tests", "host_fast_div.cpp"), "-o", exe], check=True,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE)
        r = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
        assert r.returncode == 0, r.stdout
        assert "bad 0" in r.stdout
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_vgg_stack_recipe_keeps_the_code_levels_populated(oracle):
    """The synthetic VGG-16-shaped stack is only a fair workload if its activations use the code
    range the way a trained network's would: with the recipe's per-channel scales, the 4-bit codes
    that every layer hands to the next must populate at least 8 of the 16 levels, and no single
    level may hold almost everything.  Checked on the oracle alone, on 2 images of 32x32 (the
    recipe's scales do not depend on the image size)."""
    import numpy as np
    from paper_2106_09886_amd import inputs
    w = inputs.VGG16
    X0, layers = inputs.make_stack(w, Nb=2, H=32, W=32)
    codes = X0
    for l, (Wt, s, pool) in enumerate(layers, start=1):
        acc = oracle.conv3x3(codes, Wt)
        y = oracle.scale_f32(acc, s)
        codes = oracle.requant(oracle.maxpool2x2(y) if pool else y, w.ab)
        levels, counts = np.unique(codes, return_counts=True)
        if codes.size >= 2048:             # the last layers of the small case hold too few values to say
            assert len(levels) >= 8, "layer %d populates only %d levels" % (l, len(levels))
            assert counts.max() <= 0.6 * codes.size, "layer %d: one level holds %d of %d" % (l, counts.max(), codes.size)
