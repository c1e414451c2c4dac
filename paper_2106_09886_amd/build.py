"""Build libqnn.so (HIP, gfx950 only) in-tree with hipcc.

``python -m paper_2106_09886_amd.build`` or ``build()``.  The branch kernels are compiled
once per activation bit width (eight objects, in parallel), then everything is linked into
``paper_2106_09886_amd/libqnn.so``.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqnn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(job):
    src, obj, extra = job
    cmd = [HIPCC] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(jobs=None, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    work = [("qnn_api.hip", os.path.join(OBJ, "qnn_api.o"), []),
            ("qnn_pack.hip", os.path.join(OBJ, "qnn_pack.o"), []),
            ("qnn_epilogue.hip", os.path.join(OBJ, "qnn_epilogue.o"), []),
            ("qnn_requant.hip", os.path.join(OBJ, "qnn_requant.o"), []),
            ("qnn_compare_mfma.hip", os.path.join(OBJ, "qnn_compare_mfma.o"), []),
            ("qnn_compare_dot.hip", os.path.join(OBJ, "qnn_compare_dot.o"), [])]
    for ab in range(1, 9):
        work.append(("qnn_branch.hip", os.path.join(OBJ, "qnn_branch_ab%d.o" % ab), ["-DQNN_AB=%d" % ab]))
        work.append(("qnn_conv_small.hip", os.path.join(OBJ, "qnn_conv_small_ab%d.o" % ab), ["-DQNN_AB=%d" % ab]))
        work.append(("qnn_conv_general.hip", os.path.join(OBJ, "qnn_conv_general_ab%d.o" % ab), ["-DQNN_AB=%d" % ab]))
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(_compile, work):
            if verbose and out.strip():
                print(out)
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [w[1] for w in work]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
