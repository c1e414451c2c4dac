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


# Sources whose device assembly is kept beside the object (<dir of the object>/<source>-hip-amdgcn-
# amd-amdhsa-gfx950.s): the kernels with hand-issued scalar loads, which the test suite checks
# statically in exactly the form that is linked.
KEEP_ASM = ("qnn_branch.hip", "qnn_conv_small.hip")


def _compile(job):
    src, obj, extra = job
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    keep = src in KEEP_ASM
    cmd = [HIPCC] + FLAGS + extra + (["-save-temps=obj"] if keep else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    if keep:                                   # of the intermediate files only the device assembly stays
        d, stem = os.path.dirname(obj), src.split(".")[0]
        for f in os.listdir(d):
            if f.startswith(stem + "-") or f.startswith(src + "-"):
                if not f.endswith("-gfx950.s"):
                    os.remove(os.path.join(d, f))
    return out


def _fresh(job, newest_header):
    src, obj, _ = job
    return os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(os.path.join(CSRC, src)), newest_header)


def build(jobs=None, verbose=False, incremental=False):
    """Compile and link.  incremental=True skips objects newer than their source and every header
    (a convenience while editing; the default always compiles everything)."""
    os.makedirs(OBJ, exist_ok=True)
    work = [("qnn_api.hip", os.path.join(OBJ, "qnn_api.o"), []),
            ("qnn_pack.hip", os.path.join(OBJ, "qnn_pack.o"), []),
            ("qnn_epilogue.hip", os.path.join(OBJ, "qnn_epilogue.o"), []),
            ("qnn_requant.hip", os.path.join(OBJ, "qnn_requant.o"), []),
            ("qnn_elementwise.hip", os.path.join(OBJ, "qnn_elementwise.o"), []),
            ("qnn_backward.hip", os.path.join(OBJ, "qnn_backward.o"), []),
            ("qnn_compare_mfma.hip", os.path.join(OBJ, "qnn_compare_mfma.o"), []),
            ("qnn_compare_dot.hip", os.path.join(OBJ, "qnn_compare_dot.o"), [])]
    for ab in range(1, 9):
        sub = os.path.join(OBJ, "ab%d" % ab)      # one folder per width: the kept assembly is named after the source
        work.append(("qnn_branch.hip", os.path.join(sub, "qnn_branch.o"), ["-DQNN_AB=%d" % ab]))
        work.append(("qnn_conv_small.hip", os.path.join(sub, "qnn_conv_small.o"), ["-DQNN_AB=%d" % ab]))
        work.append(("qnn_conv_general.hip", os.path.join(sub, "qnn_conv_general.o"), ["-DQNN_AB=%d" % ab]))
    if incremental:
        headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
        headers.append(os.path.join(ROOT, "include", "qnn.h"))
        newest = max(os.path.getmtime(h) for h in headers)
        todo = [w for w in work if not _fresh(w, newest)]
    else:
        todo = work
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(_compile, todo):
            if verbose and out.strip():
                print(out)
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [w[1] for w in work]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
