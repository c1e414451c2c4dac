"""Static check of the hand-placed scalar loads in the generated gfx950 assembly.

The branch kernels (qnn_branch.hip, qnn_conv_small.hip) request activation words with s_load_dword* written as inline asm and
wait for them with an explicit s_waitcnt; the compiler does not know the destination SGPRs
are in flight in between.  This module takes their assembly for every activation bit width --
the files the library build keeps beside its objects (the very code that was linked), or a
compilation of its own where those are missing or older than the sources -- and verifies,
kernel by kernel, that
  * no instruction addresses scratch memory (a kernel may reserve a few bytes that the register
    allocator set aside and never used; that is reported by size only if something accesses it), and
  * on no path of the control-flow graph does an instruction outside an asm block (a spill
    to a VGPR lane included) name a requested SGPR between its s_load and the next
    `s_waitcnt lgkmcnt(0)`.
Run: python tests/scalar_pipeline_check.py   (exit status 0 = clean); tests/test_scalar_pipeline.py
runs the same check for all eight widths in the CPU suite.
"""
import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "paper_2106_09886_amd", "csrc")          # the kernel sources
BUILD = os.path.join(ROOT, "paper_2106_09886_amd", "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


SOURCES = ("qnn_branch.hip", "qnn_conv_small.hip")


def compile_asm(job):
    src, ab, out = job
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-ffp-contract=off", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", HERE, "-DQNN_AB=%d" % ab, "-S", "--cuda-device-only",
           os.path.join(HERE, src), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    return out


def built_asm(src, ab):
    """The assembly the library build kept for (source, activation width), or None if it is missing
    or older than what it is compiled from (its source, every header)."""
    path = os.path.join(BUILD, "ab%d" % ab, src.split(".")[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(path):
        return None
    deps = [os.path.join(HERE, f) for f in os.listdir(HERE) if f.endswith(".h")]
    deps.append(os.path.join(HERE, src))
    deps.append(os.path.join(ROOT, "include", "qnn.h"))
    return path if os.path.getmtime(path) >= max(os.path.getmtime(d) for d in deps) else None


def asm_files(tmpdir, widths=range(1, 9)):
    """{(source, ab): path} for every width: the build's files where fresh, else compiled here
    (in parallel: a compilation takes one to two minutes)."""
    out, jobs = {}, []
    for src in SOURCES:
        for ab in widths:
            p = built_asm(src, ab)
            if p is not None:
                out[(src, ab)] = p
            else:
                jobs.append((src, ab, os.path.join(tmpdir, "%s_ab%d.s" % (src.split(".")[0], ab))))
    if jobs:
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            for job, path in zip(jobs, ex.map(compile_asm, jobs)):
                out[(job[0], job[1])] = path
    return out


def sregs(tok):
    """SGPR numbers named by an operand token like s5 or s[8:15]."""
    m = re.fullmatch(r"s(\d+)", tok)
    if m:
        return {int(m.group(1))}
    m = re.fullmatch(r"s\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def parse_kernel(lines):
    """-> list of instructions (lineno, text, op, in_asm) and label -> instruction index."""
    insts, labels = [], {}
    in_asm = False
    for ln, raw in lines:
        l = raw.strip()
        if l.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if l.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = len(insts)
            continue
        if not l or l.startswith(";") or l.startswith("."):
            continue
        l = l.split(";")[0].strip()
        if not l:
            continue
        insts.append((ln, l, l.split()[0], in_asm))
    return insts, labels


def check_kernel(name, lines):
    """Forward may-analysis over the control-flow graph: the set of SGPRs with a hand-issued
    scalar load in flight.  A non-asm instruction that names one of them is a violation."""
    insts, labels = parse_kernel(lines)
    n = len(insts)
    # The kernels have no lane-divergent control flow (blocks are always full, every branch
    # condition is wave-uniform).  If nothing in the kernel writes EXEC, it stays all-ones and
    # the EXEC-tested branches the compiler leaves behind are decided statically.
    exec_const = not any(
        op.startswith("v_cmpx") or "saveexec" in op or re.search(r"^\S+\s+exec(_lo|_hi)?\b", l)
        for (_, l, op, _) in insts)
    succ = [[] for _ in range(n)]
    for i, (ln, l, op, _) in enumerate(insts):
        if op == "s_endpgm":
            continue
        if op == "s_branch":
            succ[i] = [labels[l.split()[1]]]
        elif exec_const and op == "s_cbranch_execz":
            succ[i] = [i + 1] if i + 1 < n else []
        elif exec_const and op == "s_cbranch_execnz":
            succ[i] = [labels[l.split()[1]]]
        elif op.startswith("s_cbranch"):
            succ[i] = [labels[l.split()[1]]] + ([i + 1] if i + 1 < n else [])
        elif i + 1 < n:
            succ[i] = [i + 1]
    regs = [set().union(*[sregs(t) for t in re.findall(r"s\[\d+:\d+\]|\bs\d+\b", l)] or [set()])
            for (_, l, _, _) in insts]
    gen = [set() for _ in range(n)]
    kill = [False] * n
    for i, (ln, l, op, in_asm) in enumerate(insts):
        if op == "s_waitcnt" and "lgkmcnt(0)" in l:
            kill[i] = True
        elif in_asm and op.startswith("s_load_dword"):
            toks = re.findall(r"s\[\d+:\d+\]|\bs\d+\b", l)
            gen[i] = sregs(toks[0])
    pend_in = [set() for _ in range(n)]
    work = list(range(n))
    while work:
        i = work.pop()
        out = set() if kill[i] else (pend_in[i] | gen[i])
        for j in succ[i]:
            if not out <= pend_in[j]:
                pend_in[j] |= out
                work.append(j)
    problems = []
    for i, (ln, l, op, in_asm) in enumerate(insts):
        if in_asm or kill[i]:
            continue
        hit = regs[i] & pend_in[i]
        if hit:
            problems.append("%s:%d touches in-flight s%s: %s" % (name, ln, sorted(hit), l))
    spills = sum(1 for (_, _, op, _) in insts if op in ("v_writelane_b32", "v_readlane_b32"))
    return problems, spills


def uses_scratch(lines):
    """Does any instruction of the kernel address scratch memory?"""
    for _, raw in lines:
        l = raw.strip()
        if l.startswith("scratch_") or (l.startswith("buffer_") and "s[0:3]" in l and "offen" not in l.split(";")[0] and " off" in l):
            return True
        if l.startswith("buffer_") and re.search(r"s\[0:3\],\s*0(\s|$)", l.split(";")[0]):      # stack accesses: soffset 0 on the scratch descriptor
            return True
    return False


def check_file(path):
    text = open(path).read().split("\n")
    problems, nk, nspill = [], 0, 0
    cur, name = None, None
    touches_scratch = {}
    last_kernel = None
    for i, l in enumerate(text, 1):
        m = re.match(r"^(_ZN3qnn\S*_kernel\S*):", l)
        if m:
            name, cur = m.group(1), []
            continue
        if cur is not None:
            cur.append((i, l))
            if l.startswith(".Lfunc_end"):
                p, sp = check_kernel(name, cur)
                problems += p
                nspill += sp
                nk += 1
                touches_scratch[name] = uses_scratch(cur)
                cur = None
        m = re.match(r"^\s*\.amdhsa_kernel\s+(\S+)", l)
        if m:
            last_kernel = m.group(1)
        m = re.match(r"^\s*\.amdhsa_private_segment_fixed_size\s+(\d+)", l)
        if m and int(m.group(1)) != 0:
            # the descriptor may come before the function's end label: then `cur` is the kernel's text so far
            touched = uses_scratch(cur) if (cur is not None and name == last_kernel) else touches_scratch.get(last_kernel, True)
            if touched:
                problems.append("%s: kernel %s uses %s bytes of scratch" % (path, last_kernel, m.group(1)))
    return nk, problems, nspill


def main():
    tmp = tempfile.mkdtemp(prefix="qnn_asm_")
    files = list(asm_files(tmp).values())
    total, bad, spills = 0, [], 0
    for f in files:
        nk, p, sp = check_file(f)
        total += nk
        bad += p
        spills += sp
    print("%d kernels checked, %d problems (%d SGPR spill instructions, none touching a register in flight"
          " unless listed)" % (total, len(bad), spills))
    for p in bad[:40]:
        print("  " + p)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
