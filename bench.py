#!/usr/bin/env python3
"""Benchmark of the {-1,+1} multi-branch binary product hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic activations that are
already resident in HBM: encode + pack the activation codes, then the branch product
(implicit-im2col convolution or GEMM) with fused weighted accumulation and fp32 scale epilogue.
The weights are static parameters and are packed once before the timed region.

Default workload: `resnet18_s1`, the ResNet-18-stage-1-shaped W2A2 3x3 convolution the target
is quoted on.  Other workloads (`--workload`): `resnet50_s3`, `fc4096`, `gemm64`, `gemm8192`
(`--bits b`, with the two comparison lines: int8 matrix cores and packed int8 dot product), `vgg16_stack` (13 chained layers: conv +
scale, then max-pool / re-encode / pack per layer), `vgg16_stack_fused` (the same through the
fused kernels), and side suites that print their own tables: `hbm_kernels` (the
memory-bound kernels at chip-filling sizes), `conv_geometries` (`qnn_conv2d_general`),
`resnet18_mixed` and `backward_products` (the training-side products of Alg. 1).

Prints ONE JSON line.  `value` is the effective quantized throughput 2*M*N*K / t_step in
GOPS.  `roofline` prices the dominant kernel (the branch kernel) against the chip's integer
vector-ALU rate; `cpu_baseline` is the CPU oracle timed on the host cores of this machine.

Before the W warm-up steps the device is kept busy with the same step for a quarter of a
second, untimed, so that its clocks have settled.  Extras: `--wave-trace` (one traced launch:
wavefronts per SIMD, active windows, shader clock), `--batch N` (the convolution workloads on
another number of images: fixed cost of a launch), `--graph`, `--copy-calibration`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import ctypes
import hashlib
import json
import math
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Integer vector-ALU peak: compute units x 64 lanes x shader clock, one 32-bit integer lane-op per
# lane and clock (v_xor_b32, v_bcnt_u32_b32 are full rate, not packed).  The counts come from the
# device the run is on (device_peak); these are MI355X's published figures, used as the fallback.
NOMINAL_CUS, NOMINAL_GHZ = 256, 2.4
PEAK_LANE_OPS = NOMINAL_CUS * 64 * NOMINAL_GHZ * 1e9

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
# what the kernels with a stored traffic figure (branch GEMM / convolution) and their launch sizing are built from
KERNEL_SOURCES = ("include/qnn.h", "paper_2106_09886_amd/csrc/qnn_branch.hip", "paper_2106_09886_amd/csrc/qnn_device_util.h",
                  "paper_2106_09886_amd/csrc/qnn_internal.h", "paper_2106_09886_amd/csrc/qnn_api.hip")


def device_peak(q):
    """(lane-op/s, description): CU count and peak shader clock as the HIP runtime reports them."""
    global PEAK_LANE_OPS
    try:
        cus, khz = q.device_info()
    except RuntimeError:
        cus, khz = 0, 0
    cus = cus or NOMINAL_CUS
    ghz = float(khz) / 1e6 if khz else None
    said = "device"
    if not ghz or not (0.5 < ghz < 5.0):
        ghz, said = NOMINAL_GHZ, "nominal (the runtime reported none)"
    PEAK_LANE_OPS = cus * 64 * ghz * 1e9
    return PEAK_LANE_OPS, "%d CU x 64 lanes x %.3f GHz (%s clock), one 32-bit integer vector op per lane and clock" % (
        cus, ghz, said)


def kernel_source_hash():
    """sha256 over the sources of the measured kernels: ties a stored traffic figure to the code it was measured on."""
    h = hashlib.sha256()
    files = []
    for rel in KERNEL_SOURCES:
        path = os.path.join(ROOT, rel)
        if os.path.isdir(path):
            files += [os.path.join(path, f) for f in sorted(os.listdir(path)) if f.endswith((".hip", ".h"))]
        else:
            files.append(path)
    for f in files:
        h.update(os.path.relpath(f, ROOT).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def stored_traffic(key):
    """HBM bytes per launch of the dominant kernel of workload `key`, from the counter runs recorded in
    profiles/traffic.json (written by --record-traffic) -- or None when the kernel sources have changed
    since (a stale figure is worse than none)."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    if rec.get("source_sha256") != kernel_source_hash():
        return None
    e = rec.get("workloads", {}).get(key)
    return None if e is None else e.get("bytes_per_launch")


def record_traffic(args):
    """--record-traffic KEY KERNEL FETCH.csv WRITE.csv: read two rocprofv3 --pmc counter CSVs (FETCH_SIZE
    and WRITE_SIZE, KiB per dispatch; each run made with --copy-calibration), scale them by what the same
    counter shows for the 256 MiB device copy in that run, and store the per-launch bytes of the kernel
    whose name contains KERNEL in profiles/traffic.json together with the hash of the kernel sources."""
    import csv
    key, kernel, fetch_csv, write_csv = args

    def per_dispatch(path, counter):
        rows = list(csv.DictReader(open(path)))
        vals = lambda sub: [float(r["Counter_Value"]) for r in rows
                            if r.get("Counter_Name") == counter and sub in r.get("Kernel_Name", "")]
        cal, ker = vals("copyBuffer"), vals(kernel)
        if not cal or not ker:
            raise SystemExit("%s: no %s rows for the copy or for '%s'" % (path, counter, kernel))
        # the calibration copy (262144 KiB each way) is the largest device copy of the run; smaller ones
        # (torch's own) share the kernel name
        factor = (256 << 10) / max(cal)
        if not 0.9 <= factor <= 2.2:
            raise SystemExit("%s: the largest copy shows %s = %.1f KiB, not a 256 MiB copy" % (path, counter, max(cal)))
        return statistics.median(ker) * 1024.0 * factor, factor, len(ker)
    fb, ff, nf = per_dispatch(fetch_csv, "FETCH_SIZE")
    wb, wf, nw = per_dispatch(write_csv, "WRITE_SIZE")
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        rec = {}
    src = kernel_source_hash()
    if rec.get("source_sha256") != src:
        rec = {"source_sha256": src, "workloads": {}}
    try:
        rec["git_head_when_recorded"] = subprocess.run(["git", "-C", ROOT, "rev-parse", "HEAD"], capture_output=True,
                                                       text=True).stdout.strip() or None
    except OSError:
        rec["git_head_when_recorded"] = None
    rec["workloads"][key] = {"kernel": kernel, "bytes_per_launch": round(fb + wb), "fetch_bytes": round(fb),
                             "write_bytes": round(wb), "fetch_scale": round(ff, 4), "write_scale": round(wf, 4),
                             "dispatches": [nf, nw]}
    json.dump(rec, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
    print(json.dumps(rec["workloads"][key]))
    return 0


def timed(torch, fn, n):
    """Average duration in microseconds of n back-to-back calls on the current stream."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n * 1e3


def timed_regions(torch, fn, k, min_samples=100, min_ms=50.0, lead_in=3, max_regions=400):
    """Timed regions of EXACTLY k calls each, repeated until at least min_samples calls and min_ms of
    device time have been measured, so that the result does not depend on the caller's k.  A region is
    bracketed by synchronisations; inside, `lead_in` untimed calls go first so that the queue is not
    empty when the first event is reached (otherwise each region also times one launch latency).
    Returns microseconds per call: median, min and mean over the regions."""
    per_call, total_ms = [], 0.0
    while len(per_call) < max_regions and (len(per_call) * k < min_samples or total_ms < min_ms):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        for _ in range(lead_in):
            fn()
        a.record()
        for _ in range(k):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        total_ms += ms
        per_call.append(ms / k * 1e3)
    return {"median": statistics.median(per_call), "min": min(per_call), "mean": statistics.fmean(per_call),
            "regions": len(per_call), "calls_per_region": k}


def conv_tap_pixels(Nb, H, W):
    """(output pixel, tap) pairs of a 3x3 / stride 1 / pad 1 layer whose tap lies inside the image: the
    products the kernels really form (taps outside are skipped, they contribute exactly 0)."""
    vh = 3 * H - 2 if H >= 2 else H
    vw = 3 * W - 2 if W >= 2 else W
    return Nb * vh * vw


def axis_taps(size_in, size_out, k, stride, pad, dil, transposed):
    """Sum over the output positions of one axis of the number of kernel elements that meet the image."""
    n = 0
    for o in range(size_out):
        for j in range(k):
            if transposed:
                num = o + pad - j * dil
                if num % stride == 0 and 0 <= num // stride < size_in:
                    n += 1
            elif 0 <= o * stride - pad + j * dil < size_in:
                n += 1
    return n


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def traced_launch(torch, np, q, launch):
    """One launch with the per-wavefront trace on: every wavefront records its start and end on
    the shader clock (s_memtime), its hardware position and its start on the chip-wide 100 MHz
    clock.  The ratio of the two clocks between the first and the last wavefront of a SIMD is
    the shader clock the kernel really ran at."""
    cap = 1 << 20
    buf = torch.zeros(cap * 4, dtype=torch.int64, device="cuda")
    q.set_wave_trace(buf)
    launch()
    torch.cuda.synchronize()
    q.set_wave_trace(None)
    t = buf.cpu().numpy().reshape(cap, 4)
    t = t[t[:, 0] != 0]
    if len(t) == 0:
        return None
    start, end, hw, rt = t[:, 0], t[:, 1], t[:, 2] & 0xffffffff, t[:, 3]
    xcc = (t[:, 2] >> 32) & 15
    simd, cu, sh, se = (hw >> 4) & 3, (hw >> 8) & 15, (hw >> 12) & 1, (hw >> 13) & 7
    key = ((((xcc * 8 + se) * 2 + sh) * 16 + cu) * 4 + simd).astype(np.int64)
    ids, idx = np.unique(key, return_inverse=True)
    big = np.iinfo(np.int64).max

    def per_simd(values, fn, init):
        out = np.full(len(ids), init, dtype=np.int64)
        fn.at(out, idx, values)
        return out
    first_start, last_start = per_simd(start, np.minimum, big), per_simd(start, np.maximum, 0)
    first_rt, last_rt = per_simd(rt, np.minimum, big), per_simd(rt, np.maximum, 0)
    last_end = per_simd(end, np.maximum, 0)
    counts = np.bincount(idx, minlength=len(ids))
    window = last_end - first_start
    spread = (last_rt - first_rt) > 500                      # SIMDs whose wavefront starts span > 5 us
    ghz = float(np.median((last_start - first_start)[spread] / (last_rt - first_rt)[spread])) / 10.0 if spread.any() else None
    return {"wavefronts": int(len(t)), "simds": int(len(ids)),
            "wavefronts_per_simd_min_max": [int(counts.min()), int(counts.max())],
            "simd_active_window_cycles_p0_p50_p100": [int(x) for x in np.percentile(window, [0, 50, 100])],
            "first_start_spread_us": round(float(first_rt.max() - first_rt.min()) / 100.0, 2),
            "shader_clock_GHz": None if ghz is None else round(ghz, 3)}


def side_suites(name, args, steps, warmup, torch, np, q, dev):
    """Micro-benchmarks outside the headline: the memory-bound kernels at sizes that fill the chip,
    and qnn_conv2d_general on layer shapes of the networks the paper evaluates.  One JSON line."""
    def avg_us(fn):
        t_end = time.time() + 0.1                       # untimed: let the clocks settle under this kernel
        while time.time() < t_end:
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
        for _ in range(warmup):
            fn()
        return timed_regions(torch, fn, steps, min_samples=60, min_ms=20.0)["median"]

    rows = []
    if name == "hbm_kernels":
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        t = avg_us(lambda: dst.copy_(src))
        rows.append({"kernel": "device copy 1 GiB (reference)", "us": round(t, 1), "GBps": round(2 * (1 << 30) / t / 1e3, 1)})
        del src, dst
        for bits in (2, 4):
            r, K = 65536, 8192
            codes = (torch.randint(0, 1 << bits, (r, K), dtype=torch.int8, device=dev) * 2 - ((1 << bits) - 1)).to(torch.int8)
            out = torch.empty((r, bits, K // 32), dtype=torch.int32, device=dev)
            t = avg_us(lambda: q.encode_pack(codes, bits, out=out))
            rows.append({"kernel": "qnn_encode_pack int8 %dx%d, %d bits" % (r, K, bits), "us": round(t, 1),
                         "GBps": round(r * K * (1 + bits / 8) / t / 1e3, 1)})
            del codes, out
        for (Nb, H, W, C, pool) in ((16, 224, 224, 64, False), (16, 224, 224, 64, True), (64, 56, 56, 256, False)):
            y = torch.randn((Nb, H, W, C), device=dev) * 5
            t = avg_us(lambda: q.requant_pack(y, 4, pool=pool, want_codes=False))
            n_out = Nb * H * W * C / (4 if pool else 1)
            rows.append({"kernel": "qnn_requant_pack %dx%dx%dx%d -> 4-bit planes%s" % (Nb, H, W, C, ", 2x2 pool" if pool else ""),
                         "us": round(t, 1), "GBps": round((Nb * H * W * C * 4 + n_out / 2) / t / 1e3, 1)})
            del y
        x = torch.randn((65536, 4096), device=dev)
        t = avg_us(lambda: q.encode_real(x, 4, want_codes=False))
        rows.append({"kernel": "qnn_encode_real 65536x4096 -> 4-bit planes", "us": round(t, 1),
                     "GBps": round(x.numel() * 4.5 / t / 1e3, 1)})
        del x
        acc = torch.randint(-1000, 1000, (65536, 4096), dtype=torch.int32, device=dev)
        s = torch.rand(4096, device=dev)
        t = avg_us(lambda: q.scale_epilogue(acc, s))
        rows.append({"kernel": "qnn_scale_epilogue 65536x4096", "us": round(t, 1), "GBps": round(acc.numel() * 8 / t / 1e3, 1)})
        head = rows[1]
        res = {"metric": "GB/s of qnn_encode_pack (algorithmic bytes: codes in + planes out)", "value": head["GBps"],
               "unit": "GB/s", "roofline": {"bound": "hbm", "kernel": "pack_kernel", "achieved": head["GBps"], "peak": 8000.0,
                                            "unit": "GB/s", "frac": round(head["GBps"] / 8000.0, 4), "traffic": None}}
    elif name == "backward_products":
        # Alg. 1's backward lines through the product of a fully connected layer: real gradient times the
        # codes held as bit planes, on the fp32 matrix cores (dense peak 157.3 TFLOP/s).  flops = 2 * M * N * K
        # per call (the 2^(m-1) / 2^(k-1) copies are exact multiples, written, not recomputed).
        PEAK_F32_MFMA = 157.3e12
        for (label, M, N, K, ab, wb) in (("FC 256 x 4096 x 4096, W2A2", 256, 4096, 4096, 2, 2),
                                         ("FC 4096 x 4096 x 4096, W2A2", 4096, 4096, 4096, 2, 2),
                                         ("FC 4096 x 4096 x 4096, W4A4", 4096, 4096, 4096, 4, 4),
                                         ("FC 1024 x 1000 x 512, W6A4", 1024, 1000, 512, 4, 6)):
            Kw = (K + 31) // 32
            Ap = torch.randint(-2 ** 31, 2 ** 31 - 1, (M, ab, Kw), dtype=torch.int32, device=dev)
            Wp = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, wb, Kw), dtype=torch.int32, device=dev)
            g = torch.randn((M, N), device=dev)
            sd = torch.rand(N, device=dev) + 0.5
            flops = 2.0 * M * N * K
            for which, fn, out_bytes in (("towards the activations", lambda: q.branch_gemm_backward_input(g, Wp, wb, K, ab, scale=sd), ab * M * K * 4),
                                         ("towards the weights", lambda: q.branch_gemm_backward_weight(g, Ap, ab, K, wb, scale=sd), wb * N * K * 4)):
                t = avg_us(fn)
                rows.append({"layer": label, "gradient": which, "us": round(t, 1), "TFLOPs": round(flops / t / 1e6, 2),
                             "frac_of_f32_matrix_peak": round(flops / (t * 1e-6) / PEAK_F32_MFMA, 3),
                             "output_MB": round(out_bytes / 1e6, 1)})
            del Ap, Wp, g, sd
        # the same lines through 3x3 convolutions: flops = 2 * pixels * 9 * Cout * C per gradient
        for (label, Nb, H, W, C, Cout, ab, wb) in (("conv 32 x 56 x 56 x 64 -> 64, W2A2 (the headline layer)", 32, 56, 56, 64, 64, 2, 2),
                                                  ("conv 64 x 14 x 14 x 256 -> 256, W3A4", 64, 14, 14, 256, 256, 4, 3),
                                                  ("conv 16 x 112 x 112 x 128 -> 128, W2A4", 16, 112, 112, 128, 128, 4, 2)):
            Cw = (C + 31) // 32
            pixels = Nb * H * W
            Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (pixels, ab, Cw), dtype=torch.int32, device=dev)
            Wp = torch.randint(-2 ** 31, 2 ** 31 - 1, (Cout * 9, wb, Cw), dtype=torch.int32, device=dev)
            g = torch.randn((Nb, H, W, Cout), device=dev)
            sd = torch.rand(Cout, device=dev) + 0.5
            ws = torch.empty(max(16, int(q.lib().qnn_conv2d_backward_weight_workspace_bytes(Nb, H, W, C, Cout))), dtype=torch.uint8, device=dev)
            flops = 2.0 * pixels * 9 * Cout * C
            for which, fn, out_bytes in (("towards the activations", lambda: q.conv2d_backward_input(g, Wp, wb, C, ab, scale=sd), ab * pixels * C * 4),
                                         ("towards the weights", lambda: q.conv2d_backward_weight(g, Xp, ab, C, wb, scale=sd, workspace=ws), wb * Cout * 9 * C * 4)):
                t = avg_us(fn)
                rows.append({"layer": label, "gradient": which, "us": round(t, 1), "TFLOPs": round(flops / t / 1e6, 2),
                             "frac_of_f32_matrix_peak": round(flops / (t * 1e-6) / PEAK_F32_MFMA, 3),
                             "output_MB": round(out_bytes / 1e6, 1)})
            del Xp, Wp, g, sd, ws
        head = rows[3]
        res = {"metric": "TFLOP/s of qnn_branch_gemm_backward_weight, 4096^3 W2A2", "value": head["TFLOPs"], "unit": "TFLOP/s",
               "roofline": {"bound": "mfma", "kernel": "backward_gemm_kernel", "achieved": head["TFLOPs"], "peak": 157.3,
                            "unit": "TFLOP/s", "frac": head["frac_of_f32_matrix_peak"], "traffic": None}}
    elif name == "resnet18_mixed":
        # The paper's mixed-precision example (Sec. 5.1, Table 4, second precision column): ResNet-18 with
        # 4-bit activations and 5 / 3 / 2 / 2-bit weights in the four residual stages, a 6-bit fully
        # connected layer and an 8-bit first convolution (the table's Conv1 entry is garbled; the first
        # layer is taken at 8-bit activations and weights like the table's other column).  Every
        # convolution of the network once, batch 32; operands are random bit patterns (the cost does not
        # depend on the data; parity of these shapes and widths is in tests/test_gpu_general_conv.py).
        Nb = 32
        net = [("conv1 7x7/2 3->64 (row-dense input)", 1, 224, 3, 64, 8, 8, 7, 2, 3)]
        for (stage, cin, cout, hw, wb_) in (("conv2_x", 64, 64, 56, 5), ("conv3_x", 64, 128, 56, 3),
                                            ("conv4_x", 128, 256, 28, 2), ("conv5_x", 256, 512, 14, 2)):
            if cin == cout:
                net.append(("%s 3x3 %d->%d" % (stage, cin, cout), 4, hw, cin, cout, 4, wb_, 3, 1, 1))
            else:
                net.append(("%s 3x3/2 %d->%d" % (stage, cin, cout), 1, hw, cin, cout, 4, wb_, 3, 2, 1))
                net.append(("%s shortcut 1x1/2 %d->%d" % (stage, cin, cout), 1, hw, cin, cout, 4, wb_, 1, 2, 0))
                net.append(("%s 3x3 %d->%d" % (stage, cout, cout), 3, hw // 2, cout, cout, 4, wb_, 3, 1, 1))
        total_us, total_lane, total_ops = 0.0, 0.0, 0.0
        for (label, count, hw, C, Cout, ab, wb, k, st, pd) in net:
            Cw = (C + 31) // 32
            dense = C < 32
            if dense:
                Rw = (hw * C + 31) // 32
                Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (Nb * hw, ab, Rw), dtype=torch.int32, device=dev)
                if (hw * C) % 32:
                    Xp[:, :, -1] &= (1 << ((hw * C) % 32)) - 1
            else:
                Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (Nb * hw * hw, ab, Cw), dtype=torch.int32, device=dev)
            Wp = torch.randint(0, 1 << min(C, 30), (Cout, k * k, wb, Cw), dtype=torch.int32, device=dev)
            sd = torch.rand(Cout, device=dev)
            geo = q.conv_geometry(k, k, stride=st, pad=pd, dense_rows=dense)
            Ho, Wo = q.conv2d_general_output_size(hw, hw, geo)
            t = avg_us(lambda: q.conv2d_general(Xp, ab, Wp, wb, Nb, hw, hw, C, Cout, geo, scale=sd))
            tap_pixels = Nb * axis_taps(hw, Ho, k, st, pd, 1, False) ** 2
            # packed-window layers (few channels) work on window words, not on a word per tap
            kw_words = tap_pixels * Cw if not dense else Nb * Ho * Wo * (-(-(k * k * C) // 32))
            lane = 2.0 * ab * wb * kw_words * Cout
            ops = 2.0 * Nb * Ho * Wo * Cout * k * k * C
            rows.append({"layer": label, "times_in_network": count, "W%dA%d" % (wb, ab): True, "out": "%dx%d" % (Ho, Wo),
                         "us": round(t, 1), "effective_GOPS": round(ops / t / 1e3, 1),
                         "frac_of_lane_op_peak": round(lane / (t * 1e-6) / PEAK_LANE_OPS, 3)})
            total_us += count * t
            total_lane += count * lane
            total_ops += count * ops
            del Xp, Wp
        # the fully connected layer: 512 -> 1000, 4-bit activations, 6-bit weights
        A = torch.randint(-2 ** 31, 2 ** 31 - 1, (Nb, 4, 16), dtype=torch.int32, device=dev)
        Wf = torch.randint(-2 ** 31, 2 ** 31 - 1, (1000, 6, 16), dtype=torch.int32, device=dev)
        sd = torch.rand(1000, device=dev)
        t = avg_us(lambda: q.branch_gemm(A, 4, Wf, 6, 512, scale=sd))
        rows.append({"layer": "fc 512->1000", "times_in_network": 1, "W6A4": True, "out": "32x1000", "us": round(t, 1),
                     "effective_GOPS": round(2.0 * Nb * 1000 * 512 / t / 1e3, 1),
                     "frac_of_lane_op_peak": round(2.0 * 24 * Nb * 1000 * 16 / (t * 1e-6) / PEAK_LANE_OPS, 3),
                     "note": "launch-latency bound at this size"})
        total_us += t
        total_ops += 2.0 * Nb * 1000 * 512
        total_lane += 2.0 * 24 * Nb * 1000 * 16
        res = {"metric": "effective quantized GOPS over every convolution and the FC layer of the mixed-precision ResNet-18 "
                         "(sum of the layers' times, each timed on its own)",
               "value": round(total_ops / total_us / 1e3, 1), "unit": "GOPS", "ms_per_step": round(total_us / 1e3, 4),
               "roofline": {"bound": "alu", "kernel": "all branch kernels of the network", "achieved": round(total_lane / (total_us * 1e-6) / 1e12, 3),
                            "peak": round(PEAK_LANE_OPS / 1e12, 3), "unit": "Tlane-op/s",
                            "frac": round(total_lane / (total_us * 1e-6) / PEAK_LANE_OPS, 4), "traffic": None}}
    else:
        cases = [("ResNet stem 7x7 stride 2, 3->64, 224^2, W2A8", 32, 224, 224, 3, 64, 8, 2, 7, 7, 2, 3, 1, False),
                 ("3x3 stride 2, 128->128, 56^2, W2A2", 32, 56, 56, 128, 128, 2, 2, 3, 3, 2, 1, 1, False),
                 ("1x1 stride 2, 256->512, 56^2, W2A2", 32, 56, 56, 256, 512, 2, 2, 1, 1, 2, 0, 1, False),
                 ("1x1 stride 1, 256->64, 56^2, W2A2", 32, 56, 56, 256, 64, 2, 2, 1, 1, 1, 0, 1, False),
                 ("3x3 stride 1, 64->64, 56^2, W2A2 (general kernel kept on the headline shape)", 32, 56, 56, 64, 64, 2, 2, 3, 3, 1, 1, 1, False),
                 ("3x3 stride 1, 64->64, 56^2, W2A2 (as called: handed to the 3x3 kernel)", 32, 56, 56, 64, 64, 2, 2, 3, 3, 1, 1, 1, False),
                 ("3x3 dilation 2, 256->256, 33^2, W3A4 (general kernel kept)", 16, 33, 33, 256, 256, 4, 3, 3, 3, 1, 2, 2, False),
                 ("3x3 dilation 2, 256->256, 33^2, W3A4", 16, 33, 33, 256, 256, 4, 3, 3, 3, 1, 2, 2, False),
                 ("3x3 dilation 4, 512->512, 17^2, W2A4", 16, 17, 17, 512, 512, 4, 2, 3, 3, 1, 4, 4, False),
                 ("5x5 stride 1, 128->128, 28^2, W2A4", 32, 28, 28, 128, 128, 4, 2, 5, 5, 1, 2, 1, False),
                 ("5x5 stride 1, 64->64, 56^2, W2A4", 16, 56, 56, 64, 64, 4, 2, 5, 5, 1, 2, 1, False),
                 ("5x5 stride 1, 96->96, 28^2, W2A2 (half of the second 64-filter tile is idle)", 32, 28, 28, 96, 96, 2, 2, 5, 5, 1, 2, 1, False),
                 ("4x4 stride 2 transposed, 256->128, 28^2, W2A2", 16, 28, 28, 256, 128, 2, 2, 4, 4, 2, 1, 1, True)]
        cases.insert(1, ("ResNet stem 7x7 stride 2, 3->64, 224^2, W2A8, row-dense input", 32, 224, 224, 3, 64, 8, 2,
                         7, 7, 2, 3, 1, False))
        if args.only:
            cases = [c for c in cases if args.only in c[0]]
            if not cases:
                raise SystemExit("--only %r matches no layer of the suite" % args.only)
        for (label, Nb, H, W, C, Cout, ab, wb, KH, KW, st, pd, dl, tr) in cases:
            Cw = (C + 31) // 32
            dense = label.endswith("row-dense input")
            if dense:                                  # one packed row per image row, W*C bits (tail bits zero)
                Rw = (W * C + 31) // 32
                Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (Nb * H, ab, Rw), dtype=torch.int32, device=dev)
                if (W * C) % 32:
                    Xp[:, :, -1] &= (1 << ((W * C) % 32)) - 1
            else:
                Xp = torch.randint(-2 ** 31, 2 ** 31 - 1, (Nb * H * W, ab, Cw), dtype=torch.int32, device=dev)
                if C < 32:
                    Xp &= (1 << C) - 1
            Wp = torch.randint(0, 1 << min(C, 30), (Cout, KH * KW, wb, Cw), dtype=torch.int32, device=dev)
            sd = torch.rand(Cout, device=dev)
            geo = q.conv_geometry(KH, KW, stride=st, pad=pd, dilation=dl, transposed=tr, dense_rows=dense)
            Ho, Wo = q.conv2d_general_output_size(H, W, geo)
            q.tune(general_only=1 if "general kernel kept" in label else 0)
            t = avg_us(lambda: q.conv2d_general(Xp, ab, Wp, wb, Nb, H, W, C, Cout, geo, scale=sd))
            q.tune(general_only=0)
            taps = KH * KW / (st * st if tr else 1)
            ops = 2.0 * Nb * Ho * Wo * Cout * taps * C
            # (output pixel, tap) pairs that meet the image: the products the kernel forms
            tap_pixels = Nb * axis_taps(H, Ho, KH, st, pd, dl, tr) * axis_taps(W, Wo, KW, st, pd, dl, tr)
            rows.append({"layer": label, "out": "%dx%d" % (Ho, Wo), "us": round(t, 1), "effective_GOPS": round(ops / t / 1e3, 1),
                         # word-per-tap lane-ops; not meaningful on the packed-window path (few channels)
                         "frac_of_lane_op_peak": None if C < 32 else round(
                             2.0 * ab * wb * tap_pixels * Cout * Cw / (t * 1e-6) / PEAK_LANE_OPS, 3),
                         "frac_if_padded_taps_counted": None if C < 32 else round(
                             2.0 * ab * wb * Nb * Ho * Wo * Cout * taps * Cw / (t * 1e-6) / PEAK_LANE_OPS, 3)})
            del Xp, Wp
        res = {"metric": "effective quantized GOPS of qnn_conv2d_general, first listed layer", "value": rows[0]["effective_GOPS"],
               "unit": "GOPS"}
    res.update({"n_gpus": 1, "steps": steps, "warmup": warmup, "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "u32", "data": "synthetic", "config": {"workload": name, "results": rows}})
    print(json.dumps(res))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="resnet18_s1",
                    choices=["resnet18_s1", "resnet50_s3", "fc4096", "gemm64", "gemm8192", "vgg16_stack",
                             "vgg16_stack_fused", "hbm_kernels", "conv_geometries", "resnet18_mixed", "backward_products"])
    ap.add_argument("--bits", type=int, default=None,
                    help="gemm8192 only: activation = weight bit width (1..6 in the paper's sweep; default 2)")
    ap.add_argument("--batch", type=int, default=None,
                    help="resnet18_s1 / resnet50_s3 only: run the same layer on this many images instead of the "
                         "configuration's batch (a side measurement: how much of a launch is fixed cost)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None, metavar="TEXT",
                    help="conv_geometries: time only the layers whose label contains TEXT (for counter runs on one kernel)")
    ap.add_argument("--graph", action="store_true",
                    help="additionally capture one step into a HIP graph and report the time per replay "
                         "(config.graph_ms_per_step); the headline value stays the eagerly launched step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain device copy of 256 MiB (a kernel of known HBM traffic) "
                         "so that a counter run can be scaled against it")
    ap.add_argument("--record-traffic", nargs=4, metavar=("KEY", "KERNEL", "FETCH_CSV", "WRITE_CSV"),
                    help="no GPU: turn two rocprofv3 --pmc counter CSVs (FETCH_SIZE, WRITE_SIZE; runs made with "
                         "--copy-calibration) into the entry KEY of profiles/traffic.json, which roofline.traffic reads")
    ap.add_argument("--wave-trace", action="store_true",
                    help="additionally run ONE launch of the branch kernel with the per-wavefront trace "
                         "(qnn_set_wave_trace) and report config.wave_trace: wavefronts per SIMD, the SIMDs' "
                         "active windows in shader cycles and the shader clock during the kernel")
    args = ap.parse_args()
    if args.record_traffic:
        return record_traffic(args.record_traffic)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the path on ONE GPU only (the path shards over the batch "
              "with no communication, so a second GPU would run the same kernel on its own share); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    name = args.workload
    fused = name == "vgg16_stack_fused"
    if fused:
        name = "vgg16_stack"
    big = name in ("vgg16_stack", "gemm8192")
    steps = args.steps if args.steps is not None else (20 if big else 200)
    warmup = args.warmup if args.warmup is not None else (3 if big else 20)

    import numpy as np
    import torch
    from paper_2106_09886_amd import binding as q, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    L = q.lib()                                   # raises if the HIP library is not built
    dev = torch.device("cuda:0")
    peak, peak_from = device_peak(q)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())

    if args.copy_calibration:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def check(st):
        assert st == 0, L.qnn_status_string(st)

    if name in ("hbm_kernels", "conv_geometries", "resnet18_mixed", "backward_products"):
        return side_suites(name, args, steps, warmup, torch, np, q, dev)

    cpu = cpu1 = None
    if name == "vgg16_stack":
        w = inputs.VGG16
        X0, layers = inputs.make_stack(w)
        Nb, H, W, C = X0.shape
        x0 = torch.from_numpy(X0).to(dev)
        plan, ops, lane_ops, keep = [], 0.0, 0.0, []

        def kwords(c):
            """32-bit words per plane of one output pixel's K axis: nine per-tap runs, or the single
            word of the few-channel first layer (9 * c <= 32 bits)."""
            return 1 if 9 * c <= 32 else 9 * ((c + 31) // 32)

        def layer_lane_ops(ab, h, wd, c, cout):
            """xor + popcount per word, branch and tap that lies inside the image (the few-channel first
            layer works on one word per plane and pixel whatever the border)."""
            if 9 * c <= 32:
                return 2.0 * ab * w.wb * Nb * h * wd * cout
            return 2.0 * ab * w.wb * conv_tap_pixels(Nb, h, wd) * cout * ((c + 31) // 32)

        h, wd, c = H, W, C
        planes_in = torch.empty((Nb * h * wd, w.ab_first, 1), dtype=torch.int32, device=dev)
        first_planes = planes_in
        for l, (Wt, s, pool) in enumerate(layers, start=1):
            cout = Wt.shape[0]
            ab = w.ab_first if l == 1 else w.ab
            Wp = q.encode_pack(torch.from_numpy(Wt.reshape(cout * 9, c)).to(dev), w.wb)
            sd = torch.from_numpy(s).to(dev)
            acc = torch.empty((Nb, h, wd, cout), dtype=torch.int32, device=dev)
            out = torch.empty((Nb, h, wd, cout), dtype=torch.float32, device=dev)
            ho, wo = (h // 2, wd // 2) if pool else (h, wd)
            planes_out = torch.empty((Nb * ho * wo, w.ab, (cout + 31) // 32), dtype=torch.int32, device=dev)
            # fused variant: planes before pooling (the partial sums of multi-pass layers live in `acc`)
            planes_mid = (torch.empty((Nb * h * wd, w.ab, (cout + 31) // 32), dtype=torch.int32, device=dev)
                          if (fused and pool) else planes_out)
            plan.append((ab, p(planes_in), p(Wp), h, wd, c, cout, p(acc), p(sd), p(out), 1 if pool else 0,
                         p(planes_out), p(planes_mid), acc.numel() * 4))
            keep.append((Wp, sd, acc, out, planes_in, planes_out, planes_mid))
            ops += 2.0 * Nb * h * wd * cout * 9 * c
            lane_ops += layer_lane_ops(ab, h, wd, c, cout)
            planes_in, h, wd, c = planes_out, ho, wo, cout
        pX, pF = p(x0), p(first_planes)

        ws_bytes = int(L.qnn_conv2d_im2col_workspace_bytes(Nb, H, W, C, w.ab_first))
        assert ws_bytes <= first_planes.numel() * 4

        def pack():
            pass                                  # the first layer packs inside qnn_conv2d_im2col

        ws1 = None
        if fused:
            ws1_bytes = int(L.qnn_conv2d_im2col_requant_workspace_bytes(Nb, H, W, C, w.ab_first, layers[0][0].shape[0]))
            ws1 = torch.empty(ws1_bytes, dtype=torch.uint8, device=dev)
        pW1 = p(ws1)

        def layer(i):
            """Every launch of layer i (product, re-encoding, pooling)."""
            ab, pin, pw, h, wd, c, cout, pa, ps, po, pool, pout, pmid, accb = plan[i]
            if fused:
                if i == 0:
                    check(L.qnn_conv2d_im2col_requant(pX, 2, ab, pw, w.wb, Nb, h, wd, c, cout, ps, w.ab, pmid, None,
                                                      None, pW1, ws1_bytes, stream))
                else:
                    check(L.qnn_conv2d_packed_requant(pin, ab, pw, w.wb, Nb, h, wd, c, cout, ps, w.ab, pmid, None,
                                                      None, pa, accb, stream))
                if pool:
                    check(L.qnn_maxpool2x2_planes(pmid, Nb, h, wd, cout, w.ab, pout, stream))
            else:
                if i == 0:
                    check(L.qnn_conv2d_im2col(pX, 2, ab, pw, w.wb, Nb, h, wd, c, cout, pa, ps, po, pF, ws_bytes,
                                              stream))
                else:
                    check(L.qnn_conv2d_packed(pin, ab, pw, w.wb, Nb, h, wd, c, cout, pa, ps, po, stream))
                check(L.qnn_requant_pack(po, Nb, h, wd, cout, pool, w.ab, None, pout, stream))

        def branch():
            for i in range(len(plan)):
                layer(i)

        def per_layer_table():
            """Each layer on its own, K back-to-back repetitions (inputs are whatever the last full
            pass left in the buffers: the kernels' cost does not depend on the data)."""
            rows_ = []
            for i, (ab, _, _, h, wd, c, cout, *_rest) in enumerate(plan):
                us = timed_regions(torch, lambda i=i: layer(i), steps, min_samples=40, min_ms=20.0)["median"]
                lo = layer_lane_ops(ab, h, wd, c, cout)
                rows_.append({"layer": i + 1, "shape": "%dx%dx%d -> %d" % (h, wd, c, cout), "us": round(us, 1),
                              "frac_of_lane_op_peak": round(lo / (us * 1e-6) / PEAK_LANE_OPS, 3)})
            return rows_

        desc = ("vgg16_stack: 13 chained 3x3 conv layers, batch %d, %dx%dx%d input, W%dA%d (first layer A%d), "
                "2x2 max-pool after each block, re-encode + pack between layers"
                % (Nb, H, W, C, w.wb, w.ab, w.ab_first))
        kernel_name = "13 x (conv_kernel + requant_pack_kernel); lane-ops of the conv kernels only"
        B = None
        outputs = "int32 + fp32 per layer"
        if fused:
            desc += "; fused kernels: only bit planes travel between layers"
            kernel_name = "13 x fused conv_kernel (+ 5 x pool_planes_kernel); lane-ops of the conv kernels only"
            outputs = "bit planes of the next layer only"
    else:
        w = inputs.WORKLOADS[name]
        if name == "gemm8192" and args.bits is not None:
            w = inputs.with_bits(w, args.bits)
        is_conv = hasattr(w, "Cout")
        if args.batch is not None:
            if not is_conv or args.batch < 1:
                print("bench.py: --batch applies to the convolution workloads", file=sys.stderr)
                return 2
            w = w._replace(Nb=args.batch, name="%s_batch%d" % (w.name, args.batch))
        if is_conv:
            X, Wt, s = inputs.make_conv(w)
            rows, N, K, Kw = w.Nb * w.H * w.W, w.Cout, 9 * w.C, 9 * ((w.C + 31) // 32)
            kin, kbits = w.C, (w.C + 31) // 32
            Wp = q.encode_pack(torch.from_numpy(Wt.reshape(w.Cout * 9, w.C)).to(dev), w.wb)
            shape = (w.Nb, w.H, w.W, w.Cout)
        else:
            X, Wm, s = inputs.make_gemm(w)
            rows, N, K, Kw = w.M, w.N, w.K, (w.K + 31) // 32
            kin, kbits = w.K, Kw
            Wp = q.encode_pack(torch.from_numpy(np.ascontiguousarray(Wm.T)).to(dev), w.wb)
            shape = (w.M, w.N)
        Xd = torch.from_numpy(X).to(dev)
        B = w.ab * w.wb
        sd = torch.from_numpy(s).to(dev) if s is not None else None
        acc = torch.empty(shape, dtype=torch.int32, device=dev)
        out = torch.empty(shape, dtype=torch.float32, device=dev) if s is not None else None
        planes = torch.empty((rows, w.ab, kbits), dtype=torch.int32, device=dev)
        pX, pW, pS, pA, pO, pP = p(Xd), p(Wp), p(sd), p(acc), p(out), p(planes)
        esz = Xd.element_size()

        def pack():
            check(L.qnn_encode_pack(pX, esz, rows, kin, w.ab, pP, None, 0, stream))

        # "cold" variant: rotate through more than 512 MB of distinct operand/output buffers so that
        # no launch finds its data in the last-level cache
        set_bytes = planes.numel() * 4 + acc.numel() * 4 * (2 if out is not None else 1)
        n_sets = min(64, max(2, -(-(600 << 20) // set_bytes)))
        cold_sets, cold_i = [], [0]
        if set_bytes * n_sets < (8 << 30):
            for _ in range(n_sets):
                cp, ca = planes.clone(), torch.empty_like(acc)
                co = torch.empty_like(out) if out is not None else None
                cold_sets.append((cp, ca, co, p(cp), p(ca), p(co)))

        if is_conv:
            def branch():
                check(L.qnn_conv2d_packed(pP, w.ab, pW, w.wb, w.Nb, w.H, w.W, w.C, w.Cout, pA, pS, pO, stream))

            def branch_cold():
                _, _, _, cP, cA, cO = cold_sets[cold_i[0] % n_sets]
                cold_i[0] += 1
                check(L.qnn_conv2d_packed(cP, w.ab, pW, w.wb, w.Nb, w.H, w.W, w.C, w.Cout, cA, pS, cO, stream))
            desc = "%s: 3x3 conv NHWC %dx%dx%dx%d -> %d filters, W%dA%d (M=%d, N=%d, K=%d)" % (
                w.name, w.Nb, w.H, w.W, w.C, w.Cout, w.wb, w.ab, rows, N, K)
            kernel_name = "conv_kernel (branch convolution)"
        else:
            def branch():
                check(L.qnn_branch_gemm(pP, w.ab, pW, w.wb, w.M, w.N, w.K, pA, pS, pO, stream))

            def branch_cold():
                _, _, _, cP, cA, cO = cold_sets[cold_i[0] % n_sets]
                cold_i[0] += 1
                check(L.qnn_branch_gemm(cP, w.ab, pW, w.wb, w.M, w.N, w.K, cA, pS, cO, stream))
            desc = "%s: GEMM C[%dx%d] = A[%dx%d] . W[%dx%d], W%dA%d" % (
                w.name, w.M, w.N, w.M, w.K, w.K, w.N, w.wb, w.ab)
            kernel_name = "gemm_kernel (branch GEMM)"
        ops = 2.0 * rows * N * K                      # effective quantized operations per step
        # xor + popcount-accumulate per 32-bit word and branch; a convolution forms no product for a
        # tap outside the image, so only (pixel, tap) pairs inside it count
        lane_ops_padded = 2.0 * B * rows * N * Kw
        lane_ops = (2.0 * B * conv_tap_pixels(w.Nb, w.H, w.W) * N * kbits) if is_conv else lane_ops_padded
        outputs = "int32" + (" + fp32 scaled" if s is not None else "")

        cpu_rows = rows if rows * N * K <= 2e10 else max(1, int(2e10 / (N * K)))   # bound the CPU work
        cpu_ops = ops * cpu_rows / rows

        def cpu():
            import oracle
            if is_conv:
                o = oracle.conv3x3(X.astype(np.int16), Wt.astype(np.int16))
            else:
                o = oracle.gemm(X[:cpu_rows].astype(np.int16), Wm.astype(np.int16))
            if s is not None:
                oracle.scale_f64(o, s)

        # one-thread sample: about 1.5e9 multiply-adds (whole images / whole rows)
        if is_conv:
            n1 = max(1, min(w.Nb, int(1.5e9 / (w.H * w.W * N * K))))
            cpu1_sample = "first %d of %d images" % (n1, w.Nb)
        else:
            n1 = max(1, min(rows, int(1.5e9 / (N * K))))
            cpu1_sample = "first %d of %d rows" % (n1, rows)

        def cpu1():
            import oracle
            if is_conv:
                o = oracle.conv3x3(X[:n1].astype(np.int16), Wt.astype(np.int16))
                done = 2.0 * n1 * w.H * w.W * N * K
            else:
                o = oracle.gemm(X[:n1].astype(np.int16), Wm.astype(np.int16))
                done = 2.0 * n1 * N * K
            if s is not None:
                oracle.scale_f64(o, s)
            return done

    def step():
        pack()
        branch()

    # Untimed: bring the device to its steady clocks first (the shader clock takes tens of
    # milliseconds of load to settle; a short run right after start-up measures the ramp), then the
    # W warm-up steps the caller asked for.
    t_end = time.time() + 0.25
    while time.time() < t_end:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed regions of exactly K steps each, repeated until >= 100 steps and >= 50 ms are on
    # record; the reported time per step is the median region (min and mean beside it)
    t_step = timed_regions(torch, step, steps)
    ms_per_step = t_step["median"] / 1e3
    # ---- each kernel on its own, same protocol: regions of K back-to-back launches between one pair
    # of events on the launch stream (launch duration of that kernel, operands resident)
    t_branch = timed_regions(torch, branch, steps)
    branch_us = t_branch["median"]
    pack_us = timed_regions(torch, pack, steps, min_ms=10.0)["median"]
    cold_us = None
    if name != "vgg16_stack" and cold_sets:
        pack()                                    # planes of every set hold the packed activations
        for cs in cold_sets:
            cs[0].copy_(planes)
        cold_us = timed_regions(torch, branch_cold, max(steps, n_sets), min_ms=10.0)["median"]

    # comparison line (GEMM workloads with codes that fit int8): the same decoded product on the
    # int8 matrix cores, operands arranged once beforehand
    compare = compare_dot = None
    if name in ("gemm8192", "fc4096") and w.ab <= 7 and w.wb <= 7:
        Aa = q.compare_mfma_arrange(Xd)
        Wa = q.compare_mfma_arrange(torch.from_numpy(np.ascontiguousarray(Wm.T)).to(dev))
        pAa, pWa = p(Aa), p(Wa)

        def mfma():
            check(L.qnn_compare_mfma_gemm(pAa, pWa, w.M, w.N, w.K, pA, stream))
        mfma_us = timed_regions(torch, mfma, steps, min_samples=40, min_ms=20.0)["median"]
        compare = {"what": "same decoded int8 product on v_mfma_i32_32x32x32_i8 (comparison line, untuned kernel)",
                   "us": round(mfma_us, 2), "GOPS": round(ops / (mfma_us * 1e-6) / 1e9, 1),
                   "frac_of_int8_mfma_peak_5000_TOPS": round(ops / (mfma_us * 1e-6) / 5.0e15, 4)}
        # second comparison line: the packed int8 dot product of the vector ALU (v_dot4_i32_i8)
        if w.K % 4 == 0:
            Wtd = torch.from_numpy(np.ascontiguousarray(Wm.T)).to(dev)
            pXc, pWc = p(Xd), p(Wtd)

            def dot4():
                check(L.qnn_compare_dot4_gemm(pXc, pWc, w.M, w.N, w.K, pA, stream))
            dot_us = timed_regions(torch, dot4, steps, min_samples=40, min_ms=20.0)["median"]
            compare_dot = {"what": "same decoded int8 product with v_dot4_i32_i8 (comparison line)",
                           "us": round(dot_us, 2), "GOPS": round(ops / (dot_us * 1e-6) / 1e9, 1)}
        branch()                                  # leave the branch result in the output buffer

    layers_table = per_layer_table() if name == "vgg16_stack" else None
    wave_trace = None
    if args.wave_trace and name != "vgg16_stack":
        wave_trace = traced_launch(torch, np, q, branch)

    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stream = ctypes.c_void_p(side.cuda_stream)      # the closures launch on `stream`
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            step()
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        graph_ms = timed_regions(torch, gr.replay, steps)["median"] / 1e3

    value = ops / (ms_per_step * 1e-3) / 1e9
    achieved = lane_ops / (branch_us * 1e-6)
    rnd = lambda t: {k: (round(v, 3) if isinstance(v, float) else v) for k, v in t.items()}
    traffic_key = ("gemm8192/%d" % (args.bits or 2)) if name == "gemm8192" else name
    res = {
        "metric": "effective quantized GOPS (2*M*N*K/s), whole step: pack activations + branch product + scale",
        "value": round(value, 1),
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {
            "workload": desc,
            "branches": B,
            "arithmetic": "xor + popcount on u32 bit-plane words, int32 accumulation, one fp32 multiply per output",
            "weights": "packed once before the timed region (static parameters)",
            "outputs": outputs,
            "bit_ops_per_s": round(B * ops / (ms_per_step * 1e-3), 1) if B else None,
            "timing": "regions of exactly `steps` steps between two events on the launch stream, each bracketed by "
                      "synchronisations (3 untimed steps lead in), repeated until >= 100 steps and >= 50 ms; "
                      "ms_per_step and value are the median region",
            "step_us": rnd(t_step),
            "branch_kernel_us_stats": rnd(t_branch),
            "pack_kernel_us": round(pack_us, 2),
            "branch_kernel_us": round(branch_us, 2),
            "branch_kernel_cold_us": None if cold_us is None else round(cold_us, 2),
            "branch_kernel_effective_GOPS": round(ops / (branch_us * 1e-6) / 1e9, 1),
            "comparison_int8_mfma": compare,
            "comparison_int8_dot4": compare_dot,
            "graph_ms_per_step": None if graph_ms is None else round(graph_ms, 5),
            "wave_trace": wave_trace,
            "layers": layers_table,
        },
        "roofline": {
            "bound": "alu",
            "kernel": kernel_name,
            "achieved": round(achieved / 1e12, 3),
            "peak": round(peak / 1e12, 3),
            "unit": "Tlane-op/s",
            "peak_from": peak_from,
            "frac": round(achieved / peak, 4),
            "lane_ops_per_launch": lane_ops,
            "counts": "xor + popcount per 32-bit word, branch and tap inside the image (taps in the zero padding "
                      "are skipped, not computed)",
            "frac_if_padded_taps_counted": (round(lane_ops_padded / (branch_us * 1e-6) / peak, 4)
                                            if name != "vgg16_stack" else None),
            "traffic": stored_traffic(traffic_key) if args.batch is None else None,
            "traffic_from": "profiles/traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a device copy; "
                            "null when the kernel sources differ from the ones it was measured on)",
        },
    }

    if not args.no_cpu_baseline and cpu is not None:
        import oracle
        oracle.build(force=False)
        reps, t0 = 0, time.time()
        while True:
            cpu()
            reps += 1
            if time.time() - t0 > 10.0 or reps >= 200:
                break
        dt = (time.time() - t0) / reps
        if name == "vgg16_stack":
            cpu_ops, cpu_rows, rows = ops, 1, 1
        res["cpu_baseline"] = {
            "value": round(cpu_ops / dt / 1e9, 2),
            "unit": "GOPS",
            "cores": oracle.threads(),
            "kind": "oracle",
            "cpu_model": cpu_model(),
            "sample": ("full workload" if cpu_rows == rows else "first %d of %d rows" % (cpu_rows, rows))
                      + ", plain int64 product + float64 scale, mean of %d passes" % reps,
        }
        if cpu1 is not None:
            # the same oracle on ONE thread, on a smaller sample (about 5 s of work)
            try:
                gomp = ctypes.CDLL("libgomp.so.1")
                gomp.omp_set_num_threads(1)
                reps1, t0 = 0, time.time()
                while True:
                    ops1 = cpu1()
                    reps1 += 1
                    if time.time() - t0 > 5.0 or reps1 >= 50:
                        break
                dt1 = (time.time() - t0) / reps1
                gomp.omp_set_num_threads(oracle.threads())
                res["cpu_baseline"]["one_thread"] = {"value": round(ops1 / dt1 / 1e9, 2), "unit": "GOPS", "cores": 1,
                                                     "sample": cpu1_sample + ", mean of %d passes" % reps1}
            except OSError:
                pass
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
