#!/usr/bin/env python3
"""Benchmark of the {-1,+1} multi-branch binary product hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic activations that are
already resident in HBM: encode + pack the activation codes, then the implicit-im2col
branch convolution with fused weighted accumulation and fp32 scale epilogue (int32 and fp32
outputs).  The weights are static parameters and are packed once before the timed region.

Prints ONE JSON line.  `value` is the effective quantized throughput 2*M*N*K / t_step in
GOPS (M output pixels, N filters, K = 9*C).  `roofline` prices the dominant kernel (the
branch convolution) against the chip's integer vector-ALU rate; `cpu_baseline` is the CPU
oracle timed on the host cores of this machine.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18_s1]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X: 256 compute units x 64 vector lanes x 2.4 GHz = one 32-bit integer lane-op per lane
# and clock (v_xor_b32, v_bcnt_u32_b32 are full rate, not packed).
PEAK_LANE_OPS = 256 * 64 * 2.4e9

# HBM bytes per launch of the dominant kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/ (scaled by the device-copy calibration described there).
MEASURED_TRAFFIC = {"resnet18_s1": 61.6e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18_s1", choices=["resnet18_s1", "resnet50_s3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain device copy of 256 MiB (a kernel of known HBM traffic) "
                         "so that a counter run can be scaled against it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the path on ONE GPU only (it shards over the batch with "
              "no communication; see DESIGN.md); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2106_09886_amd import binding as q, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    L = q.lib()                                   # raises if the HIP library is not built
    w = inputs.WORKLOADS[args.workload]
    X, Wt, s = inputs.make_conv(w)
    rows = w.Nb * w.H * w.W
    K = 9 * w.C
    Cw = (w.C + 31) // 32
    B = w.ab * w.wb

    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    Wp = q.encode_pack(torch.from_numpy(Wt.reshape(w.Cout * 9, w.C)).to(dev), w.wb)   # once: static weights
    sd = torch.from_numpy(s).to(dev) if s is not None else None
    acc = torch.empty((w.Nb, w.H, w.W, w.Cout), dtype=torch.int32, device=dev)
    out = torch.empty((w.Nb, w.H, w.W, w.Cout), dtype=torch.float32, device=dev) if s is not None else None
    planes = torch.empty((rows, w.ab, Cw), dtype=torch.int32, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    pX, pW, pS, pA, pO, pP = p(Xd), p(Wp), p(sd), p(acc), p(out), p(planes)
    esz = Xd.element_size()

    def pack():
        st = L.qnn_encode_pack(pX, esz, rows, w.C, w.ab, pP, None, 0, stream)
        assert st == 0, st

    def conv():
        st = L.qnn_conv2d_packed(pP, w.ab, pW, w.wb, w.Nb, w.H, w.W, w.C, w.Cout, pA, pS, pO, stream)
        assert st == 0, st

    def step():
        pack()
        conv()

    if args.copy_calibration:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps

    # ---- each kernel on its own: K back-to-back launches between one pair of events on the
    # launch stream (average launch duration of that kernel, input planes resident)
    def timed(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(args.steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.steps * 1e3

    conv_us = timed(conv)
    pack_us = timed(pack)

    ops = 2.0 * rows * w.Cout * K                       # effective quantized operations per step
    lane_ops = 2.0 * B * rows * w.Cout * 9 * Cw         # xor + popcount-accumulate per 32-bit word and branch
    value = ops / (ms_per_step * 1e-3) / 1e9
    achieved = lane_ops / (conv_us * 1e-6)

    res = {
        "metric": "effective quantized GOPS (2*M*N*K/s), whole step: pack activations + branch conv + scale",
        "value": round(value, 1),
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate, fp32 scale",
        "data": "synthetic",
        "config": {
            "workload": "%s: 3x3 conv NHWC %dx%dx%dx%d -> %d filters, W%dA%d (M=%d, N=%d, K=%d)"
                        % (w.name, w.Nb, w.H, w.W, w.C, w.Cout, w.wb, w.ab, rows, w.Cout, K),
            "branches": B,
            "weights": "packed once before the timed region (static parameters)",
            "outputs": "int32" + (" + fp32 scaled" if s is not None else ""),
            "bit_ops_per_s": round(2.0 * B * rows * w.Cout * K / (ms_per_step * 1e-3), 1),
            "pack_kernel_us": round(pack_us, 2),
            "branch_kernel_us": round(conv_us, 2),
            "branch_kernel_effective_GOPS": round(ops / (conv_us * 1e-6) / 1e9, 1),
        },
        "roofline": {
            "bound": "alu",
            "kernel": "conv_kernel (branch convolution)",
            "achieved": round(achieved / 1e12, 3),
            "peak": round(PEAK_LANE_OPS / 1e12, 3),
            "unit": "Tlane-op/s",
            "peak_from": "256 CU x 64 lanes x 2.4 GHz, one 32-bit integer vector op per lane and clock",
            "frac": round(achieved / PEAK_LANE_OPS, 4),
            "traffic": MEASURED_TRAFFIC.get(w.name),
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        oracle.build(force=False)
        X16, W16 = X.astype(np.int16), Wt.astype(np.int16)
        reps, t0 = 0, time.time()
        while True:
            o = oracle.conv3x3(X16, W16)
            if s is not None:
                oracle.scale_f64(o, s)
            reps += 1
            if time.time() - t0 > 1.5 or reps >= 20:
                break
        dt = (time.time() - t0) / reps
        res["cpu_baseline"] = {
            "value": round(ops / dt / 1e9, 2),
            "unit": "GOPS",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "full workload (%d images), direct int64 convolution + float64 scale, mean of %d passes"
                      % (w.Nb, reps),
        }
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
