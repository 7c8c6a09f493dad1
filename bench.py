#!/usr/bin/env python3
"""Benchmark of the nested-integer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step is one pass of the whole path over one batch of the ResNet-18-shaped 3x3
convolution (batch 32, 56x56x64 -> 64, INT8 nesting INT6): decompose-and-pack the layer's
INT8 weights, page the lower-bit page out, copy it back in from pinned host memory, run the
part-bit convolution, then the full-bit convolution (which waits for the page).  By default
the page travels on the compute stream: it is 9 KiB, its copy takes 4 us, and handing work
between two hardware queues costs more than that per hand-over; --side-stream copies it on
a second stream concurrently with the part-bit convolution instead.  Inputs are resident in
HBM before the clock starts.  Prints one JSON line; see the design doc for how the roofline
figures are derived.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E
MFMA_INT8_PEAK_TOPS = 5000.0

# HBM bytes per launch of the full-bit convolution from the FETCH_SIZE and WRITE_SIZE counters of a
# profiling run, each scaled by what the same counter read for a 64 MiB streaming kernel (factors
# 1.999 and 1.000).  They describe the kernel as it was when they were taken: `sources` is the
# digest of the kernel's source files at that time, and a different digest reports no traffic.
TRAFFIC = dict(fetch_bytes=int(6430.6 * 1024 * 1.999), write_bytes=int(25088.0 * 1024 * 1.000),
               sources="22457a7f140f36d6")
KERNEL_SOURCES = ("nq_conv_rowstream.h", "nq_epilogue.h", "nq_codec.h", "nq_gemm_params.h")


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2506_17870_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def cpu_baseline(inputs, cfg_conv, w_int, scale, x_all, s_a, bias, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample (whole images) of the same workload."""
    import numpy as np
    from oracle import nq_oracle as oracle
    n, l = cfg_conv["n_bits"], cfg_conv["l_bits"]
    Cout, Cin, KH, KW = cfg_conv["Cout"], cfg_conv["Cin"], cfg_conv["KH"], cfg_conv["KW"]
    K = KH * KW * Cin
    ops_img = 2 * 2 * cfg_conv["H"] * cfg_conv["W"] * Cout * K       # full-bit + part-bit, stride 1 pad 1

    def run(nimg):
        t0 = time.perf_counter()
        ph, pl = oracle.decompose_pack(w_int, n, l)
        outs = []
        for pages, part_l in ((None, l), (pl, 0)):
            w = oracle.weights_from_pages(ph, pages, Cout, K, n, l).reshape(Cout, KH, KW, Cin)
            acc = oracle.conv_acc(x_all[:nimg], w, cfg_conv["stride"], cfg_conv["pad"])
            outs.append(oracle.epilogue(acc, s_a, scale, part_l_bits=part_l, bias=bias, relu=True))
        return time.perf_counter() - t0, outs

    run(1)                                                    # first call pays the library load
    nimg = x_all.shape[0]
    t, outs = run(nimg)
    total, reps = t, 1
    while total < budget_s and reps < 200:                    # repeat the batch up to the time budget
        dt, _ = run(nimg)
        total, reps = total + dt, reps + 1
    return dict(value=ops_img * nimg * reps / total / 1e12, unit="TOPS", cores=oracle.threads(), kind="oracle",
                sample=f"{reps} x the {nimg}-image batch of the same convolution (decompose+pack, part-bit, "
                       f"full-bit), {total:.1f} s, plain C loops -O2 with OpenMP"), nimg, outs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--sets", type=int, default=8, help="distinct activation/output buffer sets rotated "
                    "through, so that the working set exceeds the 256 MB Infinity Cache")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="issue every call of the timed steps from Python instead of "
                    "replaying a captured HIP graph of `sets` consecutive steps")
    ap.add_argument("--side-stream", action="store_true", help="copy the lower-bit page in on a second stream, "
                    "concurrently with the part-bit convolution (default: on the compute stream, see DESIGN.md)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path needs no exchange between GPUs; "
                 "--gpus must be 1)")

    import numpy as np
    import torch

    import paper_2506_17870_amd as nq
    from paper_2506_17870_amd import binding, inputs

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    lib = binding._lib

    c = inputs.CONV_RESNET18
    B, H, W, Cin, Cout, KH, KW = c["B"], c["H"], c["W"], c["Cin"], c["Cout"], c["KH"], c["KW"]
    n_bits, l_bits = c["n_bits"], c["l_bits"]
    h_bits = n_bits - l_bits
    K = KH * KW * Cin
    Ho, Wo = H, W
    M = B * Ho * Wo
    ops_conv = 2 * M * Cout * K

    # ---- synthetic inputs, resident before the clock starts --------------------------------
    w_int, scale = inputs.weights(Cout, K, inputs.he_sigma(K), n_bits, seed=0)
    bias = inputs.small_floats(Cout, 0.1, seed=2)
    s_a = 0.02
    cfg = nq.make_cfg(n_bits, l_bits)
    d_w_int = torch.from_numpy(w_int).cuda()
    Wn = nq.NestedWeight.from_int8(d_w_int, torch.from_numpy(scale).cuda(), cfg)
    d_bias = torch.from_numpy(bias).cuda()
    R = max(1, args.sets)
    x_host = [inputs.uniform_activations((B, H, W, Cin), seed=r) for r in range(R)]
    xs = [torch.from_numpy(x).cuda() for x in x_host]
    y_part = [torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device="cuda") for _ in range(R)]
    y_full = [torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device="cuda") for _ in range(R)]

    shape = nq.nq_conv_shape(B, H, W, Cin, Cout, KH, KW, c["stride"], c["pad"])
    epi = nq.make_epilogue(s_a, d_bias, None, 0.0, True, False, 1.0, None)
    compute = torch.cuda.current_stream()
    copy = torch.cuda.Stream() if args.side_stream else compute
    cs, ps = ctypes.c_void_p(compute.cuda_stream), ctypes.c_void_p(copy.cuda_stream)
    wref, eref, sref, cref = ctypes.byref(Wn.desc), ctypes.byref(epi), ctypes.byref(shape), ctypes.byref(cfg)
    p_w, p_hi, p_lo = ctypes.c_void_p(d_w_int.data_ptr()), ctypes.c_void_p(Wn.high.data_ptr()), \
        ctypes.c_void_p(Wn.low.data_ptr())
    p_x = [ctypes.c_void_p(t.data_ptr()) for t in xs]
    p_yp = [ctypes.c_void_p(t.data_ptr()) for t in y_part]
    p_yf = [ctypes.c_void_p(t.data_ptr()) for t in y_full]

    def step(i, ev=None):
        r = i % R
        rc = lib.nq_decompose_pack(p_w, Cout, K, cref, p_hi, p_lo, cs)          # a1 + a2
        rc |= lib.nq_page_out_low(wref, cs)                                     # a3: downgrade
        rc |= lib.nq_page_in_low(wref, ps)                                      # a4: upgrade (waits for the
                                                                                # page-out point)
        rc |= lib.nq_conv_part(p_x[r], sref, wref, eref, p_yp[r], cs)           # a6 + a7
        if ev is not None:
            lib.nq_profile_next_launch(ev[0], ev[1])                            # time stamps of this dispatch
        rc |= lib.nq_conv_full(p_x[r], sref, wref, eref, p_yf[r], cs)           # a5 + a7, waits for the page
        if rc:
            raise RuntimeError(f"libnq returned an error in step {i}")

    # One plain streaming kernel of known size (reads 64 MiB, writes 64 MiB, both initialised): the
    # yardstick the HBM byte counters of a profiling run are scaled by.
    cal_src = torch.ones(16 << 20, dtype=torch.int32, device="cuda")
    cal_dst = torch.zeros_like(cal_src)
    for _ in range(3):
        torch.add(cal_src, 1, out=cal_dst)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: K steps.  The calls of R consecutive steps (one per buffer set) are captured
    # once into a HIP graph and replayed, so the host issues one launch per R steps; K % R steps
    # left over are issued call by call.
    graph = None
    if not args.eager and args.steps >= R:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cap = torch.cuda.current_stream()
            cs_saved, ps_saved = cs, ps
            cs = ctypes.c_void_p(cap.cuda_stream)
            if not args.side_stream:
                ps = cs
            for i in range(R):
                step(i)
            cs, ps = cs_saved, ps_saved
        torch.cuda.synchronize()
    n_replay = args.steps // R if graph is not None else 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_replay):
        graph.replay()
    for i in range(n_replay * R, args.steps):
        step(i)
    t_issue = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = 2 * ops_conv * args.steps / elapsed / 1e12

    # ---- duration of the dominant kernel: the same steps once more, each full-bit convolution
    # dispatch time-stamped (begin/end of the kernel itself, what a kernel trace reports)
    n_probe = min(args.steps, 200)
    events = [(ctypes.c_void_p(nq.nq_event_create()), ctypes.c_void_p(nq.nq_event_create()))
              for _ in range(n_probe)]
    for i in range(n_probe):
        step(i, events[i])
    torch.cuda.synchronize()
    kern_ms = sorted(nq.nq_event_elapsed_ms(a, b) for a, b in events)
    for a, b in events:
        nq.nq_event_destroy(a)
        nq.nq_event_destroy(b)
    full_ms = sum(kern_ms) / len(kern_ms)
    # algorithmic bytes of one full-bit convolution launch: activations once, both packed pages once,
    # scales and bias once, fp32 outputs once
    bytes_conv_full = (M * Cin * 1 + nq.nq_packed_bytes(Cout, K, h_bits) + nq.nq_packed_bytes(Cout, K, l_bits)
                       + 2 * 4 * Cout + 4 * M * Cout)
    achieved = bytes_conv_full / (full_ms * 1e-3) / 1e9
    traffic = None
    if TRAFFIC["sources"] == kernel_sources_digest():
        traffic = TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"]
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=traffic, kernel="k_nested_conv_rowstream<6,2,full> (nq_conv_full)",
                    avg_kernel_us=1e3 * full_ms, median_kernel_us=1e3 * kern_ms[len(kern_ms) // 2],
                    algorithmic_bytes=bytes_conv_full,
                    mfma_tops=ops_conv / (full_ms * 1e-3) / 1e12,
                    mfma_frac=ops_conv / (full_ms * 1e-3) / 1e12 / MFMA_INT8_PEAK_TOPS)

    out = dict(metric="nested int8 conv TOPS (full-bit + part-bit)", value=value, unit="TOPS", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="int8", data="synthetic",
               config=dict(workload="ResNet-18-shaped 3x3 conv, stride 1 pad 1, batch 32, 56x56x64 -> 64, NHWC int8 "
                                    "activations, per-channel INT8 nesting INT6 (l=2), fp32 outputs with bias+ReLU; "
                                    "step = decompose_pack + page-out + page-in + part-bit conv + full-bit conv"
                                    + (" (page-in on a second stream)" if args.side_stream else ""),
                           buffer_sets=R, ops_per_step=2 * ops_conv,
                           host_issue_ms_per_step=1e3 * (t_issue - t0) / args.steps,
                           issue="hip graph of %d steps" % R if graph is not None else "eager"),
               roofline=roofline)

    if not args.no_cpu_baseline:
        base, nimg, outs = cpu_baseline(inputs, c, w_int, scale, x_host[0], s_a, bias)
        # the timed loop's outputs for buffer set 0 must equal the oracle's on the sampled images
        step(0)
        torch.cuda.synchronize()
        ok = (np.array_equal(y_part[0][:nimg].cpu().numpy(), outs[0]) and
              np.array_equal(y_full[0][:nimg].cpu().numpy(), outs[1]))
        if not ok:
            raise RuntimeError("bench.py: GPU outputs differ from the oracle on the sampled images")
        base["gpu_matches_oracle_on_sample"] = True
        out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()
