#!/usr/bin/env python3
"""Benchmark of the nested-integer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step is one pass of the whole path over one batch of the largest single-GPU configuration: the
ResNet-101-shaped conv/fc stack (104 convolutions + fc, 44.4 M weights, every layer INT8 nesting INT6) at
batch 128, 224 x 224 x 3 input, int8 activations.  The weights are decomposed and packed once (setup), then
every step switches the model down and up again and runs it in both modes:

    nq_page_out_low_batch   downgrade: the lower-bit pages are paged out (nothing moves)
    nq_page_in_low_batch    upgrade: 11.1 MB of lower-bit pages, one pinned host -> device copy
    part-bit forward        105 nq_conv_part / nq_gemm_part launches + pooling (never reads the pages)
    full-bit forward        105 nq_conv_full / nq_gemm_full launches + pooling (waits for the copy)

By default all of it is issued on one stream; --side-stream sends the copy over a second stream so that it
travels while the part-bit forward computes.  The step is captured once into a HIP graph and replayed, so the
host issues one launch per step.  Inputs are resident in HBM before the clock starts; the only PCIe traffic in
the timed region is the page-in, which is part of the path.  Prints one JSON line: whole-job TOPS, the roofline
of the kernel instantiation that takes the largest share of the step, sub-records for the other
configurations' dominant layers, and the CPU oracle on a reduced batch.
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

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix-core peak
RIDGE = MFMA_INT8_PEAK_TOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # op per byte above which the matrix cores bound a layer

# HBM bytes per launch of the dominant kernel from the FETCH_SIZE and WRITE_SIZE counters of a profiling run
# (scaled by what the same counters read for a plain copy kernel of known size), keyed by the kernel
# instantiation they were taken on and by a digest of the kernel's sources at that time: a different kernel or
# digest reports no traffic.
TRAFFIC = {   # profiles/gemm_big_conv3x3_b128_counters.txt: FETCH_SIZE x 1.999 KiB, WRITE_SIZE x 1.000 KiB, means per dispatch
    "k_nested_gemm_big<6,2,full,int8 out,TM=6,filter>": dict(sources="b88b875a50121b2e", fetch_bytes=14220322, write_bytes=6422528),
    "k_nested_gemm_big<6,2,part,int8 out,TM=6,filter>": dict(sources="b88b875a50121b2e", fetch_bytes=13006169, write_bytes=6422528),
}
KERNEL_SOURCES = ("nq_gemm_big.h", "nq_epilogue.h", "nq_codec.h", "nq_gemm_kernel.h")   # what k_nested_gemm_big is made of
FAMILY = {1: "k_nested_gemm", 2: "k_nested_conv_window", 3: "k_nested_conv_rowstream", 4: "k_nested_gemm_big",
          5: "k_nested_conv_smallcin", 6: "k_nested_gemm_skinny", 7: "k_nested_conv_grouped", 8: "k_nested_gemm_words", 9: "k_nested_gemm_stat"}


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2506_17870_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def forward_ops(ops, network, H, W):
    """Integer operations (2 per multiply-add) of one image's forward pass."""
    hw, macs = {0: (H, W)}, 0
    for op in ops:
        hs, ws = hw[op["src"]]
        if op["op"] == "conv":
            ho, wo = network.out_hw(hs, ws, op["k"], op["stride"], op["pad"])
            macs += ho * wo * op["cout"] * op["k"] ** 2 * op["cin"]
            hw[op["dst"]] = (ho, wo)
        elif op["op"] == "maxpool":
            hw[op["dst"]] = network.out_hw(hs, ws, op["k"], op["stride"], op["pad"])
        elif op["op"] == "avgpool":
            hw[op["dst"]] = (1, 1)
        else:
            macs += op["cin"] * op["cout"]
    return 2.0 * macs


def stamped_forward(model, binding, dx, s_x, full):
    """One eager forward with every GEMM / convolution dispatch time-stamped (begin and end of the kernel
    itself, what a kernel trace reports).  Returns one record per launch: the kernel instantiation the library
    chose, its duration, its operations and its algorithmic bytes (input once, pages once, residual once,
    output once)."""
    recs, names = [], ("nq_conv_full", "nq_conv_part", "nq_gemm_full", "nq_gemm_part")
    originals = {n: getattr(binding, n) for n in names}
    h_bits, l_bits = model.n_bits - model.l_bits, model.l_bits

    def stamped(name):
        orig = originals[name]

        def call(*a, **k):
            e0, e1 = binding.nq_event_create(), binding.nq_event_create()
            binding.nq_profile_next_launch(e0, e1)
            orig(*a, **k)
            fam, var = binding.nq_profile_last_kernel()
            conv = name.startswith("nq_conv")
            wd, epi = a[2], a[3]
            if conv:
                sh = a[1]
                ho = (sh.H + 2 * sh.pad - sh.KH) // sh.stride + 1
                wo = (sh.W + 2 * sh.pad - sh.KW) // sh.stride + 1
                m, x_bytes = sh.B * ho * wo, sh.B * sh.H * sh.W * sh.Cin
                layer = f"{sh.KH}x{sh.KW} s{sh.stride} {sh.H}x{sh.W} {sh.Cin}->{sh.Cout}"
                filt = sh.KH * sh.KW > 1 or sh.stride > 1
            else:
                m, x_bytes = a[1], a[1] * wd.K
                layer = f"fc {wd.K}->{wd.N}"
                filt = False
            out_bytes = m * wd.N * (1 if epi.out_int8 else 4)
            pages = binding.nq_packed_bytes(wd.N, wd.K, h_bits) + (binding.nq_packed_bytes(wd.N, wd.K, l_bits) if full else 0)
            byts = x_bytes + pages + out_bytes + (m * wd.N if epi.d_residual else 0) + 8 * wd.N
            if epi.d_residual:
                layer += " + residual"
            inst = FAMILY.get(fam, "?") + f"<{h_bits},{l_bits},{'full' if full else 'part'}"
            if fam == 4:
                inst += f",{'int8' if epi.out_int8 else 'fp32'} out,TM={var},{'filter' if filt else 'plain'}"
            if fam == 9:
                inst += f",{'int8' if epi.out_int8 else 'fp32'} out,K={wd.K},WN={var}"
            inst += ">"
            recs.append(dict(e=(e0, e1), inst=inst, layer=layer, ops=2.0 * m * wd.N * wd.K, bytes=byts))
        return call
    for n in names:
        setattr(binding, n, stamped(n))
    try:
        model.forward(dx, s_x, full=full)
        import torch
        torch.cuda.synchronize()
    finally:
        for n, orig in originals.items():
            setattr(binding, n, orig)
    for r in recs:
        e0, e1 = r.pop("e")
        r["us"] = binding.nq_event_elapsed_ms(e0, e1) * 1e3
        binding.nq_event_destroy(e0)
        binding.nq_event_destroy(e1)
    return recs


def cpu_baseline(model_ops, float_weights, x_float, scales, n_bits, l_bits, ops_img):
    """The CPU oracle, as it stands, on a reduced batch of the same workload (whole network, full-bit and
    part-bit forward with the same activation steps): all OpenMP threads on the first images, one thread on
    the first image.  Returns the record and the oracle's logits for the comparison with the GPU's."""
    from oracle import nq_oracle as oracle
    from oracle.nq_oracle_cnn import oracle_cnn_forward
    omp = ctypes.CDLL("libgomp.so.1")
    nthreads = oracle.threads()
    # the oracle quantises the same float draws itself (Eq. 1): weights per output channel, the input batch per tensor
    weights = [None if w is None else oracle.quantize(w[0], n_bits) + (w[1],) for w in float_weights]
    x, s_x = oracle.quantize(x_float.reshape(1, -1), 8)
    x, s_x = x.reshape(x_float.shape), float(s_x[0])

    cache = {}

    def run(nimg, threads):
        omp.omp_set_num_threads(threads)
        t0 = time.perf_counter()
        lf, _, _ = oracle_cnn_forward(model_ops, weights, x[:nimg], s_x, n_bits, l_bits, True, scales, cache)
        lp, _, _ = oracle_cnn_forward(model_ops, weights, x[:nimg], s_x, n_bits, l_bits, False, scales, cache)
        omp.omp_set_num_threads(nthreads)
        return time.perf_counter() - t0, lf, lp
    # setup, not timed (as on the GPU side): the oracle decomposes, packs and unpacks every layer's weights once
    run(1, nthreads)
    n_all = 8
    t_all, lf, lp = run(n_all, nthreads)
    t_one, _, _ = run(1, 1)
    rec = dict(value=2 * ops_img * n_all / t_all / 1e12, unit="TOPS", cores=nthreads, kind="oracle",
               sample=f"whole ResNet-101-shaped network, full-bit + part-bit forward (direct convolution loops, "
                      f"fp32 epilogue, pooling) on the first {n_all} of the batch's images with {nthreads} OpenMP "
                      f"threads: {t_all:.1f} s; plain C loops -O2; weights decomposed, packed and unpacked once before",
               single_thread=dict(value=2 * ops_img / t_one / 1e12, unit="TOPS", cores=1,
                                  sample=f"the same on the first image with one thread: {t_one:.1f} s"))
    return rec, n_all, lf, lp


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=128, help="images per step (the configuration is quoted at 128)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sub-records", action="store_true", help="skip the per-layer measurements of the other "
                    "configurations (conv 56x56x64, bottleneck 3x3, ViT MLP)")
    ap.add_argument("--eager", action="store_true", help="issue every call of the timed steps from Python instead of "
                    "replaying a captured HIP graph of one step")
    ap.add_argument("--branch-stream", action="store_true", help="issue the projection shortcut of every stage's first "
                    "block on a second stream, beside the block's main path")
    ap.add_argument("--side-stream", action="store_true", help="copy the lower-bit pages in on a second stream, "
                    "concurrently with the part-bit forward (default: on the compute stream)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (the path needs no exchange between GPUs; "
                 "--gpus must be 1)")

    import numpy as np
    import torch

    import paper_2506_17870_amd as nq
    from paper_2506_17870_amd import binding, inputs, network

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)

    # ---- synthetic model and inputs, resident before the clock starts ----------------------
    n_bits, l_bits, B, HW = 8, 2, args.batch, 224
    ops = network.resnet101_plan()
    weights = network.plan_float_weights(ops, seed=0)
    model = network.NestedCNN(ops, weights, n_bits, l_bits)          # nq_quantize + nq_decompose_pack_batch: a1 + a2, once
    x_float = inputs.gaussian_floats((B, HW, HW, 3), seed=0)
    dx, s_x = network.quantize_tensor(x_float)                       # int8 codes of the input batch, on the device
    model.allocate(B, HW, HW)
    model.calibrate(dx, float(s_x))                                   # int8 steps of the activations, once
    ops_img = forward_ops(ops, network, HW, HW)
    ops_step = 2 * ops_img * B
    low_bytes = model.low_page_bytes()

    compute = torch.cuda.Stream()
    side = torch.cuda.Stream() if args.side_stream else None
    branch = torch.cuda.Stream() if args.branch_stream else None    # the projection shortcuts of the network's blocks

    def step(st):
        model.page_out_low(st)                                       # a3: downgrade
        model.page_in_low(side if side is not None else st)          # a4: upgrade travels ...
        model.forward(dx, s_x, full=False, stream=st, branch_stream=branch)   # a6 + a7 + a8: ... while part-bit computes
        model.forward(dx, s_x, full=True, stream=st, branch_stream=branch)    # a5 + a7 + a8: waits for the pages

    with torch.cuda.stream(compute):
        for _ in range(max(args.warmup, 1)):
            step(compute)
        compute.synchronize()
        graph = None
        if not args.eager:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=compute):
                step(compute)
            graph.replay()
            compute.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            if graph is not None:
                graph.replay()
            else:
                step(compute)
        t_issue = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    elapsed = t1 - t0
    host_issue_ms = 1e3 * (t_issue - t0) / args.steps
    ms_per_step = 1e3 * elapsed / args.steps
    value = ops_step * args.steps / elapsed / 1e12

    # ---- where the step's time goes: every dispatch of one part-bit and one full-bit forward stamped ----
    torch.cuda.synchronize()
    model.page_out_low()                                    # the events of the switch recorded eagerly again:
    model.page_in_low()                                     # their last record was inside the captured step
    torch.cuda.synchronize()
    recs = []
    for rep in range(3):
        recs += stamped_forward(model, binding, dx, s_x, False) + stamped_forward(model, binding, dx, s_x, True)
    groups = {}
    for r in recs:
        g = groups.setdefault(r["inst"], dict(n=0, us=0.0, ops=0.0, bytes=0.0, layers={}))
        g["n"] += 1; g["us"] += r["us"]; g["ops"] += r["ops"]; g["bytes"] += r["bytes"]
        g["layers"][r["layer"]] = g["layers"].get(r["layer"], 0) + 1
    kern_us_step = sum(r["us"] for r in recs) / 3
    inst, g = max(groups.items(), key=lambda kv: kv[1]["us"])
    avg_us = g["us"] / g["n"]
    ops_launch, bytes_launch = g["ops"] / g["n"], g["bytes"] / g["n"]
    bound = "mfma" if ops_launch / bytes_launch > RIDGE else "hbm"
    if bound == "mfma":
        achieved, peak, unit = ops_launch / avg_us / 1e6, MFMA_INT8_PEAK_TOPS, "TOP/s"
    else:
        achieved, peak, unit = bytes_launch / avg_us / 1e3, HBM_PEAK_GBS, "GB/s"
    traffic = None
    t = TRAFFIC.get(inst)
    if t and t["sources"] == kernel_sources_digest():
        traffic = t["fetch_bytes"] + t["write_bytes"]
    roofline = dict(bound=bound, achieved=achieved, peak=peak, unit=unit, frac=achieved / peak, traffic=traffic,
                    kernel=inst, launches_per_step=g["n"] // 3, avg_kernel_us=avg_us,
                    share_of_step_kernel_time=g["us"] / 3 / kern_us_step,
                    ops_per_launch=ops_launch, algorithmic_bytes=bytes_launch,
                    layers={k: v // 3 for k, v in g["layers"].items()},
                    hbm_frac=bytes_launch / avg_us / 1e3 / HBM_PEAK_GBS,
                    mfma_frac=ops_launch / avg_us / 1e6 / MFMA_INT8_PEAK_TOPS)
    by_inst = sorted(((k, v["us"] / 3, v["n"] // 3, v["ops"] / v["us"] / 1e6, v["bytes"] / v["us"] / 1e3)
                      for k, v in groups.items()), key=lambda e: -e[1])
    breakdown = [dict(kernel=k, us_per_step=round(us, 1), launches=n, tops=round(tops, 1), algorithmic_gbs=round(gbs))
                 for k, us, n, tops, gbs in by_inst[:14]]

    # ---- the switch alone: host -> device GB/s of the page-in ----
    sw = torch.cuda.Stream()
    t_in = []
    for _ in range(7):
        model.page_out_low()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        model.page_in_low(sw)
        sw.synchronize()
        t_in.append(time.perf_counter() - t0)
    t_in = sorted(t_in)[len(t_in) // 2]
    switch = dict(page_in_bytes=low_bytes, page_in_us=t_in * 1e6, h2d_gbs=low_bytes / t_in / 1e9, page_out_moves_bytes=0)

    out = dict(metric="nested int8 GEMM/conv TOPS (full-bit + part-bit)", value=value, unit="TOPS", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="int8", data="synthetic",
               config=dict(workload=f"ResNet-101-shaped conv/fc stack (104 convolutions + fc, 44.4 M He-normal weights, "
                                    f"all layers per-channel INT8 nesting INT6, l=2), batch {B}, 224x224x3 N(0,1) input, "
                                    "int8 per-layer activations; step = page-out of all lower-bit pages + page-in "
                                    f"({low_bytes / 1e6:.1f} MB pinned host->device"
                                    + (", on a second stream" if side is not None else "")
                                    + ") + part-bit forward + full-bit forward",
                           batch=B, ops_per_step=ops_step, gmac_per_image=ops_img / 2e9,
                           host_issue_ms_per_step=host_issue_ms,
                           issue="hip graph of one step" if graph is not None else "eager",
                           kernel_us_per_step=kern_us_step, mfma_frac_whole_step=value / MFMA_INT8_PEAK_TOPS),
               roofline=roofline, kernels=breakdown, switch=switch)

    if not args.no_sub_records:
        import contextlib
        import io
        import bench_configs as bc
        with contextlib.redirect_stdout(io.StringIO()):
            sub = []
            sub += bc.conv("c2 conv 3x3 56x56x64->64 batch 32 l=2", 32, 56, 56, 64, 64, 3, 1, 1, 2, out8=False, sets=8, quiet=True)
            sub += bc.conv("c3 conv 3x3 14x14x256->256 batch 64 l=2", 64, 14, 14, 256, 256, 3, 1, 1, 2, quiet=True)
            sub += bc.conv("c3 conv 3x3 14x14x256->256 batch 64 l=4", 64, 14, 14, 256, 256, 3, 1, 1, 4, quiet=True)
            sub += bc.gemm("c5 ViT fc1 12608x768->3072 l=3", 12608, 768, 3072, 3, quiet=True)
            sub += bc.gemm("c5 ViT fc1 12608x768->3072 l=3", 12608, 768, 3072, 3, out8=True, quiet=True)
            sub += bc.gemm("c5 ViT fc2 12608x3072->768 l=3", 12608, 3072, 768, 3, quiet=True)
            sub += bc.gemm("c5 ViT fc2 12608x3072->768 l=3", 12608, 3072, 768, 3, out8=True, quiet=True)
        for r in sub:
            us = r["kernel_us"]
            r["tops"] = r.pop("ops") / us / 1e6
            r["mfma_frac"] = r["tops"] / MFMA_INT8_PEAK_TOPS
            r["hbm_frac"] = r["algorithmic_bytes"] / us / 1e3 / HBM_PEAK_GBS
        out["sub_records"] = sub

    if not args.no_cpu_baseline:
        scales = {t: s for t, s in enumerate(model.out_scale) if s is not None}
        base, nimg, lf, lp = cpu_baseline(ops, weights, x_float, scales, n_bits, l_bits, ops_img)
        # the GPU's logits for the sampled images must equal the oracle's, in both modes
        g_part = model.forward(dx, s_x, full=False).cpu().numpy()[:nimg].copy()
        g_full = model.forward(dx, s_x, full=True).cpu().numpy()[:nimg].copy()
        if not (np.array_equal(g_part, lp) and np.array_equal(g_full, lf)):
            raise RuntimeError("bench.py: GPU logits differ from the oracle's on the sampled images")
        base["gpu_matches_oracle_on_sample"] = True
        out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()
