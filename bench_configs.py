"""Per-configuration measurements: one table per configuration of the evaluation (bench.py stays the one-line
benchmark).  Every kernel time is the begin/end time stamp of the dispatch itself; buffers are rotated so that
activations and outputs come from HBM, not from the Infinity Cache.

    python bench_configs.py [c1] [c2] [c3] [c4] [c5] [pack] [page] [sweep] [words] [dw] [lib] [cpu]
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2506_17870_amd as nq  # noqa: E402
from paper_2506_17870_amd import inputs, network  # noqa: E402

MFMA_PEAK, HBM_PEAK = 5000.0, 8000.0   # TOPS (int8 dense), GB/s


def weights(N, K, sigma, n_bits=8, seed=0):
    """INT-n codes [N,K] and per-channel steps of N(0, sigma) weights, quantised on the device (nq_quantize,
    Eq. 1) and copied back as NumPy arrays."""
    d_w = torch.from_numpy(inputs.float_weights(N, K, sigma, seed)).cuda()
    d_int = torch.empty((N, K), dtype=torch.int8, device="cuda")
    d_step = torch.empty(N, dtype=torch.float32, device="cuda")
    nq.nq_quantize(d_w, N, K, n_bits, d_int, d_step)
    return d_int.cpu().numpy(), d_step.cpu().numpy()


def kernel_us(fn, n=50):
    """Median and minimum dispatch duration of the GEMM/conv launch made by fn(events).  The warm-up is long
    enough for the clocks to settle (a handful of launches is not: the first figures then read 15 % high)."""
    t0 = time.perf_counter()
    for i in range(400):
        fn(None)
        if i >= 24 and i % 8 == 0:
            torch.cuda.synchronize()
            if time.perf_counter() - t0 > 0.02:
                break
    torch.cuda.synchronize()
    evs = [(nq.nq_event_create(), nq.nq_event_create()) for _ in range(n)]
    for a, b in evs:
        fn((a, b))
    torch.cuda.synchronize()
    ts = sorted(nq.nq_event_elapsed_ms(a, b) * 1e3 for a, b in evs)
    for a, b in evs:
        nq.nq_event_destroy(a)
        nq.nq_event_destroy(b)
    return ts[len(ts) // 2], ts[0]


def wall_us(fn, n=50):
    """Back-to-back launches between two stream events (for kernels without the time-stamp hook)."""
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def row(name, mode, us, ops, byts):
    tops = ops / us / 1e6
    gbs = byts / us / 1e3
    print(f"| {name} | {mode} | {us:.2f} | {tops:.1f} | {100 * tops / MFMA_PEAK:.1f} | {gbs:.0f} | {100 * gbs / HBM_PEAK:.1f} |")


def header(title):
    print(f"\n### {title}\n")
    print("| layer | mode | kernel us | TOPS | % int8 MFMA peak | algorithmic GB/s | % HBM peak |")
    print("|---|---|---|---|---|---|---|")


def gemm(name, M, K, N, l, out8=False, sets=4, sigma=0.02, n_bits=8, layout=None, quiet=False):
    layout = nq.NQ_LAYOUT_DENSE if layout is None else layout
    w_int, scale = weights(N, K, sigma, n_bits, 0)
    W = nq.NestedWeight.from_int8(torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda(),
                                  nq.make_cfg(n_bits, l, layout=layout))
    # INT6 nesting runs with 6-bit activations (Sec. 4.2): int8 codes in [-32, 31]
    xs = [torch.from_numpy(inputs.uniform_activations((M, K), i) >> (8 - n_bits)).cuda() for i in range(sets)]
    ys = [torch.empty((M, N), dtype=torch.int8 if out8 else torch.float32, device="cuda") for _ in range(sets)]
    epi = nq.make_epilogue(0.02, out_int8=out8, inv_out_scale=3.0)
    results = []
    for full in (True, False):
        cnt = [0]

        def fn(ev):
            i = cnt[0] % sets
            cnt[0] += 1
            if ev:
                nq.nq_profile_next_launch(ev[0], ev[1])
            (nq.nq_gemm_full if full else nq.nq_gemm_part)(xs[i], M, W.desc, epi, ys[i])
        med, _ = kernel_us(fn)
        wb = nq.nq_packed_bytes(N, K, n_bits - l, layout) + (nq.nq_packed_bytes(N, K, l, layout) if full else 0)
        mode = ("full" if full else "part") + (" int8 out" if out8 else " fp32 out")
        ops, byts = 2.0 * M * N * K, M * K + wb + M * N * (1 if out8 else 4)
        if not quiet:
            row(name, mode, med, ops, byts)
        results.append(dict(layer=name, mode=mode, kernel_us=med, ops=ops, algorithmic_bytes=byts))
    return results


def conv(name, B, H, W_, Cin, Cout, k, stride, pad, l, out8=True, sets=4, quiet=False, layout=None):
    K = k * k * Cin
    w_int, scale = weights(Cout, K, inputs.he_sigma(K), 8, 0)
    cfg = nq.make_cfg(8, l) if layout is None else nq.make_cfg(8, l, layout=layout)
    W = nq.NestedWeight.from_int8(torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda(), cfg)
    Ho, Wo = network.out_hw(H, W_, k, stride, pad)
    xs = [torch.from_numpy(inputs.uniform_activations((B, H, W_, Cin), i)).cuda() for i in range(sets)]
    ys = [torch.empty((B, Ho, Wo, Cout), dtype=torch.int8 if out8 else torch.float32, device="cuda")
          for _ in range(sets)]
    epi = nq.make_epilogue(0.02, relu=True, out_int8=out8, inv_out_scale=3.0)
    cs = nq.nq_conv_shape(B, H, W_, Cin, Cout, k, k, stride, pad)
    results = []
    for full in (True, False):
        cnt = [0]

        def fn(ev):
            i = cnt[0] % sets
            cnt[0] += 1
            if ev:
                nq.nq_profile_next_launch(ev[0], ev[1])
            (nq.nq_conv_full if full else nq.nq_conv_part)(xs[i], cs, W.desc, epi, ys[i])
        med, _ = kernel_us(fn)
        M = B * Ho * Wo
        lay = nq.NQ_LAYOUT_DENSE if layout is None else layout
        wb = nq.nq_packed_bytes(Cout, K, 8 - l, lay) + (nq.nq_packed_bytes(Cout, K, l, lay) if full else 0)
        mode = ("full" if full else "part") + (" int8 out" if out8 else " fp32 out")
        ops, byts = 2.0 * M * Cout * K, B * H * W_ * Cin + wb + M * Cout * (1 if out8 else 4)
        if not quiet:
            row(name, mode, med, ops, byts)
        results.append(dict(layer=name, mode=mode, kernel_us=med, ops=ops, algorithmic_bytes=byts))
    return results


def gconv(name, B, H, W_, C, groups, k, stride, l, sets=6, Cout=None):
    """One depthwise / grouped layer, int8 in and out with bias and ReLU; full-bit and part-bit."""
    Cin, C = C, (Cout or C)
    gs = Cin // groups
    K = k * k * gs
    pad = k // 2
    w_int, scale = weights(C, K, inputs.he_sigma(K), 8, 0)
    W = nq.NestedWeight.from_int8(torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda(), nq.make_cfg(8, l))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W_ + 2 * pad - k) // stride + 1
    xs = [torch.from_numpy(inputs.uniform_activations((B, H, W_, Cin), i)).cuda() for i in range(sets)]
    ys = [torch.empty((B, Ho, Wo, C), dtype=torch.int8, device="cuda") for _ in range(sets)]
    bias = torch.from_numpy(inputs.small_floats(C, 0.1, 1)).cuda()
    epi = nq.make_epilogue(0.02, d_bias=bias, relu=True, out_int8=True, inv_out_scale=3.0)
    cs = nq.nq_conv_shape(B, H, W_, Cin, C, k, k, stride, pad)
    for full in (True, False):
        cnt = [0]

        def fn(ev):
            i = cnt[0] % sets
            cnt[0] += 1
            if ev:
                nq.nq_profile_next_launch(ev[0], ev[1])
            (nq.nq_gconv_full if full else nq.nq_gconv_part)(xs[i], cs, groups, W.desc, epi, ys[i])
        med, _ = kernel_us(fn)
        M = B * Ho * Wo
        byts = B * H * W_ * Cin + M * C + nq.nq_packed_bytes(C, K, 8 - l) + (nq.nq_packed_bytes(C, K, l) if full else 0)
        gbs = byts / med / 1e3
        print(f"| {name} | {'full' if full else 'part'} | {med:.2f} | {byts / 1e6:.2f} | {gbs:.0f} | "
              f"{100 * gbs / HBM_PEAK:.1f} | {2.0 * M * C * K / med / 1e6:.2f} |")


def dw():
    print("\n### depthwise / grouped layers of the lightweight CNNs, batch 32, int8 in and out, bias + ReLU, INT(8|5)\n")
    print("| layer | mode | kernel us | algorithmic MB | GB/s | % HBM peak | useful TOPS |")
    print("|---|---|---|---|---|---|---|")
    # MobileNet (224 x 224 input): every distinct depthwise layer
    for hw, c, s in ((112, 32, 1), (112, 64, 2), (56, 128, 1), (56, 128, 2), (28, 256, 1), (28, 256, 2), (14, 512, 1),
                     (14, 512, 2), (7, 1024, 1)):
        gconv(f"MobileNet dw 3x3 {hw}x{hw}x{c} s{s}", 32, hw, hw, c, c, 3, s, 3)
    # MobileNetV2 / EfficientNet-B0 expanded widths, 5x5 filters, and a ResNeXt 32x4d grouped layer
    gconv("MobileNetV2 dw 3x3 56x56x144 s1", 32, 56, 56, 144, 144, 3, 1, 3)
    gconv("MobileNetV2 dw 3x3 14x14x576 s1", 32, 14, 14, 576, 576, 3, 1, 3)
    gconv("EfficientNet-B0 dw 5x5 28x28x240 s1", 32, 28, 28, 240, 240, 5, 1, 3)
    gconv("EfficientNet-B0 dw 5x5 14x14x672 s1", 32, 14, 14, 672, 672, 5, 1, 3)
    gconv("ResNeXt 32x4d 3x3 56x56x128 g32", 32, 56, 56, 128, 32, 3, 1, 3)
    # wider groups and unequal channel counts: the direct kernel (vector ALU)
    gconv("ResNeXt 32x8d 3x3 56x56x256 g32 (groups of 8)", 32, 56, 56, 256, 32, 3, 1, 3)
    gconv("ShuffleNet g3 1x1 28x28 240->60", 32, 28, 28, 240, 3, 1, 1, 3, Cout=60)
    gconv("ShuffleNet g3 1x1 28x28 60->240", 32, 28, 28, 60, 3, 1, 1, 3, Cout=240)


def lib():
    """Context, not a target: the vendor library's plain int8 GEMM (torch._int_mm -> hipBLASLt; int32 outputs, no
    decode, no epilogue) on the GEMM shapes of the configurations, next to the nested kernels on the same shapes
    (INT(8|5), int8 outputs with the fused epilogue; convolutions as the implicit GEMM they are)."""
    print("\n### vendor library plain int8 GEMM (hipBLASLt through torch._int_mm) against the nested kernels\n")
    print("| shape M x K x N | library us (back-to-back launches) | library TOPS | nested full-bit us | nested part-bit us |")
    print("|---|---|---|---|---|")
    for name, M, K, N in (("ViT fc1", 12608, 768, 3072), ("ViT fc2", 12608, 3072, 768),
                          ("bottleneck 1x1 1024->256", 12544, 1024, 256), ("bottleneck 1x1 256->1024", 12544, 256, 1024),
                          ("square", 8192, 4096, 4096)):
        a = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
        bt = torch.randint(-128, 128, (N, K), dtype=torch.int8, device="cuda")
        try:
            us_lib = wall_us(lambda: torch._int_mm(a, bt.t()), n=30)
        except Exception as e:   # the library path is optional context
            print(f"| {name} | not available ({type(e).__name__}) | | | |")
            continue
        w_int, scale = weights(N, K, 0.02, 8, 0)
        W = nq.NestedWeight.from_int8(torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda(), nq.make_cfg(8, 3))
        ys = [torch.empty((M, N), dtype=torch.int8, device="cuda") for _ in range(2)]
        epi = nq.make_epilogue(0.02, out_int8=True, inv_out_scale=3.0)
        ours = []
        for full in (True, False):
            cnt = [0]

            def fn(ev):
                cnt[0] += 1
                if ev:
                    nq.nq_profile_next_launch(ev[0], ev[1])
                (nq.nq_gemm_full if full else nq.nq_gemm_part)(a, M, W.desc, epi, ys[cnt[0] % 2])
            ours.append(kernel_us(fn)[0])
        print(f"| {name} {M} x {K} x {N} | {us_lib:.1f} | {2.0 * M * K * N / us_lib / 1e6:.0f} | {ours[0]:.1f} | {ours[1]:.1f} |")
        del a, bt, W, ys


def cpu():
    """The CPU oracle (plain C loops, -O2, no intrinsics, no BLAS) on the host's cores: one thread and all
    threads OpenMP gives it, integer accumulators only (the part the GPU's TOPS are quoted on)."""
    import ctypes
    import platform
    from oracle import nq_oracle as oracle
    model = platform.processor() or "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    omp = ctypes.CDLL("libgomp.so.1")
    nthreads = oracle.threads()

    def oracle_weights(N, K, sigma, n_bits, seed):
        return oracle.quantize(inputs.float_weights(N, K, sigma, seed), n_bits)
    print(f"\n### CPU oracle timing: {model}, os.cpu_count() = {os.cpu_count()}, OpenMP threads used = {nthreads}\n")
    print("| configuration | GOP | 1 thread s | 1 thread GOPS | all threads s | all threads GOPS |")
    print("|---|---|---|---|---|---|")

    def timed(fn, threads):
        omp.omp_set_num_threads(threads)
        t0 = time.perf_counter()
        fn()
        return time.perf_counter() - t0

    def row(name, gop, fn, single=True):
        t_all = timed(fn, nthreads)
        t_one = timed(fn, 1) if single else None
        one = f"{t_one:.2f} | {gop / t_one:.1f}" if t_one else "not run | "
        print(f"| {name} | {gop:.2f} | {one} | {t_all:.3f} | {gop / t_all:.1f} |", flush=True)
    c = inputs.LINEAR_SMALL
    w = oracle_weights(c["N"], c["K"], c["sigma"], 8, 0)[0].astype(np.int16)
    x = inputs.uniform_activations((c["M"], c["K"]), 0)
    row("c1 linear 64x512->512", 2e-9 * c["M"] * c["N"] * c["K"], lambda: oracle.gemm_acc(x, w))
    c = inputs.CONV_RESNET18
    K = 9 * c["Cin"]
    w = oracle_weights(c["Cout"], K, inputs.he_sigma(K), 8, 0)[0].astype(np.int16).reshape(c["Cout"], 3, 3, c["Cin"])
    x = inputs.uniform_activations((c["B"], c["H"], c["W"], c["Cin"]), 0)
    row("c2 conv 3x3 56x56x64->64, batch 32", 2e-9 * c["B"] * c["H"] * c["W"] * c["Cout"] * K, lambda: oracle.conv_acc(x, w, 1, 1))
    for g in inputs.BOTTLENECK_RESNET101:
        K = g["KH"] * g["KW"] * g["Cin"]
        w = oracle_weights(g["Cout"], K, inputs.he_sigma(K), 8, 0)[0].astype(np.int16).reshape(g["Cout"], g["KH"], g["KW"], g["Cin"])
        x = inputs.uniform_activations((64, 14, 14, g["Cin"]), 0)
        row(f"c3 {g['KH']}x{g['KW']} {g['Cin']}->{g['Cout']}, batch 64, 14x14", 2e-9 * 64 * 196 * g["Cout"] * K,
            lambda: oracle.conv_acc(x, w, g["stride"], g["pad"]))
    for g in inputs.VIT_MLP:
        w = oracle_weights(g["N"], g["K"], g["sigma"], 8, 0)[0].astype(np.int16)
        x = inputs.uniform_activations((g["M"], g["K"]), 0)
        row(f"c5 ViT {g['K']}->{g['N']}, M = {g['M']}", 2e-9 * g["M"] * g["N"] * g["K"], lambda: oracle.gemm_acc(x, w))
    omp.omp_set_num_threads(nthreads)
    print("\n(c4, 2 TOP per forward: bench.py's cpu_baseline runs the whole network on the oracle, 8 images on all threads and "
          "one image on one thread.)")


def c1():
    header("config 1: linear 64x512 -> 512 (launch bound) and weight-bound stand-ins (M = 64 and 16, 8192 x 8192)")
    gemm("64x512->512 l=2", 64, 512, 512, 2)
    gemm("64x8192->8192 l=2", 64, 8192, 8192, 2, sets=3)
    gemm("16x8192->8192 l=2", 16, 8192, 8192, 2, sets=3)
    gemm("16x8192->8192 l=4", 16, 8192, 8192, 4, sets=3)
    c1_stack()


def c1_stack():
    """1024 distinct 512 x 512 layers (268 MB of packed pages: more than the Infinity Cache) as one sequence of
    launches, replayed as a HIP graph so that the host is out of the picture."""
    L, M, K, N = 1024, 64, 512, 512
    cfg = nq.make_cfg(8, 2)
    w_int, scale = weights(N, K, 0.02, 8, 0)
    d_w, d_s = torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda()
    low_bytes = nq.nq_packed_bytes(N, K, 2)
    arena = torch.empty(L * low_bytes, dtype=torch.uint8, device="cuda")
    host = torch.empty(L * low_bytes, dtype=torch.uint8, pin_memory=True)
    layers = []
    for i in range(L):
        W = nq.NestedWeight(N, K, cfg, low=arena[i * low_bytes:(i + 1) * low_bytes],
                            low_host=host[i * low_bytes:(i + 1) * low_bytes])
        W.fill_from_int8(d_w, d_s)
        layers.append(W)
    x = torch.from_numpy(inputs.uniform_activations((M, K), 0)).cuda()
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    epi = nq.make_epilogue(0.02)
    print("\n* stack of 1024 distinct 64x512->512 layers (packed pages 268 MB full-bit, 201 MB part-bit), one HIP graph:")
    for full in (True, False):
        fn = nq.nq_gemm_full if full else nq.nq_gemm_part
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for W in layers[:8]:
                fn(x, M, W.desc, epi, y)
            st.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=st):
                for W in layers:
                    fn(x, M, W.desc, epi, y)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 5
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        wb = L * (nq.nq_packed_bytes(N, K, 6) + (low_bytes if full else 0))
        print(f"  {'full' if full else 'part'}-bit: {ms:.2f} ms = {ms * 1e3 / L:.2f} us per layer, {wb / ms / 1e6:.0f} GB/s of packed "
              f"weights, {2.0 * M * N * K * L / ms / 1e9:.1f} TOPS (launch bound: a 64-row layer is one wave of 16 blocks)")
        del graph
    # the same stack as ONE launch: nq_gemm_batch, the problems as a table in device memory
    jobs = [(x, M, W.desc, epi, y) for W in layers]
    ws = torch.empty(nq.nq_gemm_batch_workspace_bytes(L), dtype=torch.uint8, device="cuda")
    for full in (True, False):
        us = wall_us(lambda: nq.nq_gemm_batch(jobs, full, ws), n=10)

        def fn(ev):
            if ev:
                nq.nq_profile_next_launch(ev[0], ev[1])
            nq.nq_gemm_batch(jobs, full, ws)
        kus, _ = kernel_us(fn, n=10)
        wb = L * (nq.nq_packed_bytes(N, K, 6) + (low_bytes if full else 0))
        print(f"  {'full' if full else 'part'}-bit, one nq_gemm_batch call: kernel {kus:.0f} us = {kus / L:.3f} us per layer, "
              f"{wb / kus / 1e3:.0f} GB/s of packed weights ({100 * wb / kus / 1e3 / HBM_PEAK:.1f} % of HBM peak), "
              f"{2.0 * M * N * K * L / kus / 1e6:.1f} TOPS; call to call, with the host filling the table of {L} problems: "
              f"{us / 1e3:.2f} ms")


def c2():
    header("config 2: ResNet-18 3x3 conv, batch 32, 56x56x64 -> 64, l=2")
    conv("3x3 64->64", 32, 56, 56, 64, 64, 3, 1, 1, 2, out8=False, sets=8)
    conv("3x3 64->64", 32, 56, 56, 64, 64, 3, 1, 1, 2, out8=True, sets=8)


def c3():
    header("config 3: ResNet-101 stage-3 bottleneck, batch 64, 14x14")
    for l in (2, 4):
        conv(f"1x1 1024->256 l={l}", 64, 14, 14, 1024, 256, 1, 1, 0, l)
        conv(f"3x3 256->256 l={l}", 64, 14, 14, 256, 256, 3, 1, 1, l)
        conv(f"1x1 256->1024 l={l}", 64, 14, 14, 256, 1024, 1, 1, 0, l)
    conv("1x1 256->1024 l=2", 64, 14, 14, 256, 1024, 1, 1, 0, 2, out8=False)


def c5():
    header("config 5: ViT-B/16 MLP at batch 64 (M = 12608), l=3")
    gemm("fc1 768->3072", 12608, 768, 3072, 3)
    gemm("fc1 768->3072", 12608, 768, 3072, 3, out8=True)
    gemm("fc2 3072->768", 12608, 3072, 768, 3)
    gemm("fc2 3072->768", 12608, 3072, 768, 3, out8=True)


def c4():
    print("\n### config 4: ResNet-101 conv/fc stack, batch 128, 224x224x3, all layers INT(8|6)\n")
    ops = network.resnet101_plan()
    weights = network.plan_float_weights(ops, seed=0)
    model = network.NestedCNN(ops, weights, 8, 2)
    B = 128
    dx, s_x = network.quantize_tensor(inputs.gaussian_floats((B, 224, 224, 3), seed=0))
    model.calibrate(dx, s_x)
    macs = 0
    h = w = 224
    hw = {0: (224, 224)}
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
    ops_fwd = 2.0 * macs * B

    def fwd(full):
        for _ in range(2):
            model.forward(dx, s_x, full=full)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = 5
        for _ in range(n):
            model.forward(dx, s_x, full=full)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3
    ms_full = fwd(True)
    print(f"* full-bit forward: {ms_full:.2f} ms per batch of {B} ({ops_fwd / ms_full / 1e9:.1f} TOPS, "
          f"{macs / 1e9:.2f} GMAC per image)")
    t0 = time.perf_counter()
    model.page_out_low()
    t_out = (time.perf_counter() - t0) * 1e6
    ms_part = fwd(False)
    print(f"* downgrade (nq_page_out_low on 105 layers): {t_out:.0f} us of host time, nothing moved")
    print(f"* part-bit forward: {ms_part:.2f} ms ({ops_fwd / ms_part / 1e9:.1f} TOPS)")
    side = torch.cuda.Stream()
    low = model.low_page_bytes()
    model.page_in_low(side)                       # first use of the stream and of the pinned arena: not timed
    side.synchronize()
    t_in = []
    for _ in range(5):
        model.page_out_low()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        model.page_in_low(side)
        side.synchronize()
        t_in.append((time.perf_counter() - t0) * 1e6)
    t_in = sorted(t_in)[len(t_in) // 2]
    print(f"* upgrade (nq_page_in_low_batch, {low / 1e6:.2f} MB of 105 pages as one pinned copy on a second stream): "
          f"{t_in:.0f} us = {low / t_in / 1e3:.1f} GB/s host to device")
    model.page_out_low()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model.page_in_low(side)
    model.forward(dx, s_x, full=True)
    torch.cuda.synchronize()
    print(f"* upgrade + first full-bit forward: {(time.perf_counter() - t0) * 1e3:.2f} ms")

    # per-layer: the time stamps of every GEMM / convolution dispatch of one full-bit forward, by layer shape
    from paper_2506_17870_amd import binding
    recs = []
    originals = {name: getattr(binding, name) for name in ("nq_conv_full", "nq_gemm_full")}

    def stamped(name):
        orig = originals[name]

        def call(*a, **k):
            e0, e1 = binding.nq_event_create(), binding.nq_event_create()
            binding.nq_profile_next_launch(e0, e1)
            orig(*a, **k)
            recs.append((e0, e1, a[1] if name == "nq_conv_full" else None, a[2], bool(a[3].d_residual)))
        return call
    for name in originals:
        setattr(binding, name, stamped(name))
    try:
        model.forward(dx, s_x, full=True)
        torch.cuda.synchronize()
    finally:
        for name, orig in originals.items():
            setattr(binding, name, orig)
    layers = {}
    total = 0.0
    for e0, e1, shape, wd, has_res in recs:
        us = binding.nq_event_elapsed_ms(e0, e1) * 1e3
        binding.nq_event_destroy(e0)
        binding.nq_event_destroy(e1)
        total += us
        if shape is not None:
            ho = (shape.H + 2 * shape.pad - shape.KH) // shape.stride + 1
            wo = (shape.W + 2 * shape.pad - shape.KW) // shape.stride + 1
            m, k = shape.B * ho * wo, shape.KH * shape.KW * shape.Cin
            key = f"{shape.KH}x{shape.KW} s{shape.stride} {shape.H}x{shape.W} {shape.Cin}->{shape.Cout}"
            lops, byts = 2.0 * m * shape.Cout * k, shape.B * shape.H * shape.W * shape.Cin + m * shape.Cout + shape.Cout * k
            if has_res:                      # the block's last layer also reads the skip tensor
                key += " + residual"
                byts += m * shape.Cout
        else:
            key, lops, byts = f"fc {wd.K}->{wd.N}", 2.0 * B * wd.N * wd.K, B * wd.K + 4 * B * wd.N + wd.N * wd.K
        a = layers.setdefault(key, [0, 0.0, 0.0, 0.0])
        a[0] += 1; a[1] += us; a[2] += lops; a[3] += byts
    print(f"\nper layer shape, full-bit (sum of the {len(recs)} kernel times {total / 1e3:.2f} ms; the rest of the forward is "
          "pooling and launch gaps):\n")
    print("| layer | launches | us each | TOPS | % int8 MFMA peak | algorithmic GB/s | % HBM peak |")
    print("|---|---|---|---|---|---|---|")
    for key, (cnt, us, lops, byts) in sorted(layers.items(), key=lambda kv: -kv[1][1]):
        tops, gbs = lops / us / 1e6, byts / us / 1e3
        print(f"| {key} | {cnt} | {us / cnt:.1f} | {tops:.0f} | {100 * tops / MFMA_PEAK:.1f} | {gbs:.0f} | {100 * gbs / HBM_PEAK:.1f} |")


def pack():
    print("\n### decompose-and-pack (1 B read + 1 B written per weight)\n")
    print("| tensor | us | GB/s (read+write) | % HBM peak |")
    print("|---|---|---|---|")
    cfg = nq.make_cfg(8, 2)
    for name, N, K in (("ResNet-101 largest layer 512x4608", 512, 4608), ("4096 x 4096", 4096, 4096),
                       ("1 GiB: 32768 x 32768", 32768, 32768)):
        w = torch.randint(-128, 128, (N, K), dtype=torch.int8, device="cuda")
        ph = torch.empty(nq.nq_packed_bytes(N, K, 6), dtype=torch.uint8, device="cuda")
        pl = torch.empty(nq.nq_packed_bytes(N, K, 2), dtype=torch.uint8, device="cuda")
        us = wall_us(lambda: nq.nq_decompose_pack(w, N, K, cfg, ph, pl), n=20)
        gbs = 2.0 * N * K / us / 1e3
        print(f"| {name} | {us:.1f} | {gbs:.0f} | {100 * gbs / HBM_PEAK:.1f} |")
        del w, ph, pl
    # the whole ResNet-101 weight set (105 tensors, 44.4 M weights), one launch per layer, back to back
    plan = network.resnet101_plan()
    ws = network.plan_float_weights(plan, seed=0)
    tensors = []
    for wgt in ws:
        if wgt is None:
            continue
        n_, k_ = wgt[0].shape
        d_int = torch.empty((n_, k_), dtype=torch.int8, device="cuda")
        nq.nq_quantize(torch.from_numpy(wgt[0]).cuda(), n_, k_, 8, d_int, torch.empty(n_, dtype=torch.float32, device="cuda"))
        tensors.append((d_int, n_, k_,
                        torch.empty(nq.nq_packed_bytes(n_, k_, 6), dtype=torch.uint8, device="cuda"),
                        torch.empty(nq.nq_packed_bytes(n_, k_, 2), dtype=torch.uint8, device="cuda")))
    total = sum(n_ * k_ for _, n_, k_, _, _ in tensors)

    def all_layers():
        for w, n_, k_, ph, pl in tensors:
            nq.nq_decompose_pack(w, n_, k_, cfg, ph, pl)
    us = wall_us(all_layers, n=10)
    gbs = 2.0 * total / us / 1e3
    print(f"| ResNet-101, all {len(tensors)} tensors ({total / 1e6:.1f} M weights), one launch per tensor | {us:.1f} | {gbs:.0f} | "
          f"{100 * gbs / HBM_PEAK:.1f} |")
    jobs = [(w, n_, k_, ph, pl) for w, n_, k_, ph, pl in tensors]
    us = wall_us(lambda: nq.nq_decompose_pack_batch(jobs, cfg), n=10)
    gbs = 2.0 * total / us / 1e3
    print(f"| the same as nq_decompose_pack_batch (two launches of up to 64 tensors) | {us:.1f} | {gbs:.0f} | "
          f"{100 * gbs / HBM_PEAK:.1f} |")
    del tensors
    print("\n### quantise, decompose and pack from fp32 weights (Eq. 1 fused in front; 4 B read + 1 B written per "
          "weight\ncounted, the second pass over the fp32 weights not counted)\n")
    print("| tensor | us | GB/s (counted bytes) | % HBM peak | two calls: nq_quantize + nq_decompose_pack, us |")
    print("|---|---|---|---|---|")
    for name, N, K in (("ResNet-101 largest layer 512x4608", 512, 4608), ("4096 x 4096", 4096, 4096),
                       ("16384 x 16384 (1 GiB of fp32)", 16384, 16384)):
        w = torch.randn((N, K), dtype=torch.float32, device="cuda") * 0.02
        wi = torch.empty((N, K), dtype=torch.int8, device="cuda")
        sc = torch.empty(N, dtype=torch.float32, device="cuda")
        ph = torch.empty(nq.nq_packed_bytes(N, K, 6), dtype=torch.uint8, device="cuda")
        pl = torch.empty(nq.nq_packed_bytes(N, K, 2), dtype=torch.uint8, device="cuda")
        us = wall_us(lambda: nq.nq_quantize_decompose_pack(w, N, K, cfg, sc, ph, pl), n=20)

        def two_calls():
            nq.nq_quantize(w, N, K, 8, wi, sc)
            nq.nq_decompose_pack(wi, N, K, cfg, ph, pl)
        us2 = wall_us(two_calls, n=20)
        gbs = 5.0 * N * K / us / 1e3
        print(f"| {name} | {us:.1f} | {gbs:.0f} | {100 * gbs / HBM_PEAK:.1f} | {us2:.1f} |")
        del w, wi, ph, pl


def page():
    print("\n### page-in of the lower-bit page (pinned host -> device, `nq_page_in_low`)\n")
    print("| page | us | GB/s |")
    print("|---|---|---|")
    for name, N, K, l in (("ViT fc1 low page l=3 (0.88 MB)", 3072, 768, 3), ("64 MiB page", 16384, 16384, 2)):
        cfg = nq.make_cfg(8, l)
        W = nq.NestedWeight(N, K, cfg)
        side = torch.cuda.Stream()
        best = 1e30
        for _ in range(10):
            nq.nq_page_out_low(W.desc)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            nq.nq_page_in_low(W.desc, side)
            side.synchronize()
            best = min(best, (time.perf_counter() - t0) * 1e6)
        b = nq.nq_packed_bytes(N, K, l)
        print(f"| {name} | {best:.0f} | {b / best / 1e3:.1f} |")
    # overlap: part-bit GEMMs on the compute stream while a page travels on the other stream.  The GEMM is timed
    # by the time stamps of its own dispatch (what a kernel trace shows), so host-side costs of the switching
    # calls cannot leak into it; those are timed separately, call by call, on the host clock.
    M, K, N, l = 12608, 3072, 768, 3
    w_int, scale = weights(N, K, 0.02, 8, 0)
    W = nq.NestedWeight.from_int8(torch.from_numpy(w_int).cuda(), torch.from_numpy(scale).cuda(), nq.make_cfg(8, l))
    x = torch.from_numpy(inputs.uniform_activations((M, K), 0)).cuda()
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    epi = nq.make_epilogue(0.02)
    side = torch.cuda.Stream()

    def gemm_fn(ev):
        if ev:
            nq.nq_profile_next_launch(ev[0], ev[1])
        nq.nq_gemm_part(x, M, W.desc, epi, y)
    alone, _ = kernel_us(gemm_fn)
    print(f"\npart-bit fc2 GEMM (12608 x 3072 -> 768, fp32 out), kernel time alone: {alone:.1f} us")
    print("\n| page travelling meanwhile | GEMM kernel us (median of the launches that ran during the copy) | copy us | GB/s |")
    print("|---|---|---|---|")
    big = nq.NestedWeight(16384, 16384, nq.make_cfg(8, 2))          # a 64 MiB lower-bit page of its own
    for name, Wp, n_gemm in (("its own 0.88 MB page", W, 1), ("a 64 MiB page", big, 24)):
        times, copies = [], []
        for _ in range(7):
            nq.nq_page_out_low(Wp.desc)
            torch.cuda.synchronize()
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            evs = [(nq.nq_event_create(), nq.nq_event_create()) for _ in range(n_gemm)]
            with torch.cuda.stream(side):
                c0.record()
                nq.nq_page_in_low(Wp.desc, side)
                c1.record()
            for ev in evs:
                gemm_fn(ev)
            torch.cuda.synchronize()
            copy_us = c0.elapsed_time(c1) * 1e3
            ks = [nq.nq_event_elapsed_ms(a, b) * 1e3 for a, b in evs]
            # the launches that can have overlapped the copy: those that began within its duration
            during = ks[:max(1, min(n_gemm, int(copy_us / max(alone, 1.0))))]
            times += during
            copies.append(copy_us)
            for a, b in evs:
                nq.nq_event_destroy(a)
                nq.nq_event_destroy(b)
        times.sort()
        copies.sort()
        byts = nq.nq_packed_bytes(Wp.N, Wp.K, Wp.cfg.l_bits)
        cu = copies[len(copies) // 2]
        print(f"| {name} | {times[len(times) // 2]:.1f} | {cu:.0f} | {byts / cu / 1e3:.1f} |")
    # host cost of the switching calls (one descriptor; host clock around each call, median of 200)
    def host_us(fn):
        ts = []
        for _ in range(200):
            t0 = time.perf_counter()
            fn()
            ts.append((time.perf_counter() - t0) * 1e6)
        torch.cuda.synchronize()
        return sorted(ts)[len(ts) // 2]
    t_out = host_us(lambda: nq.nq_page_out_low(W.desc))
    t_in = host_us(lambda: (nq.nq_page_out_low(W.desc), nq.nq_page_in_low(W.desc, side)))
    t_launch = host_us(lambda: nq.nq_gemm_part(x, M, W.desc, epi, y))
    print(f"\nhost time per call: nq_page_out_low {t_out:.1f} us, page-out + nq_page_in_low (event wait, copy, event "
          f"record) {t_in:.1f} us, nq_gemm_part launch {t_launch:.1f} us")


def sweep():
    """Throughput against the nesting (Sec. 4.2: INT8 nesting INT7..INT2, INT6 nesting INT5..INT2 with 6-bit
    activations).  Part-bit weight bytes scale as h/n, which shows where the weight stream matters: a skinny
    GEMM (16 rows against 8192 x 8192 weights); the ViT fc2 shape is matrix-core bound and barely moves."""
    header("nesting sweep, skinny GEMM 16 x 8192 -> 8192 (weight-stream bound)")
    for n, ls in ((8, (1, 2, 3, 4, 5, 6)), (6, (1, 2, 3, 4))):
        for l in ls:
            gemm(f"INT({n}|{n - l})", 16, 8192, 8192, l, sets=2, n_bits=n)
    header("nesting sweep, ViT fc2 12608 x 3072 -> 768, int8 out (matrix-core bound)")
    for n, ls in ((8, (1, 2, 3, 4, 5, 6)), (6, (1, 2, 3, 4))):
        for l in ls:
            gemm(f"INT({n}|{n - l})", 12608, 3072, 768, l, out8=True, sets=3, n_bits=n)


def words():
    """The paper's own page format (64 // k fields per unsigned 64-bit word, Sec. 3.3.4) against the dense
    tile pages: bits per weight, the cost of taking a model stored in words to the dense pages on the GPU
    (nq_unpack of the word pages + nq_pack into tiles), and the GEMM that reads the word pages as they are."""
    print("\n### word pages (64 // k fields per uint64) -> dense tile pages, 4096 x 4096 weights\n")
    print("| nesting | word pages bit/weight | dense pages bit/weight | unpack + pack us | GB/s (all four streams) |")
    print("|---|---|---|---|---|")
    N = K = 4096
    for l in (1, 2, 3, 4):
        h = 8 - l
        w_int, scale = weights(N, K, 0.02, 8, l)
        cw = nq.make_cfg(8, l, layout=nq.NQ_LAYOUT_PAPER_U64)
        cd = nq.make_cfg(8, l)
        bw = nq.nq_packed_bytes(N, K, h, nq.NQ_LAYOUT_PAPER_U64) + nq.nq_packed_bytes(N, K, l, nq.NQ_LAYOUT_PAPER_U64)
        bd = nq.nq_packed_bytes(N, K, h) + nq.nq_packed_bytes(N, K, l)
        d_w = torch.from_numpy(w_int).cuda()
        wh = torch.zeros(nq.nq_packed_bytes(N, K, h, nq.NQ_LAYOUT_PAPER_U64), dtype=torch.uint8, device="cuda")
        wl = torch.zeros(nq.nq_packed_bytes(N, K, l, nq.NQ_LAYOUT_PAPER_U64), dtype=torch.uint8, device="cuda")
        nq.nq_decompose_pack(d_w, N, K, cw, wh, wl)
        hi = torch.empty((N, K), dtype=torch.int8, device="cuda")
        lo = torch.empty((N, K), dtype=torch.int8, device="cuda")
        dh = torch.zeros(nq.nq_packed_bytes(N, K, h), dtype=torch.uint8, device="cuda")
        dl = torch.zeros(nq.nq_packed_bytes(N, K, l), dtype=torch.uint8, device="cuda")

        def fn():
            nq.nq_unpack(wh, wl, N, K, cw, hi, lo)
            nq.nq_pack(hi, lo, N, K, cd, dh, dl)
        us = wall_us(fn, 20)
        # check: the dense pages made from the word pages equal the ones made from the weights directly
        rh, rl = torch.zeros_like(dh), torch.zeros_like(dl)
        nq.nq_decompose_pack(d_w, N, K, cd, rh, rl)
        assert torch.equal(rh, dh) and torch.equal(rl, dl), "transcoded pages differ"
        print(f"| INT(8\\|{h}) | {8.0 * bw / (N * K):.2f} | {8.0 * bd / (N * K):.2f} | {us:.1f} | "
              f"{(bw + 4 * N * K + bd) / us / 1e3:.0f} |")


    header("GEMM straight from the word pages against the dense pages, 16 x 8192 -> 8192 (the pages are the traffic)")
    for l in (1, 2, 3, 4):
        gemm(f"INT(8|{8 - l}) dense pages", 16, 8192, 8192, l, sets=2)
        gemm(f"INT(8|{8 - l}) word pages", 16, 8192, 8192, l, sets=2, layout=nq.NQ_LAYOUT_PAPER_U64)
    header("the same for a large batch: ViT fc1 12608 x 768 -> 3072, fp32 out (word pages are read once per 32 rows)")
    gemm("INT(8|5) dense pages", 12608, 768, 3072, 3, sets=2)
    gemm("INT(8|5) word pages", 12608, 768, 3072, 3, sets=2, layout=nq.NQ_LAYOUT_PAPER_U64)
    header("convolutions straight from the word pages (rows gathered from the NHWC input), batch 8, int8 out")
    conv("3x3 14x14 256->256 dense pages", 8, 14, 14, 256, 256, 3, 1, 1, 2, sets=2)
    conv("3x3 14x14 256->256 word pages", 8, 14, 14, 256, 256, 3, 1, 1, 2, sets=2, layout=nq.NQ_LAYOUT_PAPER_U64)
    conv("7x7 s2 224x224 3->64 dense pages", 8, 224, 224, 3, 64, 7, 2, 3, 2, sets=2)
    conv("7x7 s2 224x224 3->64 word pages", 8, 224, 224, 3, 64, 7, 2, 3, 2, sets=2, layout=nq.NQ_LAYOUT_PAPER_U64)


if __name__ == "__main__":
    torch.cuda.set_device(0)
    which = sys.argv[1:] or ["c1", "c2", "c3", "c4", "c5", "pack", "page", "sweep", "words", "dw", "lib", "cpu"]
    for name in which:
        {"c1": c1, "c2": c2, "c3": c3, "c4": c4, "c5": c5, "pack": pack, "page": page, "sweep": sweep, "dw": dw, "lib": lib, "cpu": cpu,
         "words": words}[name]()
