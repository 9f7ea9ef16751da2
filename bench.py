"""Throughput of the hot path on one MI355X.

Headline (one JSON line): the ONNX Gemm sweep (M=N=K in {1024, 2048, 4096}, transB=1, 1xN bias,
alpha=beta=1), fp32, inputs resident in HBM; one step = the three Gemms.  The same line carries
  roofline      the matrix-core kernel on the 4096 case against the fp32 MFMA peak, from HIP
                events recorded around that launch inside the timed region;
  cpu_baseline  the CPU oracle timed on one whole step on this machine's host cores;
  details       per-size TFLOP/s; ResNet-50 img/s at batch 32, 1 and a batch sweep, with the per-layer
                sum of rooflines; the attribute-sweep convolutions and MatMuls; the 16-bit Gemm; LSTM;
                the HBM-bound operators (element-wise, reductions, softmax, pooling, depthwise
                convolution) on buffer sets larger than the Infinity Cache.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_FP32_PEAK_TFLOPS = 157.3      # 256 CU x 256 flop/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0
MFMA_16BIT_PEAK_TFLOPS = 2500.0    # dense fp16 / bf16
RAMP_SECONDS = 0.3

# Memory traffic of one Gemm 4096^3 launch from the FETCH_SIZE / WRITE_SIZE counter passes summarised in
# profiles/gemm4096_hbm_traffic.md (fetch scaled by the 2.000 a plain copy shows, write exact).  The
# counters sit between the eight L2s and the fabric, so this is L2 fill + write-back traffic (served by
# the Infinity Cache or HBM).  Reported only while the kernel sources are the ones that were measured.
TRAFFIC_4096 = {"sources_sha256_16": "6d9478fbf125c623", "bytes_per_launch": (196763.6 * 2.000 + 65536.0) * 1024.0}
KERNEL_SOURCES = ("paper_2008_08272_amd/csrc/contraction.h", "paper_2008_08272_amd/csrc/contraction.hip")


def measured_traffic():
    import hashlib
    h = hashlib.sha256()
    try:
        for f in KERNEL_SOURCES:
            with open(os.path.join(ROOT, f), "rb") as fh:
                h.update(fh.read())
    except OSError:
        return None
    return TRAFFIC_4096["bytes_per_launch"] if h.hexdigest()[:16] == TRAFFIC_4096["sources_sha256_16"] else None


def profile_kernels(torch, lib, workloads, dev, with_copy):
    """The four launches of the counter profiles, each 3 untimed + 5 timed calls."""
    def up(a):
        return torch.from_numpy(a).to(dev)

    ws = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    lib.onnx_set_workspace(ws)
    if with_copy:                     # known-size kernel to scale the byte counters with
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    jobs = []
    c = workloads.gemm_case(4096)
    A, B, C = up(c["A"]), up(c["B"]), up(c["C"])
    Y = torch.empty((4096, 4096), dtype=torch.float32, device=dev)
    jobs.append(("gemm_4096", 2.0 * 4096 ** 3, lambda: lib.onnx_gemm(A, B, C, 1.0, 1.0, 0, 1, out=Y)))
    g = torch.Generator(device="cpu").manual_seed(workloads.SEED_BASE)
    X1 = torch.randn(32, 64, 56, 56, generator=g).to(dev)
    W1 = (torch.randn(64, 64, 3, 3, generator=g) * (2.0 / 576) ** 0.5).to(dev)
    B1 = torch.zeros(64, device=dev)
    Y1 = torch.empty(32, 64, 56, 56, device=dev)
    jobs.append(("conv3x3_32x64x56x56", 2.0 * Y1.numel() * 576,
                 lambda: lib.onnx_conv(X1, W1, B1, (1, 1, 1, 1), (1, 1), (1, 1), 1, act=1, out=Y1)))
    for name in ("dilated", "depthwise"):
        cc = workloads.attr_sweep_case(name)
        Xc, Wc, Bc = up(cc["X"]), up(cc["W"]), up(cc["B"])
        yd = lib.onnx_conv_infer(Xc.shape, Wc.shape, cc["pads"], cc["strides"], cc["dilations"], cc["group"])
        Yc = torch.empty(yd, dtype=torch.float32, device=dev)
        flop = 2.0 * Yc.numel() * Wc.shape[1] * Wc.shape[2] * Wc.shape[3]
        jobs.append(("conv_" + name, flop,
                     lambda Xc=Xc, Wc=Wc, Bc=Bc, cc=cc, Yc=Yc: lib.onnx_conv(
                         Xc, Wc, Bc, cc["pads"], cc["strides"], cc["dilations"], cc["group"], out=Yc)))
    out = {}
    for name, flop, fn in jobs:
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        out[name] = {"ms": round(ms, 4), "tflops": round(flop / (ms * 1e-3) / 1e12, 2)}
    print(json.dumps({"profile_kernels": out}))


CONV_LP_SHAPES = (
    # name, N, C, H, W, M, stride, dilation: ResNet-50's 3x3 layers at batch 32, a dilated and a large one
    ("56x56_64", 32, 64, 56, 56, 64, 1, 1),
    ("28x28_128", 32, 128, 28, 28, 128, 1, 1),
    ("14x14_256", 32, 256, 14, 14, 256, 1, 1),
    ("7x7_512", 32, 512, 7, 7, 512, 1, 1),
    ("56x56_128_stride2", 32, 128, 56, 56, 128, 2, 1),
    ("64x64_256_dilation2", 8, 256, 64, 64, 256, 1, 2),
    ("56x56_256_batch64", 64, 256, 56, 56, 256, 1, 1),
)


def profile_conv_lp(torch, lib, dev):
    """3x3 convolutions on bf16 tensors (bf16 result, Relu), each 3 untimed + 5 timed calls."""
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    lib.onnx_set_workspace(ws)
    g = torch.Generator(device="cpu").manual_seed(11)
    out = {}
    for name, n, c, h, w, m, st, dl in CONV_LP_SHAPES:
        X = torch.randn(n, c, h, w, generator=g).to(dev).to(torch.bfloat16)
        W = (torch.randn(m, c, 3, 3, generator=g) * (2.0 / (9 * c)) ** 0.5).to(dev).to(torch.bfloat16)
        Bv = torch.zeros(m, device=dev)
        pads, strides, dil = (dl, dl, dl, dl), (st, st), (dl, dl)
        Y = torch.empty(lib.onnx_conv_infer(X.shape, W.shape, pads, strides, dil), dtype=torch.bfloat16, device=dev)
        fn = lambda: lib.onnx_conv_lp(X, W, Bv, pads, strides, dil, 1, act=1, out=Y)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        out[name] = {"ms": round(ms, 4), "tflops": round(2.0 * Y.numel() * 9 * c / (ms * 1e-3) / 1e12, 1),
                     "launch": lib.onnx_last_launch()}
        del X, W, Y
    print(json.dumps({"profile_conv_lp": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-details", action="store_true", help="skip the ResNet-50 / attribute-sweep extras")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a known-size kernel against which "
                         "hardware byte counters of a profiler run can be scaled)")
    ap.add_argument("--profile-kernels", action="store_true",
                    help="run only the four launches whose hardware counters are summarised under profiles/ "
                         "(Gemm 4096^3, 3x3 conv 32x64x56x56, dilated 3x3 conv, depthwise 3x3 conv), a few "
                         "times each, print their mean times and exit")
    ap.add_argument("--profile-conv-lp", action="store_true",
                    help="run only the 3x3 convolutions on bf16 tensors whose kernel trace and counters are summarised "
                         "under profiles/, a few times each, print their mean times and exit")
    ap.add_argument("--profile-resnet", type=int, nargs="?", const=32, default=0, metavar="BATCH",
                    help="run only ResNet-50 at the given batch (default 32; 3 untimed + 10 timed passes, one call per "
                         "node), print the mean time and exit: the run behind the per-kernel traces under profiles/")
    ap.add_argument("--profile-bf16", action="store_true", help="with --profile-resnet: run the network on bf16 tensors")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads
    import paper_2008_08272_amd as lib

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    def up(a):
        return torch.from_numpy(a).to(dev)

    if args.profile_kernels:
        profile_kernels(torch, lib, workloads, dev, with_copy=args.copy_calibration)
        return
    if args.profile_conv_lp:
        profile_conv_lp(torch, lib, dev)
        return
    if args.profile_resnet:
        from paper_2008_08272_amd.runner import GraphRunner
        r = GraphRunner(workloads.resnet50(args.profile_resnet), dev, dtype=torch.bfloat16 if args.profile_bf16 else None)
        for _ in range(3):
            r.run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            r.run()
        e1.record()
        torch.cuda.synchronize()
        print(json.dumps({"profile_resnet": {"batch": args.profile_resnet, "dtype": "bf16" if args.profile_bf16 else "f32",
                                             "ms": round(e0.elapsed_time(e1) / 10, 4)}}))
        return

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- headline: Gemm sweep -------------------------------------------------------------
    cases = []
    for n in workloads.GEMM_SWEEP_SIZES:
        c = workloads.gemm_case(n)
        A, B, C = up(c["A"]), up(c["B"]), up(c["C"])
        Y = torch.empty((n, n), dtype=torch.float32, device=dev)
        cases.append((n, A, B, C, Y, c))
    flop_step = sum(2.0 * n ** 3 for n in workloads.GEMM_SWEEP_SIZES)

    def step(events=None):
        for n, A, B, C, Y, _ in cases:
            if events is not None and n == 4096:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                lib.onnx_gemm(A, B, C, 1.0, 1.0, 0, 1, out=Y)
                e1.record()
                events.append((e0, e1))
            else:
                lib.onnx_gemm(A, B, C, 1.0, 1.0, 0, 1, out=Y)

    # The device clock needs some tens of milliseconds of load to settle (the first ~25 steps after
    # an idle period run up to 15 % slower): run untimed steps for RAMP_SECONDS, then the W warmup steps.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < RAMP_SECONDS:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flop_step / (ms_per_step * 1e-3) / 1e12
    k4096_ms = float(np.mean([a.elapsed_time(b) for a, b in events]))
    n = 4096
    flop_4096 = 2.0 * n ** 3
    bytes_4096 = 4.0 * (n * n + n * n + n + n * n)
    achieved = flop_4096 / (k4096_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 3), "peak": MFMA_FP32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / MFMA_FP32_PEAK_TFLOPS, 4), "traffic": measured_traffic(),
                "traffic_unit": "bytes per launch at the L2/fabric boundary",
                "kernel": "contraction_kernel<256,256,16; KC,KC; 16-byte loads> on Gemm 4096^3",
                "avg_launch_ms": round(k4096_ms, 4), "algorithmic_flop": flop_4096,
                "algorithmic_bytes": bytes_4096}

    def time_call(fn, iters=50, warm=10):
        """Mean over `iters` back-to-back calls (one event pair around the loop), plus median and
        minimum of the same number of calls timed one by one (an event pair around each)."""
        t_ramp = time.perf_counter()              # host-side set-up let the clock drop: ramp again
        while time.perf_counter() - t_ramp < RAMP_SECONDS / 2:
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        pairs = []
        for _ in range(iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        each = sorted(a.elapsed_time(b) for a, b in pairs)
        return e0.elapsed_time(e1) / iters, each[len(each) // 2], each[0]

    def timing(ms3):
        return {"ms": round(ms3[0], 4), "ms_median": round(ms3[1], 4), "ms_min": round(ms3[2], 4)}

    details = {}
    per_size = {}
    for n, A, B, C, Y, _ in cases:
        t3 = time_call(lambda: lib.onnx_gemm(A, B, C, 1.0, 1.0, 0, 1, out=Y))
        tf = 2.0 * n ** 3 / (t3[0] * 1e-3) / 1e12
        per_size[str(n)] = dict(timing(t3), tflops=round(tf, 2), frac_mfma_peak=round(tf / MFMA_FP32_PEAK_TFLOPS, 4))
    details["gemm_sweep"] = per_size

    if not args.no_details:
        from paper_2008_08272_amd.runner import GraphRunner
        for batch in (32, 1):
            m = workloads.resnet50(batch)
            st = workloads.graph_stats(m)
            r = GraphRunner(m, dev)
            if batch == 1:
                r.capture()             # launch-bound: one HIP graph launch per forward pass
                t3 = time_call(r.replay, iters=50, warm=10)
            else:
                t3 = time_call(r.run, iters=20, warm=5)
            ms = t3[0]
            tf = 2.0 * st["macs"] / (ms * 1e-3) / 1e12
            # per-layer sum of rooflines: each node at the better of the MFMA peak and the HBM peak
            floor_ms = sum(max(2.0 * mac / (MFMA_FP32_PEAK_TFLOPS * 1e12), nb / (HBM_PEAK_GBS * 1e9))
                           for _, _, mac, nb in st["per_node"]) * 1e3
            details["resnet50_b%d" % batch] = dict(timing(t3), img_per_s=round(batch / (ms * 1e-3), 1),
                                                   tflops=round(tf, 2),
                                                   frac_mfma_peak=round(tf / MFMA_FP32_PEAK_TFLOPS, 4),
                                                   sum_of_layer_rooflines_ms=round(floor_ms, 4),
                                                   frac_of_layer_rooflines=round(floor_ms / ms, 4))
            del r
        # the same network on bf16 tensors (weights and activations in bf16, fp32 accumulation, fp32 logits)
        m = workloads.resnet50(32)
        st = workloads.graph_stats(m)
        r = GraphRunner(m, dev, dtype=torch.bfloat16)
        t3 = time_call(r.run, iters=20, warm=5)
        details["resnet50_b32_bf16"] = dict(timing(t3), img_per_s=round(32 / (t3[0] * 1e-3), 1),
                                            tflops=round(2.0 * st["macs"] / (t3[0] * 1e-3) / 1e12, 2))
        del r
        r = GraphRunner(workloads.resnet50(1), dev, dtype=torch.bfloat16)
        r.capture()
        t3 = time_call(r.replay, iters=50, warm=10)
        details["resnet50_b1_bf16"] = dict(timing(t3), img_per_s=round(1 / (t3[0] * 1e-3), 1))
        del r
        # the MNIST-shaped small CNN (1.6 MFLOP): one call per node (5 launches: pure launch latency) and the
        # whole model as one launch (onnx_chain: weights and activations in LDS), at batch 1 and one workgroup
        # per image at batch 64
        r = GraphRunner(workloads.small_cnn(), dev, fuse_chain=False)
        t_eager = time_call(r.run, iters=50, warm=10)
        r.capture()
        t_graph = time_call(r.replay, iters=50, warm=10)
        calls = len(r.calls)
        del r
        r = GraphRunner(workloads.small_cnn(), dev)
        assert r.chain is not None
        t_chain = time_call(r.run, iters=200, warm=20)
        del r
        m64 = workloads.small_cnn()
        m64["inputs"] = {"x": np.random.default_rng(7).uniform(0, 1, (64, 1, 28, 28)).astype(np.float32)}
        m64["graph"] = [dict(nd, shape=(64, 256)) if nd["op"] == "reshape" else nd for nd in m64["graph"]]
        r = GraphRunner(m64, dev)
        assert r.chain is not None
        t_chain64 = time_call(r.run, iters=200, warm=20)
        del r
        details["small_cnn_b1"] = {"us_per_node_calls": round(t_eager[0] * 1e3, 2), "us_per_node_graph": round(t_graph[0] * 1e3, 2),
                                   "calls": calls, "us_one_launch": round(t_chain[0] * 1e3, 2),
                                   "us_one_launch_batch64": round(t_chain64[0] * 1e3, 2)}
        # Gemm on 16-bit inputs (fp32 accumulation), against the 2.5 PFLOP/s dense fp16 / bf16 MFMA peak
        for kind, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
            for n in (4096, 8192):
                A16 = torch.randn(n, n, device=dev).to(tdt)
                B16 = torch.randn(n, n, device=dev).to(tdt)
                C32 = torch.randn(1, n, device=dev)
                Y16 = torch.empty(n, n, device=dev, dtype=tdt)
                t3 = time_call(lambda: lib.onnx_gemm_lp(A16, B16, C32, out=Y16), iters=20, warm=5)
                tf = 2.0 * n ** 3 / (t3[0] * 1e-3) / 1e12
                details["gemm_%s_%d" % (kind, n)] = dict(timing(t3), tflops=round(tf, 1),
                                                         frac_mfma_peak_16bit=round(tf / MFMA_16BIT_PEAK_TFLOPS, 4))
                del A16, B16, C32, Y16
        # 16-bit MatMul and Conv (row-contiguous B through the tuned Gemm kernel; the 3x3 through the LDS-patch kernel)
        A16 = torch.randn(8, 512, 768, device=dev).to(torch.bfloat16)
        B16 = torch.randn(768, 3072, device=dev).to(torch.bfloat16)
        Y16 = torch.empty(8, 512, 3072, device=dev, dtype=torch.bfloat16)
        t3 = time_call(lambda: lib.onnx_matmul_lp(A16, B16, out=Y16), iters=20, warm=5)
        details["matmul_bf16_proj_8x512x768_x_768x3072"] = dict(timing(t3), tflops=round(2.0 * 8 * 512 * 768 * 3072 / (t3[0] * 1e-3) / 1e12, 1))
        del A16, B16, Y16
        for cname, xs, ws_, pads, st in (("conv_bf16_3x3_32x128x28x28", (32, 128, 28, 28), (128, 128, 3, 3), (1, 1, 1, 1), (1, 1)),
                                         ("conv_bf16_1x1_32x1024x14x14", (32, 1024, 14, 14), (256, 1024, 1, 1), (0, 0, 0, 0), (1, 1)),
                                         ("conv_bf16_stem_7x7s2_32x3x224x224", (32, 3, 224, 224), (64, 3, 7, 7), (3, 3, 3, 3), (2, 2))):
            X16 = torch.randn(*xs, device=dev).to(torch.bfloat16)
            W16 = (torch.randn(*ws_, device=dev) * 0.05).to(torch.bfloat16)
            yd = lib.onnx_conv_infer(xs, ws_, pads, st)
            Y16 = torch.empty(yd, device=dev, dtype=torch.bfloat16)
            t3 = time_call(lambda: lib.onnx_conv_lp(X16, W16, None, pads, st, act=1, out=Y16), iters=20, warm=5)
            fl = 2.0 * Y16.numel() * ws_[1] * ws_[2] * ws_[3]
            details[cname] = dict(timing(t3), tflops=round(fl / (t3[0] * 1e-3) / 1e12, 1))
            del X16, W16, Y16
        # ResNet-50's stem alone at batch 32 (7x7 stride 2, 3 -> 64 channels: the resident-filter kernel)
        Xs = torch.randn(32, 3, 224, 224, device=dev)
        Ws = torch.randn(64, 3, 7, 7, device=dev) * 0.1
        Bs = torch.randn(64, device=dev)
        Ys = torch.empty(32, 64, 112, 112, device=dev)
        t3 = time_call(lambda: lib.onnx_conv(Xs, Ws, Bs, (3, 3, 3, 3), (2, 2), act=1, out=Ys), iters=30, warm=5)
        fl = 2.0 * Ys.numel() * 147
        details["conv_stem_7x7s2_32x3x224x224"] = dict(timing(t3), tflops=round(fl / (t3[0] * 1e-3) / 1e12, 2),
                                                       frac_mfma_peak=round(fl / (t3[0] * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS, 4))
        del Xs, Ws, Bs, Ys
        # LSTM: one Gemm for the input projection of the sequence, then one fused launch per time step
        seq, bsz, nin, hid = 64, 32, 512, 512
        Xl = torch.randn(seq, bsz, nin, device=dev)
        Wl = torch.randn(1, 4 * hid, nin, device=dev) / nin ** 0.5
        Rl = torch.randn(1, 4 * hid, hid, device=dev) / hid ** 0.5
        Bl = torch.randn(1, 8 * hid, device=dev) * 0.1
        t3 = time_call(lambda: lib.onnx_lstm(Xl, Wl, Rl, Bl), iters=10, warm=3)
        fl = 2.0 * seq * bsz * 4 * hid * (nin + hid)
        details["lstm_seq64_b32_512_512"] = dict(timing(t3), tflops=round(fl / (t3[0] * 1e-3) / 1e12, 2),
                                                 us_per_step=round(t3[0] * 1e3 / seq, 2))
        del Xl, Wl, Rl, Bl
        # batch sweep through the same runner and kernels (shapes are run-time values: nothing is re-tuned)
        sweep = {}
        for batch in (2, 4, 8, 16, 64):
            m = workloads.resnet50(batch)
            r = GraphRunner(m, dev)
            t3 = time_call(r.run, iters=20, warm=5)
            sweep[str(batch)] = {"ms": round(t3[0], 4), "img_per_s": round(batch / (t3[0] * 1e-3), 1)}
            del r, m
        details["resnet50_batch_sweep"] = sweep
        for name in workloads.ATTR_SWEEP_CONV:
            c = workloads.attr_sweep_case(name)
            X, W, Bv = up(c["X"]), up(c["W"]), up(c["B"])
            yd = lib.onnx_conv_infer(X.shape, W.shape, c["pads"], c["strides"], c["dilations"], c["group"])
            Y = torch.empty(yd, dtype=torch.float32, device=dev)
            t3 = time_call(lambda: lib.onnx_conv(X, W, Bv, c["pads"], c["strides"], c["dilations"], c["group"], out=Y))
            ms = t3[0]
            macs = Y.numel() * W.shape[1] * W.shape[2] * W.shape[3]
            byts = 4.0 * (X.numel() + W.numel() + Y.numel())
            details["conv_" + name] = dict(timing(t3), tflops=round(2.0 * macs / (ms * 1e-3) / 1e12, 3),
                                           frac_mfma_peak=round(2.0 * macs / (ms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS, 4),
                                           gbytes_per_s=round(byts / (ms * 1e-3) / 1e9, 1),
                                           frac_hbm_peak=round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
        for name in workloads.ATTR_SWEEP_MATMUL:
            c = workloads.attr_sweep_case(name)
            A, B = up(c["A"]), up(c["B"])
            Y = torch.empty(lib.onnx_matmul_infer(A.shape, B.shape), dtype=torch.float32, device=dev)
            t3 = time_call(lambda: lib.onnx_matmul(A, B, out=Y))
            ms = t3[0]
            macs = Y.numel() * A.shape[-1]
            byts = 4.0 * (A.numel() + B.numel() + Y.numel())
            details[name] = dict(timing(t3), tflops=round(2.0 * macs / (ms * 1e-3) / 1e12, 3),
                                 frac_mfma_peak=round(2.0 * macs / (ms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS, 4),
                                 gbytes_per_s=round(byts / (ms * 1e-3) / 1e9, 1),
                                 frac_hbm_peak=round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))

    if not args.no_details:
        # Element-wise / reduction / softmax operators and the two HBM-bound window kernels, quoted
        # against the 8 TB/s HBM peak.  Each call of a case works on the next of several buffer sets
        # (at least 4, together above 600 MB) so that the 256 MB Infinity Cache cannot serve them.
        def hbm(name, nbytes, make):
            nsets = max(4, int(600e6 // nbytes) + 1)
            sets = [make() for _ in range(nsets)]
            for f in sets:
                f()
            torch.cuda.synchronize()
            # one HIP graph holding one call per buffer set: these kernels take 10-50 us, less than the
            # host needs to marshal a call, so launching them one by one would time the host
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for f in sets:
                    f()
            t3 = tuple(t / nsets for t in time_call(graph.replay, iters=20, warm=5))
            gb = nbytes / (t3[0] * 1e-3) / 1e9
            details[name] = dict(timing(t3), gbytes_per_s=round(gb, 1), frac_hbm_peak=round(gb / HBM_PEAK_GBS, 4),
                                 buffer_sets=nsets)
            del graph, sets

        shape = (32, 256, 56, 56)                                 # 102.8 MB, ResNet-50's largest activation
        nb = 4.0 * 32 * 256 * 56 * 56

        def rnd(*sh):
            return torch.randn(*sh, device=dev)

        def mk_add():
            a, b, y = rnd(*shape), rnd(*shape), torch.empty(shape, device=dev)
            return lambda: lib.onnx_add(a, b, out=y)

        def mk_bias():
            a, b, y = rnd(*shape), rnd(256, 1, 1), torch.empty(shape, device=dev)
            return lambda: lib.onnx_add(a, b, out=y)

        def mk_relu():
            a, y = rnd(*shape), torch.empty(shape, device=dev)
            return lambda: lib.onnx_relu(a, out=y)

        def mk_leaky():
            a, y = rnd(*shape), torch.empty(shape, device=dev)
            return lambda: lib.onnx_leakyrelu(a, 0.01, out=y)

        def mk_sum_hw():
            a, y = rnd(*shape), torch.empty(32, 256, 1, 1, device=dev)
            return lambda: lib.onnx_reducesum(a, (2, 3), 1, out=y)

        def mk_sum_all():
            a, y = rnd(*shape), torch.empty((), device=dev)
            return lambda: lib.onnx_reducesum(a, None, 0, out=y)

        def mk_softmax():
            a = rnd(8192, 1000)
            y = torch.empty_like(a)
            return lambda: lib.onnx_softmax(a, 1, out=y)

        def mk_maxpool():
            x, y = rnd(32, 64, 112, 112), torch.empty(32, 64, 56, 56, device=dev)
            return lambda: lib.onnx_maxpool(x, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0, out=y)

        def mk_depthwise():
            x, w, b = rnd(8, 256, 56, 56), rnd(256, 1, 3, 3), rnd(256)
            y = torch.empty(8, 256, 56, 56, device=dev)
            return lambda: lib.onnx_conv(x, w, b, (1, 1, 1, 1), (1, 1), (1, 1), 256, out=y)

        # the same operators on bfloat16 tensors (half the bytes)
        def rnd16(*sh):
            return torch.randn(*sh, device=dev).to(torch.bfloat16)

        def mk_add16():
            a, b, y = rnd16(*shape), rnd16(*shape), torch.empty(shape, device=dev, dtype=torch.bfloat16)
            return lambda: lib.onnx_add_lp(a, b, out=y)

        def mk_bias16():
            a, b, y = rnd16(*shape), rnd16(256, 1, 1), torch.empty(shape, device=dev, dtype=torch.bfloat16)
            return lambda: lib.onnx_add_lp(a, b, out=y)

        def mk_leaky16():
            a, y = rnd16(*shape), torch.empty(shape, device=dev, dtype=torch.bfloat16)
            return lambda: lib.onnx_leakyrelu_lp(a, 0.01, out=y)

        def mk_maxpool16():
            x, y = rnd16(32, 64, 112, 112), torch.empty(32, 64, 56, 56, device=dev, dtype=torch.bfloat16)
            return lambda: lib.onnx_maxpool_lp(x, (3, 3), (1, 1, 1, 1), (2, 2), (1, 1), 0, out=y)

        hbm("hbm_add_32x256x56x56", 3 * nb, mk_add)
        hbm("hbm_add_channel_bias_32x256x56x56", 2 * nb, mk_bias)
        hbm("hbm_relu_32x256x56x56", 2 * nb, mk_relu)
        hbm("hbm_leakyrelu_32x256x56x56", 2 * nb, mk_leaky)
        hbm("hbm_reducesum_32x256x56x56_over_hw", nb, mk_sum_hw)
        hbm("hbm_reducesum_all_25.7M", nb, mk_sum_all)
        hbm("hbm_softmax_8192x1000", 8.0 * 8192 * 1000, mk_softmax)
        hbm("hbm_maxpool_3x3s2_32x64x112x112", 4.0 * (32 * 64 * 112 * 112 + 32 * 64 * 56 * 56), mk_maxpool)
        hbm("hbm_depthwise_3x3_8x256x56x56", 4.0 * 2 * 8 * 256 * 56 * 56, mk_depthwise)
        hbm("hbm_add_bf16_32x256x56x56", 1.5 * nb, mk_add16)
        hbm("hbm_add_channel_bias_bf16_32x256x56x56", nb, mk_bias16)
        hbm("hbm_leakyrelu_bf16_32x256x56x56", nb, mk_leaky16)
        hbm("hbm_maxpool_bf16_3x3s2_32x64x112x112", 2.0 * (32 * 64 * 112 * 112 + 32 * 64 * 56 * 56), mk_maxpool16)

    # ---- CPU oracle beside it (a reported baseline, not the target) ---------------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.gemm(cases[0][5]["A"][:8], cases[0][5]["B"], cases[0][5]["C"], 1.0, 1.0, 0, 1)   # load the library
        t0 = time.perf_counter()
        for _, _, _, _, _, c in cases:
            oracle.gemm(c["A"], c["B"], c["C"], 1.0, 1.0, 0, 1)
        dt = time.perf_counter() - t0
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        extra = {}
        if not args.no_details:              # the same oracle on one ResNet-50 image (8.2 GFLOP), for the img/s figures
            from oracle import chain
            m1 = workloads.resnet50(1)
            t0 = time.perf_counter()
            chain.run(m1, keep=())
            extra = {"resnet50_b1_seconds": round(time.perf_counter() - t0, 3)}
        cpu = {"value": round(flop_step / dt / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": "one whole step (the 1024^3, 2048^3 and 4096^3 Gemms) through the fp64-accumulating "
                         "C loop nest, OpenMP over output rows"}
        cpu.update(extra)

    out = {"metric": "ONNX Gemm fp32 throughput on the Gemm sweep (M=N=K in 1024,2048,4096; transB=1, 1xN bias)",
           "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "gemm_sweep_fp32 (three ONNX Gemm calls per step: 1024^3, 2048^3, 4096^3)",
                      "flop_per_step": flop_step},
           "roofline": roofline, "cpu_baseline": cpu, "details": details}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
