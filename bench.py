#!/usr/bin/env python3
"""Benchmark of the dense-op hot path on one MI355X.

A step is one MobileNet-v1 1.0/224 batch-1 inference (stem conv, 13 x (depthwise + pointwise),
pool, fully connected, softmax) through tfx_mobilenet_v1_forward, with weights and the image
already resident in HBM: the quantity Table 1 of the TensorFlow.js paper reports (Section 3.9),
on seeded random weights of the same shapes.  After the timed steps the same process times each
layer, the single-op workloads (small matMul, the 8 x 1024^3 batchMatMul, 1x1 pointwise conv and
3x3 conv2d at batch 1 / 8 / 64, 3x3 depthwise conv at stride 1 and 2 with warm and cold caches)
against the fp32-MFMA or HBM roofline, the whole network at batch 8 and 64, and the CPU oracle on
the host cores as a baseline.

Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3e12   # FLOP/s, dense fp32 matrix peak of MI355X
PEAK_MFMA_F16 = 2.5e15     # FLOP/s, dense fp16 matrix peak (fp32 accumulate)
PEAK_HBM = 8.0e12          # B/s

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by the same counters'
# reading for a plain 205.5 MB copy (profiles/hbm_traffic_counters.txt).  Each entry names the kernel
# source it was measured on, with the digest of that file followed by the shared headers csrc/tfx_internal.h and
# csrc/stream_f16.h; if any of them has changed since, the entry is reported as null.
MEASURED_TRAFFIC = {
    "batch_matmul_8x1024x1024x1024_tB": (100848549, "gemm.hip", "bac39288fc357e2c8673f7ea33783fd405976589242fc0199c98fa77957e03ca"),
    "pointwise_64x56x56x128_to_128": (206181264, "pointwise.hip", "0a9baa78bfad3ce283cef204e55f924712128b899e78c4fe2fc3060cb0f5c4d8"),
    "conv3x3_64x56x56x64_to_64": (104528320, "gemm.hip", "bac39288fc357e2c8673f7ea33783fd405976589242fc0199c98fa77957e03ca"),
    "depthwise_64x112x112x64_s1_cold_rotation": (411139682, "depthwise.hip", "5bf610ceb3e6bbe368ffc0883ae29a9d12cb14357f03d0d20b13db3d36e3b37e"),
    "depthwise_64x112x112x64_s2_cold_rotation": (257119699, "depthwise.hip", "5bf610ceb3e6bbe368ffc0883ae29a9d12cb14357f03d0d20b13db3d36e3b37e"),
    "batch_matmul_f16_1x4096x4096x4096_tB": (235078145, "gemm_f16.hip", "924ffb57eaeeb75ba9838b04777ece730400211aedcaf1172be3e0061bfdce75"),
    "batch_matmul_f16_8x1024x1024x1024_tB": (50493600, "gemm_f16.hip", "924ffb57eaeeb75ba9838b04777ece730400211aedcaf1172be3e0061bfdce75"),
    "pointwise_f16_64x56x56x128_to_128": (104298589, "pointwise_f16.hip", "ce1b39f22ab2de85935114032f7da23fa19670dd2587c5787ce442e1a65ef9ae"),
    "depthwise_f16_64x112x112x64_s1_cold_rotation": (205682029, "conv_f16.hip", "afe6f8ef43c1ef8148e17ecfb1317d9bb5da79a3024c8dff8ff47b6ebdc20a4d"),
    "depthwise_f16_64x112x112x64_s2_cold_rotation": (128552106, "conv_f16.hip", "afe6f8ef43c1ef8148e17ecfb1317d9bb5da79a3024c8dff8ff47b6ebdc20a4d"),
    "pointwise_f16_64x14x14x512_to_512": (30193140, "pointwise_slab_f16.hip", "af2faf347eb820ccf9a29fb135a9ca89ecf628f4ce49a11949d8b30c7e1a5587"),
    "conv3x3_f16_64x56x56x64_to_64": (55026506, "conv_stream_f16.hip", "5d25ba83ebb077dcddf0dcaed1a88b53a1395351810b957ba4056c3c06bc7fe9"),
    "add_f32_64M": (805262989, "elementwise.hip", "7f84a8e7a8ec924bce5600deb9d686a5a76abe82b88ca3d841c7cda5219bee52"),
    "add_f16_64M": (402651879, "elementwise.hip", "7f84a8e7a8ec924bce5600deb9d686a5a76abe82b88ca3d841c7cda5219bee52"),
    "mobilenet_chain_kernel": (121651524, "chain.hip", "d6e4fe4eea090fda5555f06e369f20246b30e6da62bbd03727c1832248106007"),
}


def measured_traffic(name):
    """Counter-measured HBM bytes for a workload, or None if unknown or its kernel source changed since."""
    import hashlib
    if name not in MEASURED_TRAFFIC:
        return None
    nbytes, fname, digest = MEASURED_TRAFFIC[name]
    csrc = os.path.join(ROOT, "paper_1901_05350_amd", "csrc")
    try:
        h = hashlib.sha256()
        for part in (fname, "tfx_internal.h", "stream_f16.h"):
            with open(os.path.join(csrc, part), "rb") as f:
                h.update(f.read())
        return nbytes if h.hexdigest() == digest else None
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-ops", action="store_true", help="skip the per-layer and single-op measurements")
    ap.add_argument("--op", default=None, help="time only this single-op workload (for profiling), e.g. "
                                               "batch_matmul_8x1024x1024x1024_tB; 'list' prints the names")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU; use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1901_05350_amd as tfx
    from paper_1901_05350_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    tfx.lib()
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")

    def time_loop(fn, reps, warmup=5, inner=None):
        """Mean seconds per call of `fn`, GPU-side: `inner` back-to-back launches are captured into a
        HIP graph and the graph is replayed, so the host's per-call cost (about 10 us through Python)
        does not hide the kernels' own duration.  Timed with HIP events on the launch stream."""
        inner = inner or min(reps, 20)
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(inner):
                fn()
        g.replay()
        torch.cuda.synchronize()
        n_rep = max(1, reps // inner)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_rep):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (n_rep * inner)

    def time_single(fn, reps=20):
        """Median seconds of one isolated launch (events around a single call, queue drained before)."""
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3)
        return float(np.median(ts))

    # ---------------- the single-op workloads (each returns its result entry) ----------------
    reps = max(20, min(args.steps, 200))

    def mfma_entry(fn, flop, nbytes, name=None):
        t = time_loop(fn, reps)
        return {"us": round(t * 1e6, 3), "single_launch_us": round(time_single(fn) * 1e6, 2),
                "TFLOPs": round(flop / t / 1e12, 4), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                "roofline": {"bound": "mfma", "achieved": round(flop / t / 1e12, 4), "peak": PEAK_MFMA_F32 / 1e12,
                             "unit": "TFLOP/s", "frac": round(flop / t / PEAK_MFMA_F32, 5),
                             "traffic": measured_traffic(name)}}

    def op_matmul():
        d = inputs.matmul_small(seed=0)
        a, b = dev(d["a"]), dev(d["b"])
        c = tfx.tfx_matmul(a, b)
        return mfma_entry(lambda: tfx.tfx_matmul(a, b, out=c), 2 * 64 * 128 * 64, 81920)

    def op_batch_matmul():
        d = inputs.batch_matmul(seed=3)
        a, b = dev(d["a"]), dev(d["b"])
        c = tfx.tfx_batch_matmul(a, b, False, True)
        return mfma_entry(lambda: tfx.tfx_batch_matmul(a, b, False, True, out=c), 2 * 8 * 1024 ** 3, 3 * 8 * 1024 * 1024 * 4,
                          "batch_matmul_8x1024x1024x1024_tB")

    def op_pointwise(n):
        def build():
            d = inputs.pointwise_conv(seed=1, n=n)
            xx, ff, bb = dev(d["x"]), dev(d["filter"]), dev(d["bias"])
            yy = tfx.tfx_conv2d(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6)
            return mfma_entry(lambda: tfx.tfx_conv2d(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6, out=yy),
                              2 * n * 56 * 56 * 128 * 128, 4 * (xx.numel() + yy.numel() + 128 * 128 + 128),
                              "pointwise_%dx56x56x128_to_128" % n)
        return build

    def op_conv3x3(n):
        """3x3 conv2d 56x56x64 -> 64, stride 1, SAME, bias + ReLU6 (implicit GEMM on the matrix cores)."""
        def build():
            d = inputs.conv_general(5, n, 56, 56, 64, 64, 3, 3)
            xx, ff, bb = dev(d["x"]), dev(d["filter"]), dev(d["bias"])
            yy = tfx.tfx_conv2d(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6)
            return mfma_entry(lambda: tfx.tfx_conv2d(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6, out=yy),
                              2 * n * 56 * 56 * 64 * 64 * 9, 4 * (xx.numel() + yy.numel() + 9 * 64 * 64 + 64),
                              "conv3x3_%dx56x56x64_to_64" % n)
        return build

    def op_depthwise(n, s, copies):
        """copies > 1: rotate over distinct tensors whose total size exceeds the 256 MB last-level cache."""
        def build():
            d = inputs.depthwise_conv(seed=2, n=n)
            ff, bb = dev(d["filter"]), dev(d["bias"])
            xs = [dev(d["x"])]
            for _ in range(copies - 1):
                xs.append(xs[0].clone())
            ys = [tfx.tfx_depthwise_conv2d(xv, ff, bb, s, tfx.PAD_SAME, tfx.ACT_RELU6) for xv in xs]
            nbytes = 4 * (xs[0].numel() + ys[0].numel() + 9 * 64 + 64)
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % copies
                tfx.tfx_depthwise_conv2d(xs[i], ff, bb, s, tfx.PAD_SAME, tfx.ACT_RELU6, out=ys[i])
            t = time_loop(fn, max(reps, copies * 2), warmup=copies, inner=copies if copies > 1 else None)
            e = {"us": round(t * 1e6, 3), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                 "roofline": {"bound": "hbm", "achieved": round(nbytes / t / 1e9, 1), "peak": PEAK_HBM / 1e9,
                              "unit": "GB/s", "frac": round(nbytes / t / PEAK_HBM, 5),
                              "traffic": measured_traffic("depthwise_%dx112x112x64_s%d_%s" % (
                                  n, s, "cold_rotation" if copies > 1 else "warm"))}}
            if copies == 1:
                e["single_launch_us"] = round(time_single(fn) * 1e6, 2)
            return e
        return build

    def op_depthwise_f16(n, s, copies):
        """Depthwise 3x3 112x112x64 + bias + ReLU6 on 16-bit float storage (cold rotation as op_depthwise)."""
        def build():
            d = inputs.depthwise_conv(seed=2, n=n)
            h16 = lambda a: dev(a).to(torch.float16)
            ff, bb = h16(d["filter"]), h16(d["bias"])
            xs = [h16(d["x"])]
            for _ in range(copies - 1):
                xs.append(xs[0].clone())
            ys = [tfx.tfx_depthwise_conv2d_f16(xv, ff, bb, s, tfx.PAD_SAME, tfx.ACT_RELU6) for xv in xs]
            nbytes = 2 * (xs[0].numel() + ys[0].numel() + 9 * 64 + 64)
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % copies
                tfx.tfx_depthwise_conv2d_f16(xs[i], ff, bb, s, tfx.PAD_SAME, tfx.ACT_RELU6, out=ys[i])
            t = time_loop(fn, max(reps, copies * 2), warmup=copies, inner=copies if copies > 1 else None)
            return {"us": round(t * 1e6, 3), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                    "roofline": {"bound": "hbm", "achieved": round(nbytes / t / 1e9, 1), "peak": PEAK_HBM / 1e9,
                                 "unit": "GB/s", "frac": round(nbytes / t / PEAK_HBM, 5),
                                 "traffic": measured_traffic("depthwise_f16_%dx112x112x64_s%d_cold_rotation" % (n, s))}}
        return build

    def op_copy():
        """Plain device-to-device copy of 205.5 MB (a framework elementwise kernel, not part of the library):
        the known-size reference that the HBM traffic counters are scaled by."""
        src = torch.empty(64 * 112 * 112 * 64, device="cuda:0").uniform_(-1, 1)
        dsts = [torch.empty_like(src) for _ in range(2)]
        state = {"i": 0}

        def fn():
            i = state["i"] = (state["i"] + 1) % 2
            dsts[i].copy_(src)
        t = time_loop(fn, reps, inner=4)
        nbytes = 2 * src.numel() * 4
        return {"us": round(t * 1e6, 3), "GBps": round(nbytes / t / 1e9, 1), "bytes_read": src.numel() * 4,
                "bytes_written": src.numel() * 4,
                "roofline": {"bound": "hbm", "achieved": round(nbytes / t / 1e9, 1), "peak": PEAK_HBM / 1e9,
                             "unit": "GB/s", "frac": round(nbytes / t / PEAK_HBM, 5), "traffic": None}}

    def op_add(n, half):
        """Element-wise c = a + b over n elements, rotating over distinct buffer sets (> the 256 MB last-level cache)."""
        def build():
            dt, esz = (torch.float16, 2) if half else (torch.float32, 4)
            copies = max(2, int(1.2e9 // (3 * n * esz)) + 1)
            sets = [(torch.empty(n, device="cuda:0").uniform_(-1, 1).to(dt), torch.empty(n, device="cuda:0").uniform_(-1, 1).to(dt),
                     torch.empty(n, device="cuda:0", dtype=dt)) for _ in range(copies)]
            f = tfx.tfx_add_f16 if half else tfx.tfx_add
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % copies
                f(sets[i][0], sets[i][1], out=sets[i][2])
            t = time_loop(fn, max(reps, copies * 2), warmup=copies, inner=copies)
            nbytes = 3 * n * esz
            return {"us": round(t * 1e6, 3), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                    "roofline": {"bound": "hbm", "achieved": round(nbytes / t / 1e9, 1), "peak": PEAK_HBM / 1e9,
                                 "unit": "GB/s", "frac": round(nbytes / t / PEAK_HBM, 5),
                                 "traffic": measured_traffic("add_f16_64M" if half else "add_f32_64M") if n == 1 << 26 else None}}
        return build

    def op_matmul_f16(batch, m, n, k, tb=True):
        """batchMatMul on 16-bit float storage (fp32 accumulation on the matrix cores); B stored [N,K] if tb."""
        def build():
            a = torch.empty((batch, m, k), device="cuda:0").normal_().to(torch.float16)
            b = torch.empty((batch, n, k) if tb else (batch, k, n), device="cuda:0").normal_().to(torch.float16)
            c = tfx.tfx_batch_matmul_f16(a, b, False, tb)
            fn = lambda: tfx.tfx_batch_matmul_f16(a, b, False, tb, out=c)
            t = time_loop(fn, reps)
            flop, nbytes = 2 * batch * m * n * k, 2 * batch * (m * k + n * k + m * n)
            return {"us": round(t * 1e6, 3), "single_launch_us": round(time_single(fn) * 1e6, 2),
                    "TFLOPs": round(flop / t / 1e12, 3), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                    "roofline": {"bound": "mfma", "achieved": round(flop / t / 1e12, 3), "peak": PEAK_MFMA_F16 / 1e12,
                                 "unit": "TFLOP/s", "frac": round(flop / t / PEAK_MFMA_F16, 5),
                                 "traffic": measured_traffic("batch_matmul_f16_%dx%dx%dx%d%s" % (batch, m, n, k, "_tB" if tb else ""))}}
        return build

    def op_pointwise_f16(n, hw=56, k=128, co=128):
        """1x1 conv hw x hw x k -> co + bias + ReLU6 on 16-bit storage, as a matMul of x [N*hw*hw,k] with the
        filter stored [k,co] (inC, outC).  56x56x128 -> 128 has 3.3 flop per byte moved, 14x14x512 -> 512 has 250
        (the balance of the chip is 312): bound by HBM, not by the matrix cores."""
        def build():
            m = n * hw * hw
            copies = 1 if n < 64 else -(-(3 << 28) // (2 * m * (k + co)))   # rotate over 3 x 256 MB of activations at batch 64
            xs = [torch.empty((1, m, k), device="cuda:0").uniform_(-1, 1).to(torch.float16) for _ in range(copies)]
            f = (torch.empty((1, k, co), device="cuda:0").normal_() * (2.0 / k) ** 0.5).to(torch.float16)
            bias = (torch.empty(co, device="cuda:0").normal_() * 0.01).to(torch.float16)
            ys = [tfx.tfx_batch_matmul_f16(x, f, False, False, bias, tfx.ACT_RELU6) for x in xs]
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % copies
                tfx.tfx_batch_matmul_f16(xs[i], f, False, False, bias, tfx.ACT_RELU6, out=ys[i])
            t = time_loop(fn, max(reps, copies * 2), warmup=copies, inner=copies if copies > 1 else None)
            flop, nbytes = 2 * m * k * co, 2 * (m * k + m * co + k * co + co)
            return {"us": round(t * 1e6, 3), "TFLOPs": round(flop / t / 1e12, 3), "GBps": round(nbytes / t / 1e9, 1),
                    "algorithmic_bytes": nbytes,
                    "roofline": {"bound": "hbm", "achieved": round(nbytes / t / 1e9, 1), "peak": PEAK_HBM / 1e9,
                                 "unit": "GB/s", "frac": round(nbytes / t / PEAK_HBM, 5),
                                 "traffic": measured_traffic("pointwise_f16_%dx%dx%dx%d_to_%d" % (n, hw, hw, k, co))}}
        return build

    def op_conv3x3_f16(n):
        """3x3 conv2d 56x56x64 -> 64, stride 1, SAME, bias + ReLU6 on 16-bit storage (implicit GEMM, fp32 accumulation)."""
        def build():
            d = inputs.conv_general(5, n, 56, 56, 64, 64, 3, 3)
            xx, ff, bb = (dev(d[k]).to(torch.float16) for k in ("x", "filter", "bias"))
            yy = tfx.tfx_conv2d_f16(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6)
            fn = lambda: tfx.tfx_conv2d_f16(xx, ff, bb, 1, tfx.PAD_SAME, tfx.ACT_RELU6, out=yy)
            t = time_loop(fn, reps)
            flop, nbytes = 2 * n * 56 * 56 * 64 * 64 * 9, 2 * (xx.numel() + yy.numel() + 9 * 64 * 64 + 64)
            return {"us": round(t * 1e6, 3), "single_launch_us": round(time_single(fn) * 1e6, 2),
                    "TFLOPs": round(flop / t / 1e12, 3), "GBps": round(nbytes / t / 1e9, 1), "algorithmic_bytes": nbytes,
                    "roofline": {"bound": "mfma", "achieved": round(flop / t / 1e12, 3), "peak": PEAK_MFMA_F16 / 1e12,
                                 "unit": "TFLOP/s", "frac": round(flop / t / PEAK_MFMA_F16, 5),
                                 "traffic": measured_traffic("conv3x3_f16_%dx56x56x64_to_64" % n),
                                 # 144 FLOP per algorithmic byte against the chip's 312: on the HBM side of the roofline
                                 "hbm_frac_of_the_same_launch": round(nbytes / t / PEAK_HBM, 5)}}
        return build

    single_ops = {"matmul_64x128x64": op_matmul, "batch_matmul_8x1024x1024x1024_tB": op_batch_matmul}
    single_ops["batch_matmul_f16_8x1024x1024x1024_tB"] = op_matmul_f16(8, 1024, 1024, 1024)
    single_ops["batch_matmul_f16_1x4096x4096x4096_tB"] = op_matmul_f16(1, 4096, 4096, 4096)
    single_ops["batch_matmul_f16_1x4096x4096x4096"] = op_matmul_f16(1, 4096, 4096, 4096, tb=False)
    single_ops["pointwise_f16_64x56x56x128_to_128"] = op_pointwise_f16(64)
    single_ops["pointwise_f16_8x56x56x128_to_128"] = op_pointwise_f16(8)
    single_ops["pointwise_f16_64x14x14x512_to_512"] = op_pointwise_f16(64, 14, 512, 512)
    single_ops["conv3x3_f16_64x56x56x64_to_64"] = op_conv3x3_f16(64)
    single_ops["conv3x3_f16_8x56x56x64_to_64"] = op_conv3x3_f16(8)
    single_ops["depthwise_f16_64x112x112x64_s1_cold_rotation"] = op_depthwise_f16(64, 1, 6)
    single_ops["depthwise_f16_64x112x112x64_s2_cold_rotation"] = op_depthwise_f16(64, 2, 6)
    single_ops["add_f32_64M"] = op_add(1 << 26, False)
    single_ops["add_f16_64M"] = op_add(1 << 26, True)
    calibration_ops = {"copy_calibration_205MB": op_copy}

    def op_network(nb, f16):
        """The whole network at batch nb alone (for a per-kernel profile of the batched forward pass)."""
        def build():
            dd = (inputs.mobilenet_v1_f16 if f16 else inputs.mobilenet_v1)(seed=4, batch=1)
            model = (tfx.MobileNetV1F16 if f16 else tfx.MobileNetV1)(dd["weights"], batch=nb)
            imgs = torch.empty((nb, 224, 224, 3), device="cuda:0").uniform_(-1, 1)
            imgs = imgs.to(torch.float16) if f16 else imgs
            t = time_loop(lambda: model.forward(imgs), max(20, reps // 4), warmup=3, inner=5)
            return {"ms_per_batch": round(t * 1e3, 4), "images_per_s": round(nb / t, 1),
                    "TFLOPs": round(nb * 1.137480704e9 / t / 1e12, 3)}
        return build
    network_ops = {"mobilenet_v1_batch64": op_network(64, False), "mobilenet_v1_f16_batch64": op_network(64, True),
                   "mobilenet_v1_batch8": op_network(8, False), "mobilenet_v1_f16_batch8": op_network(8, True)}
    for n in (1, 8, 64):
        single_ops["pointwise_%dx56x56x128_to_128" % n] = op_pointwise(n)
        single_ops["conv3x3_%dx56x56x64_to_64" % n] = op_conv3x3(n)
    for s in (1, 2):
        single_ops["depthwise_1x112x112x64_s%d_warm" % s] = op_depthwise(1, s, 1)
        single_ops["depthwise_1x112x112x64_s%d_cold_rotation" % s] = op_depthwise(1, s, 96)
        single_ops["depthwise_8x112x112x64_s%d_warm" % s] = op_depthwise(8, s, 1)
        single_ops["depthwise_64x112x112x64_s%d_cold_rotation" % s] = op_depthwise(64, s, 3)
    if args.op is not None:
        every = {**single_ops, **calibration_ops, **network_ops}
        if args.op not in every:
            print("\n".join(every))
            sys.exit(0 if args.op == "list" else 2)
        print(json.dumps({"op": args.op, **every[args.op]()}))
        return

    # ---------------- the timed steps: MobileNet-v1 b1 ----------------
    data = inputs.mobilenet_v1(seed=4, batch=1)
    model = tfx.MobileNetV1(data["weights"], batch=1)
    image = dev(data["image"])
    step = lambda: model.forward(image)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # The interpreter's cyclic garbage collector is kept out of the timed region (as timeit does): a full
    # collection takes tens of ms in a process that has imported torch, and when it falls into the K steps
    # the GPU runs dry while the host is stopped (measured: 37 ms, twice the whole timed region).
    import gc
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gc.enable()
    ms_per_step = wall * 1e3 / args.steps
    ms_events = e0.elapsed_time(e1) / args.steps
    probs = model.probs.cpu().numpy()
    assert np.isfinite(probs).all() and abs(float(probs.sum()) - 1.0) < 1e-4

    # same forward pass replayed from a captured graph (no memset nodes: the library uses none)
    graph_ms = None
    try:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        ge0, ge1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ge0.record()
        for _ in range(args.steps):
            g.replay()
        ge1.record()
        torch.cuda.synchronize()
        graph_ms = ge0.elapsed_time(ge1) / args.steps
        torch.cuda.synchronize()
        assert np.array_equal(model.probs.cpu().numpy(), probs)
    except Exception as exc:  # reported, not fatal
        graph_ms = None
        print("bench.py: graph replay unavailable: %r" % (exc,), file=sys.stderr)

    out = {
        "metric": "MobileNet-v1 1.0/224 batch-1 ms/inference",
        "value": round(ms_per_step, 5), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "MobileNet-v1 1.0/224 forward, batch 1, fp32 NHWC, random He-normal weights (seed 4), "
                               "input uniform[-1,1)",
                   "launch": "stream enqueue, one C-ABI call per inference = 4 kernel launches (stem + block 1; blocks 2, "
                             "3 and 4 as three stages of one launch; block 5; one chained kernel for blocks 6-13 + pool + "
                             "FC + softmax)"},
        "ms_per_step_hip_events": round(ms_events, 5),
        "graph_replay_ms_per_inference": None if graph_ms is None else round(graph_ms, 5),
        "paper_table1_ms": {"plain JS (MacBook Pro 2014)": 3426, "WebGL Intel Iris Pro": 49, "WebGL GTX 1080": 5,
                            "Node.js CPU AVX2": 87, "Node.js CUDA GTX 1080": 3},
    }

    # ---------------- per-layer times inside the network, and the roofline of its dominant kernel ----------
    if not args.no_ops:
        CH, ST = inputs.MOBILENET_V1_CHANNELS, inputs.MOBILENET_V1_STRIDES
        w = model.tensors
        layers = []
        x = torch.empty((1, 224, 224, 3), device="cuda:0").uniform_(-1, 1)
        y = tfx.tfx_conv2d(x, w["conv0_w"], w["conv0_b"], 2, tfx.PAD_SAME, tfx.ACT_RELU6)
        t = time_loop(lambda: tfx.tfx_conv2d(x, w["conv0_w"], w["conv0_b"], 2, tfx.PAD_SAME, tfx.ACT_RELU6, out=y), reps)
        layers.append({"layer": "conv0", "kind": "stem", "us": t * 1e6, "flop": 2 * 112 * 112 * 32 * 27,
                       "bytes": 4 * (x.numel() + y.numel() + 27 * 32 + 32)})
        x = y
        for i in range(13):
            s, cin, cout = ST[i], x.shape[3], CH[i]
            y = tfx.tfx_depthwise_conv2d(x, w["dw_w"][i], w["dw_b"][i], s, tfx.PAD_SAME, tfx.ACT_RELU6)
            t = time_loop(lambda: tfx.tfx_depthwise_conv2d(x, w["dw_w"][i], w["dw_b"][i], s, tfx.PAD_SAME, tfx.ACT_RELU6, out=y), reps)
            layers.append({"layer": "dw%d" % (i + 1), "kind": "depthwise", "us": t * 1e6, "flop": 2 * 9 * y.numel(),
                           "bytes": 4 * (x.numel() + y.numel() + 10 * cin)})
            x = y
            y = tfx.tfx_conv2d(x, w["pw_w"][i], w["pw_b"][i], 1, tfx.PAD_SAME, tfx.ACT_RELU6)
            t = time_loop(lambda: tfx.tfx_conv2d(x, w["pw_w"][i], w["pw_b"][i], 1, tfx.PAD_SAME, tfx.ACT_RELU6, out=y), reps)
            layers.append({"layer": "pw%d" % (i + 1), "kind": "pointwise", "us": t * 1e6,
                           "flop": 2 * y.numel() * cin, "bytes": 4 * (x.numel() + y.numel() + cin * cout + cout)})
            x = y
        pw = [l for l in layers if l["kind"] == "pointwise"]
        dw = [l for l in layers if l["kind"] == "depthwise"]
        pw_flop, pw_s = sum(l["flop"] for l in pw), sum(l["us"] for l in pw) * 1e-6
        dw_bytes, dw_s = sum(l["bytes"] for l in dw), sum(l["us"] for l in dw) * 1e-6

        # The step's top kernel by time is mobilenet_chain_kernel (blocks 6-13, pool, fully connected layer, softmax
        # in one launch: about 65 % of the step).  The C ABI enqueues it inside the forward call, so its duration is
        # taken as the difference of two graph replays timed with HIP events on the launch stream: the whole forward
        # pass (4 launches) minus its 3 leading launches (stem + block 1, blocks 2 - 4, block 5), which the C ABI runs
        # on their own as tfx_mobilenet_v1_variant_features(end_block = 5).
        head_in = torch.empty((1, 224, 224, 3), device="cuda:0").uniform_(-1, 1)
        head_out = model.features(head_in, 5)

        def head():
            model.features(head_in, 5, out=head_out)
        t_head = time_loop(head, reps, inner=10)
        t_full = time_loop(step, reps, inner=10)
        t_chain = max(t_full - t_head, 1e-9)
        tail_layers = [l for l in layers if l["layer"] in ["dw%d" % i for i in range(6, 14)] + ["pw%d" % i for i in range(6, 14)]]
        chain_flop = sum(l["flop"] for l in tail_layers) + 2 * 1024 * 1000
        chain_bytes = sum(l["bytes"] for l in tail_layers) + 4 * (1024 * 1000 + 1000 + 1000 + 1000)
        out["roofline"] = {
            "kernel": "mobilenet_chain_kernel", "bound": "mfma",
            "achieved": round(chain_flop / t_chain / 1e12, 4), "peak": PEAK_MFMA_F32 / 1e12, "unit": "TFLOP/s",
            "frac": round(chain_flop / t_chain / PEAK_MFMA_F32, 5), "traffic": measured_traffic("mobilenet_chain_kernel"),
            "launches_per_step": 1, "avg_launch_us": round(t_chain * 1e6, 3),
            "algorithmic_flop": chain_flop, "algorithmic_bytes": chain_bytes,
            "hbm_frac_of_the_same_launch": round(chain_bytes / t_chain / PEAK_HBM, 5),
            "how_timed": "graph replay of the whole forward pass (%.2f us) minus graph replay of its 3 leading launches "
                         "(%.2f us), HIP events on the launch stream" % (t_full * 1e6, t_head * 1e6),
            "note": "16 dependent convolution layers + pool + FC + softmax at batch 1: bound by the latency of 18 "
                    "producer-consumer steps (1.3-1.8 us each on this GPU), not by a throughput roofline"}
        head_layers = [l for l in layers if l["layer"] in ("conv0", "dw1", "pw1", "dw2", "pw2", "dw3", "pw3", "dw4", "pw4", "dw5", "pw5")]
        head_flop = sum(l["flop"] for l in head_layers)
        # algorithmic bytes of the 4 launches: the image in, each block's output written once and read once by the
        # next launch (the last one only written), every filter and bias once; the stem's and the depthwise layers'
        # outputs never leave the chip
        head_bytes = 4 * (224 * 224 * 3 + 2 * (112 * 112 * 64 + 56 * 56 * 128 + 56 * 56 * 128 + 28 * 28 * 256) + 28 * 28 * 256 +
                          (27 * 32 + 32) + sum(10 * c for c in (32, 64, 128, 128, 256)) +
                          sum(ci * co + co for ci, co in ((32, 64), (64, 128), (128, 128), (128, 256), (256, 256))))
        out["roofline_other_kernels_of_the_step"] = [
            {"kernel": "separable_block_kernel (stem + block 1; block 5) and separable_chain_kernel (blocks 2, 3, 4 as three "
                       "stages): 3 launches, 11 layers", "bound": "mfma",
             "achieved": round(head_flop / t_head / 1e12, 4), "peak": PEAK_MFMA_F32 / 1e12, "unit": "TFLOP/s",
             "frac": round(head_flop / t_head / PEAK_MFMA_F32, 5), "avg_launch_us": round(t_head * 1e6 / 3, 3),
             "algorithmic_flop": head_flop, "algorithmic_bytes": head_bytes,
             "hbm_frac_of_the_same_launches": round(head_bytes / t_head / PEAK_HBM, 5),
             "the_same_11_layers_as_single_op_launches_us": round(sum(l["us"] for l in head_layers), 2),
             "note": "bound by five dependent steps (argument fetch or flag hand-over, one round trip for the previous "
                     "block's output, split-K reduction, store), not by a throughput roofline"},
            {"kernel": "all 13 pointwise layers as single-op launches (the multi-kernel path of batch > 1; not part of the batch-1 step)", "bound": "mfma",
             "achieved": round(pw_flop / pw_s / 1e12, 4), "peak": PEAK_MFMA_F32 / 1e12, "unit": "TFLOP/s",
             "frac": round(pw_flop / pw_s / PEAK_MFMA_F32, 5), "avg_launch_us": round(pw_s * 1e6 / 13, 3)},
            {"kernel": "all 13 depthwise layers as single-op launches (not part of the batch-1 step)", "bound": "hbm",
             "achieved": round(dw_bytes / dw_s / 1e9, 1), "peak": PEAK_HBM / 1e9, "unit": "GB/s",
             "frac": round(dw_bytes / dw_s / PEAK_HBM, 5), "avg_launch_us": round(dw_s * 1e6 / 13, 3)}]
        out["mobilenet_layers"] = {
            "sum_layer_us": round(sum(l["us"] for l in layers), 2),
            "pointwise_us": round(pw_s * 1e6, 2), "depthwise_us": round(dw_s * 1e6, 2),
            "depthwise_GBps": round(dw_bytes / dw_s / 1e9, 1),
            "per_layer_us": {l["layer"]: round(l["us"], 2) for l in layers}}

        out["ops"] = {name: build() for name, build in single_ops.items()}

        # ---------------- whole network at larger batches (same weights; throughput, not latency) ----------
        batched = {}
        for nb in (8, 64):
            mb = tfx.MobileNetV1(data["weights"], batch=nb)
            imgs = torch.empty((nb, 224, 224, 3), device="cuda:0").uniform_(-1, 1)
            t = time_loop(lambda: mb.forward(imgs), max(20, reps // 4), warmup=3, inner=5)
            batched["batch_%d" % nb] = {"ms_per_batch": round(t * 1e3, 4), "images_per_s": round(nb / t, 1),
                                        "TFLOPs": round(nb * 1.137480704e9 / t / 1e12, 3),
                                        "form": "three parts of the batch on three streams" if nb >= 60 and not os.environ.get("TFX_ONE_STREAM")
                                        else "one chain of kernels"}
            del mb, imgs
        out["mobilenet_batched"] = batched

        # ---------------- other members of the family (width alpha = q/4, input size), batch 1 ----------
        family = {}
        for q, size in ((1, 128), (2, 160), (3, 192)):
            dv = inputs.mobilenet_v1(seed=4, batch=1, image_size=size, width_quarters=q)
            mv = tfx.MobileNetV1(dv["weights"], batch=1, image_size=size, width_quarters=q)
            img = dev(dv["image"])
            t = time_loop(lambda: mv.forward(img), reps, warmup=3, inner=10)
            family["%.2f_%d" % (q / 4, size)] = {"ms_per_inference": round(t * 1e3, 5)}
            del mv, img
        out["mobilenet_family_b1"] = family

        # ---------------- the same network on 16-bit float storage (fp32 accumulation), batch 1 / 8 / 64 ----------
        d16 = inputs.mobilenet_v1_f16(seed=4, batch=1)
        half = {}
        for nb in (1, 8, 64):
            m16 = tfx.MobileNetV1F16(d16["weights"], batch=nb)
            imgs = torch.empty((nb, 224, 224, 3), device="cuda:0").uniform_(-1, 1).to(torch.float16)
            t = time_loop(lambda: m16.forward(imgs), max(20, reps // 4), warmup=3, inner=5)
            half["batch_%d" % nb] = {"ms_per_batch": round(t * 1e3, 4), "images_per_s": round(nb / t, 1),
                                     "TFLOPs": round(nb * 1.137480704e9 / t / 1e12, 3)}
            del m16, imgs
        out["mobilenet_f16"] = half

    # ---------------- CPU oracle on the host cores (baseline only), beside every workload ----------------
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.get_max_threads()

        def cpu_ms(fn, budget_s):
            """Mean ms of fn() on the host: at least one call, then repeated while the budget lasts."""
            fn()
            n, t0 = 0, time.perf_counter()
            while n < 1 or (time.perf_counter() - t0 < budget_s and n < 200):
                fn()
                n += 1
            return (time.perf_counter() - t0) * 1e3 / n, n

        def both(fn, budget_s=0.5, scale=1.0, sample="the whole workload"):
            """Oracle time with one thread and with all of the host's threads; `scale` extrapolates a sample."""
            oracle.set_threads(1)
            one, _ = cpu_ms(fn, budget_s)
            oracle.set_threads(threads)
            many, _ = cpu_ms(fn, budget_s)
            return {"ms_1_thread": round(one * scale, 4), "ms_all_threads": round(many * scale, 4), "threads": threads,
                    "nproc": os.cpu_count(), "kind": "oracle", "sample": sample}

        oracle.set_threads(threads)
        oracle.mobilenet_v1_forward(data["image"], data["weights"])  # warm
        n_inf, t0 = 0, time.perf_counter()
        while n_inf < 3 or (time.perf_counter() - t0 < 8.0 and n_inf < 200):
            oracle.mobilenet_v1_forward(data["image"], data["weights"])
            n_inf += 1
        cpu_all = (time.perf_counter() - t0) * 1e3 / n_inf
        oracle.set_threads(1)
        cpu_one, n_one = cpu_ms(lambda: oracle.mobilenet_v1_forward(data["image"], data["weights"]), 3.0)
        oracle.set_threads(threads)
        out["cpu_baseline"] = {"value": round(cpu_all, 3), "unit": "ms", "cores": threads, "kind": "oracle",
                               "sample": "%d whole MobileNet-v1 b1 inferences (same seeded input), plain C loops with "
                                         "double accumulation, OpenMP over output rows" % n_inf,
                               "value_1_thread": round(cpu_one, 3), "nproc": os.cpu_count()}
        if not args.no_ops:
            ops = out["ops"]
            d = inputs.matmul_small(seed=0)
            ops["matmul_64x128x64"]["cpu_baseline"] = both(lambda: oracle.matmul(d["a"], d["b"]))
            d4 = inputs.batch_matmul(seed=3)
            ops["batch_matmul_8x1024x1024x1024_tB"]["cpu_baseline"] = both(
                lambda: oracle.batch_matmul(d4["a"], d4["b"], False, True), budget_s=0.0, sample="the whole workload, once")
            for n in (1, 8, 64):
                dp = inputs.pointwise_conv(seed=1, n=n)
                ops["pointwise_%dx56x56x128_to_128" % n]["cpu_baseline"] = both(
                    lambda: oracle.conv2d(dp["x"], dp["filter"], dp["bias"], 1, oracle.PAD_SAME, oracle.ACT_RELU6),
                    budget_s=0.3 if n < 64 else 0.0)
                k = min(n, 8)   # 3x3: 9 times the multiply-adds; the batch-64 line times 8 images and scales
                dc = inputs.conv_general(5, k, 56, 56, 64, 64, 3, 3)
                ops["conv3x3_%dx56x56x64_to_64" % n]["cpu_baseline"] = both(
                    lambda: oracle.conv2d(dc["x"], dc["filter"], dc["bias"], 1, oracle.PAD_SAME, oracle.ACT_RELU6),
                    budget_s=0.3 if n == 1 else 0.0, scale=n / k,
                    sample="the whole workload" if k == n else "%d of the %d images, scaled" % (k, n))
            for n, tag in ((1, "warm"), (1, "cold_rotation"), (8, "warm"), (64, "cold_rotation")):
                dd = inputs.depthwise_conv(seed=2, n=n)
                for st in (1, 2):
                    ops["depthwise_%dx112x112x64_s%d_%s" % (n, st, tag)]["cpu_baseline"] = both(
                        lambda: oracle.depthwise_conv2d(dd["x"], dd["filter"], dd["bias"], st, oracle.PAD_SAME, oracle.ACT_RELU6),
                        budget_s=0.2 if n < 64 else 0.0)
            # 16-bit storage: bounded samples (the oracle decodes binary16 element by element)
            r16 = np.random.Generator(np.random.PCG64(6))
            a16 = r16.standard_normal((1, 64, 1024)).astype(np.float16)
            b16 = r16.standard_normal((1, 1024, 1024)).astype(np.float16)
            for name, full_rows in (("batch_matmul_f16_8x1024x1024x1024_tB", 8 * 1024), ("batch_matmul_f16_1x4096x4096x4096_tB", 4096 * 16),
                                    ("batch_matmul_f16_1x4096x4096x4096", 4096 * 16)):
                ops[name]["cpu_baseline"] = both(lambda: oracle.batch_matmul_f16(a16, b16, False, True), budget_s=0.0,
                                                 scale=full_rows / 64, sample="64 rows x 1024 x 1024 of binary16 operands, scaled by the multiply-add count")
            xa = r16.standard_normal(1 << 22).astype(np.float32)
            xb = r16.standard_normal(1 << 22).astype(np.float32)
            ops["add_f32_64M"]["cpu_baseline"] = both(lambda: oracle.add(xa, xb), budget_s=0.0, scale=16, sample="4 Mi of the 64 Mi elements, scaled")
            ha, hb = xa.astype(np.float16), xb.astype(np.float16)
            ops["add_f16_64M"]["cpu_baseline"] = both(lambda: oracle.add_f16(ha, hb), budget_s=0.0, scale=16, sample="4 Mi of the 64 Mi elements, scaled")
            h16 = lambda a: np.ascontiguousarray(a).astype(np.float16)
            dp = inputs.pointwise_conv(seed=1, n=1)
            for n in (8, 64):
                ops["pointwise_f16_%dx56x56x128_to_128" % n]["cpu_baseline"] = both(
                    lambda: oracle.conv2d_f16(h16(dp["x"]), h16(dp["filter"]), h16(dp["bias"]), 1, oracle.PAD_SAME, oracle.ACT_RELU6),
                    budget_s=0.0, scale=n, sample="1 of the %d images, scaled" % n)
            dc = inputs.conv_general(5, 1, 56, 56, 64, 64, 3, 3)
            for n in (8, 64):
                ops["conv3x3_f16_%dx56x56x64_to_64" % n]["cpu_baseline"] = both(
                    lambda: oracle.conv2d_f16(h16(dc["x"]), h16(dc["filter"]), h16(dc["bias"]), 1, oracle.PAD_SAME, oracle.ACT_RELU6),
                    budget_s=0.0, scale=n, sample="1 of the %d images, scaled" % n)
            dd = inputs.depthwise_conv(seed=2, n=4)
            for st in (1, 2):
                ops["depthwise_f16_64x112x112x64_s%d_cold_rotation" % st]["cpu_baseline"] = both(
                    lambda: oracle.depthwise_conv2d_f16(h16(dd["x"]), h16(dd["filter"]), h16(dd["bias"]), st, oracle.PAD_SAME, oracle.ACT_RELU6),
                    budget_s=0.0, scale=16, sample="4 of the 64 images, scaled")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
