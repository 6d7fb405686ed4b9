#!/usr/bin/env python3
"""Benchmark of the block-rotation MXFP4 hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic activations that are
already resident in HBM: fused block rotation + MXFP4 quantization of X (B = 32), then the
W4A4 product against weights that were rotated and quantized offline.  The default
workload is the 8B-shaped MLP layer (X 8192x4096 bf16, W 14336x4096), the largest product
shape, which the MFMA target is quoted on; the HBM target of the rotate+quantize kernel is
quoted on X 16384x8192, measured in the same run and reported under "rotate_quant_16384x8192";
"swiglu_rotate_quant_8192x14336" is the same online step with its producer (silu(gate) * up) fused in.

Prints ONE JSON line.
  value        whole-step throughput: 2*M*N*K useful flops of the layer per second of step
               time (rotate+quantize included), TFLOP/s
  kernels      per-kernel averages: back-to-back launch trains between HIP events on the launch stream
  roofline     the dominant kernel of the step against its roof
  cpu_baseline the C oracle on a bounded sample of the same workload, on the host cores
Buffers rotate through several sets so that no step finds its operands in the 256 MB
last-level cache left behind by the previous one.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MXFP4_PEAK_TFLOPS = 10100.0      # MI355X dense fp4 MFMA, published
BYTES_PER_ELEM = 2 + 0.5 + 1.0 / 32     # bf16 in, 4-bit code out, one scale byte per 32
# Bytes per launch that leave the L2s (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, scaled by a plain copy
# of known size), from the committed counter summary under profiles/; a counter run is not part of a
# bench run, so other workloads (and the row-major layout) report null.
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # 39.3: one fp32 lane-operation per lane and cycle, 256 CUs x 4
                                               # SIMDs x 16 lanes at 2.4 GHz (the 157.3 TFLOP/s figure counts an
                                               # FMA as two and packed fp32 as two more; packed fp32 is not used)
# fp32 lane-operations per element of the SwiGLU-fused online step, bf16 in, B = 32, activation through bf16:
# 2 widenings, 22 of the activation's fixed sequence, 1.5 bf16 rounding, 5 butterfly stages + 1 normalisation,
# 2.5 group maximum / scale / encode / zero fix
SWIGLU_FUSED_OPS_PER_ELEM = 34.0
PROFILED_TRAFFIC = {"mxfp4_gemm_mlp8b_bf16": 617.2e6, "rotate_quant_16384x8192": 340.8e6,
                    "matrix_rotate_quant_16384x8192": 340.9e6, "block_stats_16384x8192": 302.1e6,
                    "swiglu_rotate_quant_8192x14336": 532.2e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--settle-ms", type=float, default=30.0,
                    help="untimed: keep running the step for this long before the warm-up steps, so that the "
                         "clocks have left their idle state (inputs are generated on the CPU while the GPU idles)")
    ap.add_argument("--workload", default="mlp8b", help="llama1b_up | down_sweep | mlp8b | decode")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--layout", default="tiled", choices=["tiled", "rowmajor"],
                    help="layout of the quantized operands between the two kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-aux", action="store_true", help="skip the 16384x8192 rotate+quantize measurement")
    ap.add_argument("--no-library", action="store_true", help="skip the torch._scaled_mm comparison")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy 4 times (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (rows shard without "
              "communication; nothing here uses a second GPU)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2511_04214_amd as brq
    from paper_2511_04214_amd import inputs

    brq.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = inputs.CONFIGS[args.workload]
    M, K, N, B = cfg["M"], cfg["K"], cfg["N"], 32
    gemm_M = 16 if args.workload == "decode" else M
    out_dtype = torch.bfloat16 if args.out_dtype == "bf16" else torch.float32
    out_es = 2 if args.out_dtype == "bf16" else 4

    def to_dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    x_np = inputs.make_x(cfg)
    w_np = inputs.make_w(cfg)
    LAY = args.layout
    import hashlib
    input_sha256 = {"x": hashlib.sha256(np.ascontiguousarray(x_np).tobytes()).hexdigest(),
                    "w": hashlib.sha256(np.ascontiguousarray(w_np).tobytes()).hexdigest()}
    wq0, ws0 = brq.rotate_quantize_fused(to_dev(w_np), B, layout=LAY)          # offline weight preparation
    del w_np
    set_bytes = M * K * BYTES_PER_ELEM + N * K * 0.53125 + gemm_M * N * out_es
    nsets = int(max(2, min(6, 600e6 // set_bytes + 1)))
    xs = [to_dev(x_np)] + [None] * (nsets - 1)
    for i in range(1, nsets):
        xs[i] = xs[0].clone()
    wqs = [wq0] + [wq0.clone() for _ in range(nsets - 1)]
    wss = [ws0] + [ws0.clone() for _ in range(nsets - 1)]
    cbytes, sbytes = brq.operand_bytes(M, K, LAY)
    cshape, sshape = ((M, K // 2), (M, K // 32)) if LAY == "rowmajor" else ((cbytes,), (sbytes,))
    codes = [torch.empty(cshape, dtype=torch.uint8, device="cuda") for _ in range(nsets)]
    scales = [torch.empty(sshape, dtype=torch.uint8, device="cuda") for _ in range(nsets)]

    def rq(j):
        brq.rotate_quantize_fused(xs[j], B, codes=codes[j], scales=scales[j], stream=stream, layout=LAY)

    def gemm(j):
        # the product reads the first gemm_M rows of the quantized activations (all of them but for "decode")
        a_c, a_s = (codes[j][:gemm_M], scales[j][:gemm_M]) if LAY == "rowmajor" else (codes[j], scales[j])
        brq.mxfp4_gemm(a_c, a_s, wqs[j], wss[j], out=ys[j], stream=stream, a_layout=LAY, w_layout=LAY,
                       M=gemm_M, N=N, K=K)
    ys = [torch.empty((gemm_M, N), dtype=out_dtype, device="cuda") for _ in range(nsets)]
    stream = torch.cuda.Stream()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(i):
        j = i % nsets
        rq(j)
        gemm(j)

    # The GPU has idled while the inputs were generated on the CPU, and its clocks take some
    # milliseconds of load to come up (10 warm-up steps alone measure 280 us per step, 100 measure 245):
    # untimed steps for --settle-ms first, then the W warm-up steps, then the K timed ones.
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for i in range(8):
            step(i)
        stream.synchronize()
    for i in range(args.warmup):
        step(i)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # Per-kernel time: a train of back-to-back launches of that kernel alone between two events on the
    # launch stream, repeated 5 times (a pair of events around every single launch would add the
    # launch gap, 5-6 us, to the short row-wise kernel).
    def train(launch, reps=5):
        # the clocks take a few milliseconds of load to settle: run the kernel for about that long first
        for i in range(max(args.warmup, 200 if launch is rq else 20)):
            launch(i % nsets)
        stream.synchronize()
        out = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(args.steps):
                launch(i % nsets)
            b.record(stream)
            stream.synchronize()
            out.append(a.elapsed_time(b) / args.steps)
        return np.array(out)

    rq_ms = train(rq)
    gm_ms = train(gemm)
    # the same product on ONE buffer set: operands stay in the 256 MB memory-side cache ("warm")
    gm_warm_ms = train(lambda j: gemm(0), reps=3)
    # the same launch on constant operands (all codes 0, all scales 2^0): what the schedule does when the
    # chip's clock management is not reacting to switching activity in the matrix cores
    zc, zs = torch.zeros_like(codes[0]), torch.full_like(scales[0], 127)
    zwc, zws = torch.zeros_like(wqs[0]), torch.full_like(wss[0], 127)

    def gemm_const(j):
        a_c, a_s = (zc[:gemm_M], zs[:gemm_M]) if LAY == "rowmajor" else (zc, zs)
        brq.mxfp4_gemm(a_c, a_s, zwc, zws, out=ys[0], stream=stream, a_layout=LAY, w_layout=LAY, M=gemm_M, N=N, K=K)
    gm_const_ms = train(gemm_const, reps=3)
    # the shader clock the chip holds during the product (cycle and 100 MHz counters of the kernel's first
    # workgroup), on the workload's operands and on the constant ones
    gm_clock = {}
    if gemm_M > 128 and N % 256 == 0:
        clk = torch.zeros(2, dtype=torch.int64, device="cuda")

        def clocked(a_c, a_s, w_c, w_s):
            vals = []
            for _ in range(3):      # the last launch of a train of back-to-back ones (every launch overwrites clk)
                for i in range(20):
                    brq.mxfp4_gemm(a_c, a_s, w_c, w_s, out=ys[0], stream=stream, a_layout=LAY, w_layout=LAY, M=gemm_M, N=N,
                                   K=K, clock=clk)
                stream.synchronize()
                c, t = clk.tolist()
                vals.append(0.1 * c / max(t, 1))
            return float(np.mean(vals))
        for i in range(40):
            gemm(i % nsets)
        a_c, a_s = (codes[0][:gemm_M], scales[0][:gemm_M]) if LAY == "rowmajor" else (codes[0], scales[0])
        gm_clock["shader_clock_GHz"] = clocked(a_c, a_s, wqs[0], wss[0])
        for i in range(40):
            gemm_const(0)
        a_c, a_s = (zc[:gemm_M], zs[:gemm_M]) if LAY == "rowmajor" else (zc, zs)
        gm_clock["constant_operands_shader_clock_GHz"] = clocked(a_c, a_s, zwc, zws)
    del zc, zs, zwc, zws

    ms_per_step = wall * 1e3 / args.steps
    rq_bytes = M * K * BYTES_PER_ELEM
    gemm_flops = 2.0 * gemm_M * N * K
    gemm_bytes = (gemm_M + N) * K * 0.53125 + gemm_M * N * out_es
    rq_avg, gm_avg = float(rq_ms.mean()), float(gm_ms.mean())
    if "shader_clock_GHz" in gm_clock:   # the published peak is quoted at 2.4 GHz: the same ratio at the clock held
        gm_clock["frac_mxfp4_peak_at_held_clock"] = (2.0 * gemm_M * N * K / float(gm_ms.mean()) / 1e9 / MXFP4_PEAK_TFLOPS
                                                     * 2.4 / gm_clock["shader_clock_GHz"])
    kernels = {
        "rotate_quantize_fused": {"avg_ms": rq_avg, "median_ms": float(np.median(rq_ms)), "min_ms": float(rq_ms.min()),
                                  "alg_bytes": rq_bytes,
                                  "GB/s": rq_bytes / rq_avg / 1e6,
                                  "frac_hbm_peak": rq_bytes / rq_avg / 1e6 / HBM_PEAK_GBS},
        "mxfp4_gemm": {"avg_ms": gm_avg, "median_ms": float(np.median(gm_ms)), "min_ms": float(gm_ms.min()),
                       "warm_cache_avg_ms": float(gm_warm_ms.mean()),
                       "constant_operands_avg_ms": float(gm_const_ms.mean()),
                       "constant_operands_frac_mxfp4_peak": gemm_flops / float(gm_const_ms.mean()) / 1e9 / MXFP4_PEAK_TFLOPS,
                       **gm_clock,
                       "flops": gemm_flops, "alg_bytes": gemm_bytes,
                       "TFLOP/s": gemm_flops / gm_avg / 1e9,
                       "frac_mxfp4_peak": gemm_flops / gm_avg / 1e9 / MXFP4_PEAK_TFLOPS,
                       "GB/s": gemm_bytes / gm_avg / 1e6, "frac_hbm_peak": gemm_bytes / gm_avg / 1e6 / HBM_PEAK_GBS},
    }
    if args.workload == "decode":     # M = 16 product: weight streaming, HBM bound
        roofline = {"kernel": "mxfp4_gemm (M=16, weight streaming)", "bound": "hbm",
                    "achieved": kernels["mxfp4_gemm"]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": kernels["mxfp4_gemm"]["frac_hbm_peak"], "traffic": None}
    else:
        roofline = {"kernel": "mxfp4_gemm", "bound": "mfma", "achieved": kernels["mxfp4_gemm"]["TFLOP/s"],
                    "peak": MXFP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": kernels["mxfp4_gemm"]["frac_mxfp4_peak"],
                    "traffic": PROFILED_TRAFFIC.get("mxfp4_gemm_%s_%s" % (args.workload, args.out_dtype))
                    if LAY == "tiled" else None}

    # ---- what the chip sustains on the block-scaled MFMA alone, fed from registers with bit patterns
    # of this workload (the first 2 KB of quantized activations): the ceiling of any product kernel
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty((ncu * 256,), dtype=torch.float32, device="cuda")
    with torch.cuda.stream(stream):
        ops = codes[0].flatten()[:2048].clone()
    c_iters = 2000
    c_flops = brq.diag_mfma_ceiling(ops, 50, ncu, sink=sink, stream=stream)
    c_ms = []
    for _ in range(3):
        a, b = ev(), ev()
        a.record(stream)
        for _ in range(3):
            c_flops = brq.diag_mfma_ceiling(ops, c_iters, ncu, sink=sink, stream=stream)
        b.record(stream)
        stream.synchronize()
        c_ms.append(a.elapsed_time(b) / 3)
    c_clk = sink[:2].tolist()
    zops = torch.zeros_like(ops)
    z_ms = []
    for _ in range(3):
        a, b = ev(), ev()
        a.record(stream)
        for _ in range(3):
            brq.diag_mfma_ceiling(zops, c_iters, ncu, sink=sink, stream=stream)
        b.record(stream)
        stream.synchronize()
        z_ms.append(a.elapsed_time(b) / 3)
    z_clk = sink[:2].tolist()
    ceiling = {"TFLOP/s": c_flops / (sum(c_ms) / len(c_ms)) / 1e9,
               "frac_mxfp4_peak": c_flops / (sum(c_ms) / len(c_ms)) / 1e9 / MXFP4_PEAK_TFLOPS,
               "shader_clock_GHz": 0.1 * c_clk[0] / max(c_clk[1], 1.0),
               "zero_operands_shader_clock_GHz": 0.1 * z_clk[0] / max(z_clk[1], 1.0),
               "zero_operands_TFLOP/s": c_flops / (sum(z_ms) / len(z_ms)) / 1e9,
               "zero_operands_frac_mxfp4_peak": c_flops / (sum(z_ms) / len(z_ms)) / 1e9 / MXFP4_PEAK_TFLOPS,
               "note": "v_mfma_scale_f32_32x32x64 fp4 back to back from registers on every CU, operand "
                       "bit patterns from this workload's quantized activations"}

    # ---- context: the same product through the vendor library as PyTorch exposes it
    # (torch._scaled_mm on float4_e2m1fn_x2 operands with e8m0 group scales = hipBLASLt), on
    # row-major copies of this workload's operands
    library = None
    if not args.no_library and gemm_M >= 32:
        try:
            a_c, a_s = (codes[0], scales[0]) if LAY == "rowmajor" else brq.to_rowmajor(codes[0], scales[0], M, K, stream=stream)
            w_c, w_s = (wq0, ws0) if LAY == "rowmajor" else brq.to_rowmajor(wq0, ws0, N, K, stream=stream)
            stream.synchronize()
            f4, e8 = torch.float4_e2m1fn_x2, torch.float8_e8m0fnu
            ta, tb = a_c[:gemm_M].view(f4), w_c.view(f4).t()
            tsa, tsb = a_s[:gemm_M].contiguous().view(e8), w_s.view(e8)
            with torch.cuda.stream(stream):
                for _ in range(20):
                    torch._scaled_mm(ta, tb, scale_a=tsa, scale_b=tsb, out_dtype=out_dtype)
                l_ms = []
                for _ in range(3):
                    a, b = ev(), ev()
                    a.record(stream)
                    for _ in range(args.steps):
                        torch._scaled_mm(ta, tb, scale_a=tsa, scale_b=tsb, out_dtype=out_dtype)
                    b.record(stream)
                    stream.synchronize()
                    l_ms.append(a.elapsed_time(b) / args.steps)
            l_avg = sum(l_ms) / len(l_ms)
            library = {"what": "torch._scaled_mm (hipBLASLt MXFP4) on the same operands, warm cache",
                       "avg_ms": l_avg, "TFLOP/s": gemm_flops / l_avg / 1e9,
                       "this_kernel_warm_cache_avg_ms": float(gm_warm_ms.mean())}
            del a_c, a_s, w_c, w_s, ta, tb, tsa, tsb
        except Exception as e:      # the comparison is context, never a reason to fail the bench
            library = {"what": "torch._scaled_mm unavailable: %s" % str(e)[:200]}

    # ---- the rotate+quantize kernel on the shape its HBM target is quoted on
    aux = None
    aux_m = None
    aux_s = None
    if not args.no_aux:
        del xs, codes, scales, ys, wqs, wss
        torch.cuda.empty_cache()
        acfg = inputs.CONFIGS["decode"]
        aM, aK = acfg["M"], acfg["K"]
        ax_np = inputs.make_x(acfg) if args.workload != "decode" else x_np
        axs = [to_dev(ax_np)]
        axs.append(axs[0].clone())
        axs.append(axs[0].clone())
        acb, asb = brq.operand_bytes(aM, aK, LAY)
        ac = [torch.empty((aM, aK // 2) if LAY == "rowmajor" else (acb,), dtype=torch.uint8, device="cuda") for _ in range(3)]
        asc = [torch.empty((aM, aK // 32) if LAY == "rowmajor" else (asb,), dtype=torch.uint8, device="cuda") for _ in range(3)]
        for i in range(max(args.warmup, 200)):      # ~12 ms: the clocks settle only under sustained load
            brq.rotate_quantize_fused(axs[i % 3], B, codes=ac[i % 3], scales=asc[i % 3], stream=stream, layout=LAY)
        stream.synchronize()
        ams = []
        for _ in range(5):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(args.steps):
                brq.rotate_quantize_fused(axs[i % 3], B, codes=ac[i % 3], scales=asc[i % 3], stream=stream, layout=LAY)
            b.record(stream)
            stream.synchronize()
            ams.append(a.elapsed_time(b) / args.steps)
        ams = np.array(ams)
        ab = aM * aK * BYTES_PER_ELEM
        aux = {"kernel": "rotate_quantize_fused", "bound": "hbm", "avg_ms": float(ams.mean()),
               "min_ms": float(ams.min()), "alg_bytes": ab, "achieved": ab / float(ams.mean()) / 1e6,
               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ab / float(ams.mean()) / 1e6 / HBM_PEAK_GBS,
               "traffic": PROFILED_TRAFFIC["rotate_quant_16384x8192"] if LAY == "tiled" else None}
        # what the online rotation costs (Sec. 4.2 "reduced online computing", Table "latency overhead"): the same
        # activations through the quantizer alone, with the block rotation, and with the global one (B = K)
        rot = {}
        for name, fn in (("quantize_only", lambda i: brq.mxfp4_quantize(axs[i % 3], codes=ac[i % 3], scales=asc[i % 3],
                                                                      stream=stream, layout=LAY)),
                         ("block_128", lambda i: brq.rotate_quantize_fused(axs[i % 3], 128, codes=ac[i % 3], scales=asc[i % 3],
                                                                          stream=stream, layout=LAY)),
                         ("global_%d" % aK, lambda i: brq.rotate_quantize_fused(axs[i % 3], aK, codes=ac[i % 3],
                                                                               scales=asc[i % 3], stream=stream, layout=LAY))):
            for i in range(100):
                fn(i)
            stream.synchronize()
            ts = []
            for _ in range(3):
                a, b = ev(), ev()
                a.record(stream)
                for i in range(args.steps):
                    fn(i)
                b.record(stream)
                stream.synchronize()
                ts.append(a.elapsed_time(b) / args.steps)
            rot[name + "_ms"] = float(np.mean(ts))
        rot["block_%d_ms" % B] = float(ams.mean())
        aux["online_rotation_cost"] = rot
        # the same step with caller-supplied orthogonal 32x32 blocks (one per block of K) on the matrix cores
        rng_r = np.random.default_rng(11)
        Rb = torch.from_numpy(np.stack([np.linalg.qr(rng_r.standard_normal((32, 32)))[0]
                                        for _ in range(aK // 32)]).astype(np.float32)).cuda()
        for i in range(200):
            brq.matrix_rotate_quantize_fused(axs[i % 3], Rb, codes=ac[i % 3], scales=asc[i % 3], stream=stream, layout=LAY)
        stream.synchronize()
        mms = []
        for _ in range(5):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(args.steps):
                brq.matrix_rotate_quantize_fused(axs[i % 3], Rb, codes=ac[i % 3], scales=asc[i % 3], stream=stream, layout=LAY)
            b.record(stream)
            stream.synchronize()
            mms.append(a.elapsed_time(b) / args.steps)
        mms = np.array(mms)
        aux_m = {"kernel": "matrix_rotate_quantize_fused", "blocks": "%d orthogonal 32x32 fp32 matrices" % (aK // 32),
                 "bound": "hbm", "avg_ms": float(mms.mean()), "min_ms": float(mms.min()), "alg_bytes": ab,
                 "achieved": ab / float(mms.mean()) / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": ab / float(mms.mean()) / 1e6 / HBM_PEAK_GBS,
                 "traffic": PROFILED_TRAFFIC["matrix_rotate_quant_16384x8192"] if LAY == "tiled" else None,
                 "mfma_flops": 3 * 2.0 * aM * aK * 32}
        # block statistics of the same activations after the block rotation (scales, loss, two thresholds)
        st_counts = torch.zeros(2, dtype=torch.int64, device="cuda")
        for i in range(100):
            brq.block_stats(axs[i % 3], B, (1.5, 3.0), counts=st_counts, stream=stream)
        stream.synchronize()
        sms = []
        for _ in range(5):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(args.steps):
                brq.block_stats(axs[i % 3], B, (1.5, 3.0), counts=st_counts, stream=stream)
            b.record(stream)
            stream.synchronize()
            sms.append(a.elapsed_time(b) / args.steps)
        # the same call with the FP16-scale loss as a fourth output (8 divisions per 8 values more)
        st_b = torch.empty((aM, aK // 32), dtype=torch.float32, device="cuda")
        st_a, st_q = torch.empty_like(st_b), torch.empty_like(st_b)
        bms = []
        for _ in range(3):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(args.steps):
                brq.block_stats(axs[i % 3], B, (1.5, 3.0), counts=st_counts, amax=st_a, sqerr=st_q, sqerr_bfp4=st_b, stream=stream)
            b.record(stream)
            stream.synchronize()
            bms.append(a.elapsed_time(b) / args.steps)
        sbytes = aM * aK * (2 + 8.0 / 32)
        aux_s = {"kernel": "block_stats", "what": "block-wise scale + MXFP4 loss per block + counts above 1.5 and 3.0, B = 32",
                 "bound": "hbm", "avg_ms": float(np.mean(sms)), "alg_bytes": sbytes,
                 "achieved": sbytes / float(np.mean(sms)) / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": sbytes / float(np.mean(sms)) / 1e6 / HBM_PEAK_GBS,
                 "traffic": PROFILED_TRAFFIC["block_stats_16384x8192"],
                 "with_fp16_scale_loss_ms": float(np.mean(bms))}
        del axs, ac, asc, Rb, st_a, st_q, st_b

    # ---- the online step with its producer fused in: silu(gate) * up -> rotation -> MXFP4 on the
    # down_proj input of the 8B MLP (8192 tokens x 14336), against the two-kernel path
    aux2 = None
    if not args.no_aux:
        sM, sK = 8192, 14336
        gen = torch.Generator(device="cuda")
        gen.manual_seed(7)
        gus = [(torch.randn((sM, 2 * sK), device="cuda", generator=gen) * 1.5).to(torch.bfloat16) for _ in range(2)]
        scb, ssb = brq.operand_bytes(sM, sK, LAY)
        sc = [torch.empty((sM, sK // 2) if LAY == "rowmajor" else (scb,), dtype=torch.uint8, device="cuda") for _ in range(2)]
        ss = [torch.empty((sM, sK // 32) if LAY == "rowmajor" else (ssb,), dtype=torch.uint8, device="cuda") for _ in range(2)]
        hbuf = torch.empty((sM, sK), dtype=torch.bfloat16, device="cuda")

        def fused(i):
            g = gus[i % 2]
            brq.swiglu_rotate_quantize_fused(g[:, :sK], g[:, sK:], B, h_dtype=torch.bfloat16, codes=sc[i % 2],
                                             scales=ss[i % 2], stream=stream, layout=LAY)

        def two_kernels(i):
            g = gus[i % 2]
            brq.swiglu(g[:, :sK], g[:, sK:], out=hbuf, stream=stream)
            brq.rotate_quantize_fused(hbuf, B, codes=sc[i % 2], scales=ss[i % 2], stream=stream, layout=LAY)

        res = {}
        for name, fn in (("fused", fused), ("two_kernels", two_kernels)):
            for i in range(100):
                fn(i)
            stream.synchronize()
            ts = []
            for _ in range(5):
                a, b = ev(), ev()
                a.record(stream)
                for i in range(args.steps):
                    fn(i)
                b.record(stream)
                stream.synchronize()
                ts.append(a.elapsed_time(b) / args.steps)
            res[name] = float(np.mean(ts))
        sb_ = sM * sK * (4 + 0.5 + 1.0 / 32)
        ops = sM * sK * SWIGLU_FUSED_OPS_PER_ELEM
        aux2 = {"kernel": "swiglu_rotate_quantize_fused", "shape": "gate, up 8192x14336 bf16 (one 8192x28672 buffer)",
                "bound": "alu", "avg_ms": res["fused"], "ops_per_elem": SWIGLU_FUSED_OPS_PER_ELEM,
                "achieved": ops / res["fused"] / 1e9, "peak": VALU_PEAK_TOPS, "unit": "Tlane-op/s",
                "frac": ops / res["fused"] / 1e9 / VALU_PEAK_TOPS,
                "alg_bytes": sb_, "GB/s": sb_ / res["fused"] / 1e6, "frac_hbm_peak": sb_ / res["fused"] / 1e6 / HBM_PEAK_GBS,
                "two_kernel_path_ms": res["two_kernels"],
                "traffic": PROFILED_TRAFFIC["swiglu_rotate_quant_8192x14336"] if LAY == "tiled" else None}
        del gus, sc, ss, hbuf

    # ---- decode batches: the product M x 28672 x 8192 (gate_up of the 8B MLP against one batch of tokens),
    # weight streaming, HBM bound: two weight copies alternate so that no launch finds them in the cache
    aux3 = None
    if not args.no_aux:
        dN, dK = 28672, 8192
        gen = torch.Generator(device="cuda")
        gen.manual_seed(8)
        dws = []
        for _ in range(2):
            wbf = (torch.randn((dN, dK), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
            dws.append(brq.rotate_quantize_fused(wbf, B, layout=LAY))
            del wbf
        dx = torch.randn((128, dK), device="cuda", generator=gen).to(torch.bfloat16)
        aux3 = {"kernel": "mxfp4_gemm", "shape": "M x 28672 x 8192, bf16 out", "bound": "hbm", "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "alg_bytes_weights": dN * dK * 0.53125, "batches": {}}
        for dM in (16, 32, 64, 128):
            dq = brq.rotate_quantize_fused(dx[:dM].contiguous(), B, layout=LAY)
            dy = torch.empty((dM, dN), dtype=torch.bfloat16, device="cuda")

            def dgemm(i):
                brq.mxfp4_gemm(dq[0], dq[1], dws[i % 2][0], dws[i % 2][1], out=dy, stream=stream, a_layout=LAY,
                               w_layout=LAY, M=dM, N=dN, K=dK)
            for i in range(60):
                dgemm(i)
            stream.synchronize()
            ts = []
            for _ in range(3):
                a, b = ev(), ev()
                a.record(stream)
                for i in range(args.steps):
                    dgemm(i)
                b.record(stream)
                stream.synchronize()
                ts.append(a.elapsed_time(b) / args.steps)
            t = float(np.mean(ts))
            by = (dN + dM) * dK * 0.53125 + dM * dN * 2
            aux3["batches"][str(dM)] = {"avg_ms": t, "achieved": by / t / 1e6, "frac": by / t / 1e6 / HBM_PEAK_GBS}
        del dws, dx

    if args.calibrate_copy:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        o = oracle.default()
        threads = o.get_threads()
        rows = int(min(M, max(64, 6e7 // K)))
        t0 = time.perf_counter()
        rc, rs = o.rotate_quantize_fused(x_np[:rows], B)
        t_rq = time.perf_counter() - t0
        grows = int(min(gemm_M, rows, max(1, 2e11 // (N * K))))       # some 10 s of oracle work
        wq_r, ws_r = (wq0, ws0) if LAY == "rowmajor" else brq.to_rowmajor(wq0, ws0, N, K)
        wq_h, ws_h = wq_r.cpu().numpy(), ws_r.cpu().numpy()
        t0 = time.perf_counter()
        o.mxfp4_gemm(rc[:grows], rs[:grows], wq_h, ws_h, want_bound=False)
        t_g = time.perf_counter() - t0
        # the same unit as `value`: useful layer flops per second of (rotate+quantize + product) time,
        # both legs scaled to the full M rows
        t_full = t_rq * (M / rows) + t_g * (gemm_M / grows)
        # the same two legs on one thread, on smaller samples (1/8 and 1/32)
        o.set_threads(1)
        r1, g1 = max(1, rows // 8), max(1, grows // 32)
        t0 = time.perf_counter()
        o.rotate_quantize_fused(x_np[:r1], B)
        t_rq1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        o.mxfp4_gemm(rc[:g1], rs[:g1], wq_h, ws_h, want_bound=False)
        t_g1 = time.perf_counter() - t0
        o.set_threads(threads)
        t_full1 = t_rq1 * (M / r1) + t_g1 * (gemm_M / g1)
        cpu_baseline = {
            "value": gemm_flops / t_full / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "value_one_thread": gemm_flops / t_full1 / 1e12,
            "sample": "rotate+quantize of the first %d of %d rows in %.2f s (%.2f GB/s); product of %d rows "
                      "x N=%d x K=%d in %.2f s incl. dequantizing W (%.4f TFLOP/s); both scaled linearly to M=%d"
                      % (rows, M, t_rq, rows * K * BYTES_PER_ELEM / t_rq / 1e9, grows, N, K, t_g,
                         2.0 * grows * N * K / t_g / 1e12, M)}

    out = {
        "metric": "rotate+quant GB/s (% HBM peak); MXFP4 GEMM TFLOPS (% MXFP4 MFMA peak)",
        "value": gemm_flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "value_note": "whole step: 2*M*N*K of the layer / (rotate+quantize + product) wall time",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_settle_ms": args.settle_ms,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "mxfp4",
        "data": "synthetic",
        "config": {"workload": "%s: X %dx%d bf16 -> block Hadamard B=32 + MXFP4; product M=%d N=%d K=%d, %s out"
                               % (args.workload, M, K, gemm_M, N, K, args.out_dtype), "buffer_sets": nsets,
                   "operand_layout": LAY, "input_sha256": input_sha256},
        "rotate_quant_GBps": kernels["rotate_quantize_fused"]["GB/s"],
        "gemm_TFLOPs": kernels["mxfp4_gemm"]["TFLOP/s"],
        "roofline": roofline,
        "mfma_loop_ceiling": ceiling,
        "library_baseline": library,
        "rotate_quant_16384x8192": aux,
        "matrix_rotate_quant_16384x8192": aux_m,
        "block_stats_16384x8192": aux_s,
        "decode_batches_28672x8192": aux3,
        "swiglu_rotate_quant_8192x14336": aux2,
        "kernels": kernels,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
