#!/usr/bin/env python3
"""Benchmark of the block-rotation MXFP4 hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic activations that are
already resident in HBM: fused block rotation + MXFP4 quantization of X (B = 32), then the
W4A4 product against weights that were rotated and quantized offline.  The default
workload is the 8B-shaped MLP layer (X 8192x4096 bf16, W 14336x4096), the largest product
shape, which the MFMA target is quoted on; the HBM target of the rotate+quantize kernel is
quoted on X 16384x8192, measured in the same run and reported under "rotate_quant_16384x8192".
"configs" holds both kernels on every other workload of the benchmark definition (the tiny layer, the
1B-shaped up-projection, the down-projection at every rotation block of its sweep) and the fp32-output
product of the default one; "swiglu_rotate_quant_8192x14336" is the online step with its producer
(silu(gate) * up) fused in.

Prints ONE JSON line.
  value        whole-step throughput: 2*M*N*K useful flops of the layer per second of step
               time (rotate+quantize included), TFLOP/s
  kernels      per-kernel averages: back-to-back launch trains between HIP events on the launch stream
  roofline     the dominant kernel of the step against its roof
  cpu_baseline the C oracle on a bounded sample of the same workload, on the host cores
Buffers rotate through several sets so that no step finds its operands in the 256 MB
last-level cache left behind by the previous one.  Every launch train is preceded by at least
--train-warm-ms of the same kernel, so that the result does not depend on --warmup.
"""
import argparse
import hashlib
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
# of known size), from the committed counter summary named below; a counter run is not part of a
# bench run, so other workloads (and the row-major layout) report null.
TRAFFIC_SOURCE = "profiles/bench_mlp8b_pmc_hbm_traffic.txt"
PROFILED_TRAFFIC = {"mxfp4_gemm_mlp8b_bf16": 609.8e6, "rotate_quant_16384x8192": 339.8e6,
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
    ap.add_argument("--train-warm-ms", type=float, default=30.0,
                    help="untimed: every per-kernel launch train first runs its kernel for at least this long")
    ap.add_argument("--workload", default="mlp8b", help="llama1b_up | down_sweep | mlp8b | decode")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--layout", default="tiled", choices=["tiled", "rowmajor"],
                    help="layout of the quantized operands between the two kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-aux", action="store_true", help="skip every leg but the default step")
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
    LAY = args.layout
    stream = torch.cuda.Stream()

    def to_dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def sha(a):
        return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()

    # ---- timing of one kernel: a train of back-to-back launches between two events on the launch stream,
    # repeated `reps` times (a pair of events around every single launch would add the launch gap, 5-6 us,
    # to the short row-wise kernels), after at least --train-warm-ms of the same launches: the clocks take
    # milliseconds of load to settle, and what they settle at depends on the kernel.
    def train(launch, reps=5, steps=None):
        steps = args.steps if steps is None else steps
        t0, i = time.perf_counter(), 0
        while True:
            for _ in range(16):
                launch(i)
                i += 1
            stream.synchronize()
            if (time.perf_counter() - t0) * 1e3 >= args.train_warm_ms:
                break
        out = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record(stream)
            for i in range(steps):
                launch(i)
            b.record(stream)
            stream.synchronize()
            out.append(a.elapsed_time(b) / steps)
        return np.array(out)

    # The same launches replayed from a HIP graph (n launches captured once): what a serving loop that replays a
    # captured step sees.  For kernels of a few microseconds the eager train above is bound by the host's launch
    # rate (the Python binding, 5-10 us a call), not by the GPU; the graph figure is reported next to it.
    def train_graph(launch, n=16, reps=3):
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for i in range(n):
                launch(i)
        t0 = time.perf_counter()
        with torch.cuda.stream(stream):
            while True:
                for _ in range(4):
                    g.replay()
                stream.synchronize()
                if (time.perf_counter() - t0) * 1e3 >= args.train_warm_ms:
                    break
            out = []
            for _ in range(reps):
                a, b = ev(), ev()
                a.record(stream)
                for _ in range(4):
                    g.replay()
                b.record(stream)
                stream.synchronize()
                out.append(a.elapsed_time(b) / (4 * n))
        del g
        return np.array(out)

    def hbm_leg(kernel, ms, alg_bytes, **extra):
        t = float(np.mean(ms))
        return {"kernel": kernel, "bound": "hbm", "avg_ms": t, "min_ms": float(np.min(ms)), "alg_bytes": alg_bytes,
                "achieved": alg_bytes / t / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": alg_bytes / t / 1e6 / HBM_PEAK_GBS, **extra}

    def mfma_leg(ms, m, n, k, es, **extra):
        t = float(np.mean(ms))
        fl = 2.0 * m * n * k
        return {"kernel": "mxfp4_gemm", "bound": "mfma", "avg_ms": t, "min_ms": float(np.min(ms)), "flops": fl,
                "alg_bytes": (m + n) * k * 0.53125 + m * n * es, "achieved": fl / t / 1e9,
                "peak": MXFP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fl / t / 1e9 / MXFP4_PEAK_TFLOPS, **extra}

    def q_buffers(rows, k, n):
        cb, sb = brq.operand_bytes(rows, k, LAY)
        cs = (rows, k // 2) if LAY == "rowmajor" else (cb,)
        ss = (rows, k // 32) if LAY == "rowmajor" else (sb,)
        return ([torch.empty(cs, dtype=torch.uint8, device="cuda") for _ in range(n)],
                [torch.empty(ss, dtype=torch.uint8, device="cuda") for _ in range(n)])

    x_np = inputs.make_x(cfg)
    w_np = inputs.make_w(cfg)
    input_sha256 = {"x": sha(x_np), "w": sha(w_np)}
    wq0, ws0 = brq.rotate_quantize_fused(to_dev(w_np), B, layout=LAY)          # offline weight preparation
    del w_np
    set_bytes = M * K * BYTES_PER_ELEM + N * K * 0.53125 + gemm_M * N * out_es
    nsets = int(max(2, min(6, 600e6 // set_bytes + 1)))
    xs = [to_dev(x_np)]
    xs += [xs[0].clone() for _ in range(nsets - 1)]
    wqs = [wq0] + [wq0.clone() for _ in range(nsets - 1)]
    wss = [ws0] + [ws0.clone() for _ in range(nsets - 1)]
    codes, scales = q_buffers(M, K, nsets)
    ys = [torch.empty((gemm_M, N), dtype=out_dtype, device="cuda") for _ in range(nsets)]
    torch.cuda.synchronize()      # everything above ran on the null stream; the launches below use `stream`

    def rq(i):
        j = i % nsets
        brq.rotate_quantize_fused(xs[j], B, codes=codes[j], scales=scales[j], stream=stream, layout=LAY)

    def a_operand(c, s, rows):
        # the product reads the first `rows` rows of the quantized activations (all of them but for "decode")
        return (c[:rows], s[:rows]) if LAY == "rowmajor" else (c, s)

    def gemm(i, out=None):
        j = i % nsets
        a_c, a_s = a_operand(codes[j], scales[j], gemm_M)
        brq.mxfp4_gemm(a_c, a_s, wqs[j], wss[j], out=ys[j] if out is None else out[j], stream=stream, a_layout=LAY,
                       w_layout=LAY, M=gemm_M, N=N, K=K)

    def step(i):
        rq(i)
        gemm(i)

    # ---- the step.  The GPU has idled while the inputs were generated on the CPU, and its clocks take some
    # milliseconds of load to come up: untimed steps for --settle-ms first, then the W warm-up steps, then
    # the K timed ones.
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
    ms_per_step = wall * 1e3 / args.steps

    rq_ms = train(rq)
    gm_ms = train(gemm)
    # the same product on ONE buffer set: operands stay in the 256 MB memory-side cache ("warm")
    gm_warm_ms = train(lambda i: gemm(0), reps=3)
    # the same launch on constant operands (all codes 0, all scales 2^0): what the schedule does when the
    # chip's clock management is not reacting to switching activity in the matrix cores
    with torch.cuda.stream(stream):
        zc, zs = torch.zeros_like(codes[0]), torch.full_like(scales[0], 127)
        zwc, zws = torch.zeros_like(wqs[0]), torch.full_like(wss[0], 127)

    def gemm_const(i):
        a_c, a_s = a_operand(zc, zs, gemm_M)
        brq.mxfp4_gemm(a_c, a_s, zwc, zws, out=ys[0], stream=stream, a_layout=LAY, w_layout=LAY, M=gemm_M, N=N, K=K)
    gm_const_ms = train(gemm_const, reps=3)
    # the shader clock the chip holds during the product (cycle and 100 MHz counters of the kernel's first
    # workgroup), on the workload's operands and on the constant ones
    gm_clock = {}
    if gemm_M > 128 and N % 256 == 0:
        with torch.cuda.stream(stream):
            clk = torch.zeros(6, dtype=torch.int64, device="cuda")
        split = {}

        def clocked(a_c, a_s, w_c, w_s, key=None):
            vals = []
            for _ in range(3):      # the last launch of a train of back-to-back ones (every launch overwrites clk)
                for i in range(20):
                    brq.mxfp4_gemm(a_c, a_s, w_c, w_s, out=ys[0], stream=stream, a_layout=LAY, w_layout=LAY, M=gemm_M, N=N,
                                   K=K, clock=clk)
                stream.synchronize()
                c, t, loop, epi, tiles, pro = clk.tolist()
                vals.append(0.1 * c / max(t, 1))
                if key:     # cycles of the kernel's first wavefront: per tile inside the K loop / the epilogue; prologue
                    split[key] = {"tiles": tiles, "k_loop_cycles_per_tile": loop / max(tiles, 1),
                                  "epilogue_cycles_per_tile": epi / max(tiles, 1), "prologue_cycles": pro, "total_cycles": c,
                                  "mfma_cycles_per_tile_at_32": (K // 64) * 16 * 32 * (gemm_M > 0)}
            return float(np.mean(vals))
        for i in range(40):
            gemm(i)
        a_c, a_s = a_operand(codes[0], scales[0], gemm_M)
        gm_clock["shader_clock_GHz"] = clocked(a_c, a_s, wqs[0], wss[0], "workload_operands")
        for i in range(40):
            gemm_const(0)
        a_c, a_s = a_operand(zc, zs, gemm_M)
        gm_clock["constant_operands_shader_clock_GHz"] = clocked(a_c, a_s, zwc, zws, "constant_operands")
        gm_clock["cycle_split_first_wavefront"] = split
        # the same kernel without its refill loads (a measurement instantiation whose output is not the product):
        # what the product would take if moving its operands from the L2s into LDS cost nothing
        if out_dtype == torch.bfloat16 and ((gemm_M + 255) // 256) * (N // 256) >= 1024:
            a_c, a_s = a_operand(codes[0], scales[0], gemm_M)
            with torch.cuda.stream(stream):
                y_nl = torch.empty_like(ys[0])

            def gemm_no_loads(i):
                j = i % nsets
                a_cj, a_sj = a_operand(codes[j], scales[j], gemm_M)
                brq.mxfp4_gemm(a_cj, a_sj, wqs[j], wss[j], out=y_nl, stream=stream, a_layout=LAY, w_layout=LAY, M=gemm_M,
                               N=N, K=K, clock=clk, no_loads=True)
            nl_ms = float(train(gemm_no_loads, reps=3).mean())
            stream.synchronize()
            c, t = clk.tolist()[:2]
            gm_clock["without_refill_loads"] = {"avg_ms": nl_ms, "frac_mxfp4_peak": 2.0 * gemm_M * N * K / nl_ms / 1e9 / MXFP4_PEAK_TFLOPS,
                                                "shader_clock_GHz": 0.1 * c / max(t, 1), "total_cycles": c,
                                                "note": "measurement instantiation: every MFMA, LDS read, barrier and output store "
                                                        "of the product, no operand loads after the first 512 of K; its output "
                                                        "is not the product"}
            del y_nl
    stream.synchronize()
    del zc, zs, zwc, zws

    rq_bytes = M * K * BYTES_PER_ELEM
    gemm_flops = 2.0 * gemm_M * N * K
    gemm_bytes = (gemm_M + N) * K * 0.53125 + gemm_M * N * out_es
    rq_avg, gm_avg = float(rq_ms.mean()), float(gm_ms.mean())
    if "shader_clock_GHz" in gm_clock:   # the published peak is quoted at 2.4 GHz: the same ratio at the clock held
        gm_clock["frac_mxfp4_peak_at_held_clock"] = (gemm_flops / gm_avg / 1e9 / MXFP4_PEAK_TFLOPS
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
        traffic = PROFILED_TRAFFIC.get("mxfp4_gemm_%s_%s" % (args.workload, args.out_dtype)) if LAY == "tiled" else None
        roofline = {"kernel": "mxfp4_gemm", "bound": "mfma", "achieved": kernels["mxfp4_gemm"]["TFLOP/s"],
                    "peak": MXFP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": kernels["mxfp4_gemm"]["frac_mxfp4_peak"],
                    "traffic": traffic, "traffic_source": TRAFFIC_SOURCE if traffic else None}

    # ---- what the chip sustains on the block-scaled MFMA alone, fed from registers with bit patterns
    # of this workload (the first 8 KB of quantized activations): the ceiling of any product kernel
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    with torch.cuda.stream(stream):
        sink = torch.empty((ncu * 256,), dtype=torch.float32, device="cuda")
        ops = codes[0].flatten()[:8192].clone()
        zops = torch.zeros_like(ops)
    c_iters = 2000
    c_flops = brq.diag_mfma_ceiling(ops, c_iters, ncu, sink=sink, stream=stream)
    c_ms = train(lambda i: brq.diag_mfma_ceiling(ops, c_iters, ncu, sink=sink, stream=stream), reps=3, steps=3)
    stream.synchronize()
    c_clk = sink[:2].tolist()
    z_ms = train(lambda i: brq.diag_mfma_ceiling(zops, c_iters, ncu, sink=sink, stream=stream), reps=3, steps=3)
    stream.synchronize()
    z_clk = sink[:2].tolist()
    ceiling = {"TFLOP/s": c_flops / float(c_ms.mean()) / 1e9,
               "frac_mxfp4_peak": c_flops / float(c_ms.mean()) / 1e9 / MXFP4_PEAK_TFLOPS,
               "shader_clock_GHz": 0.1 * c_clk[0] / max(c_clk[1], 1.0),
               "zero_operands_shader_clock_GHz": 0.1 * z_clk[0] / max(z_clk[1], 1.0),
               "zero_operands_TFLOP/s": c_flops / float(z_ms.mean()) / 1e9,
               "zero_operands_frac_mxfp4_peak": c_flops / float(z_ms.mean()) / 1e9 / MXFP4_PEAK_TFLOPS,
               "product_kernel_frac_of_this_ceiling": (gemm_flops / gm_avg) / (c_flops / float(c_ms.mean())),
               "note": "v_mfma_scale_f32_32x32x64 fp4 back to back from registers on every CU: the product kernel's "
                       "4 x 4 register tile (8 operand fragments, 16 accumulators) with nothing else in the loop, "
                       "operand bit patterns from this workload's quantized activations"}

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

            def lib_mm(i):
                with torch.cuda.stream(stream):
                    torch._scaled_mm(ta, tb, scale_a=tsa, scale_b=tsb, out_dtype=out_dtype)
            l_ms = train(lib_mm, reps=3)
            l_avg = float(l_ms.mean())
            library = {"what": "torch._scaled_mm (hipBLASLt MXFP4) on the same operands, warm cache",
                       "avg_ms": l_avg, "TFLOP/s": gemm_flops / l_avg / 1e9,
                       "this_kernel_warm_cache_avg_ms": float(gm_warm_ms.mean())}
            del a_c, a_s, w_c, w_s, ta, tb, tsa, tsb
        except Exception as e:      # the comparison is context, never a reason to fail the bench
            library = {"what": "torch._scaled_mm unavailable: %s" % str(e)[:200]}

    # ---- the other output type of the default product (fp32: 470 MB of output per launch on mlp8b)
    other_out = None
    if not args.no_aux and gemm_M > 128:
        o_dt, o_es, o_name = (torch.float32, 4, "f32") if args.out_dtype == "bf16" else (torch.bfloat16, 2, "bf16")
        with torch.cuda.stream(stream):
            ys2 = [torch.empty((gemm_M, N), dtype=o_dt, device="cuda") for _ in range(nsets)]
        o_ms = train(lambda i: gemm(i, out=ys2), reps=3)
        other_out = mfma_leg(o_ms, gemm_M, N, K, o_es, out_dtype=o_name)
        stream.synchronize()
        del ys2

    del xs, codes, scales, ys, wqs, wss
    torch.cuda.empty_cache()

    # ---- both kernels on every other workload of the benchmark definition, same launch configuration
    # as the tests check against the oracle (tiled operands, bf16 out except for the tiny fp32 layer)
    configs = None
    if not args.no_aux:
        configs = {}
        for name in ("tiny", "llama1b_up", "down_sweep"):
            if name == args.workload:
                continue
            c = inputs.CONFIGS[name]
            cM, cK, cN = c["M"], c["K"], c["N"]
            cx, cw = inputs.make_x(c), inputs.make_w(c)
            c_es = 4 if c["dtype"] == "f32" else 2
            c_out = torch.float32 if c["dtype"] == "f32" else torch.bfloat16
            n2 = int(max(2, min(8, 600e6 // (cM * cK * (c_es + 0.53125) + cN * cK * 0.53125 + cM * cN * c_es) + 1)))
            with torch.cuda.stream(stream):
                cxs = [to_dev(cx)]
                cxs += [cxs[0].clone() for _ in range(n2 - 1)]
                cwd = to_dev(cw)
                cy = [torch.empty((cM, cN), dtype=c_out, device="cuda") for _ in range(n2)]
            cc, cs = q_buffers(cM, cK, n2)
            entry = {"shape": "X %dx%d %s, W %dx%d" % (cM, cK, c["dtype"], cN, cK), "buffer_sets": n2,
                     "input_sha256": {"x": sha(cx), "w": sha(cw)}, "by_rotation_block": {}}
            for cB in c["B"]:
                with torch.cuda.stream(stream):
                    w_sets = [brq.rotate_quantize_fused(cwd, cB, stream=stream, layout=LAY) for _ in range(n2)]

                def c_rq(i):
                    brq.rotate_quantize_fused(cxs[i % n2], cB, codes=cc[i % n2], scales=cs[i % n2], stream=stream, layout=LAY)

                def c_gemm(i):
                    j = i % n2
                    brq.mxfp4_gemm(cc[j], cs[j], w_sets[j][0], w_sets[j][1], out=cy[j], stream=stream, a_layout=LAY,
                                   w_layout=LAY, M=cM, N=cN, K=cK)
                r_ms = train(c_rq, reps=3)
                g_ms = train(c_gemm, reps=3)
                r_gr, g_gr = float(train_graph(c_rq).mean()), float(train_graph(c_gemm).mean())
                entry["by_rotation_block"]["global_%d" % cB if cB == cK else str(cB)] = {
                    "rotate_quantize_fused": hbm_leg("rotate_quantize_fused", r_ms, cM * cK * (c_es + 0.53125),
                                                     graph_replay_avg_ms=r_gr,
                                                     graph_replay_frac=cM * cK * (c_es + 0.53125) / r_gr / 1e6 / HBM_PEAK_GBS),
                    "mxfp4_gemm": mfma_leg(g_ms, cM, cN, cK, c_es, graph_replay_avg_ms=g_gr,
                                           graph_replay_frac=2.0 * cM * cN * cK / g_gr / 1e9 / MXFP4_PEAK_TFLOPS)}
                stream.synchronize()
                del w_sets
            configs[name] = entry
            del cxs, cwd, cy, cc, cs
            torch.cuda.empty_cache()
        if other_out is not None:
            configs["%s_%s_out" % (args.workload, other_out["out_dtype"])] = {"mxfp4_gemm": other_out}

    # ---- the rotate+quantize kernel on the shape its HBM target is quoted on
    aux = aux_m = aux_s = None
    if not args.no_aux:
        acfg = inputs.CONFIGS["decode"]
        aM, aK = acfg["M"], acfg["K"]
        ax_np = inputs.make_x(acfg) if args.workload != "decode" else x_np
        with torch.cuda.stream(stream):
            axs = [to_dev(ax_np)]
            axs += [axs[0].clone(), axs[0].clone()]
        ac, asc = q_buffers(aM, aK, 3)
        ab = aM * aK * BYTES_PER_ELEM

        def a_rq(blk):
            return lambda i: brq.rotate_quantize_fused(axs[i % 3], blk, codes=ac[i % 3], scales=asc[i % 3], stream=stream,
                                                       layout=LAY)
        ams = train(a_rq(B))
        aux = hbm_leg("rotate_quantize_fused", ams, ab, input_sha256=sha(ax_np),
                      traffic=PROFILED_TRAFFIC["rotate_quant_16384x8192"] if LAY == "tiled" else None,
                      traffic_source=TRAFFIC_SOURCE if LAY == "tiled" else None)
        # what the online rotation costs (Sec. 4.3 "reduced online computing", Sec. 5.3 table of prefill
        # overheads): the same activations through the quantizer alone, with the block rotation, and with the
        # global one (B = K)
        rot = {"quantize_only_ms": float(train(lambda i: brq.mxfp4_quantize(axs[i % 3], codes=ac[i % 3], scales=asc[i % 3],
                                                                            stream=stream, layout=LAY), reps=3).mean()),
               "block_%d_ms" % B: float(ams.mean()),
               "block_128_ms": float(train(a_rq(128), reps=3).mean()),
               "global_%d_ms" % aK: float(train(a_rq(aK), reps=3).mean())}
        aux["online_rotation_cost"] = rot
        # the same step with caller-supplied orthogonal 32x32 blocks (one per block of K) on the matrix cores
        rng_r = np.random.default_rng(11)
        with torch.cuda.stream(stream):
            Rb = torch.from_numpy(np.stack([np.linalg.qr(rng_r.standard_normal((32, 32)))[0]
                                            for _ in range(aK // 32)]).astype(np.float32)).cuda()
        mms = train(lambda i: brq.matrix_rotate_quantize_fused(axs[i % 3], Rb, codes=ac[i % 3], scales=asc[i % 3],
                                                               stream=stream, layout=LAY))
        aux_m = hbm_leg("matrix_rotate_quantize_fused", mms, ab, blocks="%d orthogonal 32x32 fp32 matrices" % (aK // 32),
                        traffic=PROFILED_TRAFFIC["matrix_rotate_quant_16384x8192"] if LAY == "tiled" else None,
                        traffic_source=TRAFFIC_SOURCE if LAY == "tiled" else None, mfma_flops=3 * 2.0 * aM * aK * 32)
        # block statistics of the same activations after the block rotation (scales, loss, two thresholds)
        with torch.cuda.stream(stream):
            st_counts = torch.zeros(2, dtype=torch.int64, device="cuda")
            st_b = torch.empty((aM, aK // 32), dtype=torch.float32, device="cuda")
            st_a, st_q = torch.empty_like(st_b), torch.empty_like(st_b)
        sms = train(lambda i: brq.block_stats(axs[i % 3], B, (1.5, 3.0), counts=st_counts, amax=st_a, sqerr=st_q, stream=stream))
        # the same call with the FP16-scale loss as a fourth output (8 divisions per 8 values more)
        bms = train(lambda i: brq.block_stats(axs[i % 3], B, (1.5, 3.0), counts=st_counts, amax=st_a, sqerr=st_q,
                                              sqerr_bfp4=st_b, stream=stream), reps=3)
        aux_s = hbm_leg("block_stats", sms, aM * aK * (2 + 8.0 / 32),
                        what="block-wise scale + MXFP4 loss per block + counts above 1.5 and 3.0, B = 32",
                        traffic=PROFILED_TRAFFIC["block_stats_16384x8192"], traffic_source=TRAFFIC_SOURCE,
                        with_fp16_scale_loss_ms=float(bms.mean()))
        # the paper's comparison from those outputs (Sec. 4.2, Appendix "Rotation Comparison"): scales and losses
        # after no / block / global rotation, blocks classified by their untransformed scale
        with torch.cuda.stream(stream):
            ref_a = torch.empty_like(st_a)
        brq.block_stats(axs[0], 1, (), amax=ref_a, sqerr=st_q, stream=stream)
        cmp_res = {}
        with torch.cuda.stream(stream):
            h_ = torch.zeros(8, dtype=torch.int64, device="cuda")
            c_ = torch.zeros(4, dtype=torch.int64, device="cuda")
            s_ = torch.zeros(4, dtype=torch.float64, device="cuda")

        def summarize(i=0):
            brq.block_stats_summary(st_a.view(-1), st_q.view(-1), ref_a.view(-1), outlier_threshold=60.0,
                                    edges=(1.0, 2.0, 4.0, 8.0, 16.0, 32.0, 64.0), hist=h_, counts=c_, sums=s_, stream=stream)
        for name, blk in (("none", 1), ("block_%d" % B, B), ("global_%d" % aK, aK)):
            brq.block_stats(axs[0], blk, (), amax=st_a, sqerr=st_q, stream=stream)
            with torch.cuda.stream(stream):
                h_.zero_(), c_.zero_(), s_.zero_()
            summarize()
            stream.synchronize()
            c_l, s_l = c_.tolist(), s_.tolist()
            cmp_res[name] = {"scale_histogram": h_.tolist(), "regular_blocks": c_l[0], "outlier_blocks": c_l[1],
                             "regular_blocks_whose_scale_grew": c_l[2] / max(c_l[0], 1),
                             "mean_scale_regular": s_l[2] / max(c_l[0], 1), "mean_scale_outlier": s_l[3] / max(c_l[1], 1),
                             "mean_loss_regular": s_l[0] / max(c_l[0], 1), "mean_loss_outlier": s_l[1] / max(c_l[1], 1)}
        sum_ms = train(summarize, reps=3)
        aux_s["rotation_comparison"] = {"what": "blocks of 32 classified by untransformed scale > 60; scale histogram edges "
                                                "1, 2, 4, ..., 64", "summary_kernel_ms": float(sum_ms.mean()), **cmp_res}
        stream.synchronize()
        del axs, ac, asc, Rb, st_a, st_q, st_b, ref_a
        torch.cuda.empty_cache()

    # ---- the online step with its producer fused in: silu(gate) * up -> rotation -> MXFP4 on the
    # down_proj input of the 8B MLP (8192 tokens x 14336), against the two-kernel path
    aux2 = None
    if not args.no_aux:
        sM, sK = 8192, 14336
        gen = torch.Generator(device="cuda")
        gen.manual_seed(7)
        with torch.cuda.stream(stream):
            gus = [(torch.randn((sM, 2 * sK), device="cuda", generator=gen) * 1.5).to(torch.bfloat16) for _ in range(2)]
            hbuf = torch.empty((sM, sK), dtype=torch.bfloat16, device="cuda")
        sc, ss = q_buffers(sM, sK, 2)

        def fused(i):
            g = gus[i % 2]
            brq.swiglu_rotate_quantize_fused(g[:, :sK], g[:, sK:], B, h_dtype=torch.bfloat16, codes=sc[i % 2],
                                             scales=ss[i % 2], stream=stream, layout=LAY)

        def two_kernels(i):
            g = gus[i % 2]
            brq.swiglu(g[:, :sK], g[:, sK:], out=hbuf, stream=stream)
            brq.rotate_quantize_fused(hbuf, B, codes=sc[i % 2], scales=ss[i % 2], stream=stream, layout=LAY)
        f_ms = train(fused)
        t_ms = train(two_kernels, reps=3)
        aux2 = hbm_leg("swiglu_rotate_quantize_fused", f_ms, sM * sK * (4 + 0.5 + 1.0 / 32),
                       shape="gate, up 8192x14336 bf16 (one 8192x28672 buffer)",
                       two_kernel_path_ms=float(t_ms.mean()),
                       traffic=PROFILED_TRAFFIC["swiglu_rotate_quant_8192x14336"] if LAY == "tiled" else None,
                       traffic_source=TRAFFIC_SOURCE if LAY == "tiled" else None)
        stream.synchronize()
        del gus, sc, ss, hbuf
        torch.cuda.empty_cache()

    # ---- decode batches: the product M x 28672 x 8192 (gate_up of the 8B MLP against one batch of tokens),
    # weight streaming, HBM bound: two weight copies alternate so that no launch finds them in the cache
    aux3 = None
    if not args.no_aux:
        dN, dK = 28672, 8192
        gen = torch.Generator(device="cuda")
        gen.manual_seed(8)
        dws = []
        with torch.cuda.stream(stream):
            for _ in range(2):
                wbf = (torch.randn((dN, dK), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
                dws.append(brq.rotate_quantize_fused(wbf, B, layout=LAY, stream=stream))
                del wbf
            dx = torch.randn((128, dK), device="cuda", generator=gen).to(torch.bfloat16)
        aux3 = {"kernel": "mxfp4_gemm", "shape": "M x 28672 x 8192, bf16 out", "bound": "hbm", "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "alg_bytes_weights": dN * dK * 0.53125, "batches": {}}
        for dM in (1, 4, 16, 32, 64, 128):
            with torch.cuda.stream(stream):
                dq = brq.rotate_quantize_fused(dx[:dM].contiguous(), B, layout=LAY, stream=stream)
                dy = torch.empty((dM, dN), dtype=torch.bfloat16, device="cuda")

            def dgemm(i):
                brq.mxfp4_gemm(dq[0], dq[1], dws[i % 2][0], dws[i % 2][1], out=dy, stream=stream, a_layout=LAY,
                               w_layout=LAY, M=dM, N=dN, K=dK)
            t = float(train(dgemm, reps=3).mean())
            by = (dN + dM) * dK * 0.53125 + dM * dN * 2
            aux3["batches"][str(dM)] = {"avg_ms": t, "achieved": by / t / 1e6, "frac": by / t / 1e6 / HBM_PEAK_GBS,
                                        "graph_replay_avg_ms": float(train_graph(dgemm).mean())}
            if dM <= 16:
                # the whole online path of a decode step (Sec. 4.3): rotate + quantize the bf16 activations, then the
                # product - as two launches, and as the one launch that carries the online step in its prologue
                dxm = dx[:dM].contiguous()
                dqc, dqs = q_buffers(dM, dK, 1)

                def two_launches(i):
                    brq.rotate_quantize_fused(dxm, B, codes=dqc[0], scales=dqs[0], stream=stream, layout=LAY)
                    brq.mxfp4_gemm(dqc[0], dqs[0], dws[i % 2][0], dws[i % 2][1], out=dy, stream=stream, a_layout=LAY,
                                   w_layout=LAY, M=dM, N=dN, K=dK)

                def one_launch(i):
                    brq.rotate_quantize_gemm_fused(dxm, B, dws[i % 2][0], dws[i % 2][1], dN, out=dy, stream=stream, w_layout=LAY)
                aux3["batches"][str(dM)]["online_step_plus_product_two_launches_ms"] = float(train(two_launches, reps=3).mean())
                aux3["batches"][str(dM)]["online_step_inside_the_product_ms"] = float(train(one_launch, reps=3).mean())
                aux3["batches"][str(dM)]["graph_replay_two_launches_ms"] = float(train_graph(two_launches).mean())
                aux3["batches"][str(dM)]["graph_replay_one_launch_ms"] = float(train_graph(one_launch).mean())
        stream.synchronize()
        del dws, dx
        torch.cuda.empty_cache()

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
        rows = int(min(M, max(64, 3e7 // K)))
        t0 = time.perf_counter()
        rc, rs = o.rotate_quantize_fused(x_np[:rows], B)
        t_rq = time.perf_counter() - t0
        grows = int(min(gemm_M, rows, max(1, 1.2e11 // (N * K))))       # some 5 s of oracle work
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
        "train_warm_ms": args.train_warm_ms,
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
        "configs": configs,
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
