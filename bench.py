#!/usr/bin/env python3
"""Benchmark of the SwitchBack linear layer (Algorithm 1 of arxiv 2304.13013) on one MI355X.

One "step" is the whole hot path over the ViT-H/14-shaped workload: for each of the four transformer linear
layers (qkv, proj, fc1, fc2; b = 128 x 257 tokens) a forward pass, the input gradient and the weight gradient
through the C ABI.  The headline value counts 6*b*n*m flop per layer (the three products; quantization is
overhead).  Beside it: the same three products as bf16 torch matmuls on the same GPU (the paper's baseline), the
per-kernel times with the roofline of the dominant kernel, and the CPU oracle timed on a bounded sample.

Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm_GBps": 8000.0, "int8_TOPs": 5000.0, "bf16_TFLOPs": 2500.0}

# HBM-side bytes per launch (mean over the launches of one step) of each kernel group on the vit_h14 workload, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (FETCH_SIZE x2, WRITE_SIZE x1 after calibration against
# copy kernels of known size; summary and commands in profiles/bench_vit_h14_hbm_traffic.md).  Not re-measured at run
# time: the table belongs to the kernels as they were when that profile was taken (tile walk, grid and split choices
# decide the figures), and is null for other workloads.
TRAFFIC_BYTES_PER_LAUNCH_VIT_H14 = {
    "gemm_int8_dequant": 318.4e6 + 168.8e6,        # 8 launches per step; algorithmic mean 257.6e6
    "gemm_bf16_weight_grad": 583.7e6 + 97.9e6,     # 4 launches per step, fp32 split-K partials included; the reduction
                                                   # kernel of the same step adds 96.7e6 + 9.8e6; algorithmic 346.7e6
    "quantize_rowwise": 258.2e6,                   # 8 launches per step, 4 of them with the absmax pass of W riding
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="vit_h14", help="workload (default: the headline ViT-H/14 shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch three 256 MiB device-to-device copy kernels (known traffic) so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--no-clocks", action="store_true",
                    help="skip the rocm-smi clock reading (it queues about a second of extra steps)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured-ceilings leg (matrix-instruction loops, main-loop-only product, copy); "
                         "measured_peak / frac_of_measured are then null")
    ap.add_argument("--cpu-sample-rows", type=int, default=0, help="token rows of the oracle sample (0 = auto)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
                         "--gpus %d is not supported, use --gpus 1\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2304_13013_amd import inputs as I
    from paper_2304_13013_amd import switchback as sb

    sb.load_library()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = I.CONFIGS[args.config]
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def draw(shape, kind, sigma):
        z = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
        if kind == "student_t3":
            chi2 = sum(torch.randn(shape, generator=gen, device=dev) ** 2 for _ in range(3))
            z = z / torch.sqrt(chi2 / 3.0)
        elif kind == "outlier":
            cols = torch.randperm(shape[1], generator=gen, device=dev)[: -(-shape[1] // 1000)]
            z[:, cols] *= 100.0
        return (z * sigma).to(torch.bfloat16)

    layers = []
    for L in cfg.layers:
        x = draw((L.b, L.n), *cfg.x_dist)
        w = draw((L.m, L.n), "normal", (1.0 / L.n) ** 0.5)
        dy = draw((L.b, L.m), *cfg.dy_dist)
        e = lambda shape, dt=torch.bfloat16: torch.empty(shape, dtype=dt, device=dev)
        layers.append(dict(L=L, x=x, w=w, dy=dy, bufs=sb.LayerBuffers(L.b, L.n, L.m, dev),
                           y=e((L.b, L.m)), dx=e((L.b, L.n)), dw=e((L.m, L.n))))
    flop_per_step = sum(6.0 * t["L"].b * t["L"].n * t["L"].m for t in layers)

    def switchback_step():
        for t in layers:
            sb.forward(t["x"], t["w"], bufs=t["bufs"], y=t["y"])
            sb.backward_input(t["dy"], t["bufs"], dx=t["dx"])
            sb.backward_weight(t["dy"], t["x"], t["bufs"], dw=t["dw"])

    def switchback_step_requant():
        # Algorithm 1 as printed: the backward pass quantizes (and transposes) W again instead of keeping the codes.
        for t in layers:
            bufs = t["bufs"]
            sb.forward(t["x"], t["w"], bufs=bufs, y=t["y"])
            sb.quantize_tensorwise(t["w"], bufs.wq, bufs.wq_t, bufs.state_w, bufs.ws_fwd)
            sb.backward_input(t["dy"], bufs, dx=t["dx"])
            sb.backward_weight(t["dy"], t["x"], bufs, dw=t["dw"])

    x_hat = torch.empty((max(L.b * L.n for L in cfg.layers),), dtype=torch.bfloat16, device=dev)

    def switchback_m_step():
        # The memory-efficient variant (SwitchBackM): only X_int8 and state_X survive the forward pass; the weight
        # gradient rebuilds X by row-wise dequantization.
        for t in layers:
            L = t["L"]
            sb.forward(t["x"], t["w"], bufs=t["bufs"], y=t["y"])
            sb.backward_input(t["dy"], t["bufs"], dx=t["dx"])
            sb.backward_weight_m(t["dy"], t["bufs"], x_hat=x_hat[: L.b * L.n].view(L.b, L.n), dw=t["dw"])

    q_bufs = {}

    def switchback_q_step():
        # SwitchBackQ: row-wise weight quantization in the forward pass, column-wise (transposed) in the backward pass.
        for i, t in enumerate(layers):
            L = t["L"]
            if i not in q_bufs:
                q_bufs[i] = sb.LayerBuffersQ(L.b, L.n, L.m, dev)
            sb.forward_q(t["x"], t["w"], bufs=q_bufs[i], y=t["y"])
            sb.backward_input_q(t["dy"], t["w"], q_bufs[i], dx=t["dx"])
            sb.backward_weight(t["dy"], t["x"], t["bufs"], dw=t["dw"])

    def switchback_f8_step():
        # The float8 variant: float8cast(x / absmax) quantizers (E4M3 for X and W, E5M2 for dY), float8 MFMA products.
        # Shares the layer buffers with the int8 path (same sizes), so it runs after the int8 measurements.
        for t in layers:
            sb.forward_f8(t["x"], t["w"], bufs=t["bufs"], y=t["y"])
            sb.backward_input_f8(t["dy"], t["bufs"], dx=t["dx"])
            sb.backward_weight(t["dy"], t["x"], t["bufs"], dw=t["dw"])

    def bf16_step():
        for t in layers:
            torch.matmul(t["x"], t["w"].t(), out=t["y"])
            torch.matmul(t["dy"], t["w"], out=t["dx"])
            torch.matmul(t["dy"].t(), t["x"], out=t["dw"])

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return max(e0.elapsed_time(e1) / steps, 0.0), wall

    sb_ms, sb_wall_ms = timed(switchback_step, args.steps, args.warmup)
    bf_ms, _ = timed(bf16_step, args.steps, args.warmup)
    requant_ms, _ = timed(switchback_step_requant, max(3, args.steps // 2), 2)

    # Per layer: forward + input gradient + weight gradient of that layer alone, back to back, both ways.
    per_layer = []
    for t in layers:
        def one_sb(t=t):
            sb.forward(t["x"], t["w"], bufs=t["bufs"], y=t["y"])
            sb.backward_input(t["dy"], t["bufs"], dx=t["dx"])
            sb.backward_weight(t["dy"], t["x"], t["bufs"], dw=t["dw"])

        def one_bf(t=t):
            torch.matmul(t["x"], t["w"].t(), out=t["y"])
            torch.matmul(t["dy"], t["w"], out=t["dx"])
            torch.matmul(t["dy"].t(), t["x"], out=t["dw"])

        n_rep = max(5, args.steps // 2)
        a, _ = timed(one_sb, n_rep, 2)
        c, _ = timed(one_bf, n_rep, 2)
        L = t["L"]
        per_layer.append({"layer": L.name, "b": L.b, "n": L.n, "m": L.m, "switchback_ms": round(a, 4),
                          "bf16_linear_ms": round(c, 4), "speedup": round(c / a, 4),
                          "TFLOPs": round(6.0 * L.b * L.n * L.m / a / 1e9, 1)})
    variant_m_ms, _ = timed(switchback_m_step, max(3, args.steps // 2), 2)
    variant_q_ms, _ = timed(switchback_q_step, max(3, args.steps // 2), 2)
    q_bufs.clear()
    variant_f8_ms = None
    if all(L.n % 128 == 0 and L.m % 128 == 0 for L in cfg.layers):
        variant_f8_ms, _ = timed(switchback_f8_step, max(3, args.steps // 2), 2)

    # ---- per-kernel times: the same kernels on the same shapes, one event pair around each launch group ------
    ops = {}  # name -> [total ms over reps, algorithmic work, unit kind]

    def time_op(name, fn, work, kind, reps):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        rec = ops.setdefault(name, [0.0, 0.0, kind])
        rec[0] += e0.elapsed_time(e1) / reps
        rec[1] += work

    reps = max(5, min(args.steps, 20))
    adamw_rms = torch.empty(1, dtype=torch.float32, device=dev)
    adamw_ws = torch.empty(sb.workspace_bytes(sb.SB_OP_STABLE_ADAMW, 0, 0, 0), dtype=torch.uint8, device=dev)
    for t in layers:
        L, bufs = t["L"], t["bufs"]
        b, n, m = L.b, L.n, L.m
        time_op("quantize_rowwise", lambda: sb.quantize_rowwise(t["x"], bufs.xq, bufs.state_x),
                b * n * 3.0 + 4.0 * b, "bytes", reps)
        time_op("quantize_rowwise", lambda: sb.quantize_rowwise(t["dy"], bufs.gq, bufs.state_g),
                b * m * 3.0 + 4.0 * b, "bytes", reps)
        time_op("dequantize_rowwise (SwitchBackM only)",
                lambda: sb.dequantize_rowwise(bufs.xq, bufs.state_x, out=x_hat[: b * n].view(b, n)),
                b * n * 3.0 + 4.0 * b, "bytes", reps)
        time_op("quantize_tensorwise",
                lambda: sb.quantize_tensorwise(t["w"], bufs.wq, bufs.wq_t, bufs.state_w, bufs.ws_fwd),
                m * n * 6.0, "bytes", reps)
        time_op("gemm_int8_dequant",
                lambda: sb.matmul_int8_dequant(bufs.xq, bufs.state_x, bufs.wq, bufs.state_w, out=t["y"]),
                2.0 * b * n * m, "int8", reps)
        time_op("gemm_int8_dequant",
                lambda: sb.matmul_int8_dequant(bufs.gq, bufs.state_g, bufs.wq_t, bufs.state_w, out=t["dx"]),
                2.0 * b * n * m, "int8", reps)
        time_op("gemm_bf16_weight_grad", lambda: sb.backward_weight(t["dy"], t["x"], bufs, dw=t["dw"]),
                2.0 * b * n * m, "bf16", reps)
        if L.n % 128 == 0 and L.m % 128 == 0:
            # float8 variant: quantize into the same buffers (afterwards they hold float8 bytes), then the two products
            sb.forward_f8(t["x"], t["w"], bufs=bufs, y=t["y"])
            sb.backward_input_f8(t["dy"], bufs, dx=t["dx"])
            u8 = lambda q: q.view(torch.uint8)
            time_op("gemm_f8_dequant (float8 variant)",
                    lambda: sb.matmul_f8_dequant(u8(bufs.xq), sb.SB_E4M3, bufs.state_x, u8(bufs.wq), sb.SB_E4M3,
                                                 bufs.state_w, out=t["y"]),
                    2.0 * b * n * m, "f8", reps)
            time_op("gemm_f8_dequant (float8 variant)",
                    lambda: sb.matmul_f8_dequant(u8(bufs.gq), sb.SB_E5M2, bufs.state_g, u8(bufs.wq_t), sb.SB_E4M3,
                                                 bufs.state_w, out=t["dx"]),
                    2.0 * b * n * m, "f8", reps)
        # The optimizer step that consumes dW (binary32 master weights and moments, bf16 gradient): 34 bytes per
        # parameter (g 2, v and u read + written 16, theta/v/u read 12, theta written 4).  Not part of the step.
        opt = [torch.zeros(m * n, dtype=torch.float32, device=dev) for _ in range(3)]
        opt[0].copy_(t["w"].view(-1))
        opt[2].fill_(1e-6)
        time_op("stable_adamw_step (optimizer, outside the step)",
                lambda: sb.stable_adamw_step(opt[0], opt[1], opt[2], t["dw"], 1e-3, 0.9, 0.98, 1e-6, 0.2, 10,
                                             rms_out=adamw_rms, ws=adamw_ws),
                34.0 * m * n, "bytes", reps)
        del opt

    # The same optimizer step for the four weights of the block in one launch pair.
    opt_all = [tuple(torch.zeros(t["L"].m * t["L"].n, dtype=torch.float32, device=dev) for _ in range(3)) + (t["dw"],)
               for t in layers]
    for o in opt_all:
        o[2].fill_(1e-6)
    plan = sb.AdamwPlan(opt_all)
    time_op("stable_adamw_step_multi (optimizer, the block's 4 weights in one launch pair)",
            lambda: sb.stable_adamw_step_multi(plan, 1e-3, 0.9, 0.98, 1e-6, 0.2, 10),
            34.0 * sum(t["L"].m * t["L"].n for t in layers), "bytes", reps)
    del plan, opt_all

    # ---- measured ceilings (outside the timed region): what this GPU sustains for code that does nothing but issue
    # matrix instructions from registers, on the workload's own operand values (the clock the GPU holds under load
    # depends on how many operand bits toggle), and for a plain copy.  Launch shape of the product kernels: eight waves
    # per workgroup, two per SIMD; four workgroups per compute unit in a row so that a launch lasts several ms.
    def ceiling(kind, a, b_, reps=3):
        wgs, iters = 4 * torch.cuda.get_device_properties(dev).multi_processor_count, 2000
        sink = torch.empty(wgs * 8 * 64, dtype=torch.float32, device=dev)
        sb.ceiling_mfma(kind, a, b_, wgs, 8, iters, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            work, _ = sb.ceiling_mfma(kind, a, b_, wgs, 8, iters, sink)
        e1.record()
        torch.cuda.synchronize()
        return work * reps / e0.elapsed_time(e1) / 1e9

    ceilings, measured = None, {"int8": None, "bf16": None, "f8": None, "bytes": None}
    if not args.no_ceilings:
        big = max(layers, key=lambda t: t["L"].n * t["L"].m)
        sb.forward(big["x"], big["w"], bufs=big["bufs"], y=big["y"])           # int8 codes back into the buffers
        sb.backward_input(big["dy"], big["bufs"], dx=big["dx"])
        zeros = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
        ceilings = {
            "mfma_int8_workload_codes": round(ceiling(sb.SB_CEILING_I8, big["bufs"].gq, big["bufs"].wq), 1),
            "mfma_int8_zero_operands": round(ceiling(sb.SB_CEILING_I8, zeros, zeros), 1),
            "mfma_bf16_workload_values": round(ceiling(sb.SB_CEILING_BF16, big["dy"], big["x"]), 1),
            "mfma_bf16_zero_operands": round(ceiling(sb.SB_CEILING_BF16, zeros, zeros), 1),
        }
        if big["L"].n % 128 == 0 and big["L"].m % 128 == 0:
            sb.forward_f8(big["x"], big["w"], bufs=big["bufs"], y=big["y"])
            ceilings["mfma_float8_workload_codes"] = round(
                ceiling(sb.SB_CEILING_F8, big["bufs"].xq.view(torch.uint8), big["bufs"].wq.view(torch.uint8)), 1)
            ceilings["mfma_float8_zero_operands"] = round(ceiling(sb.SB_CEILING_F8, zeros, zeros), 1)
        # The product kernel's own main loop on the workload's codes, with the tile boundary amortized away: one 256x256 tile
        # per workgroup (4096 x 4096 outputs) and a contraction of 32768, i.e. 256 k-tiles per epilogue instead of 10.
        # What separates this figure from the matrix-instruction loop above is the operand traffic (L2 -> LDS -> registers);
        # what separates the workload's products from this figure is the tile boundary (epilogue, output stores) and
        # the rounds that do not fill the GPU.
        sb.forward(big["x"], big["w"], bufs=big["bufs"], y=big["y"])
        sb.backward_input(big["dy"], big["bufs"], dx=big["dx"])
        need = 4096 * 32768
        if big["bufs"].gq.numel() >= need:
            a_long = big["bufs"].gq.view(-1)[:need].view(4096, 32768)
            b_src = torch.cat([big["bufs"].wq.view(-1), big["bufs"].wq_t.view(-1)])
            b_long = b_src.repeat(-(-need // b_src.numel()))[:need].view(4096, 32768).contiguous()
            out_long = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
            run = lambda: sb.matmul_int8_dequant(a_long, big["bufs"].state_g[:4096].contiguous(), b_long,
                                                 big["bufs"].state_w, out=out_long)
            run()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                run()
            e1.record()
            torch.cuda.synchronize()
            ceilings["gemm_int8_main_loop_only_workload_codes"] = round(
                5 * 2.0 * 4096 * 4096 * 32768 / e0.elapsed_time(e1) / 1e9, 1)
            del a_long, b_long, b_src, out_long
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        sb.ceiling_copy(src, dst)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            sb.ceiling_copy(src, dst)
        e1.record()
        torch.cuda.synchronize()
        ceilings["copy_read_plus_write_GBps"] = round(5 * 2.0 * src.numel() / e0.elapsed_time(e1) / 1e6, 1)
        ceilings["unit"] = "T(FL)OP/s for the matrix-instruction loops (register-resident, no LDS or memory traffic), GB/s for the copy"
        del src, dst
        measured = {"int8": ceilings["mfma_int8_workload_codes"], "bf16": ceilings["mfma_bf16_workload_values"],
                    "f8": ceilings.get("mfma_float8_workload_codes"), "bytes": ceilings["copy_read_plus_write_GBps"]}

    kernels = {}
    for name, (ms, work, kind) in ops.items():
        if kind == "bytes":
            ach, peak, unit, bound = work / ms / 1e6, PEAK["hbm_GBps"], "GB/s", "hbm"
        else:
            ach, unit, bound = work / ms / 1e9, "TFLOP/s", "mfma"
            peak = PEAK["bf16_TFLOPs"] if kind == "bf16" else PEAK["int8_TOPs"]  # int8 and float8: 5.0 P(FL)OP/s dense
        kernels[name] = {"ms_per_step": round(ms, 4), "bound": bound, "achieved": round(ach, 1), "peak": peak,
                         "unit": unit, "frac": round(ach / peak, 4), "measured_peak": measured[kind],
                         "frac_of_measured": round(ach / measured[kind], 4) if measured[kind] else None}
    in_step = [k for k in kernels if "(" not in k]  # names with a parenthesis are measured beside the step
    dominant = max(in_step, key=lambda k: kernels[k]["ms_per_step"])
    roofline = {"kernel": dominant, "bound": kernels[dominant]["bound"], "achieved": kernels[dominant]["achieved"],
                "peak": kernels[dominant]["peak"], "unit": kernels[dominant]["unit"],
                "frac": kernels[dominant]["frac"],
                "measured_peak": kernels[dominant]["measured_peak"],
                "frac_of_measured": kernels[dominant]["frac_of_measured"],
                "measured_peak_is": "the register-resident matrix-instruction loop of this run on the workload's operand "
                                    "values (see ceilings); the published peak assumes 2.4 GHz, which the GPU does "
                                    "not hold under this load",
                "traffic": TRAFFIC_BYTES_PER_LAUNCH_VIT_H14.get(dominant) if args.config == "vit_h14" else None,
                "traffic_unit": "bytes per launch (mean over this kernel's launches of a step), HBM side, from profiles/"}
    op_sum = sum(kernels[k]["ms_per_step"] for k in in_step)
    quant_ms = kernels["quantize_rowwise"]["ms_per_step"] + kernels["quantize_tensorwise"]["ms_per_step"]

    # Clocks under load: rocm-smi is read by a child process while about a second of steps is still queued.
    clocks = None
    if not args.no_clocks:
        import re
        import subprocess
        for _ in range(max(1, int(1200.0 / max(sb_ms, 0.1)))):
            switchback_step()
        try:
            txt = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
            found = {}
            for name in ("sclk", "mclk", "fclk"):
                m = re.search(name + r" clock level:? *\d* *:? *\(?(\d+) ?[Mm][Hh]z", txt)
                if m:
                    found[name + "_MHz"] = int(m.group(1))
            clocks = found or None
        except Exception:
            clocks = None
        torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.ones(128 << 20, dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU oracle on a bounded sample of the same workload --------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import switchback_oracle as oracle
        L = max(cfg.layers, key=lambda l: l.n * l.m)
        rows = args.cpu_sample_rows or max(8, int(4.5e11 / (3.0 * L.n * L.m)))
        rows = min(rows, L.b)
        idx = np.linspace(0, L.b - 1, rows).astype(np.int64)
        li = cfg.layers.index(L)
        d = I.make_layer_inputs(args.config, li, token_rows=idx)
        t0 = time.perf_counter()
        f = oracle.forward(d["x"], d["w"])
        oracle.backward_input(d["dy"], f["wq_t"], f["state_w"])
        oracle.backward_weight(d["dy"], d["x"])
        secs = time.perf_counter() - t0
        cpu = {"value": round(6.0 * rows * L.n * L.m / secs / 1e12, 5), "unit": "TFLOP/s",
               "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(secs, 2),
               "sample": "%s layer %s (n=%d, m=%d): forward + dX + dW on %d of %d token rows (evenly spaced), "
                         "W whole" % (args.config, L.name, L.n, L.m, rows, L.b)}

    out = {
        "metric": "SwitchBack linear fwd+bwd TFLOP/s + speedup vs bf16 linear, ViT-H shapes",
        "value": round(flop_per_step / sb_ms / 1e9, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sb_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8+bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %s; forward + input gradient + weight gradient of each layer" % (
            args.config, ", ".join("%s %dx(%d->%d)" % (l.name, l.b, l.n, l.m) for l in cfg.layers))},
        "speedup_vs_bf16_linear": round(bf_ms / sb_ms, 4),
        "bf16_linear_ms_per_step": round(bf_ms, 4),
        "bf16_linear_TFLOPs": round(flop_per_step / bf_ms / 1e9, 2),
        "wall_ms_per_step": round(sb_wall_ms, 4),
        "ms_per_step_w_requantized_in_backward": round(requant_ms, 4),
        "ms_per_step_switchback_m": round(variant_m_ms, 4),
        "ms_per_step_switchback_q": round(variant_q_ms, 4),
        "ms_per_step_switchback_float8": None if variant_f8_ms is None else round(variant_f8_ms, 4),
        "per_layer": per_layer,
        "roofline": roofline,
        "kernels": kernels,
        "ceilings": ceilings,
        "sum_of_kernel_ms": round(op_sum, 4),
        "quantize_share_of_kernel_time": round(quant_ms / op_sum, 4),
        "clocks_under_load": clocks,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
