#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A step is one pass of the whole path -- dvdq_qlinear: block-Hadamard rotation,
per-token auto-scale, quantization, INT4 x INTb GEMM, dequantizing epilogue --
over one batch of synthetic activations of the small-video-DiT QKV projection
(M=32760 tokens, K=1536, N=4608, W4A4, Hadamard block 256).  Inputs are resident
in HBM before the timed region; weights are pre-packed offline.  W4A4 runs on the
FP6 matrix path (4-bit codes carried as E2M3 patterns, integer-exact, twice the INT8
matrix rate; --w4a4-path int8 selects the INT8 matrix path with codes packed two per
byte); other bit-widths run on the INT8 matrix path with the int8 container.

Prints ONE JSON line: whole-path throughput in TOP/s (2*M*N*K per step), the
roofline of the dominant kernel (the GEMM, against the matrix peak of the operand
type it runs on) from per-launch HIP-event timings, the same for the HBM-bound
rotate+quantize kernel, the other W4A4 matrix path for reference, and the CPU oracle
timed on this machine's host cores on a bounded token sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # published dense INT8 matrix peak, MI355X
FP6_MFMA_PEAK_TOPS = 10100.0     # published dense FP6 / FP4 matrix peak, MI355X
HBM_PEAK_GBPS = 8000.0           # published HBM3E bandwidth, MI355X

# HBM bytes per launch (read + written) from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# very command, scaled by the same counters' reading for dvdq_bench_copy; the summaries with the
# commands are profiles/bench_<workload>_hbm_counters.md.  None where no counter run exists.
MEASURED_HBM_TRAFFIC = {   # keyed by (workload, container of the codes between the two kernels)
    ("small_dit_qkv_w4a4", "fp6"): {"gemm": 496.2e6, "rotate_quant": 138.7e6},
    ("small_dit_qkv_w4a4", "packed4"): {"gemm": 368.0e6, "rotate_quant": 126.2e6},
    ("small_dit_ffn_up_w4a6", "int8"): {"gemm": 795.7e6, "rotate_quant": 151.3e6},
    ("large_dit_proj_w4a4", "fp6"): {"gemm": 2545.7e6, "rotate_quant": 1004.3e6},
    ("large_dit_proj_w4a4", "packed4"): {"gemm": 2000.1e6, "rotate_quant": 914.3e6},
    ("large_dit_ffn_down_w4a4", "fp6"): {"gemm": 3587.2e6, "rotate_quant": 1245.9e6},
    ("large_dit_ffn_down_w4a4", "packed4"): {"gemm": 3446.7e6, "rotate_quant": 1133.3e6},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=1, help="index into the five configs (default: the headline one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--w4a4-path", choices=("fp6", "int8"), default="fp6",
                    help="matrix path of 4-bit activations: FP6 (E2M3 patterns, default) or INT8 (packed nibbles)")
    ap.add_argument("--bufs", type=int, default=3, help="input/output buffer sets rotated through (cache defeat)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; the path shards by tokens with no collective, "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import dvdq_inputs as di
    import paper_2505_18663_amd as dvdq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dvdq.lib()   # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    wl = di.WORKLOADS[args.workload]
    M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    nb = max(1, args.bufs)
    x0 = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(dev)
    xs = [x0] + [x0.clone() for _ in range(nb - 1)]
    wp_dev = torch.from_numpy(wp).to(dev)
    ws_dev = torch.from_numpy(ws).to(dev)
    use_fp6 = bits == 4 and args.w4a4_path == "fp6"
    if use_fp6:
        fmt, lay, w_native = dvdq.CODES_FP6, dvdq.W_NATIVE_FP6, dvdq.w4_prepack_fp6(wp_dev)
    else:
        fmt, lay, w_native = (dvdq.CODES_PACKED4 if bits == 4 else dvdq.CODES_INT8), dvdq.W_NATIVE, dvdq.w4_prepack(wp_dev)
    fmt_name = {dvdq.CODES_INT8: "int8", dvdq.CODES_PACKED4: "packed4", dvdq.CODES_FP6: "fp6"}[fmt]
    peak_tops = FP6_MFMA_PEAK_TOPS if use_fp6 else INT8_MFMA_PEAK_TOPS
    need = dvdq.qlinear_workspace_bytes(M, K, fmt)
    wsp = [torch.empty((need,), dtype=torch.uint8, device=dev) for _ in range(nb)]
    ys = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(nb)]
    torch.cuda.synchronize()

    def step(i):
        j = i % nb
        dvdq.qlinear(xs[j], w_native, ws_dev, B, bits, lay, y=ys[j], workspace=wsp[j], codes_format=fmt)

    # ---- timed region: whole path.  Before the W warm-up steps the same step runs for about half a
    # second: coming out of idle the chip needs tens of milliseconds to settle its clocks, and
    # without this the first timed steps run up to 25 % slower than the steady state.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.5:
        for i in range(20):
            step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    ops = 2.0 * M * N * K
    tops = ops / t_step / 1e12

    # ---- per-kernel launch durations (HIP events on the launch stream, around groups of 5
    # back-to-back launches so that the event overhead does not inflate short kernels)
    def time_launches(fn, n, group=5):
        n_groups = max(1, n // group)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_groups)]
        for i in range(min(args.warmup, 5)):
            fn(i)
        torch.cuda.synchronize()
        for g in range(n_groups):
            ev[g][0].record()
            for i in range(group):
                fn(g * group + i)
            ev[g][1].record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) / group for a, b in ev)
        return sum(ms) / len(ms), ms[len(ms) // 2]

    views = [dvdq.workspace_views(w_, M, K, fmt) for w_ in wsp]

    def rq(i):
        j = i % nb
        dvdq.rotate_quant(xs[j], B, bits, codes=views[j][0], x_scale=views[j][1], codes_format=fmt)

    def gemm(i):
        j = i % nb
        dvdq.w4ax_gemm(views[j][0], views[j][1], w_native, ws_dev, bits, lay, y=ys[j], codes_format=fmt, K=K)

    # The two kernels of the path in the order the fused call runs them, one event after every
    # kernel: a kernel's duration is the time between the events around it.  Measured in this
    # context (the quantizer runs while the GEMM's output is still draining from the memory-side
    # cache; the GEMM finds the codes the quantizer just wrote) the two durations add up to the step.
    def time_in_context(n, rq=rq, gemm=gemm):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n + 1)]
        for i in range(min(args.warmup, 5)):
            rq(i)
            gemm(i)
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(n):
            rq(i)
            evs[2 * i + 1].record()
            gemm(i)
            evs[2 * i + 2].record()
        torch.cuda.synchronize()
        t_rq = sorted(evs[2 * i].elapsed_time(evs[2 * i + 1]) for i in range(n))
        t_gemm = sorted(evs[2 * i + 1].elapsed_time(evs[2 * i + 2]) for i in range(n))
        return sum(t_rq) / n, t_rq[n // 2], sum(t_gemm) / n, t_gemm[n // 2]

    rq_avg, rq_med, gemm_avg, gemm_med = time_in_context(args.steps)
    # the same kernels launched back to back on their own (no other kernel in between)
    rq_alone, _ = time_launches(rq, args.steps)
    gemm_alone, _ = time_launches(gemm, args.steps)
    # ---- W4A4 only: the other matrix path on the same inputs (separate workspaces), same in-context timing
    other_path = None
    if bits == 4:
        if use_fp6:
            o_fmt, o_lay, o_w, o_name, o_peak = dvdq.CODES_PACKED4, dvdq.W_NATIVE, dvdq.w4_prepack(wp_dev), "int8 matrix path, packed4 codes", INT8_MFMA_PEAK_TOPS
        else:
            o_fmt, o_lay, o_w, o_name, o_peak = dvdq.CODES_FP6, dvdq.W_NATIVE_FP6, dvdq.w4_prepack_fp6(wp_dev), "fp6 matrix path", FP6_MFMA_PEAK_TOPS
        o_wsp = [torch.empty((dvdq.qlinear_workspace_bytes(M, K, o_fmt),), dtype=torch.uint8, device=dev) for _ in range(nb)]
        o_views = [dvdq.workspace_views(w_, M, K, o_fmt) for w_ in o_wsp]

        def o_rq(i):
            j = i % nb
            dvdq.rotate_quant(xs[j], B, bits, codes=o_views[j][0], x_scale=o_views[j][1], codes_format=o_fmt)

        def o_gemm(i):
            j = i % nb
            dvdq.w4ax_gemm(o_views[j][0], o_views[j][1], o_w, ws_dev, bits, o_lay, y=ys[j], codes_format=o_fmt, K=K)
        o_rq_avg, _, o_gemm_avg, _ = time_in_context(args.steps, o_rq, o_gemm)
        o_step = o_rq_avg + o_gemm_avg
        other_path = {"path": o_name, "ms_per_step": round(o_step, 4), "value": round(ops / (o_step * 1e-3) / 1e12, 2),
                      "unit": "TOP/s", "gemm_avg_launch_ms": round(o_gemm_avg, 4),
                      "gemm_frac_of_its_peak": round(ops / (o_gemm_avg * 1e-3) / 1e12 / o_peak, 4), "gemm_peak": o_peak,
                      "rotate_quant_avg_launch_ms": round(o_rq_avg, 4)}
        del o_wsp, o_views, o_w

    code_bytes = {dvdq.CODES_INT8: 1.0, dvdq.CODES_PACKED4: 0.5, dvdq.CODES_FP6: 0.75}[fmt]
    rq_bytes = 2.0 * M * K + code_bytes * M * K + 4.0 * M      # bf16 in, codes out, fp32 scales out
    rq_gbps = rq_bytes / (rq_avg * 1e-3) / 1e9
    # the same kernel writing the int8 container (3 bytes per element), for reference
    codes8 = [torch.empty((M, K), dtype=torch.int8, device=dev) for _ in range(nb)]
    rq8_avg, _ = time_launches(lambda i: dvdq.rotate_quant(xs[i % nb], B, bits, codes=codes8[i % nb],
                                                           x_scale=views[i % nb][1]), args.steps)
    rq8_bytes = 3.0 * M * K + 4.0 * M
    del codes8
    gemm_tops = ops / (gemm_avg * 1e-3) / 1e12

    # ---- calibration: what this chip sustains for a plain copy and a register-only INT8 MFMA loop
    src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    copy_avg, _ = time_launches(lambda i: dvdq.bench_copy(src, dst), 10, group=2)
    copy_gbps = 2.0 * src.numel() / (copy_avg * 1e-3) / 1e9
    sink = torch.zeros((4,), dtype=torch.int32, device=dev)
    mfma_ops = [0.0]

    # register-only MFMA loops: on constant operands (only MFMA issue limits them) and on random 4-bit codes in
    # every lane and register (the chip's power management then holds a lower clock: the rate the matrix cores
    # sustain on the layer's kind of data, before any operand traffic)
    def mfma_rate(fn, data):
        def launch(i):
            mfma_ops[0] = fn(8000, sink, data=data)
        avg, _ = time_launches(launch, 4, group=2)
        return mfma_ops[0] / (avg * 1e-3) / 1e12
    mfma_ceiling = mfma_rate(dvdq.bench_mfma_i8, 0)
    mfma_ceiling_codes = mfma_rate(dvdq.bench_mfma_i8, 1)
    mfma6_ceiling = mfma_rate(dvdq.bench_mfma_fp6, 0)
    mfma6_ceiling_codes = mfma_rate(dvdq.bench_mfma_fp6, 1)
    del src, dst

    # ---- the delta-GBS controller step on a 720p-class latent (16 x 33 x 90 x 160 bf16 values):
    # two HBM reads of the tensor, one scalar out
    n_lat = 16 * 33 * 90 * 160
    f_prev = torch.randn((n_lat,), device=dev).to(torch.bfloat16)
    f_cur = (f_prev.float() + 0.05 * torch.randn((n_lat,), device=dev)).to(torch.bfloat16)
    ctl = dvdq.GbsController(delta=0.1)
    gbs_avg, _ = time_launches(lambda i: ctl.step(f_cur, f_prev), 20, group=10)

    # ---- the block-wise scaled variant of the same layer (4-bit codes with power-of-two group steps in
    # the int8 container; the GEMM then runs its int8-code path), as two calls on separate buffers
    blockwise = None
    if bits in (4, 6):
        vals = [torch.empty((M, K), dtype=torch.int8, device=dev) for _ in range(nb)]
        w_int8_path = w_native if lay == dvdq.W_NATIVE else dvdq.w4_prepack(wp_dev)

        def bw(i):
            j = i % nb
            dvdq.rotate_quant_blockwise(xs[j], B, bits, 128, values=vals[j], x_scale=views[j][1])
            dvdq.w4ax_gemm(vals[j], views[j][1], w_int8_path, ws_dev, 8, dvdq.W_NATIVE, y=ys[j])
        bw_avg, _ = time_launches(bw, args.steps)
        blockwise = {"group": 128, "ms_per_step": round(bw_avg, 4), "value": round(ops / (bw_avg * 1e-3) / 1e12, 2),
                     "unit": "TOP/s", "codes_format": "int8"}
        del vals

    # ---- the offline weight quantizer on this layer's weight shape (runs once per layer, fp64)
    w_f32 = (torch.randn((N, K), device=dev) * 0.02).contiguous()
    bgr_ms, _ = time_launches(lambda i: dvdq.bgr_quantize(w_f32), 2, group=1)
    del w_f32

    out = {
        "metric": "fused W4A4 qlinear TOPS & % INT8-MFMA peak; rotate+quant HBM GB/s",
        "value": round(tops, 2), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("fp6 e2m3 x fp6 e2m3 -> fp32, integer-exact (int4 codes; bf16 in/out)" if use_fp6
                  else "int8 x int4 -> int32 (bf16 in/out)"),
        "data": "synthetic",
        "config": {"workload": wl.name, "M": M, "K": K, "N": N, "had_block": B, "act_bits": bits,
                   "w_layout": "native_fp6" if use_fp6 else "native", "codes_format": fmt_name,
                   "matrix_path": "fp6" if use_fp6 else "int8", "buffers_rotated": nb},
        "frac_int8_mfma_peak": round(tops / INT8_MFMA_PEAK_TOPS, 4),
        "roofline": {"kernel": "w4a4_fp6_gemm" if use_fp6 else "w4ax_gemm", "bound": "mfma", "achieved": round(gemm_tops, 2),
                     "peak": peak_tops, "unit": "TOP/s", "frac": round(gemm_tops / peak_tops, 4),
                     "traffic": MEASURED_HBM_TRAFFIC.get((wl.name, fmt_name), {}).get("gemm"),
                     "avg_launch_ms": round(gemm_avg, 4), "median_launch_ms": round(gemm_med, 4),
                     "avg_launch_ms_alone": round(gemm_alone, 4),
                     "frac_of_int8_peak": round(gemm_tops / INT8_MFMA_PEAK_TOPS, 4),
                     "measured_mfma_ceiling_tops": round(mfma6_ceiling if use_fp6 else mfma_ceiling, 1),
                     "measured_mfma_ceiling_random_codes_tops": round(mfma6_ceiling_codes if use_fp6 else mfma_ceiling_codes, 1),
                     "measured_int8_mfma_ceiling_tops": round(mfma_ceiling, 1),
                     "measured_int8_mfma_ceiling_random_codes_tops": round(mfma_ceiling_codes, 1)},
        "roofline_rotate_quant": {"kernel": "rotate_quant", "bound": "hbm", "achieved": round(rq_gbps, 1),
                                  "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(rq_gbps / HBM_PEAK_GBPS, 4),
                                  "traffic": MEASURED_HBM_TRAFFIC.get((wl.name, fmt_name), {}).get("rotate_quant"),
                                  "avg_launch_ms": round(rq_avg, 4),
                                  "median_launch_ms": round(rq_med, 4), "avg_launch_ms_alone": round(rq_alone, 4),
                                  "algorithmic_bytes": rq_bytes,
                                  "measured_copy_gbps": round(copy_gbps, 1),
                                  "int8_container": {"achieved": round(rq8_bytes / (rq8_avg * 1e-3) / 1e9, 1),
                                                     "frac": round(rq8_bytes / (rq8_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                                     "avg_launch_ms": round(rq8_avg, 4),
                                                     "algorithmic_bytes": rq8_bytes}},
    }

    out["gbs_controller"] = {"elements": n_lat, "us_per_step": round(gbs_avg * 1e3, 2),
                             "achieved_gbps": round(4.0 * n_lat / (gbs_avg * 1e-3) / 1e9, 1), "bound": "hbm (launch-bound at this size)"}

    if other_path:
        out["other_w4a4_path"] = other_path
    if blockwise:
        out["blockwise_scaling"] = blockwise
    out["bgr_quantizer"] = {"rows": N, "K": K, "n_steps": 100, "max_refine": 10, "ms": round(bgr_ms, 2),
                            "note": "offline, once per layer; fp64"}

    # ---- CPU baseline: the oracle as it stands, on a bounded token sample (about 10-30 s of CPU work)
    if not args.no_cpu_baseline:
        import oracle
        probe = di.sample_rows(M, 256)
        xp = np.ascontiguousarray(xb[probe])
        oracle.qlinear(xp[:8], wp, ws, B, bits)            # build / load / warm the library
        t0 = time.perf_counter()
        oracle.qlinear(xp, wp, ws, B, bits)
        t_probe = time.perf_counter() - t0
        per_row = t_probe / probe.size
        n_rows = int(min(M, max(probe.size, 15.0 / per_row)))     # aim at ~15 s, never more than the workload
        if n_rows >= M:
            rows, what = np.arange(M), f"all {M} token rows"
        else:
            rows = di.sample_rows(M, n_rows // 2)
            what = f"{rows.size} of {M} token rows (first and last {n_rows // 2})"
        xs_rows = xb if rows.size == M else np.ascontiguousarray(xb[rows])
        t0 = time.perf_counter()
        oracle.qlinear(xs_rows, wp, ws, B, bits)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(2.0 * rows.size * N * K / t_cpu / 1e12, 5), "unit": "TOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{what}, whole layer (dense fp64 Hadamard, int64 GEMM), {t_cpu:.2f} s"
                      + ("" if rows.size == M else f"; work is linear in rows, full size extrapolates to "
                                                   f"{t_cpu * M / rows.size:.1f} s"),
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
