#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

A step is one pass of the whole path -- dvdq_qlinear: block-Hadamard rotation,
per-token auto-scale, quantization, INT4 x INTb GEMM, dequantizing epilogue --
over one batch of synthetic activations of one video-DiT linear layer.  Inputs are
resident in HBM before the timed region; weights are pre-packed offline.

By default the four DiT workloads are timed one after the other (QKV projection
and FFN up-projection of the small DiT, output projection and FFN down-projection
of the large one), each with the same K steps / W warm-ups, and reported under
`per_config`; the headline fields (`value`, `ms_per_step`, `config`, `roofline`,
`cpu_baseline`) are those of the largest one, the FFN down-projection
(M=32760, K=13824, N=5120, W4A4, Hadamard block 512).  `--workload i` times one.

W4A4 runs on the FP6 matrix path (4-bit codes carried as E2M3 patterns,
integer-exact, twice the INT8 matrix rate); its entry also carries the INT8
matrix path (codes packed two per byte) timed in the same run.  Other bit-widths
run on the INT8 matrix path with the int8 container.

Prints ONE JSON line: whole-path throughput in TOP/s (2*M*N*K per step) and as a
fraction of the published INT8 matrix peak, the roofline of the dominant kernel
(the GEMM, against the matrix peak of the operand type it runs on) from
per-launch HIP-event timings, the same for the HBM-bound rotate+quantize kernel,
and the CPU oracle timed on this machine's host cores on a bounded token sample.
"""
import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # published dense INT8 matrix peak, MI355X
FP6_MFMA_PEAK_TOPS = 10100.0     # published dense FP6 / FP4 matrix peak, MI355X
HBM_PEAK_GBPS = 8000.0           # published HBM3E bandwidth, MI355X
HEADLINE = 4                     # the largest single-GPU workload

# What the paper itself reports (Sec. 4, memory / latency table; Sec. 4.5): whole-model ratios against BF16
# on its own hardware.  Context only: another machine, another quantity than this path's kernel throughput.
PAPER_CONTEXT = {
    "source": "Sec. 4, table of memory saving and latency speedup; Sec. 4.5 (with TeaCache)",
    "hardware": "one NVIDIA RTX 4090", "workload": "HunyuanVideo, 50-step flow matching, whole model, vs BF16",
    "latency_speedup": {"W4A8": 1.75, "W4A6 (about half the steps W4A8, half W4A4)": 1.93, "W4A4": 2.12},
    "memory_reduction": 3.68, "latency_speedup_with_teacache": {"W4A8": 4.01, "W4A4": 4.85},
    "per_layer_numbers": None,
    "note": "the paper gives no GEMM or quantizer throughput for the layer in isolation, so vs_baseline is null",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=None,
                    help="index into the five configs: time this one only (default: all four DiT workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements (controller, block-wise, BGR)")
    ap.add_argument("--w4a4-path", choices=("fp6", "int8"), default="fp6",
                    help="matrix path of 4-bit activations: FP6 (E2M3 patterns, default) or INT8 (packed nibbles)")
    ap.add_argument("--bufs", type=int, default=3, help="input/output buffer sets rotated through (cache defeat)")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="CPU time aimed at per workload for the oracle leg")
    ap.add_argument("--overlap-experiment", action="store_true",
                    help="instead of the benchmark: time the layer with the quantizer of row panel p + 1 on a second stream "
                         "beside the GEMM of panel p (W4A4 workloads 1 and 3), against the plain back-to-back call")
    return ap.parse_args()


def csrc_digest():
    """Digest of the kernel sources: a profile summary records the one it was taken with."""
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(ROOT, "paper_2505_18663_amd", "csrc", "*"))):
        with open(p, "rb") as f:
            h.update(os.path.basename(p).encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def profile_traffic(workload_name):
    """{kernel name: HBM bytes per launch (read + written)} from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE
    summary of this workload (scaled there by the same counters' reading for the plain copy kernel), and the
    summary's path.  Empty when there is no summary or when it was taken with other kernel sources than the
    ones in the tree (the summary records their digest)."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload_name}_hbm_counters.md")
    if not os.path.exists(path):
        return {}, None
    rel = os.path.relpath(path, ROOT)
    text = open(path).read()
    m = re.search(r"csrc digest: `([0-9a-f]+)`", text)
    if not m or m.group(1) != csrc_digest():
        return {}, rel + " (taken with other kernel sources: not used)"
    rows = {}
    for line in text.splitlines():
        cells = [c.strip() for c in line.split("|")]
        if len(cells) >= 6 and cells[1].startswith("`"):
            try:
                rows[cells[1].strip("`")] = (float(cells[4]) + float(cells[5])) * 1e6
            except ValueError:
                pass
    return rows, rel


def first_match(rows, pattern, want_name=False):
    for name, v in rows.items():
        if re.match(pattern, name):
            return name if want_name else v
    return None


class Bench:
    def __init__(self, args):
        import numpy as np
        import torch
        import dvdq_inputs as di
        import paper_2505_18663_amd as dvdq
        self.args, self.np, self.torch, self.di, self.dvdq = args, np, torch, di, dvdq
        self.dev = "cuda:0"

    # per-kernel launch durations (HIP events on the launch stream -- torch's current stream, which is the one the
    # binding launches on -- around groups of back-to-back launches so that event overhead does not inflate short kernels)
    def time_launches(self, fn, n, group=5):
        torch = self.torch
        n_groups = max(1, n // group)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_groups)]
        for i in range(min(self.args.warmup, 5)):
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

    # The two kernels of the path in the order the fused call runs them, one event after every kernel: a kernel's
    # duration is the time between the events around it.  Measured in this context (the quantizer runs while the
    # GEMM's output is still draining from the memory-side cache; the GEMM finds the codes the quantizer just
    # wrote) the two durations add up to the step.
    def time_in_context(self, n, rq, gemm):
        torch = self.torch
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n + 1)]
        for i in range(min(self.args.warmup, 5)):
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

    def calibration(self):
        """What this chip sustains: a tuned streaming copy, and register-only MFMA loops on constant operands (only
        MFMA issue limits them) and on random 4-bit codes in every lane and register (the chip's power management
        then holds a lower clock: the rate the matrix cores sustain on the layer's kind of data, before any
        operand traffic)."""
        torch, dvdq = self.torch, self.dvdq
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=self.dev)
        dst = torch.empty_like(src)
        copy_avg, _ = self.time_launches(lambda i: dvdq.bench_copy(src, dst), 10, group=2)
        sink = torch.zeros((4,), dtype=torch.int32, device=self.dev)
        ops = [0.0]

        def rate(fn, data):
            def launch(i):
                ops[0] = fn(8000, sink, data=data)
            avg, _ = self.time_launches(launch, 4, group=2)
            return round(ops[0] / (avg * 1e-3) / 1e12, 1)
        return {"copy_gbps": round(2.0 * src.numel() / (copy_avg * 1e-3) / 1e9, 1),
                "int8_mfma_tops_constant_operands": rate(dvdq.bench_mfma_i8, 0),
                "int8_mfma_tops_random_codes": rate(dvdq.bench_mfma_i8, 1),
                "fp6_mfma_tops_constant_operands": rate(dvdq.bench_mfma_fp6, 0),
                "fp6_mfma_tops_random_codes": rate(dvdq.bench_mfma_fp6, 1)}

    def path_setup(self, wl, wp_dev, use_fp6):
        dvdq = self.dvdq
        if use_fp6:
            return dict(fmt=dvdq.CODES_FP6, lay=dvdq.W_NATIVE_FP6, w=dvdq.w4_prepack_fp6(wp_dev), fmt_name="fp6",
                        kernel="w4a4_fp6_gemm", peak=FP6_MFMA_PEAK_TOPS, code_bytes=0.75, matrix_path="fp6",
                        dtype="fp6 e2m3 x fp6 e2m3 -> fp32, integer-exact (int4 codes; bf16 in/out)")
        packed = wl.act_bits == 4
        return dict(fmt=dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8, lay=dvdq.W_NATIVE, w=dvdq.w4_prepack(wp_dev),
                    fmt_name="packed4" if packed else "int8", kernel="w4ax_gemm", peak=INT8_MFMA_PEAK_TOPS,
                    code_bytes=0.5 if packed else 1.0, matrix_path="int8", dtype="int8 x int4 -> int32 (bf16 in/out)")

    def run_workload(self, idx):
        args, np, torch, di, dvdq = self.args, self.np, self.torch, self.di, self.dvdq
        wl = di.WORKLOADS[idx]
        M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
        print(f"[bench] {wl.name}: inputs", file=sys.stderr, flush=True)
        xb = di.make_x(wl)
        wp, ws, _ = di.make_weights(wl)
        nb = max(1, args.bufs)
        x0 = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(self.dev)
        xs = [x0] + [x0.clone() for _ in range(nb - 1)]
        wp_dev = torch.from_numpy(wp).to(self.dev)
        ws_dev = torch.from_numpy(ws).to(self.dev)
        ys = [torch.empty((M, N), dtype=torch.bfloat16, device=self.dev) for _ in range(nb)]
        ops = 2.0 * M * N * K
        use_fp6 = bits == 4 and args.w4a4_path == "fp6"
        print(f"[bench] {wl.name}: timing", file=sys.stderr, flush=True)

        def measure(p, whole_step):
            wsp = [torch.empty((dvdq.qlinear_workspace_bytes(M, K, p["fmt"]),), dtype=torch.uint8, device=self.dev)
                   for _ in range(nb)]
            views = [dvdq.workspace_views(w_, M, K, p["fmt"]) for w_ in wsp]

            def step(i):
                j = i % nb
                dvdq.qlinear(xs[j], p["w"], ws_dev, B, bits, p["lay"], y=ys[j], workspace=wsp[j], codes_format=p["fmt"])

            def rq(i):
                j = i % nb
                dvdq.rotate_quant(xs[j], B, bits, codes=views[j][0], x_scale=views[j][1], codes_format=p["fmt"])

            def gemm(i):
                j = i % nb
                dvdq.w4ax_gemm(views[j][0], views[j][1], p["w"], ws_dev, bits, p["lay"], y=ys[j], codes_format=p["fmt"], K=K)

            res = {}
            if whole_step:
                # Timed region: the whole path.  Before the W warm-up steps the same step runs for about half a
                # second: coming out of idle the chip needs tens of milliseconds to settle its clocks, and without
                # this the first timed steps run up to 25 % slower than the steady state.
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
                res["t_step"] = (time.perf_counter() - t0) / args.steps
            res["rq_avg"], res["rq_med"], res["gemm_avg"], res["gemm_med"] = self.time_in_context(args.steps, rq, gemm)
            if whole_step:
                # the same kernels launched back to back on their own (no other kernel in between)
                res["rq_alone"], _ = self.time_launches(rq, args.steps)
                res["gemm_alone"], _ = self.time_launches(gemm, args.steps)
            res["views"] = views
            return res

        p = self.path_setup(wl, wp_dev, use_fp6)
        r = measure(p, True)
        t_step = r["t_step"]
        tops = ops / t_step / 1e12
        gemm_tops = ops / (r["gemm_avg"] * 1e-3) / 1e12
        rq_bytes = (2.0 + p["code_bytes"]) * M * K + 4.0 * M       # bf16 in, codes out, fp32 scales out
        rq_gbps = rq_bytes / (r["rq_avg"] * 1e-3) / 1e9
        traffic, src = profile_traffic(wl.name)
        # (whichever kernel the library's dispatch took for this shape: the summary holds the kernels of this workload's run)
        gemm_traffic = first_match(traffic, r"dvdq::(w4a4_fp6_gemm_kernel<|w4ax_gemm_wide_kernel<true, )" if use_fp6 else
                                   (r"dvdq::w4ax_gemm_native_kernel<.*, true>" if p["fmt_name"] == "packed4" else
                                    r"dvdq::(w4ax_gemm_native_kernel<.*, false>|w4ax_gemm_wide_kernel<false, )"))
        gemm_symbol = first_match(traffic, r"dvdq::(w4a4_fp6_gemm_kernel<|w4ax_gemm_wide_kernel<true, )" if use_fp6 else
                                  (r"dvdq::w4ax_gemm_native_kernel<.*, true>" if p["fmt_name"] == "packed4" else
                                   r"dvdq::(w4ax_gemm_native_kernel<.*, false>|w4ax_gemm_wide_kernel<false, )"), want_name=True)
        rq_traffic = first_match(traffic, r"dvdq::rotate_quant_kernel<\d+, \d+, %d>" % {"int8": 0, "packed4": 1, "fp6": 2}[p["fmt_name"]])
        entry = {
            "workload": wl.name, "M": M, "K": K, "N": N, "had_block": B, "act_bits": bits,
            "matrix_path": p["matrix_path"], "codes_format": p["fmt_name"], "dtype": p["dtype"],
            "ms_per_step": round(t_step * 1e3, 4), "value": round(tops, 2), "unit": "TOP/s",
            "frac_int8_mfma_peak": round(tops / INT8_MFMA_PEAK_TOPS, 4),
            "roofline": {"kernel": p["kernel"], "kernel_symbol": gemm_symbol, "bound": "mfma", "achieved": round(gemm_tops, 2), "peak": p["peak"],
                         "unit": "TOP/s", "frac": round(gemm_tops / p["peak"], 4), "traffic": gemm_traffic,
                         "traffic_source": src,
                         "avg_launch_ms": round(r["gemm_avg"], 4), "median_launch_ms": round(r["gemm_med"], 4),
                         "avg_launch_ms_alone": round(r["gemm_alone"], 4),
                         "frac_of_int8_peak": round(gemm_tops / INT8_MFMA_PEAK_TOPS, 4)},
            "roofline_rotate_quant": {"kernel": "rotate_quant", "bound": "hbm", "achieved": round(rq_gbps, 1),
                                      "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(rq_gbps / HBM_PEAK_GBPS, 4),
                                      "traffic": rq_traffic, "traffic_source": src,
                                      "avg_launch_ms": round(r["rq_avg"], 4), "median_launch_ms": round(r["rq_med"], 4),
                                      "avg_launch_ms_alone": round(r["rq_alone"], 4), "algorithmic_bytes": rq_bytes},
        }
        views = r["views"]
        del r
        # W4A4: the other matrix path on the same inputs, same in-context timing
        if bits == 4:
            po = self.path_setup(wl, wp_dev, not use_fp6)
            ro = measure(po, False)
            o_step = ro["rq_avg"] + ro["gemm_avg"]
            o_tops = ops / (o_step * 1e-3) / 1e12
            o_bytes = (2.0 + po["code_bytes"]) * M * K + 4.0 * M
            entry["other_w4a4_path"] = {
                "matrix_path": po["matrix_path"], "codes_format": po["fmt_name"], "ms_per_step": round(o_step, 4),
                "value": round(o_tops, 2), "unit": "TOP/s", "frac_int8_mfma_peak": round(o_tops / INT8_MFMA_PEAK_TOPS, 4),
                "gemm_avg_launch_ms": round(ro["gemm_avg"], 4), "gemm_peak": po["peak"],
                "gemm_frac_of_its_peak": round(ops / (ro["gemm_avg"] * 1e-3) / 1e12 / po["peak"], 4),
                "rotate_quant_avg_launch_ms": round(ro["rq_avg"], 4),
                "rotate_quant_gbps": round(o_bytes / (ro["rq_avg"] * 1e-3) / 1e9, 1),
                "rotate_quant_frac_hbm": round(o_bytes / (ro["rq_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
            del ro, po
        # the same quantizer writing the int8 container (3 bytes per element), for reference
        if p["fmt_name"] != "int8":
            codes8 = [torch.empty((M, K), dtype=torch.int8, device=self.dev) for _ in range(nb)]
            rq8_avg, _ = self.time_launches(lambda i: dvdq.rotate_quant(xs[i % nb], B, bits, codes=codes8[i % nb],
                                                                        x_scale=views[i % nb][1]), args.steps)
            rq8_bytes = 3.0 * M * K + 4.0 * M
            entry["roofline_rotate_quant"]["int8_container"] = {
                "achieved": round(rq8_bytes / (rq8_avg * 1e-3) / 1e9, 1), "frac": round(rq8_bytes / (rq8_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "avg_launch_ms": round(rq8_avg, 4), "algorithmic_bytes": rq8_bytes}
            del codes8

        if idx == 1 and not args.no_extras:
            entry["extras"] = self.extras(wl, xs, ys, views, p, wp_dev, ws_dev, ops)

        # CPU baseline: the oracle as it stands, on a bounded token sample
        if not args.no_cpu_baseline:
            print(f"[bench] {wl.name}: oracle on the host cores", file=sys.stderr, flush=True)
            import oracle
            probe = di.sample_rows(M, 32)
            xp = np.ascontiguousarray(xb[probe])
            oracle.qlinear(xp[:8], wp, ws, B, bits)            # build / load / warm the library
            t0 = time.perf_counter()
            oracle.qlinear(xp, wp, ws, B, bits)
            per_row = (time.perf_counter() - t0) / probe.size
            n_rows = int(min(M, max(probe.size, args.cpu_seconds / per_row)))
            if n_rows >= M:
                rows, what = np.arange(M), f"all {M} token rows"
            else:
                rows = di.sample_rows(M, n_rows // 2)
                what = f"{rows.size} of {M} token rows (first and last {n_rows // 2})"
            xs_rows = xb if rows.size == M else np.ascontiguousarray(xb[rows])
            t0 = time.perf_counter()
            oracle.qlinear(xs_rows, wp, ws, B, bits)
            t_cpu = time.perf_counter() - t0
            entry["cpu_baseline"] = {
                "value": round(2.0 * rows.size * N * K / t_cpu / 1e12, 5), "unit": "TOP/s",
                "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"{what}, whole layer (dense fp64 Hadamard, int64 GEMM), {t_cpu:.2f} s"
                          + ("" if rows.size == M else f"; work is linear in rows, the full size extrapolates to "
                                                       f"{t_cpu * M / rows.size:.1f} s (extrapolated)"),
            }
        del xs, ys, views, x0
        torch.cuda.empty_cache()
        return entry

    def extras(self, wl, xs, ys, views, p, wp_dev, ws_dev, ops):
        """Side measurements on the QKV workload: the delta-GBS controller step, the block-wise scaled variant of
        the layer, the offline weight quantizer."""
        torch, dvdq, args = self.torch, self.dvdq, self.args
        M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
        nb = len(xs)
        out = {}
        # the controller on a 720p-class latent (16 x 33 x 90 x 160 bf16 values): two HBM reads of the tensor, one scalar out
        n_lat = 16 * 33 * 90 * 160
        f_prev = torch.randn((n_lat,), device=self.dev).to(torch.bfloat16)
        f_cur = (f_prev.float() + 0.05 * torch.randn((n_lat,), device=self.dev)).to(torch.bfloat16)
        ctl = dvdq.GbsController(delta=0.1)
        gbs_avg, _ = self.time_launches(lambda i: ctl.step(f_cur, f_prev), 20, group=10)
        out["gbs_controller"] = {"elements": n_lat, "us_per_step": round(gbs_avg * 1e3, 2),
                                 "achieved_gbps": round(4.0 * n_lat / (gbs_avg * 1e-3) / 1e9, 1),
                                 "bound": "hbm (launch-bound at this size)"}
        # block-wise scaled variant (4-bit codes with power-of-two group steps in the int8 container; the GEMM then
        # runs its int8-code path), as two calls on separate buffers
        vals = [torch.empty((M, K), dtype=torch.int8, device=self.dev) for _ in range(nb)]
        w_int8_path = p["w"] if p["lay"] == dvdq.W_NATIVE else dvdq.w4_prepack(wp_dev)

        def bw(i):
            j = i % nb
            dvdq.rotate_quant_blockwise(xs[j], B, bits, 128, values=vals[j], x_scale=views[j][1])
            dvdq.w4ax_gemm(vals[j], views[j][1], w_int8_path, ws_dev, 8, dvdq.W_NATIVE, y=ys[j])
        bw_avg, _ = self.time_launches(bw, args.steps)
        out["blockwise_scaling"] = {"group": 128, "ms_per_step": round(bw_avg, 4), "value": round(ops / (bw_avg * 1e-3) / 1e12, 2),
                                    "unit": "TOP/s", "codes_format": "int8"}
        del vals
        # the offline weight quantizer on this layer's weight shape (runs once per layer, fp64)
        w_f32 = (torch.randn((N, K), device=self.dev) * 0.02).contiguous()
        bgr_ms, _ = self.time_launches(lambda i: dvdq.bgr_quantize(w_f32), 2, group=1)
        out["bgr_quantizer"] = {"rows": N, "K": K, "n_steps": 100, "max_refine": 10, "search": "as printed in Alg. 1",
                                "ms": round(bgr_ms, 2), "note": "offline, once per layer; fp64"}
        return out


def overlap_experiment(torch, dvdq, di):
    """Rotate/GEMM overlap by row panels: panel p + 1 is quantized on one stream while the GEMM of panel p runs on
    another (same priority), the GEMM's persistent grid optionally shortened to leave compute units free.  Every
    variant is checked bit for bit against the plain call; times are medians of event pairs around whole calls,
    host launch work included on both sides."""
    import itertools
    dev = "cuda:0"

    def med(fn, n=15, warm=4):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return sorted(ts)[n // 2]

    out = {}
    main_stream = torch.cuda.current_stream()
    sq, sg = torch.cuda.Stream(), torch.cuda.Stream()
    for idx in (1, 3):
        wl = di.WORKLOADS[idx]
        M, K, N, B = wl.M, wl.K, wl.N, wl.had_block
        g = torch.Generator(device=dev)
        g.manual_seed(idx)
        x = (torch.randn((M, K), device=dev, generator=g) *
             torch.exp(0.5 * torch.randn((M, 1), device=dev, generator=g))).to(torch.bfloat16)
        w = dvdq.w4_prepack_fp6(torch.randint(0, 256, (N, K // 2), device=dev, dtype=torch.uint8, generator=g))
        ws = torch.rand((N,), device=dev, generator=g) * 0.01 + 1e-3
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        wsb = torch.empty(dvdq.qlinear_workspace_bytes(M, K, dvdq.CODES_FP6), dtype=torch.uint8, device=dev)
        t0 = med(lambda: dvdq.qlinear(x, w, ws, B, 4, dvdq.W_NATIVE_FP6, y=y, workspace=wsb, codes_format=dvdq.CODES_FP6))
        y_ref = y.clone()
        entry = {"back_to_back_us": round(t0 * 1e3, 1), "panelled": []}
        for panels, limit in itertools.product((2, 4, 8), (0, 496, 448, 384)):
            rows = -(-(-(-M // panels)) // 256) * 256
            bounds = [(r, min(M, r + rows)) for r in range(0, M, rows)]
            cs = [torch.empty(dvdq.codes_bytes(b - a, K, dvdq.CODES_FP6), dtype=torch.uint8, device=dev) for a, b in bounds]
            ss = [torch.empty((b - a,), dtype=torch.float32, device=dev) for a, b in bounds]

            def panelled():
                sq.wait_stream(main_stream)
                sg.wait_stream(main_stream)
                for (a, b), c, sc in zip(bounds, cs, ss):
                    dvdq.rotate_quant(x[a:b], B, 4, codes=c, x_scale=sc, codes_format=dvdq.CODES_FP6, stream=sq)
                    ev = torch.cuda.Event()
                    ev.record(sq)
                    sg.wait_event(ev)
                    dvdq.w4ax_gemm(c, sc, w, ws, 4, dvdq.W_NATIVE_FP6, y=y[a:b], codes_format=dvdq.CODES_FP6, K=K, stream=sg)
                main_stream.wait_stream(sg)
                main_stream.wait_stream(sq)
            dvdq.bench_set_gemm_grid_limit(limit)
            y.zero_()
            t = med(panelled)
            same = bool(torch.equal(y.view(torch.int16), y_ref.view(torch.int16)))
            dvdq.bench_set_gemm_grid_limit(0)
            entry["panelled"].append({"panels": len(bounds), "gemm_workgroups_at_most": limit or "all", "us": round(t * 1e3, 1),
                                      "vs_back_to_back": round(t / t0, 3), "identical": same})
        out[wl.name] = entry
        del x, w, y, wsb
        torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; the path shards by tokens with no collective, "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2505_18663_amd as dvdq
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dvdq.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    if args.overlap_experiment:
        import dvdq_inputs as di
        print(json.dumps({"experiment": "rotate/GEMM overlap by row panels on two streams", "results": overlap_experiment(torch, dvdq, di)}))
        return
    b = Bench(args)
    which = [args.workload] if args.workload is not None else [1, 2, 3, 4]
    head_idx = HEADLINE if HEADLINE in which else which[-1]
    calib = b.calibration()
    per = {}
    for idx in which:
        e = b.run_workload(idx)
        per[e["workload"]] = e
    head = per[b.di.WORKLOADS[head_idx].name]
    out = {
        "metric": "fused W4A4 qlinear TOPS & % INT8-MFMA peak; rotate+quant HBM GB/s",
        "value": head["value"], "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "M": head["M"], "K": head["K"], "N": head["N"],
                   "had_block": head["had_block"], "act_bits": head["act_bits"], "matrix_path": head["matrix_path"],
                   "codes_format": head["codes_format"], "buffers_rotated": max(1, args.bufs),
                   "also_timed": [n for n in per if n != head["workload"]]},
        "frac_int8_mfma_peak": head["frac_int8_mfma_peak"],
        "roofline": dict(head["roofline"]),
        "roofline_rotate_quant": dict(head["roofline_rotate_quant"]),
        "calibration": calib,
        "targets": {"fused_frac_int8_mfma_peak": 0.5, "rotate_quant_frac_hbm": 0.7},
        "summary": {n: {"ms_per_step": e["ms_per_step"], "TOP/s": e["value"], "frac_int8_mfma_peak": e["frac_int8_mfma_peak"],
                        "matrix_path": e["matrix_path"], "gemm_frac_of_its_peak": e["roofline"]["frac"],
                        "rotate_quant_frac_hbm": e["roofline_rotate_quant"]["frac"],
                        **({"int8_matrix_path_frac_int8_mfma_peak": e["other_w4a4_path"]["frac_int8_mfma_peak"]}
                           if "other_w4a4_path" in e and e["other_w4a4_path"]["matrix_path"] == "int8" else {})}
                    for n, e in per.items()},
        "per_config": per,
        "paper_context": PAPER_CONTEXT,
    }
    out["roofline"]["measured_mfma_ceiling_tops"] = calib["fp6_mfma_tops_constant_operands" if head["matrix_path"] == "fp6" else "int8_mfma_tops_constant_operands"]
    out["roofline"]["measured_mfma_ceiling_random_codes_tops"] = calib["fp6_mfma_tops_random_codes" if head["matrix_path"] == "fp6" else "int8_mfma_tops_random_codes"]
    out["roofline_rotate_quant"]["measured_copy_gbps"] = calib["copy_gbps"]
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
