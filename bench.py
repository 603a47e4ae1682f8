#!/usr/bin/env python3
"""Benchmark of the SLiM compressed-linear forward path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--legs all|decode|prefill|none] [--no-cpu]

Workload of the headline line (`config.workload`): the largest configured layer that one GPU
holds, the LLaMA-2-70B-shaped up projection in decode: W 28672 x 8192 int4 2:4 + rank-820 fp16
adapters.  One "step" is one forward of that layer at 1 and at 16 tokens (two slim_linear_gemv
calls), every call on a copy of the layer that the calls before it have pushed out of the caches
(rotation over enough copies to exceed twice the 256 MB Infinity Cache), inputs resident in HBM.

`value` = algorithmic bytes of a step / time of a step, in GB/s, over exactly K steps between two
events on the launch stream.  The JSON line also carries
  roofline      of the dominant kernel (decode_fused_kernel, both calls of a step are launches of it),
  batches       median and minimum over five more batches of K steps,
  cpu_baseline  the CPU oracle on the same step, and on a 256-row sample of the prefill call,
  legs          every other configured shape (decode and prefill; median and minimum of five batches
                each), the dense fp16 GEMM (torch -> hipBLASLt) measured the same way, the 4-bit
                adapter variant, and the offline entry points (slim_pack, ...).
Prefill legs state two fractions of the dense fp16 matrix peak: on the dense-equivalent FLOPs
(`roofline_frac`, flops_eff = 2 m n k + adapters) and on the FLOPs the method executes
(`roofline_frac_alg`: the 2:4 mask halves the weight term).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "layer µs, GB/s & TFLOP/s (% roofline), 2:4 int4+LoRA vs dense fp16 GEMM"
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0       # dense fp16/bf16 matrix peak
CACHE_BYTES = 256 << 20         # Infinity Cache
BATCHES = 5
# HBM bytes per launch of the dominant kernel on the headline workload (mean of the 1-token and the
# 16-token call of a step), from two rocprofv3 --pmc runs of `bench.py --headline-only` (FETCH_SIZE, then
# WRITE_SIZE), each scaled by what the same counter reads for the 256 MiB device copy this script
# issues first.  Not measured by this run: the summary file holds the command and the readings.
TRAFFIC_SOURCE = "profiles/decode_gemv_llama70b_up_hbm_traffic.md"
TRAFFIC_BYTES_PER_LAUNCH = 155.12e6


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--legs", default="all", choices=["all", "decode", "prefill", "none"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--headline-only", action="store_true",
                    help="warm-up, the timed steps and the batches only (profiler runs: every launch of the "
                         "dominant kernel is then one of the headline step)")
    ap.add_argument("--tokens", default="1,16", help="token counts of one step (counter runs use one value)")
    ap.add_argument("--layer", default="llama2_70b_up_28672x8192",
                    help="profiler runs of another configured shape: the decode step on that layer instead of the "
                         "headline one (the JSON line then names it in config.workload; not the benchmark)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2
    if args.headline_only:
        args.legs, args.no_cpu = "none", True

    import numpy as np
    import torch
    from paper_2410_09615_amd import accounting as A
    from paper_2410_09615_amd import binding as B
    from paper_2410_09615_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.lib()                                       # fail loudly if libslim.so is missing
    try:
        torch.backends.cuda.preferred_blas_library("hipblaslt")
    except Exception:
        pass

    def event_time_ms(fn, iters):
        """Average ms per call of fn(i) over `iters` back-to-back calls on the current stream, between
        two events recorded on that stream (the stream the library launches on)."""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / iters

    def batches_ms(fn, iters, batches=BATCHES):
        """ms per call in each of `batches` batches of `iters` calls (the rotation continues across batches)."""
        return [event_time_ms(lambda i, b=b: fn(b * iters + i), iters) for b in range(batches)]

    class Rotating:
        """`copies` device copies of one compressed layer, plus X / Y / workspace per copy, so that
        consecutive calls touch different HBM."""

        def __init__(self, shape, ms, min_copies=2, max_bytes=6 << 30, with_dense=True, adapter_bits=16):
            self.shape = shape
            self.adapter_bits = adapter_bits
            W, L, R, _ = wl.make_layer(shape, 1)
            self.W_host = W
            self.L_host, self.R_host = L, R
            Wd = W.to(dev)
            base = B.compress(Wd, L.to(dev), R.to(dev), adapter_bits=adapter_bits)
            torch.cuda.synchronize()
            self.base = base
            self.W_dev = Wd
            layer_bytes = A.packed_weight_bytes(shape.n, shape.k) + (
                A.adapter_bytes_q4(shape.n, shape.k, shape.r) if adapter_bits == 4 else A.adapter_bytes(shape.n, shape.k, shape.r))
            copies = max(min_copies, -(-2 * CACHE_BYTES // layer_bytes))
            copies = max(2, min(copies, max_bytes // max(layer_bytes, 1)))
            self.copies = int(copies)
            self.layers = [base]
            cl = lambda t: None if t is None else t.clone()
            for _ in range(self.copies - 1):
                self.layers.append(B.SlimLayer(base.n, base.k, base.rank, base.rank_pad, base.qvals.clone(),
                                               base.meta.clone(), base.scale.clone(), cl(base.L), cl(base.R),
                                               base.adapter_bits, cl(base.Lq), cl(base.Ls), cl(base.Rq), cl(base.Rs)))
            self.X, self.Y, self.ws = {}, {}, {}
            for m in ms:
                Xh = wl.make_activations(m, shape.k, shape.outliers)
                ncp = self.copies if m <= 16 else 2
                self.X[m] = [Xh.to(dev).clone() for _ in range(ncp)]
                self.Y[m] = [torch.empty(m, shape.n, dtype=torch.float16, device=dev) for _ in range(ncp)]
                self.ws[m] = [B.alloc_workspace(base, m) for _ in range(min(ncp, 4))]
            self.dense = None
            if with_dense:
                dense_bytes = 2 * shape.n * shape.k
                dcopies = max(2, min(-(-2 * CACHE_BYTES // dense_bytes), (4 << 30) // dense_bytes))
                Wh = Wd.to(torch.float16)
                self.dense = [Wh] + [Wh.clone() for _ in range(int(dcopies) - 1)]

        def call(self, fn, m, i):
            xs = self.X[m]
            fn(self.layers[i % self.copies], xs[i % len(xs)], self.Y[m][i % len(xs)], self.ws[m][i % len(self.ws[m])])

        def dense_call(self, m, i):
            xs = self.X[m]
            torch.matmul(xs[i % len(xs)], self.dense[i % len(self.dense)].t(), out=self.Y[m][i % len(xs)])

        def check_workspaces(self):
            for wss in self.ws.values():
                for w in wss:
                    B.slim_workspace_check(w)      # raises if a decode call gave up waiting for its T

    def leg_record(rot, m, fn, iters, warm, kind):
        shape = rot.shape
        for i in range(warm):
            rot.call(fn, m, i)
        ms_b = batches_ms(lambda i: rot.call(fn, m, i), iters)
        ms = statistics.median(ms_b)
        rot.check_workspaces()
        for i in range(max(3, warm // 3)):
            rot.dense_call(m, i)
        ms_dense = statistics.median(batches_ms(lambda i: rot.dense_call(m, i), iters, 3))
        nbytes = A.layer_bytes(shape.n, shape.k, shape.r, m, rot.adapter_bits)
        feff = A.flops_eff(shape.n, shape.k, shape.r, m)
        falg = A.flops_alg(shape.n, shape.k, shape.r, m)
        rec = {
            "shape": shape.name, "tokens": m, "entry": kind, "us": round(ms * 1e3, 3), "us_min": round(min(ms_b) * 1e3, 3),
            "batches": len(ms_b), "launches_per_batch": iters,
            "GBps": round(nbytes / ms * 1e-6, 1), "TFLOPs_eff": round(feff / ms * 1e-9, 2),
            "TFLOPs_alg": round(falg / ms * 1e-9, 2),
            "dense_fp16_us": round(ms_dense * 1e3, 3), "speedup_vs_dense_fp16": round(ms_dense / ms, 3),
            "byte_ratio_ceiling": round(A.dense_bytes(shape.n, shape.k, m) / nbytes, 2),
            "copies": rot.copies,
        }
        if rot.adapter_bits == 4:
            rec["adapters"] = "4-bit group-128"
        if kind == "slim_linear_gemv":
            rec["bound"] = "hbm"
            rec["roofline_frac"] = round(nbytes / ms * 1e-6 / HBM_PEAK_GBPS, 4)
        else:
            rec["bound"] = "mfma"
            rec["roofline_frac"] = round(feff / ms * 1e-9 / MFMA_PEAK_TFLOPS, 4)
            rec["roofline_frac_counts"] = "dense-equivalent FLOPs (flops_eff) over the dense fp16 peak"
            rec["roofline_frac_alg"] = round(falg / ms * 1e-9 / MFMA_PEAK_TFLOPS, 4)
        return rec

    def fp8_leg(rot, m, iters, warm):
        """slim_linear_gemm_fp8 on the rotation's inputs quantized once (App. "Input Quantization"): codes and scale
        resident before the timed region; the quantizer itself (codes only) is timed beside it."""
        shape = rot.shape
        q = [B.slim_input_quant_fp8(x, Xq=False, codes=True) for x in rot.X[m]]
        torch.cuda.synchronize()
        fmt = int(q[0][1][1])

        def call(i):
            _, info, codes = q[i % len(q)]
            B.slim_linear_gemm_fp8(rot.layers[i % rot.copies], codes, info, fmt, rot.Y[m][i % len(q)], rot.ws[m][i % len(rot.ws[m])])
        for i in range(warm):
            call(i)
        ms_b = batches_ms(call, iters)
        ms = statistics.median(ms_b)
        ms16 = statistics.median(batches_ms(lambda i: rot.call(B.slim_linear_gemm, m, i), iters, 3))
        x0 = rot.X[m][0]
        ms_q = statistics.median(batches_ms(lambda i: B.slim_input_quant_fp8(x0, False, q[0][1], None, q[0][2]), iters, 3))
        for i in range(3):
            rot.dense_call(m, i)
        ms_dense = statistics.median(batches_ms(lambda i: rot.dense_call(m, i), iters, 3))
        feff = A.flops_eff(shape.n, shape.k, shape.r, m)
        return {"shape": shape.name, "tokens": m, "entry": "slim_linear_gemm_fp8", "inputs": "E4M3" if fmt == 0 else "E5M2",
                "adapters": "4-bit group-128 (Sec. 3.3)" if rot.adapter_bits == 4 else "fp16",
                "us": round(ms * 1e3, 3), "us_min": round(min(ms_b) * 1e3, 3), "batches": len(ms_b), "launches_per_batch": iters,
                "TFLOPs_eff": round(feff / ms * 1e-9, 2), "fp16_inputs_us": round(ms16 * 1e3, 3),
                "input_quant_us": round(ms_q * 1e3, 3), "dense_fp16_us": round(ms_dense * 1e3, 3),
                "speedup_vs_dense_fp16": round(ms_dense / ms, 3), "speedup_vs_fp16_inputs": round(ms16 / ms, 3),
                "bound": "mfma", "roofline_frac": round(feff / ms * 1e-9 / 5000.0, 4),
                "roofline_frac_counts": "dense-equivalent FLOPs (flops_eff) over the dense FP8 peak, 5.0 PFLOP/s: the weight term runs "
                                        "on the 8-bit instruction, the adapters (a fifth of the FLOPs) on fp16",
                "roofline_frac_fp16_peak": round(feff / ms * 1e-9 / MFMA_PEAK_TFLOPS, 4)}

    # ---------------- headline: LLaMA-2-70B-shaped up projection, decode ----------------
    by_name = {c.name: c for c in (wl.L7B_ATTN, wl.L7B_UP, wl.L7B_DOWN, wl.L13B_ATTN, wl.L13B_UP, wl.L70B_ATTN, wl.L70B_UP)}
    if args.layer not in by_name:
        print("bench.py: --layer is one of " + ", ".join(by_name), file=sys.stderr)
        return 2
    shape = by_name[args.layer]
    headline = shape is wl.L70B_UP
    tokens = tuple(int(t) for t in args.tokens.split(","))
    rot = Rotating(shape, tokens, with_dense=not args.headline_only)

    # reference dispatch for hardware-counter runs: a plain 256 MiB device copy (reads 256 MiB, writes
    # 256 MiB), so that FETCH_SIZE / WRITE_SIZE readings of the kernels can be scaled by a transfer of known size
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    calib_dst = torch.empty_like(calib_src)
    for _ in range(3):
        calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    nt = len(tokens)

    def step(i):
        for j, m in enumerate(tokens):
            rot.call(B.slim_linear_gemv, m, nt * i + j)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    ms_step = event_time_ms(step, args.steps)                 # exactly K steps
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_wall0
    step_b = batches_ms(step, args.steps)
    rot.check_workspaces()
    # CPU time of one call through the binding (argument checks, ctypes, the launch), queue not full
    torch.cuda.synchronize()
    t_h0 = time.perf_counter()
    for i in range(50):
        step(i)
    host_us = (time.perf_counter() - t_h0) / (50 * len(tokens)) * 1e6
    torch.cuda.synchronize()
    step_bytes = sum(A.layer_bytes(shape.n, shape.k, shape.r, m) for m in tokens)
    step_flops = sum(A.flops_eff(shape.n, shape.k, shape.r, m) for m in tokens)
    value = step_bytes / ms_step * 1e-6            # GB/s
    launch_bytes = step_bytes / nt                 # algorithmic bytes of one launch, mean over the calls of a step
    launch_us = ms_step * 1e3 / nt
    roofline = {
        "bound": "hbm",
        "kernel": "decode_fused_kernel<false,false> (slim_linear_gemv, one launch per call; a step is "
                  + " + ".join(f"{m}" for m in tokens) + " tokens)",
        "achieved": round(launch_bytes / launch_us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(launch_bytes / launch_us * 1e-3 / HBM_PEAK_GBPS, 4),
        "traffic": TRAFFIC_BYTES_PER_LAUNCH if headline and tokens == (1, 16) else None,
        "traffic_source": TRAFFIC_SOURCE if TRAFFIC_BYTES_PER_LAUNCH and headline and tokens == (1, 16) else None,
        "algorithmic_bytes": launch_bytes, "avg_launch_us": round(launch_us, 3),
        "host_enqueue_us_per_call": round(host_us, 2),
        "note": "bytes and duration per launch are means over the calls of a step; duration = event time of the "
                "timed region / launches (launch gaps included)",
    }
    batches = {"count": len(step_b), "steps_each": args.steps,
               "ms_per_step_median": round(statistics.median(step_b), 6), "ms_per_step_min": round(min(step_b), 6),
               "value_median_GBps": round(step_bytes / statistics.median(step_b) * 1e-6, 1),
               "value_best_GBps": round(step_bytes / min(step_b) * 1e-6, 1)}

    per_m, hot, achievable, legs, cpu_baseline = {}, {}, None, [], None
    if not args.headline_only:
        # per-call records of the headline layer (same rotation, same stream), and the dense fp16 GEMM
        for m in tokens:
            per_m[m] = leg_record(rot, m, B.slim_linear_gemv, args.steps, args.warmup, "slim_linear_gemv")
        # cache-resident variant (no rotation), reported separately
        for m in tokens:
            x, y, w = rot.X[m][0], rot.Y[m][0], rot.ws[m][0]
            for _ in range(10):
                B.slim_linear_gemv(rot.base, x, y, w)
            hot[m] = round(event_time_ms(lambda i: B.slim_linear_gemv(rot.base, x, y, w), args.steps) * 1e3, 3)

        # ---- what the machine delivers: streaming read, back-to-back matrix instructions ----
        # (the same workload bytes read by a plain kernel, launch to launch and cold; 1 GiB for the asymptote)
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        big = torch.empty(4 << 30, dtype=torch.uint8, device=dev).fill_(1)

        def read_rate(nbytes, iters):
            nbytes = int(nbytes) // 65536 * 65536
            iters = min(iters, big.numel() // nbytes)
            B.slim_probe_read(big, nbytes, min(3, iters), nbytes, sink)
            ms = event_time_ms(lambda i: B.slim_probe_read(big, nbytes, iters, nbytes, sink), 1) / iters
            return nbytes / ms * 1e-6, ms * 1e3
        read_small_gbps, read_small_us = read_rate(launch_bytes, 200)
        read_big_gbps, _ = read_rate(1 << 30, 4)
        del big
        mfma = {}
        for sparse in (False, True):
            B.slim_probe_mfma(sparse, 256, 512, sink)
            fl = [0.0]

            def run(i, sparse=sparse):
                fl[0] = B.slim_probe_mfma(sparse, 4096, 512, sink)
            ms = event_time_ms(run, 5)
            mfma[sparse] = fl[0] / ms * 1e-9
        achievable = {
            "hbm_read_GBps_1GiB": round(read_big_gbps, 1),
            "hbm_read_GBps_at_workload_bytes": round(read_small_gbps, 1),
            "read_kernel_us_at_workload_bytes": round(read_small_us, 3),
            "mfma_f16_dense_TFLOPs": round(mfma[False], 1),
            "smfmac_f16_TFLOPs_as_dense_product": round(mfma[True], 1),
            "note": "plain read kernel / back-to-back matrix instructions of this library's probes, same run",
        }
        roofline["frac_of_read_kernel_at_same_bytes"] = round(read_small_us / launch_us, 4)

    # ---------------- CPU oracle baseline (rank 0 = this process) ----------------
    if not args.no_cpu:
        from oracle import slim_oracle as O
        Wn = rot.W_host.numpy()
        t0 = time.perf_counter()
        ref = O.compress(Wn)
        t_pack = time.perf_counter() - t0
        Ln, Rn = rot.L_host.numpy(), rot.R_host.numpy()
        Xs = {m: rot.X[m][0].cpu().numpy() for m in tokens}
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            for m in tokens:
                O.forward(ref, Ln, Rn, Xs[m])
        t_fwd = (time.perf_counter() - t0) / reps
        cpu_baseline = {
            "value": round(step_bytes / t_fwd * 1e-9, 4), "unit": "GB/s", "cores": O.threads(), "kind": "oracle",
            "sample": f"the full step (forward at {' and '.join(str(m) for m in tokens)} tokens of {shape.name}, all "
                      f"{shape.n} output rows), fp64, mean of {reps} passes",
            "ms_per_step": round(t_fwd * 1e3, 2), "pack_ms": round(t_pack * 1e3, 2),
        }
        # parity spot check of the timed configuration against the oracle
        dom_m = max(tokens)
        Yg = rot.Y[dom_m][0].clone()
        B.slim_linear_gemv(rot.base, rot.X[dom_m][0], Yg, rot.ws[dom_m][0])
        torch.cuda.synchronize()
        Yr = O.forward(ref, Ln, Rn, Xs[dom_m])
        cpu_baseline["parity_rel_err_max_tokens"] = float(
            np.linalg.norm(Yg.cpu().numpy().astype(np.float64) - Yr) / np.linalg.norm(Yr))
        # the prefill call of the same layer (4096 tokens) on 256 of its output rows, extrapolated to all rows
        # (the adapter stage T = X R^T does not depend on the rows: timed once, counted once)
        if args.legs in ("all", "prefill"):
            mp = 4096
            Xp = wl.make_activations(mp, shape.k, shape.outliers).numpy()
            rows = np.sort(np.random.default_rng(0).choice(shape.n, size=256, replace=False))
            t0 = time.perf_counter()
            O.xr(Xp, Rn)
            t_xr = time.perf_counter() - t0
            t0 = time.perf_counter()
            O.forward(ref, Ln, Rn, Xp, rows=rows)
            t_rows = time.perf_counter() - t0
            t_full = t_xr + (t_rows - t_xr) * shape.n / rows.size
            cpu_baseline["prefill_sample"] = {
                "sample": f"forward of {shape.name} at {mp} tokens on 256 random output rows",
                "seconds_sample": round(t_rows, 3), "seconds_full_layer_extrapolated": round(t_full, 1),
                "TFLOPs_eff_extrapolated": round(A.flops_eff(shape.n, shape.k, shape.r, mp) / t_full * 1e-12, 5),
                "extrapolated": True,
            }
        del ref
    headline_copies = rot.copies
    dense_step_us = sum(per_m[m]["dense_fp16_us"] for m in tokens) if per_m else None
    del rot
    torch.cuda.empty_cache()

    # ---------------- other configured shapes ----------------
    if args.legs != "none":
        decode_cfgs = [(wl.L7B_ATTN, (1, 4, 16)), (wl.L13B_ATTN, (1,)), (wl.L13B_UP, (1,)), (wl.L70B_ATTN, (1, 16))]
        prefill_cfgs = [(wl.L7B_UP, 2048), (wl.L7B_DOWN, 2048), (wl.L13B_ATTN, 4096), (wl.L13B_UP, 4096),
                        (wl.L70B_ATTN, 4096), (wl.L70B_UP, 4096)]
        for shp, ms_ in (decode_cfgs if args.legs != "prefill" else []):
            r = Rotating(shp, ms_)
            for m in ms_:
                legs.append(leg_record(r, m, B.slim_linear_gemv, 100, 10, "slim_linear_gemv"))
            if shp is wl.L7B_ATTN:
                legs.extend(offline_legs(r, torch, B, A, wl, dev, event_time_ms))
            del r
            torch.cuda.empty_cache()
        # 4-bit group-128 adapters (Sec. 3.3): the same calls on a quarter of the adapter bytes
        q4_cfgs = [(wl.L7B_ATTN, (1, 16)), (wl.L70B_ATTN, (1,)), (wl.L70B_UP, (1, 16))]
        for shp, ms_ in (q4_cfgs if args.legs != "prefill" else []):
            r = Rotating(shp, ms_, adapter_bits=4)
            for m in ms_:
                legs.append(leg_record(r, m, B.slim_linear_gemv, 100, 10, "slim_linear_gemv"))
            del r
            torch.cuda.empty_cache()
        if args.legs in ("all", "prefill"):
            for shp, m in prefill_cfgs:
                r = Rotating(shp, (m,), min_copies=2, max_bytes=1 << 30)
                legs.append(leg_record(r, m, B.slim_linear_gemm, 8, 3, "slim_linear_gemm"))
                del r
                torch.cuda.empty_cache()
            r = Rotating(wl.L70B_ATTN, (4096,), min_copies=2, max_bytes=1 << 30, adapter_bits=4)
            legs.append(leg_record(r, 4096, B.slim_linear_gemm, 8, 3, "slim_linear_gemm"))
            del r
            torch.cuda.empty_cache()
            # 8-bit inputs (App. "Input Quantization"): the weight term on the 8-bit sparse matrix instruction
            for shp, m, bits in ((wl.L7B_UP, 2048, 16), (wl.L70B_ATTN, 4096, 16), (wl.L70B_UP, 4096, 16), (wl.L70B_ATTN, 4096, 4)):
                r = Rotating(shp, (m,), min_copies=2, max_bytes=1 << 30, adapter_bits=bits)
                legs.append(fp8_leg(r, m, 8, 3))
                del r
                torch.cuda.empty_cache()

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": ("LLaMA-2-70B-shaped up projection at one-GPU full size" if headline else shape.name) +
                               f", decode: W {shape.n}x{shape.k} int4 2:4 + rank-{shape.r} fp16 adapters, X of " +
                               " and ".join(str(m) for m in tokens) + " tokens (one step = these forwards), cold caches",
                   "n": shape.n, "k": shape.k, "rank": shape.r, "tokens": list(tokens), "layer_copies": headline_copies},
        "batches": batches,
        "layer_us": {str(m): per_m[m]["us"] for m in per_m},
        "layer_us_min": {str(m): per_m[m]["us_min"] for m in per_m},
        "layer_us_cache_resident": {str(m): hot[m] for m in hot},
        "layer_GBps": {str(m): per_m[m]["GBps"] for m in per_m},
        "layer_TFLOPs_eff": {str(m): per_m[m]["TFLOPs_eff"] for m in per_m},
        "hbm_roofline_frac": {str(m): per_m[m]["roofline_frac"] for m in per_m},
        "step_TFLOPs_eff": round(step_flops / ms_step * 1e-9, 3),
        "dense_fp16_gemm_us": {str(m): per_m[m]["dense_fp16_us"] for m in per_m},
        "speedup_vs_dense_fp16": round(dense_step_us * 1e-3 / ms_step, 3) if dense_step_us else None,
        "paper_context": "paper reports up to 4.3x (RTX 3060) and 3.8x (A100) layer-wise speed-up over dense fp16; "
                         "other machines, not a target",
        "wall_s_timed_region": round(wall, 4),
        "roofline": roofline, "achievable": achievable, "cpu_baseline": cpu_baseline, "legs": legs,
    }
    print(json.dumps(out))
    return 0


def offline_legs(rot, torch, B, A, wl, dev, event_time_ms):
    """The entry points that run once per layer, offline, on the 7B attention projection."""
    HBM = HBM_PEAK_GBPS
    shape = rot.shape
    legs = []
    q, me, sc = rot.base.qvals, rot.base.meta, rot.base.scale
    wcopies = [rot.W_dev] + [rot.W_dev.clone() for _ in range(8)]      # 9 x 64 MiB > 2 x cache
    for i in range(5):
        B.slim_pack(wcopies[i % len(wcopies)], q, me, sc)
    ms_pack = event_time_ms(lambda i: B.slim_pack(wcopies[i % len(wcopies)], q, me, sc), 45)
    pb = A.pack_bytes(shape.n, shape.k)
    legs.append({"shape": shape.name, "entry": "slim_pack", "us": round(ms_pack * 1e3, 2),
                 "GBps": round(pb / ms_pack * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(pb / ms_pack * 1e-6 / HBM, 4)})
    # slim_quant_search reads W twice (maximum, histogram); slim_pack_ex as slim_pack plus the saliency vector
    for i in range(5):
        B.slim_quant_search(wcopies[i % len(wcopies)])
    ms_qs = event_time_ms(lambda i: B.slim_quant_search(wcopies[i % len(wcopies)]), 45)
    qb = 2 * 4 * shape.n * shape.k
    legs.append({"shape": shape.name, "entry": "slim_quant_search", "us": round(ms_qs * 1e3, 2),
                 "GBps": round(qb / ms_qs * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(qb / ms_qs * 1e-6 / HBM, 4)})
    for i in range(5):
        B.slim_quant_search_rows(wcopies[i % len(wcopies)])
    ms_qr = event_time_ms(lambda i: B.slim_quant_search_rows(wcopies[i % len(wcopies)]), 45)
    legs.append({"shape": shape.name, "entry": "slim_quant_search_rows", "us": round(ms_qr * 1e3, 2),
                 "GBps": round(qb / 2 / ms_qr * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(qb / 2 / ms_qr * 1e-6 / HBM, 4)})
    sal = torch.rand(shape.k, device=dev) + 0.5
    sc_in, _ = B.slim_quant_search(rot.W_dev)
    for i in range(5):
        B.slim_pack_ex(wcopies[i % len(wcopies)], sal, sc_in)
    ms_px = event_time_ms(lambda i: B.slim_pack_ex(wcopies[i % len(wcopies)], sal, sc_in), 45)
    legs.append({"shape": shape.name, "entry": "slim_pack_ex", "us": round(ms_px * 1e3, 2),
                 "GBps": round(pb / ms_px * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(pb / ms_px * 1e-6 / HBM, 4)})
    # slim_compute_adapters: the adapters of this layer from its dense weights (16 rounds of the subspace
    # iteration); rate on the products with the error saliency alone, 2 (2 q + 2) n k rank_pad FLOPs
    xt = torch.rand(shape.k, device=dev) + 0.1
    B.slim_compute_adapters(rot.W_dev, q, me, sc, shape.r, xt)
    torch.cuda.synchronize()
    ms_ca = event_time_ms(lambda i: B.slim_compute_adapters(rot.W_dev, q, me, sc, shape.r, xt), 3)
    ca_flops = 2.0 * (2 * 16 + 2) * shape.n * shape.k * B.slim_rank_pad(shape.r)
    legs.append({"shape": shape.name, "entry": "slim_compute_adapters", "us": round(ms_ca * 1e3, 1),
                 "TFLOPs": round(ca_flops / ms_ca * 1e-9, 2), "bound": "mfma", "dtype": "f32",
                 "roofline_frac": round(ca_flops / ms_ca * 1e-9 / 157.3, 4)})
    del wcopies
    # slim_pack_adapters_q4: the layer's fp16 adapters to 4-bit group-128 codes + fp16 scales (Sec. 3.3)
    Ld, Rd = rot.L_host.to(dev), rot.R_host.to(dev)
    q4_out = B.slim_pack_adapters_q4(Ld, Rd)
    for _ in range(3):
        B.slim_pack_adapters_q4(Ld, Rd, out=q4_out)
    ms_q4 = event_time_ms(lambda i: B.slim_pack_adapters_q4(Ld, Rd, out=q4_out), 30)
    q4b = shape.r * (shape.n + shape.k) * (2 + 0.5) + 2 * (shape.n * ((shape.r + 127) // 128) + shape.r * (shape.k // 128))
    legs.append({"shape": shape.name, "entry": "slim_pack_adapters_q4", "us": round(ms_q4 * 1e3, 2),
                 "GBps": round(q4b / ms_q4 * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(q4b / ms_q4 * 1e-6 / HBM, 4), "note": "cache-resident inputs"})
    # slim_lowrank alone: Y = (X R^T) L^T on this layer's adapters, decode and prefill shaped
    for m_lr, iters in ((16, 100), (2048, 20)):
        Xl = wl.make_activations(m_lr, shape.k, seed=3).to(dev)
        Yl = torch.empty(m_lr, shape.n, dtype=torch.float16, device=dev)
        wsl = B.alloc_workspace(rot.base, m_lr)
        call = lambda i: B.slim_lowrank(Xl, rot.base.R, rot.base.L, shape.n, shape.r, Yl, False, wsl)
        for i in range(5):
            call(i)
        ms_lr = event_time_ms(call, iters)
        lr_bytes = 2 * shape.r * (shape.n + shape.k) + 2 * m_lr * (shape.n + shape.k)
        lr_flops = 2.0 * m_lr * shape.r * (shape.n + shape.k)
        rec = {"shape": shape.name, "entry": "slim_lowrank", "tokens": m_lr, "us": round(ms_lr * 1e3, 2),
               "GBps": round(lr_bytes / ms_lr * 1e-6, 1), "TFLOPs": round(lr_flops / ms_lr * 1e-9, 2),
               "note": "cache-resident adapters"}
        if m_lr <= 16:
            rec.update({"bound": "hbm", "roofline_frac": round(lr_bytes / ms_lr * 1e-6 / HBM, 4)})
        else:
            rec.update({"bound": "mfma", "roofline_frac": round(lr_flops / ms_lr * 1e-9 / MFMA_PEAK_TFLOPS, 4)})
        legs.append(rec)
        del Xl, Yl, wsl
    # slim_input_quant_fp8 on a prefill-sized input (2048 tokens): reads X twice, writes it once
    Xf = [wl.make_activations(2048, shape.k, seed=30 + c).to(dev) for c in range(4)]
    Xq8, info8 = B.slim_input_quant_fp8(Xf[0])
    ws8 = torch.empty(1024, dtype=torch.uint8, device=dev)
    for i in range(4):
        B.slim_input_quant_fp8(Xf[i % 4], Xq8, info8, ws8)
    ms_f8 = event_time_ms(lambda i: B.slim_input_quant_fp8(Xf[i % 4], Xq8, info8, ws8), 40)
    f8b = 3 * 2 * 2048 * shape.k
    legs.append({"shape": f"X 2048 x {shape.k}", "entry": "slim_input_quant_fp8", "us": round(ms_f8 * 1e3, 2),
                 "GBps": round(f8b / ms_f8 * 1e-6, 1), "bound": "hbm",
                 "roofline_frac": round(f8b / ms_f8 * 1e-6 / HBM, 4), "note": "cache-resident inputs"})
    return legs


if __name__ == "__main__":
    sys.exit(main())
