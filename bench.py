#!/usr/bin/env python3
"""Benchmark of the W4A8 (dINT4 x INT8) linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-sides] [--no-cpu] [--no-graph]

Headline (the configuration the metric's prefill half is quoted on, and the largest one): the
OPT-66B-shaped layer C5, M=4096 K=9216 N=36864, per-channel dINT4, end to end.  A step is one pass of
the online hot path -- quantize_act_int8 then w4a8_gemm, back to back on one stream -- over the
seeded C5 inputs of synthetic_inputs.make_layer (resident in HBM before the timed region).  The
offline rows (weight quantization and packing) run once before it, as in the method, and are timed
separately.  `value` = 2 M N K / step time.  The step is timed as W warm-up steps, then repeats of
EXACTLY K steps between synchronizations (at least five, and more than 0.2 s of GPU time in all);
`ms_per_step` is the median repeat.  The roofline object is for the dominant kernel, the MFMA tile
kernel, from HIP events recorded around every w4a8_gemm call of those same timed steps.

Second object (`decode`): the memory-bound half of the metric on the LLaMA-13B up-projection at 16
tokens (M=16 K=5120 N=13824 group-128; one step = one w4a8_linear call = one launch), weights streamed
from a ring of distinct quantized copies larger than the 256 MB Infinity Cache, with its own HBM roofline.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
METRIC = "W4A8 GEMM TOPS (prefill) + weight GB/s (decode), % of MI355X roofline"
# HBM-side bytes per launch of the two roofline kernels from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script on the kernels as they are (--pmc-calibration scales the counters by 256 MiB copies):
# profiles/gemm_kernel_C5_and_gemv_kernel_C4_hbm_traffic.md.  C5 tile kernel: 1,360,788,070 read (re-reads of
# the activations per group of channel tiles, served by the last-level cache) + 301,989,888 written.
TRAFFIC_BYTES = {"gemm_kernel_C5": 1662722048, "gemv_kernel_C4": 39479296}


def decode_bytes(M, N, K, G):
    """Algorithmic HBM bytes of one decode GEMM launch: packed weights, group parameters
    (fp32 step + u8 zero), int8 activations, token scales, fp16 output."""
    return N * K // 2 + N * (K // G) * 5 + M * K + 4 * M + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-graph", action="store_true", help="decode object: launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-sides", "--no-prefill", dest="no_sides", action="store_true",
                    help="skip the side measurements (other shapes, quantizers, ceilings, next rows)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline and the parity verdicts")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode object")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run of this command can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be >= 1 and --warmup >= 0", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2311_05161_amd as w
    import synthetic_inputs as syn

    lib = w.load_library()  # fails loudly if the HIP library is missing: no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    st = ctypes.c_void_p(stream.cuda_stream)
    P = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    ev = lambda: torch.cuda.Event(enable_timing=True)
    e0, e1 = ev(), ev()

    def offline(Wd, sd, G):
        codes, step, zero = w.quantize_weight_dint4(Wd, sd, G)
        return w.pack_dint4(codes, w.LAYOUT_TILED), step, zero

    # ================================================================== headline: C5 end to end
    cfg = syn.CONFIGS["C5"]
    M, K, N, G = cfg["M"], cfg["K"], cfg["N"], cfg["group_size"]
    X, W, s, _ = syn.make_layer("C5")
    Xd, sd = torch.from_numpy(X).to(dev), torch.from_numpy(s).to(dev)
    Wd = torch.from_numpy(W).to(dev)
    offline(Wd, sd, G)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    Wp, step, zero = offline(Wd, sd, G)
    torch.cuda.synchronize()
    offline_ms = (time.perf_counter() - t0) * 1e3
    del Wd
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev)
    sx = torch.empty((M,), dtype=torch.float32, device=dev)
    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
    ws_bytes = w.gemm_workspace_bytes(M, N, K, G)
    ws = torch.empty((max(1, ws_bytes),), dtype=torch.uint8, device=dev)
    aq_args = (P(Xd), w.F16, M, K, K, P(sd), P(Xq), P(sx), st)
    gm_args = (P(Xq), P(sx), M, P(Wp), w.LAYOUT_TILED, P(step), P(zero), N, K, G, P(Y), w.F16, N,
               None, P(ws), ws_bytes, st)

    def step_fn():
        rc = lib.quantize_act_int8(*aq_args)
        rc |= lib.w4a8_gemm(*gm_args)
        if rc:
            raise RuntimeError(f"kernel launch failed: status {rc}")

    steps, warmup = args.steps, args.warmup
    for _ in range(warmup):
        step_fn()
    torch.cuda.synchronize()
    # one probe step sizes the number of repeats: at least five, and more than 0.2 s of GPU time in all
    t0 = time.perf_counter()
    step_fn()
    torch.cuda.synchronize()
    probe_s = time.perf_counter() - t0
    repeats = max(5, math.ceil(0.25 / max(1e-6, probe_s * steps)))
    repeats = min(repeats, 400)
    rep_s, gemm_ms, aq_ms = [], [], []
    evs = [(ev(), ev(), ev()) for _ in range(steps)]
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):          # EXACTLY `steps` steps between the two synchronizations
            ea, eb, ec = evs[i]
            ea.record(stream)
            rc = lib.quantize_act_int8(*aq_args)
            eb.record(stream)
            rc |= lib.w4a8_gemm(*gm_args)
            ec.record(stream)
            if rc:
                raise RuntimeError(f"kernel launch failed: status {rc}")
        torch.cuda.synchronize()
        rep_s.append(time.perf_counter() - t0)
        aq_ms += [ea.elapsed_time(eb) for ea, eb, _ in evs]
        gemm_ms += [eb.elapsed_time(ec) for _, eb, ec in evs]
    elapsed = float(np.median(rep_s))
    ms_per_step = elapsed / steps * 1e3
    ops = 2.0 * M * N * K
    tops = ops / (elapsed / steps) / 1e12
    gemm_avg_ms = float(np.mean(gemm_ms))
    achieved = ops / (gemm_avg_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_kernel<256, 2, 4, per-channel> (w4a8_gemm, M > 16)",
                "achieved": round(achieved, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / INT8_PEAK_TOPS, 4), "traffic": TRAFFIC_BYTES["gemm_kernel_C5"],
                "algorithmic_bytes": M * K + N * K // 2 + 5 * N + 4 * M + 2 * M * N,
                "ops_per_launch": ops, "avg_launch_us": round(gemm_avg_ms * 1e3, 2),
                "median_launch_us": round(float(np.median(gemm_ms)) * 1e3, 2),
                "launches_timed": len(gemm_ms),
                "note": "HIP events around every w4a8_gemm call of the timed steps; the call is the tile kernel "
                        "plus its 3 us row-sum pre-pass (rowsum_kernel), both counted in the duration",
                "act_quant_avg_us": round(float(np.mean(aq_ms)) * 1e3, 2),
                "act_quant_bytes": M * K * 3 + 4 * K + 4 * M,
                "act_quant_frac_of_hbm_peak": round((M * K * 3 + 4 * K + 4 * M) / (float(np.mean(aq_ms)) * 1e-3)
                                                    / 1e9 / HBM_PEAK_GBS, 4)}
    timing = {"repeats": repeats, "steps_per_repeat": steps, "median_s": round(elapsed, 6),
              "min_s": round(min(rep_s), 6), "max_s": round(max(rep_s), 6),
              "gpu_time_timed_s": round(sum(rep_s), 4)}

    if args.pmc_calibration:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- parity of this very launch configuration and the CPU baseline: the oracle on a bounded sample
    cpu_baseline, parity = None, {}
    if not args.no_cpu:
        import oracle
        oracle.build()
        rng = np.random.default_rng(5)
        rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, size=30)]))[:32]
        cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, size=30)]))[:32]
        mi, ni = rng.integers(0, M, size=4096), rng.integers(0, N, size=4096)
        oracle.quantize_act_int8(X[:2], s)   # load + warm
        codes_d = w.unpack_dint4(Wp, N, K, w.LAYOUT_TILED)
        t0 = time.perf_counter()
        Xq_h, sx_h = oracle.quantize_act_int8(X, s)                            # full size
        t_aq = time.perf_counter() - t0
        # weights of the sampled output columns and of the full rows: quantized by the oracle itself
        t0 = time.perf_counter()
        codes_h, step_h, zero_h = oracle.quantize_weight_dint4(W, s, G)        # full size (offline row)
        t_wq = time.perf_counter() - t0
        packed_h = oracle.pack_dint4(codes_h)
        t0 = time.perf_counter()
        acc_rows = oracle.int_gemm(Xq_h[rows], packed_h, zero_h, G)            # 32 full output rows
        acc_cols = oracle.int_gemm(Xq_h, packed_h[cols], zero_h[cols], G)      # 32 full output columns
        acc_pts = oracle.int_gemm_sampled(Xq_h, packed_h, zero_h, G, mi, ni)   # 4096 single outputs
        t_gemm = time.perf_counter() - t0
        macs = (rows.size * N + M * cols.size + mi.size) * K
        full_s = t_aq + (M * N * K) / (macs / t_gemm)
        cpu_baseline = {"value": round(2.0 * M * N * K / full_s / 1e12, 6), "unit": "TOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"act-quant of all {M} tokens ({t_aq:.2f} s) + plain-loop int GEMM of {rows.size} full "
                                  f"output rows, {cols.size} full output columns and {mi.size} single outputs "
                                  f"({macs / 1e9:.1f} GMAC in {t_gemm:.1f} s = {macs / t_gemm / 1e9:.2f} GMAC/s); value = "
                                  f"2MNK over the whole step's time EXTRAPOLATED from that rate ({full_s:.0f} s); "
                                  f"offline weight quantization {t_wq:.1f} s not included"}
        # parity verdicts on the timed configuration's own outputs
        step_fn()
        torch.cuda.synchronize()
        hs = 0.5 * step_h.astype(np.float64)[:, 0]
        rt, ct = torch.from_numpy(rows).to(dev), torch.from_numpy(cols).to(dev)
        rms = (Y.float().square().mean(1).sqrt()).cpu().numpy().astype(np.float64)

        def y_ok(y_gpu, acc, r_idx, c_idx):
            y64 = sx_h.astype(np.float64)[r_idx][:, None] * hs[c_idx][None, :] * acc[:, :, 0].astype(np.float64)
            return bool(np.all(np.abs(y_gpu - y64) <= 1e-3 * np.maximum(np.abs(y64), 1e-3 * rms[r_idx][:, None])))
        yr = Y.index_select(0, rt).float().cpu().numpy().astype(np.float64)
        yc = Y.index_select(1, ct).float().cpu().numpy().astype(np.float64)
        yp = Y[torch.from_numpy(mi).to(dev), torch.from_numpy(ni).to(dev)].float().cpu().numpy().astype(np.float64)
        y64p = sx_h.astype(np.float64)[mi] * hs[ni] * acc_pts[:, 0].astype(np.float64)
        parity["C5"] = {
            "Xq_sx_bit_exact": bool(np.array_equal(Xq.cpu().numpy(), Xq_h) and np.array_equal(sx.cpu().numpy(), sx_h)),
            "codes_step_zero_bit_exact": bool(np.array_equal(codes_d.cpu().numpy(), codes_h)
                                              and np.array_equal(step.cpu().numpy(), step_h)
                                              and np.array_equal(zero.cpu().numpy(), zero_h)),
            "Y_within_1e-3": bool(y_ok(yr, acc_rows, rows, np.arange(N)) and y_ok(yc, acc_cols, np.arange(M), cols)
                                  and np.all(np.abs(yp - y64p) <= 1e-3 * np.maximum(np.abs(y64p), 1e-3 * rms[mi]))),
            "checked": f"{rows.size} full rows + {cols.size} full columns + {mi.size} outputs of Y against the oracle's "
                       "accumulators (float64 epilogue); int32 accumulators themselves: tests/test_gpu_parity.py"}
        del codes_d, codes_h, packed_h, acc_rows, acc_cols
    del X, W
    del Xd, Xq, Y, Wp, ws   # (step_fn holds raw pointers only: it is not called again)
    torch.cuda.empty_cache()

    # ================================================================== decode object: C4 up-projection, M = 16
    def time_loop(fn, n, reps=5):
        """Median over `reps` of the HIP-event time of n back-to-back calls, in ms per call."""
        out = []
        for _ in range(reps):
            e0.record(stream)
            for i in range(n):
                fn(i)
            e1.record(stream)
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / n)
        return float(np.median(out)), out

    decode = None
    if not args.no_decode:
        name = "C4_5120x13824"
        Md = 16
        Xh, Wh, sh, Gd = syn.make_layer(name, M=Md)
        Kd, Nd = Xh.shape[1], Wh.shape[0]
        Xdd, Wdd, sdd = torch.from_numpy(Xh).to(dev), torch.from_numpy(Wh).to(dev), torch.from_numpy(sh).to(dev)
        Wp0, step0, zero0 = offline(Wdd, sdd, Gd)
        per_copy = decode_bytes(Md, Nd, Kd, Gd)
        R = max(2, -(-2 * 256 * 2 ** 20 // per_copy))   # ring >= 2 x Infinity Cache
        ring = [(Wp0, step0, zero0)]
        for r in range(1, R):  # distinct buffers; rolled so that no two copies hold the same rows
            sh_r = (r * 16) % Nd
            ring.append((torch.roll(Wp0.view(Nd // 16, -1), r, 0).contiguous().view(-1),
                         torch.roll(step0, sh_r, 0).contiguous(), torch.roll(zero0, sh_r, 0).contiguous()))
        Xqd = torch.empty((Md, Kd), dtype=torch.int8, device=dev)
        sxd = torch.empty((Md,), dtype=torch.float32, device=dev)
        Yd = torch.empty((Md, Nd), dtype=torch.float16, device=dev)
        wsd_bytes = w.gemm_workspace_bytes(Md, Nd, Kd, Gd)
        wsd = torch.empty((max(1, wsd_bytes),), dtype=torch.uint8, device=dev)
        aq_d = (P(Xdd), w.F16, Md, Kd, Kd, P(sdd), P(Xqd), P(sxd), st)
        gm_d = [(P(Xqd), P(sxd), Md, P(wp), w.LAYOUT_TILED, P(sp), P(zp), Nd, Kd, Gd, P(Yd), w.F16, Nd,
                 None, P(wsd), wsd_bytes, st) for (wp, sp, zp) in ring]

        # the step as ONE call: w4a8_linear quantizes the 16 tokens inside the streaming kernel's launch
        lin_ws_bytes = int(lib.w4a8_linear_workspace_bytes(Md, Nd, Kd, Gd, w.LAYOUT_TILED))
        lin_ws = torch.empty((max(1, lin_ws_bytes),), dtype=torch.uint8, device=dev)
        lin_d = [(P(Xdd), w.F16, Md, Kd, Kd, P(sdd), P(wp), w.LAYOUT_TILED, P(sp), P(zp), Nd, Gd, P(Yd), w.F16, Nd,
                  None, None, None, P(lin_ws), lin_ws_bytes, st) for (wp, sp, zp) in ring]

        def dstep(i):
            rc = lib.w4a8_linear(*lin_d[i % R])
            if rc:
                raise RuntimeError(f"kernel launch failed: status {rc}")

        def dstep_two_calls(i):
            rc = lib.quantize_act_int8(*aq_d) | lib.w4a8_gemm(*gm_d[i % R])
            if rc:
                raise RuntimeError(f"kernel launch failed: status {rc}")

        dstep_two_calls(0)
        torch.cuda.synchronize()
        y_two = Yd.clone()
        Yd.zero_()
        dstep(0)
        torch.cuda.synchronize()
        assert torch.equal(Yd, y_two), "the one-launch step differs from quantize_act_int8 + w4a8_gemm"
        if not args.no_cpu:
            r_h = oracle.linear_w4a8(Xh, Wh, sh, Gd)
            y_gpu = Yd.float().cpu().numpy().astype(np.float64)
            y64 = r_h["Y64"]
            floor = 1e-3 * np.sqrt(np.mean(y64 ** 2, axis=1, keepdims=True))
            parity["C4_5120x13824_M16"] = {
                "Xq_sx_bit_exact": bool(np.array_equal(Xqd.cpu().numpy(), r_h["Xq"])
                                        and np.array_equal(sxd.cpu().numpy(), r_h["sx"])),
                "codes_step_zero_bit_exact": bool(
                    np.array_equal(w.unpack_dint4(Wp0, Nd, Kd, w.LAYOUT_TILED).cpu().numpy(), r_h["codes"])
                    and np.array_equal(step0.cpu().numpy(), r_h["step"]) and np.array_equal(zero0.cpu().numpy(), r_h["zero"])),
                "Y_within_1e-3": bool(np.all(np.abs(y_gpu - y64) <= 1e-3 * np.maximum(np.abs(y64), floor))),
                "checked": "the whole Y against the oracle's plain-loop layer (float64 epilogue)"}
        del Wdd
        # a step = act-quant + GEMM; launched as a HIP graph of one trip round the ring (launch-bound
        # inner loop), checked against the eager result; timed as repeats of whole trips
        use_graph = not args.no_graph
        n_trip = max(1, round(2048 / R))
        graph = None
        if use_graph:
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                st_side = ctypes.c_void_p(side.cuda_stream)
                lin_g = [a[:-1] + (st_side,) for a in lin_d]
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    for i in range(R):
                        rc = lib.w4a8_linear(*lin_g[i])
                        assert rc == 0
            stream.wait_stream(side)
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            y_graph = Yd.clone()
            dstep(R - 1)
            torch.cuda.synchronize()
            assert torch.equal(Yd, y_graph), "graph replay differs from eager launch"
        reps_s = []
        for _ in range(7):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if use_graph:
                for _ in range(n_trip):
                    graph.replay()
            else:
                for i in range(n_trip * R):
                    dstep(i)
            torch.cuda.synchronize()
            reps_s.append((time.perf_counter() - t0) / (n_trip * R))
        d_step_s = float(np.median(reps_s))
        two_ms, _ = time_loop(dstep_two_calls, 1024, reps=3)   # context: the same step as two launches (eager)
        # its roofline: the GEMV alone, HIP events on the launch stream around back-to-back launches over the ring
        for i in range(64):
            lib.w4a8_gemm(*gm_d[i % R])
        torch.cuda.synchronize()
        kern_ms, kern_all = time_loop(lambda i: lib.w4a8_gemm(*gm_d[i % R]), 1024)
        tiny_codes = torch.zeros((16, 128), dtype=torch.uint8, device=dev)
        tiny_out = torch.empty((16 * 64,), dtype=torch.uint8, device=dev)
        tiny_args = (P(tiny_codes), 16, 128, P(tiny_out), w.LAYOUT_TILED, st)
        floor_ms, _ = time_loop(lambda i: lib.pack_dint4(*tiny_args), 1024, reps=3)
        ach = per_copy / (kern_ms * 1e-3) / 1e9
        cpu_dec = None
        if not args.no_cpu:
            packed_h = oracle.pack_dint4(r_h["codes"])
            t0 = time.perf_counter()
            n_cpu = 0
            while True:   # bounded sample: whole steps until about 5 s of CPU work
                Xq_h, sx_h = oracle.quantize_act_int8(Xh, sh)
                acc_h = oracle.int_gemm(Xq_h, packed_h, r_h["zero"], Gd)
                oracle.dequant_epilogue(acc_h, sx_h, r_h["step"])
                n_cpu += 1
                cpu_s = time.perf_counter() - t0
                if cpu_s >= 5.0 or n_cpu >= 500:
                    break
            cpu_dec = {"value": round(Nd * Kd / 2 * n_cpu / cpu_s / 1e9, 4), "unit": "GB/s",
                       "cores": oracle.num_threads(), "kind": "oracle",
                       "sample": f"{n_cpu} whole steps (act-quant + int GEMM + dequant) in {cpu_s:.1f} s"}
        decode = {
            "workload": f"C4 LLaMA-13B up-projection decode: M={Md} K={Kd} N={Nd} group-{Gd} dINT4; step = "
                        f"w4a8_linear (activation quantization + GEMM in one launch, bit-identical to "
                        f"quantize_act_int8 + w4a8_gemm); ring of {R} weight copies ({R * per_copy / 2 ** 20:.0f} MiB)",
            "launch": "hip-graph" if use_graph else "eager",
            "value": round(Nd * Kd / 2 / d_step_s / 1e9, 1), "unit": "GB/s (packed weight bytes per step time)",
            "us_per_step": round(d_step_s * 1e6, 3), "steps_timed": 7 * n_trip * R,
            "us_per_step_min_max": [round(min(reps_s) * 1e6, 3), round(max(reps_s) * 1e6, 3)],
            "us_per_step_as_two_launches": round(two_ms * 1e3, 3),
            "roofline": {"bound": "hbm", "kernel": "gemv_kernel (w4a8_gemm, M <= 16: the GEMM alone, int8 activations given)",
                         "achieved": round(ach, 1),
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                         "traffic": TRAFFIC_BYTES["gemv_kernel_C4"], "bytes_per_launch": per_copy,
                         "avg_launch_us": round(kern_ms * 1e3, 3),
                         "launch_us_min_max": [round(min(kern_all) * 1e3, 3), round(max(kern_all) * 1e3, 3)],
                         "launch_floor_us": round(floor_ms * 1e3, 3)},
            "cpu_baseline": cpu_dec}
        del ring, gm_d, Wp0

    # ================================================================== side measurements
    sides = {}
    if not args.no_sides:
        sides = side_measurements(torch, w, lib, syn, dev, stream, st, P, e0, e1)

    out = {
        "metric": METRIC, "value": round(tops, 1), "unit": "TOP/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"C5 OPT-66B-shaped layer end to end: M={M} K={K} N={N} per-channel dINT4; step = "
                               f"quantize_act_int8 + w4a8_gemm on one stream; inputs: synthetic_inputs.make_layer('C5')",
                   "launch": "eager"},
        "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4),
        "timing": timing,
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity or None,
        "offline": {"what": "quantize_weight_dint4 + pack_dint4 (tiled) of the C5 weights, once per weight matrix",
                    "ms": round(offline_ms, 3),
                    "GBps": round((N * K * 2 + N * K + N * K + N * K // 2) / (offline_ms * 1e-3) / 1e9, 1)},
        "decode": decode,
    }
    out.update(sides)
    print(json.dumps(out), flush=True)


def side_measurements(torch, w, lib, syn, dev, stream, st, P, e0, e1):
    """Everything that is not the headline or the decode object: other shapes of the configurations,
    the quantizer kernels, the measured ceilings of the box, and the rows built beyond the scope table's
    first part (asymmetric activations, Value cache, scale search, formats)."""

    def draw_layer(fam, Mq, Kq, Nq, Gq, g):
        """Quantized operands of a layer drawn on the GPU by the recipe of synthetic_inputs.make_layer
        (same distributions and outlier structure, not the same bits), through the library's own
        quantizers.  The compute-bound timings need this: what the int8 operands look like decides
        the power the matrix cores draw and with it the clock (all-zero activations: 2.38 GHz,
        uniformly random int8: 1.78 GHz on the same launch)."""
        X = torch.randn((Mq, Kq), device=dev, generator=g)
        n_out = max(1, round(0.01 * Kq)) if fam == "C5" else max(1, math.ceil(0.005 * Kq))
        ch = torch.randperm(Kq, device=dev, generator=g)[:n_out]
        if fam == "C4":   # heavy-tailed outlier channels: 50 x Student-t(3)
            z = torch.randn((Mq, n_out), device=dev, generator=g)
            chi = torch.randn((3, Mq, n_out), device=dev, generator=g).square().sum(0) / 3.0
            X[:, ch] = 50.0 * z / chi.sqrt()
        else:
            X[:, ch] *= 100.0 if fam == "C5" else 50.0
        X = X.clamp_(-65504.0, 65504.0).to(torch.float16)
        s = torch.rand((Kq,), device=dev, generator=g) * 1.5 + 0.5
        xq_, sx_ = w.quantize_act_int8(X, s)
        gw = torch.Generator(device=dev)
        gw.manual_seed(g.initial_seed() + 1)
        rows = max(16, (1 << 26) // Kq // 16 * 16)   # weights in slabs of about 64 Mi elements
        codes = torch.empty((Nq, Kq), dtype=torch.uint8, device=dev)
        st_, z_ = [], []
        for r0 in range(0, Nq, rows):
            Wb = (torch.randn((min(rows, Nq - r0), Kq), device=dev, generator=gw) * 0.02).to(torch.float16)
            c_, s_b, z_b = w.quantize_weight_dint4(Wb, s, Gq)
            codes[r0:r0 + Wb.shape[0]] = c_
            st_.append(s_b)
            z_.append(z_b)
        wp_ = w.pack_dint4(codes, w.LAYOUT_TILED)
        return xq_, sx_, wp_, torch.cat(st_).contiguous(), torch.cat(z_).contiguous()

    def time_gemm(Mq, Nq, Kq, Gq, reps, ring_bytes=600 << 20, asym=False, fam=None):
        """Back-to-back w4a8_gemm (or w4a8_gemm_asym) launches (timing only).  fam = None: a ring of
        random packed weights and random int8 activations (the memory-bound side: values do not
        matter there); fam = "C3" / "C4": one set of operands quantized from that configuration's
        distributions.  Median of three timed loops."""
        g = torch.Generator(device=dev)
        g.manual_seed(20231105)
        Gs = Kq if Gq == 0 else Gq
        per = decode_bytes(Mq, Nq, Kq, Gs)
        nring = max(2, min(32, ring_bytes // per + 1))
        if fam is not None:
            xq, sxq, wp0, stq, zq = draw_layer(fam, Mq, Kq, Nq, Gq, g)
            wps, nring = [wp0], 1
        else:
            wps = [torch.randint(0, 256, (Nq * Kq // 2,), dtype=torch.uint8, device=dev, generator=g)
                   for _ in range(nring)]
            stq = torch.rand((Nq, Kq // Gs), device=dev, generator=g) * 0.01 + 0.001
            zq = torch.randint(0, 14, (Nq, Kq // Gs), dtype=torch.uint8, device=dev, generator=g)
            xq = torch.randint(-127, 128, (Mq, Kq), dtype=torch.int8, device=dev, generator=g)
            sxq = torch.rand((Mq,), device=dev, generator=g) * 0.01 + 0.001
        yq = torch.empty((Mq, Nq), dtype=torch.float16, device=dev)
        wsb = w.gemm_workspace_bytes(Mq, Nq, Kq, Gq)
        wsq = torch.empty((max(1, wsb),), dtype=torch.uint8, device=dev)
        fn = lib.w4a8_gemm
        argsq = [(P(xq), P(sxq), Mq, P(wp), w.LAYOUT_TILED, P(stq), P(zq), Nq, Kq, Gq, P(yq), w.F16, Nq,
                  None, P(wsq), wsb, st) for wp in wps]
        if asym:
            fn = lib.w4a8_gemm_asym
            zxq = torch.randint(-128, 128, (Mq,), dtype=torch.int32, device=dev, generator=g)
            wsq_ = torch.randint(-3000, 3000, (Nq, Kq // Gs), dtype=torch.int32, device=dev, generator=g)
            tsq_ = torch.randint(-3000, 3000, (Nq, Kq // 128), dtype=torch.int32, device=dev, generator=g)
            argsq = [(P(xq), P(sxq), P(zxq), Mq, P(wp), w.LAYOUT_TILED, P(stq), P(zq), P(wsq_), P(tsq_),
                      Nq, Kq, Gq, P(yq), w.F16, Nq, None, P(wsq), wsb, st) for wp in wps]
        for i in range(max(3, reps // 10)):
            assert fn(*argsq[i % nring]) == 0
        torch.cuda.synchronize()
        runs = []
        for _ in range(3):
            e0.record(stream)
            for i in range(reps):
                fn(*argsq[i % nring])
            e1.record(stream)
            torch.cuda.synchronize()
            runs.append(e0.elapsed_time(e1) / reps)
        return float(np.median(runs)), per

    # ---- measured ceilings of the box in this run (the roofline fractions stay against the nominal peaks)
    big = torch.empty((1 << 30,), dtype=torch.uint8, device=dev)
    big.random_(0, 256)
    sink = torch.zeros((4,), dtype=torch.int32, device=dev)
    reads = {}
    for label, nbytes in (("9_MB", 9_240_640), ("39_MB", 38_600_000 // 16 * 16), ("170_MB", 170_000_000 // 16 * 16)):
        slots = (1 << 30) // nbytes   # consecutive launches walk through the 1 GiB buffer: every launch reads from HBM
        for i in range(8):
            assert lib.w4a8_measure_stream_read(big.data_ptr() + (i % slots) * nbytes, nbytes, P(sink), st) == 0
        torch.cuda.synchronize()
        n_l = max(16, min(256, (4 << 30) // nbytes))
        e0.record(stream)
        for i in range(n_l):
            lib.w4a8_measure_stream_read(big.data_ptr() + (i % slots) * nbytes, nbytes, P(sink), st)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / n_l * 1e3
        reads[label] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1)}
    del big
    ops = ctypes.c_int64(0)
    iters = 20000
    for _ in range(2):
        assert lib.w4a8_measure_mfma_i8(iters, P(sink), ctypes.byref(ops), st) == 0
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(5):
        lib.w4a8_measure_mfma_i8(iters, P(sink), ctypes.byref(ops), st)
    e1.record(stream)
    torch.cuda.synchronize()
    mfma_ms = e0.elapsed_time(e1) / 5
    # the group-wise k-tile's instruction mix (16 MFMAs, 96 + 128 vector instructions per wave), operands in
    # registers / second MFMA operand read from LDS as in the kernel: ns per k-tile of a wave pair
    mix = {}
    mix_iters = 4000
    for label, frags in (("registers_only", 0), ("with_lds_fragment_reads", 1)):
        assert lib.w4a8_measure_ktile_mix(mix_iters, frags, P(sink), st) == 0
        torch.cuda.synchronize()
        e0.record(stream)
        lib.w4a8_measure_ktile_mix(mix_iters, frags, P(sink), st)
        e1.record(stream)
        torch.cuda.synchronize()
        mix[label] = round(e0.elapsed_time(e1) * 1e6 / mix_iters, 1)
    ceilings = {"what": "measured on this box in this run: a plain streaming read of as many bytes as the decode "
                        "shapes move (each launch from HBM), a register-resident v_mfma_i32_32x32x32_i8 loop, and the "
                        "instruction mix of one k-tile of the group-wise tile kernel (two workgroups of four waves per "
                        "CU) with and without its LDS fragment reads",
                "stream_read": reads, "mfma_i8_loop_TOPS": round(ops.value / (mfma_ms * 1e-3) / 1e12, 1),
                "groupwise_ktile_mix_ns": mix}

    # ---- the other decode shapes
    decode_side = []
    for (Mq, Kq, Nq, Gq) in [(16, 4096, 4096, 128), (16, 5120, 5120, 128), (16, 13824, 5120, 128), (16, 9216, 36864, 0)]:
        ms, per = time_gemm(Mq, Nq, Kq, Gq, 400)
        decode_side.append({"workload": f"M={Mq} K={Kq} N={Nq} G={Gq or Kq}", "us": round(ms * 1e3, 3),
                            "GBps": round(per / ms / 1e6, 1),
                            "frac_of_hbm_peak": round(per / ms / 1e6 / HBM_PEAK_GBS, 4)})

    # ---- the other prefill shapes (compute-bound), w4a8_gemm alone
    prefill = []
    for (name, Mp, Kp, Np, Gp) in [("C3_up", 2048, 4096, 11008, 0), ("C3_down", 2048, 11008, 4096, 0),
                                   ("C4", 2048, 5120, 13824, 128), ("C4", 512, 5120, 13824, 128)]:
        ms, _ = time_gemm(Mp, Np, Kp, Gp, 20, ring_bytes=0, fam=name[:2])
        tops = 2.0 * Mp * Np * Kp / (ms * 1e-3) / 1e12
        prefill.append({"workload": f"{name} M={Mp} K={Kp} N={Np} G={Gp or Kp}", "ms": round(ms, 4),
                        "TOPS": round(tops, 1), "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4)})

    # ---- the LLaMA-13B layer sweep: K -> N in {5120 -> 5120, 5120 -> 13824, 13824 -> 5120} x M in
    # {1, 16, 128, 512, 2048}, group-128: time per w4a8_gemm call, against both rooflines
    c4_sweep = []
    for (Kq, Nq) in [(5120, 5120), (5120, 13824), (13824, 5120)]:
        for Mq in (1, 16, 128, 512, 2048):
            ms, per = time_gemm(Mq, Nq, Kq, 128, 200 if Mq <= 128 else 20,
                                ring_bytes=(600 << 20) if Mq <= 16 else 0, fam=None if Mq <= 16 else "C4")
            tops = 2.0 * Mq * Nq * Kq / (ms * 1e-3) / 1e12
            c4_sweep.append({"workload": f"M={Mq} K={Kq} N={Nq} G=128", "us": round(ms * 1e3, 2),
                             "GBps": round(per / ms / 1e6, 1), "TOPS": round(tops, 1),
                             "frac_of_hbm_peak": round(per / ms / 1e6 / HBM_PEAK_GBS, 4),
                             "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4)})

    # ---- 17 .. 128 tokens on the C2 layer: 16-token blocks of the streaming kernel in one launch
    mid_tokens = []
    for Mq in (17, 32, 64, 128):
        ms, per = time_gemm(Mq, 4096, 4096, 128, 300, ring_bytes=0)
        mid_tokens.append({"workload": f"M={Mq} K=4096 N=4096 G=128", "us": round(ms * 1e3, 2),
                           "TOPS": round(2.0 * Mq * 4096 * 4096 / (ms * 1e-3) / 1e12, 1)})

    # ---- weight quantizer and packing (offline) on a C4 up-projection matrix
    g = torch.Generator(device=dev)
    g.manual_seed(20231107)
    Nw, Kw = 13824, 5120
    Wb = (torch.randn((Nw, Kw), device=dev, generator=g) * 0.02).to(torch.float16)
    sw = torch.rand((Kw,), device=dev, generator=g) * 1.5 + 0.5
    for _ in range(2):
        cb, _, _ = w.quantize_weight_dint4(Wb, sw, 128)
        w.pack_dint4(cb, w.LAYOUT_TILED)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(10):
        cb, _, _ = w.quantize_weight_dint4(Wb, sw, 128)
    e1.record(stream)
    torch.cuda.synchronize()
    wq_ms = e0.elapsed_time(e1) / 10
    e0.record(stream)
    for _ in range(10):
        w.pack_dint4(cb, w.LAYOUT_TILED)
    e1.record(stream)
    torch.cuda.synchronize()
    pk_ms = e0.elapsed_time(e1) / 10
    wq_bytes = Nw * Kw * 3 + 5 * Nw * Kw // 128 + 4 * Kw
    quant_side = {"what": "the offline quantizer kernels against the HBM roofline (bytes: input read + output written)",
                  "weight_quant_C4": {"workload": f"N={Nw} K={Kw} fp16 G=128", "ms": round(wq_ms, 4),
                                      "GBps": round(wq_bytes / wq_ms / 1e6, 1),
                                      "frac_of_hbm_peak": round(wq_bytes / wq_ms / 1e6 / HBM_PEAK_GBS, 4)},
                  "pack_tiled_C4": {"ms": round(pk_ms, 4), "GBps": round(Nw * Kw * 1.5 / pk_ms / 1e6, 1)}}
    del Wb, cb

    # ---- asymmetric activations
    asym_side = []
    for (name, Ma, Ka, Na, Ga, reps) in [("C2 decode", 16, 4096, 4096, 128, 400),
                                         ("C4 decode", 16, 5120, 13824, 128, 400),
                                         ("C3_up prefill", 2048, 4096, 11008, 0, 20),
                                         ("C4 prefill", 2048, 5120, 13824, 128, 20)]:
        ms, per = time_gemm(Ma, Na, Ka, Ga, reps, ring_bytes=(600 << 20) if Ma <= 16 else 0, asym=True)
        row = {"workload": f"{name} M={Ma} K={Ka} N={Na} G={Ga or Ka}", "us": round(ms * 1e3, 3)}
        if Ma <= 16:
            row["GBps"] = round(per / ms / 1e6, 1)
        else:
            row["TOPS"] = round(2.0 * Ma * Na * Ka / (ms * 1e-3) / 1e12, 1)
        asym_side.append(row)

    # ---- 4-bit Value cache: decode attention of 16 sequences x 32 heads (LLaMA-7B): one query token per head
    # against 4096 cached tokens of 128 channels, channel-wise dINT4 Value, 8-bit probabilities
    Bv, Mv, Tv, Dv = 512, 1, 4096, 128
    g = torch.Generator(device=dev)
    g.manual_seed(20231106)
    Vv = torch.randn((Bv, Tv, Dv), device=dev, generator=g).to(torch.float16)
    Pv = torch.softmax(torch.randn((Bv * Mv, Tv), device=dev, generator=g) * 2.0, dim=1)
    for _ in range(2):
        codes_v, step_v, zero_v = w.quantize_value_dint4(Vv, 0)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(5):
        w.quantize_value_dint4(Vv, 0)
    e1.record(stream)
    torch.cuda.synchronize()
    vq_ms = e0.elapsed_time(e1) / 5
    nring_v = 5
    wps_v = [w.pack_dint4(codes_v, w.LAYOUT_TILED)] + [
        torch.randint(0, 256, (Bv * Dv * Tv // 2,), dtype=torch.uint8, device=dev, generator=g)
        for _ in range(nring_v - 1)]
    del codes_v
    xq_v, sx_v = w.quantize_act_int8(Pv, None)
    y_v = torch.empty((Bv * Mv, Dv), dtype=torch.float16, device=dev)
    args_v = [(P(xq_v), P(sx_v), None, Mv, P(wp), P(step_v), P(zero_v), None, None, Dv, Tv, 0, P(y_v),
               w.F16, Dv, Bv, st) for wp in wps_v]
    for i in range(nring_v):
        assert lib.w4a8_gemm_batched(*args_v[i]) == 0
    torch.cuda.synchronize()
    reps_v = 100
    e0.record(stream)
    for i in range(reps_v):
        lib.w4a8_gemm_batched(*args_v[i % nring_v])
    e1.record(stream)
    torch.cuda.synchronize()
    av_ms = e0.elapsed_time(e1) / reps_v
    per_v = Bv * decode_bytes(Mv, Dv, Tv, Tv)
    value_side = {"what": "quantize_value_dint4 (channel-wise dINT4 of V along the tokens) and "
                          "w4a8_gemm_batched (8-bit probabilities x 4-bit Value, one launch for all heads)",
                  "workload": f"heads={Bv} query_tokens={Mv} cached_tokens={Tv} channels={Dv}",
                  "attn_value_us": round(av_ms * 1e3, 2), "attn_value_GBps": round(per_v / av_ms / 1e6, 1),
                  "attn_value_frac_of_hbm_peak": round(per_v / av_ms / 1e6 / HBM_PEAK_GBS, 4),
                  "quantize_value_ms": round(vq_ms, 4),
                  "quantize_value_GBps": round(Bv * Tv * Dv * 3 / vq_ms / 1e6, 1)}
    del Vv, Pv, wps_v

    # ---- AQAS scale search (offline) on the C2 layer, and the error split of Eq. 4
    Ms = 512   # calibration tokens
    _, Wc, _, Gc = syn.make_layer("C2")
    Xc, _, _, _ = syn.make_layer("C2", M=Ms, variant=1)
    Xc_d, Wc_d = torch.from_numpy(Xc).to(dev), torch.from_numpy(Wc).to(dev)
    w.aqas_search(Xc_d, Wc_d, Gc)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    s_best, j_best, losses_s = w.aqas_search(Xc_d, Wc_d, Gc)
    torch.cuda.synchronize()
    search_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    clip_idx, _, _ = w.aqas_clip_search(Xc_d, Wc_d, s_best, Gc)
    torch.cuda.synchronize()
    clip_ms = (time.perf_counter() - t0) * 1e3
    ls = losses_s.cpu().numpy()
    search_side = {"what": "aqas_search (17 grid points, each a full pass of the quantized layer on the GPU) and "
                           "aqas_clip_search (11 range factors per output channel) on the C2 layer",
                   "workload": f"calibration_tokens={Ms} K=4096 N=4096 G={Gc}",
                   "search_ms": round(search_ms, 3), "clip_ms": round(clip_ms, 3),
                   "best_alpha": int(j_best.item()) / 16.0,
                   "loss_at_best_over_loss_at_alpha_0_and_1": [round(float(ls.min() / ls[0]), 4),
                                                               round(float(ls.min() / ls[16]), 4)],
                   "channels_clipped": int((clip_idx > 0).sum().item())}
    terms = {}
    for fname, fid in (("int4", w.FMT_INT4), ("dint4", w.FMT_DINT4), ("dint3", w.FMT_DINT3),
                       ("dint4_special_step_over_4", w.FMT_DINT4_C4),
                       ("dint4_special_step_over_8", w.FMT_DINT4_C8)):
        tt = w.dint_error_terms(Xc_d, Wc_d, s_best, Gc, fid).cpu().numpy()
        terms[fname] = {"underflow": float(f"{tt[0]:.5g}"), "rounding": float(f"{tt[1]:.5g}"),
                        "cross": float(f"{tt[2]:.5g}"), "underflowing_weights": int(tt[3])}
    search_side["output_error_split"] = terms

    return {"decode_other_shapes": decode_side, "prefill_other_shapes": prefill, "c4_layer_sweep": c4_sweep,
            "c2_17_to_128_tokens": mid_tokens,
            "asymmetric_activations": {"what": "w4a8_gemm_asym (token zero-point taken out of the int32 "
                                               "accumulators), same shapes and protocol as the lists above",
                                       "shapes": asym_side},
            "quantizers": quant_side, "value_cache": value_side, "aqas_search": search_side,
            "ceilings": ceilings}


if __name__ == "__main__":
    main()
