#!/usr/bin/env python3
"""Benchmark of the W4A8 (dINT4 x INT8) linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-graph] [--no-prefill] [--no-cpu]

A step is one pass of the online hot path -- quantize_act_int8 then w4a8_gemm -- over one batch
of the decode workload (LLaMA-7B attention projection, M=16, K=N=4096, group-128 dINT4), with the
weights of each step taken from a ring of distinct quantized copies larger than the 256 MB
Infinity Cache so that they really stream from HBM.  The offline rows (weight quantization and
packing) run once per weight matrix before the timed region, as in the method, and are timed
separately ("offline").  Prints ONE JSON line.
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
# HBM bytes per gemv_kernel launch on this workload from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, scaled by a 256 MiB copy (profiles/gemv_kernel_C2_decode_hbm_traffic.md): 9,689,088 read + 131,072 written
GEMV_C2_TRAFFIC_BYTES = 9820160
METRIC = "W4A8 GEMM TOPS (prefill) + weight GB/s (decode), % of MI355X roofline"


def decode_bytes(M, N, K, G):
    """Algorithmic HBM bytes of one decode GEMM launch: packed weights, group parameters
    (fp32 step + u8 zero), int8 activations, token scales, fp16 output."""
    return N * K // 2 + N * (K // G) * 5 + M * K + 4 * M + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill (compute-bound) side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run of this command can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
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

    # ------------------------------------------------------------------ workload: C2, M = 16
    cfg = syn.CONFIGS["C2"]
    M, K, N, G = cfg["M"], cfg["K"], cfg["N"], cfg["group_size"]
    X, W, s, _ = syn.make_layer("C2")
    Xd, Wd, sd = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev), torch.from_numpy(s).to(dev)

    # offline rows: weight quantization + packing (timed, reported separately)
    def offline():
        codes, step, zero = w.quantize_weight_dint4(Wd, sd, G)
        return w.pack_dint4(codes, w.LAYOUT_TILED), step, zero
    offline()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        Wp, step, zero = offline()
    torch.cuda.synchronize()
    offline_ms = (time.perf_counter() - t0) / 5 * 1e3

    per_copy = decode_bytes(M, N, K, G)
    R = max(2, -(-2 * 256 * 2 ** 20 // per_copy))  # ring >= 2 x Infinity Cache
    ring = []
    for r in range(R):  # distinct buffers; rolled so that no two copies hold the same rows
        sh = (r * 16) % N
        ring.append((torch.roll(Wp.view(N // 16, -1), r, 0).contiguous().view(-1),
                     torch.roll(step, sh, 0).contiguous(), torch.roll(zero, sh, 0).contiguous()))
    ring[0] = (Wp, step, zero)

    Xq = torch.empty((M, K), dtype=torch.int8, device=dev)
    sx = torch.empty((M,), dtype=torch.float32, device=dev)
    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    aq_args = (P(Xd), w.F16, M, K, K, P(sd), P(Xq), P(sx), st)
    gm_args = [(P(Xq), P(sx), M, P(wp), w.LAYOUT_TILED, P(sp), P(zp), N, K, G, P(Y), w.F16, N,
                None, None, 0, st) for (wp, sp, zp) in ring]

    def step_fn(i):
        rc = lib.quantize_act_int8(*aq_args)
        rc |= lib.w4a8_gemm(*gm_args[i % R])
        if rc:
            raise RuntimeError(f"kernel launch failed: status {rc}")

    # parity of this very launch configuration against the CPU oracle (also the CPU baseline)
    step_fn(0)
    torch.cuda.synchronize()
    y_gpu = Y.float().cpu().numpy().astype(np.float64)
    cpu_baseline, parity = None, None
    if not args.no_cpu:
        import oracle
        oracle.build()
        oracle.linear_w4a8(X[:1], W[:16], s, G)  # load + warm
        codes_h, step_h, zero_h = oracle.quantize_weight_dint4(W, s, G)
        packed_h = oracle.pack_dint4(codes_h)
        t0 = time.perf_counter()
        n_cpu = 0
        while True:   # bounded sample: whole steps until about 10 s of CPU work
            Xq_h, sx_h = oracle.quantize_act_int8(X, s)
            acc_h = oracle.int_gemm(Xq_h, packed_h, zero_h, G)
            y32_h, y64_h = oracle.dequant_epilogue(acc_h, sx_h, step_h)
            n_cpu += 1
            cpu_s = time.perf_counter() - t0
            if cpu_s >= 10.0 or n_cpu >= 2000:
                break
        cpu_baseline = {"value": round(N * K / 2 * n_cpu / cpu_s / 1e9, 4), "unit": "GB/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"{n_cpu} whole steps (act-quant + int GEMM + dequant, M={M} K={K} N={N} "
                                  f"g{G}) in {cpu_s:.1f} s"}
        floor = 1e-3 * np.sqrt(np.mean(y64_h ** 2, axis=1, keepdims=True))
        ok = bool(np.all(np.abs(y_gpu - y64_h) <= 1e-3 * np.maximum(np.abs(y64_h), floor)))
        parity = {"Xq_bit_exact": bool(np.array_equal(Xq.cpu().numpy(), Xq_h)),
                  "codes_bit_exact": bool(np.array_equal(
                      w.unpack_dint4(Wp, N, K, w.LAYOUT_TILED).cpu().numpy(), codes_h)),
                  "Y_within_1e-3": ok}

    # ------------------------------------------------------------------ timed region
    use_graph = not args.no_graph
    steps, warmup = args.steps, args.warmup
    graph = None
    if use_graph:
        # one graph = one trip round the ring (R steps, 2R kernels); replayed steps / R times
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            st_side = ctypes.c_void_p(side.cuda_stream)
            aq_g = aq_args[:-1] + (st_side,)
            gm_g = [a[:-1] + (st_side,) for a in gm_args]
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for i in range(R):
                    rc = lib.quantize_act_int8(*aq_g) | lib.w4a8_gemm(*gm_g[i])
                    assert rc == 0
        stream.wait_stream(side)
        steps = max(R, steps // R * R)
        warmup = max(R, -(-warmup // R) * R)
        for _ in range(warmup // R):
            graph.replay()
        torch.cuda.synchronize()
        # a replay must reproduce the eager result exactly
        y_eager = Y.clone()
        step_fn(R - 1)
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager), "graph replay differs from eager launch"
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps // R):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        for i in range(warmup):
            step_fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step_fn(i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

    if args.pmc_calibration:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = elapsed / steps * 1e3
    weight_gbs = N * K / 2 / (elapsed / steps) / 1e9

    # ------------------------------------------------------------------ roofline of the dominant kernel
    # The decode GEMV, timed with HIP events on the launch stream around L back-to-back launches of
    # w4a8_gemm alone over the same weight ring (the figure a rocprofv3 kernel trace reports as the
    # kernel's average duration; event pairs around single launches add ~3 us of marker overhead).
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    L = 2048
    for i in range(64):
        lib.w4a8_gemm(*gm_args[i % R])
    torch.cuda.synchronize()
    reps_ms = []
    for _ in range(5):
        e0.record(stream)
        for i in range(L):
            lib.w4a8_gemm(*gm_args[i % R])
        e1.record(stream)
        torch.cuda.synchronize()
        reps_ms.append(e0.elapsed_time(e1) / L)
    kern_ms = float(np.median(reps_ms))
    achieved = per_copy / (kern_ms * 1e-3) / 1e9
    # context: the same loop over the smallest kernel of the library (packing one 16 x 128 tile) -- what a
    # launch costs on this stream when the kernel itself does next to nothing
    tiny_codes = torch.zeros((16, 128), dtype=torch.uint8, device=dev)
    tiny_out = torch.empty((16 * 64,), dtype=torch.uint8, device=dev)
    tiny_args = (P(tiny_codes), 16, 128, P(tiny_out), w.LAYOUT_TILED, st)
    for i in range(64):
        lib.pack_dint4(*tiny_args)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(L):
        lib.pack_dint4(*tiny_args)
    e1.record(stream)
    torch.cuda.synchronize()
    floor_us = e0.elapsed_time(e1) / L * 1e3
    roofline = {"bound": "hbm", "kernel": "gemv_kernel (w4a8_gemm, M<=16)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": GEMV_C2_TRAFFIC_BYTES,
                "bytes_per_launch": per_copy, "avg_launch_us": round(kern_ms * 1e3, 3),
                "launch_floor_us": round(floor_us, 3)}

    # ------------------------------------------------------------------ measured ceilings and the cache-resident figure
    # What a plain streaming read and a register-resident int8 MFMA loop reach on this machine in this
    # run (the roofline fractions stay against the nominal peaks), and the C2 GEMV launched over
    # one weight copy that stays in the 256 MB last-level cache (never an HBM fraction).
    ceilings = None
    if not args.no_prefill:
        big = torch.empty((1 << 30,), dtype=torch.uint8, device=dev)
        big.random_(0, 256)
        sink = torch.zeros((4,), dtype=torch.int32, device=dev)
        reads = {}
        for label, nbytes in (("9_MB", per_copy // 16 * 16), ("39_MB", 38_600_000 // 16 * 16),
                              ("170_MB", 170_000_000 // 16 * 16)):
            # consecutive launches walk through the 1 GiB buffer, so every launch reads from HBM
            slots = (1 << 30) // nbytes
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
        e0.record(stream)
        for i in range(L):
            lib.w4a8_gemm(*gm_args[0])
        e1.record(stream)
        torch.cuda.synchronize()
        resident_us = e0.elapsed_time(e1) / L * 1e3
        ceilings = {"what": "measured on this box in this run: a plain streaming read of as many bytes as "
                            "the decode shapes move (each launch from HBM), a register-resident "
                            "v_mfma_i32_32x32x32_i8 loop, and the C2 GEMV over one cache-resident weight copy",
                    "stream_read": reads,
                    "mfma_i8_loop_TOPS": round(ops.value / (mfma_ms * 1e-3) / 1e12, 1),
                    "gemv_C2_cache_resident_us": round(resident_us, 3)}

    # ------------------------------------------------------------------ larger decode shapes (side figures)
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
        wp_, st_, z_ = None, [], []
        rows = max(16, (1 << 26) // Kq // 16 * 16)   # weights in slabs of about 64 Mi elements
        if fam == "C5":   # the alpha = 0.5 point of the max-based scale family
            aw = torch.zeros((Kq,), device=dev)
            gw = torch.Generator(device=dev)
            gw.manual_seed(g.initial_seed() + 1)
            for r0 in range(0, Nq, rows):
                Wb = (torch.randn((min(rows, Nq - r0), Kq), device=dev, generator=gw) * 0.02).to(torch.float16)
                aw = torch.maximum(aw, Wb.float().abs().amax(0))
            s = (X.float().abs().amax(0).clamp_min(1e-5).sqrt() / aw.clamp_min(1e-5).sqrt()).contiguous()
        xq_, sx_ = w.quantize_act_int8(X, s)
        gw = torch.Generator(device=dev)
        gw.manual_seed(g.initial_seed() + 1)
        codes = torch.empty((Nq, Kq), dtype=torch.uint8, device=dev)
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
        matter there); fam = "C3" / "C4" / "C5": one set of operands quantized from that
        configuration's distributions."""
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
        for _ in range(3):   # median of three timed loops
            e0.record(stream)
            for i in range(reps):
                fn(*argsq[i % nring])
            e1.record(stream)
            torch.cuda.synchronize()
            runs.append(e0.elapsed_time(e1) / reps)
        return float(np.median(runs)), per

    decode_side = []
    if not args.no_prefill:
        for (Mq, Kq, Nq, Gq) in [(16, 5120, 5120, 128), (16, 5120, 13824, 128), (16, 13824, 5120, 128),
                                 (16, 9216, 36864, 0)]:
            ms, per = time_gemm(Mq, Nq, Kq, Gq, 400)
            decode_side.append({"workload": f"M={Mq} K={Kq} N={Nq} G={Gq or Kq}", "us": round(ms * 1e3, 3),
                                "GBps": round(per / ms / 1e6, 1),
                                "frac_of_hbm_peak": round(per / ms / 1e6 / HBM_PEAK_GBS, 4)})

    # ------------------------------------------------------------------ prefill side (compute-bound)
    prefill = []
    if not args.no_prefill:
        for (name, Mp, Kp, Np, Gp) in [("C3_up", 2048, 4096, 11008, 0), ("C3_down", 2048, 11008, 4096, 0),
                                       ("C4", 2048, 5120, 13824, 128), ("C4", 512, 5120, 13824, 128),
                                       ("C5", 4096, 9216, 36864, 0)]:
            ms, _ = time_gemm(Mp, Np, Kp, Gp, 20, ring_bytes=0, fam=name[:2])
            tops = 2.0 * Mp * Np * Kp / (ms * 1e-3) / 1e12
            prefill.append({"workload": f"{name} M={Mp} K={Kp} N={Np} G={Gp or Kp}", "ms": round(ms, 4),
                            "TOPS": round(tops, 1), "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4)})

    # ------------------------------------------------------------------ the LLaMA-13B layer sweep (side)
    # K -> N in {5120 -> 5120, 5120 -> 13824, 13824 -> 5120} x M in {1, 16, 128, 512, 2048}, group-128:
    # time per w4a8_gemm call, against both rooflines (M <= 16 is the HBM side, M >= 512 the matrix-core
    # side, M = 128 sits at the ridge)
    c4_sweep = []
    if not args.no_prefill:
        for (Kq, Nq) in [(5120, 5120), (5120, 13824), (13824, 5120)]:
            for Mq in (1, 16, 128, 512, 2048):
                ms, per = time_gemm(Mq, Nq, Kq, 128, 200 if Mq <= 128 else 20,
                                    ring_bytes=(600 << 20) if Mq <= 16 else 0, fam=None if Mq <= 16 else "C4")
                tops = 2.0 * Mq * Nq * Kq / (ms * 1e-3) / 1e12
                c4_sweep.append({"workload": f"M={Mq} K={Kq} N={Nq} G=128", "us": round(ms * 1e3, 2),
                                 "GBps": round(per / ms / 1e6, 1), "TOPS": round(tops, 1),
                                 "frac_of_hbm_peak": round(per / ms / 1e6 / HBM_PEAK_GBS, 4),
                                 "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4)})

    # 17 .. 128 tokens on the C2 layer: 16-token blocks of the streaming kernel in one launch
    mid_tokens = []
    if not args.no_prefill:
        for Mq in (17, 32, 64, 128):
            ms, per = time_gemm(Mq, N, K, G, 300, ring_bytes=0)
            mid_tokens.append({"workload": f"M={Mq} K={K} N={N} G={G}", "us": round(ms * 1e3, 2),
                               "TOPS": round(2.0 * Mq * N * K / (ms * 1e-3) / 1e12, 1)})

    # ------------------------------------------------------------------ quantizer kernels and C5 end to end (side)
    quant_side = None
    if not args.no_prefill:
        g = torch.Generator(device=dev)
        g.manual_seed(20231107)
        Mq, Kq, Nq = 4096, 9216, 36864                      # C5
        Xb = torch.randn((Mq, Kq), device=dev, generator=g).to(torch.float16)
        sb = torch.rand((Kq,), device=dev, generator=g) * 1.5 + 0.5
        Xqb = torch.empty((Mq, Kq), dtype=torch.int8, device=dev)
        sxb = torch.empty((Mq,), dtype=torch.float32, device=dev)
        aq_b = (P(Xb), w.F16, Mq, Kq, Kq, P(sb), P(Xqb), P(sxb), st)
        for _ in range(3):
            lib.quantize_act_int8(*aq_b)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(20):
            lib.quantize_act_int8(*aq_b)
        e1.record(stream)
        torch.cuda.synchronize()
        aq_ms = e0.elapsed_time(e1) / 20
        aq_bytes = Mq * Kq * 3 + 4 * Kq + 4 * Mq
        # end to end on C5: activation quantization + GEMM back to back on one stream
        wpb = torch.randint(0, 256, (Nq * Kq // 2,), dtype=torch.uint8, device=dev, generator=g)
        stb = torch.rand((Nq, 1), device=dev, generator=g) * 0.01 + 0.001
        zb = torch.randint(0, 14, (Nq, 1), dtype=torch.uint8, device=dev, generator=g)
        yb = torch.empty((Mq, Nq), dtype=torch.float16, device=dev)
        wsb_n = w.gemm_workspace_bytes(Mq, Nq, Kq, 0)
        wsb = torch.empty((max(1, wsb_n),), dtype=torch.uint8, device=dev)
        gm_b = (P(Xqb), P(sxb), Mq, P(wpb), w.LAYOUT_TILED, P(stb), P(zb), Nq, Kq, 0, P(yb), w.F16, Nq, None,
                P(wsb), wsb_n, st)
        for _ in range(2):
            assert lib.quantize_act_int8(*aq_b) == 0 and lib.w4a8_gemm(*gm_b) == 0
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(10):
            lib.quantize_act_int8(*aq_b)
            lib.w4a8_gemm(*gm_b)
        e1.record(stream)
        torch.cuda.synchronize()
        e2e_ms = e0.elapsed_time(e1) / 10
        del Xb, Xqb, wpb, yb
        # weight quantization + packing of a C4 up-projection matrix (offline)
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
        quant_side = {"what": "the quantizer kernels against the HBM roofline (bytes: input read + output written), "
                              "and the C5 layer end to end (quantize_act_int8 + w4a8_gemm on one stream)",
                      "act_quant_C5": {"workload": f"M={Mq} K={Kq} fp16", "ms": round(aq_ms, 4),
                                       "GBps": round(aq_bytes / aq_ms / 1e6, 1),
                                       "frac_of_hbm_peak": round(aq_bytes / aq_ms / 1e6 / HBM_PEAK_GBS, 4)},
                      "weight_quant_C4": {"workload": f"N={Nw} K={Kw} fp16 G=128", "ms": round(wq_ms, 4),
                                          "GBps": round(wq_bytes / wq_ms / 1e6, 1),
                                          "frac_of_hbm_peak": round(wq_bytes / wq_ms / 1e6 / HBM_PEAK_GBS, 4)},
                      "pack_tiled_C4": {"ms": round(pk_ms, 4), "GBps": round(Nw * Kw * 1.5 / pk_ms / 1e6, 1)},
                      "C5_end_to_end": {"workload": f"M={Mq} K={Kq} N={Nq} per-channel", "ms": round(e2e_ms, 4),
                                        "TOPS": round(2.0 * Mq * Nq * Kq / (e2e_ms * 1e-3) / 1e12, 1),
                                        "frac_of_int8_peak": round(2.0 * Mq * Nq * Kq / (e2e_ms * 1e-3) / 1e12
                                                                   / INT8_PEAK_TOPS, 4)}}
        del Wb, cb

    # ------------------------------------------------------------------ asymmetric activations (side)
    asym_side = []
    if not args.no_prefill:
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

    # ------------------------------------------------------------------ 4-bit Value cache (side)
    value_side = None
    if not args.no_prefill:
        # decode attention of 16 sequences x 32 heads (LLaMA-7B): one query token per head against 4096
        # cached tokens of 128 channels, channel-wise dINT4 Value, 8-bit probabilities
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

    # ------------------------------------------------------------------ AQAS scale search (side, offline)
    search_side = None
    if not args.no_prefill:
        Ms = 512   # calibration tokens
        Xc, _, _, _ = syn.make_layer("C2", M=Ms, variant=1)
        Xc_d = torch.from_numpy(Xc).to(dev)
        w.aqas_search(Xc_d, Wd, G)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        s_best, j_best, losses_s = w.aqas_search(Xc_d, Wd, G)
        torch.cuda.synchronize()
        search_ms = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        clip_idx, _, _ = w.aqas_clip_search(Xc_d, Wd, s_best, G)
        torch.cuda.synchronize()
        clip_ms = (time.perf_counter() - t0) * 1e3
        ls = losses_s.cpu().numpy()
        search_side = {"what": "aqas_search (17 grid points, each a full pass of the quantized layer on the GPU) and "
                               "aqas_clip_search (11 range factors per output channel) on the C2 layer",
                       "workload": f"calibration_tokens={Ms} K={K} N={N} G={G}",
                       "search_ms": round(search_ms, 3), "clip_ms": round(clip_ms, 3),
                       "best_alpha": int(j_best.item()) / 16.0,
                       "loss_at_best_over_loss_at_alpha_0_and_1": [round(float(ls.min() / ls[0]), 4),
                                                                   round(float(ls.min() / ls[16]), 4)],
                       "channels_clipped": int((clip_idx > 0).sum().item())}
        # the underflow / rounding split of the output error (weight quantization alone) on the same layer
        terms = {}
        for fname, fid in (("int4", w.FMT_INT4), ("dint4", w.FMT_DINT4), ("dint3", w.FMT_DINT3),
                           ("dint4_special_step_over_4", w.FMT_DINT4_C4),
                           ("dint4_special_step_over_8", w.FMT_DINT4_C8)):
            tt = w.dint_error_terms(Xc_d, Wd, s_best, G, fid).cpu().numpy()
            terms[fname] = {"underflow": float(f"{tt[0]:.5g}"), "rounding": float(f"{tt[1]:.5g}"),
                            "cross": float(f"{tt[2]:.5g}"), "underflowing_weights": int(tt[3])}
        search_side["output_error_split"] = terms

    out = {
        "metric": METRIC, "value": round(weight_gbs, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"C2 LLaMA-7B attention projection decode: M={M} K={K} N={N} group-{G} dINT4; "
                               f"step = quantize_act_int8 + w4a8_gemm; ring of {R} weight copies "
                               f"({R * per_copy / 2 ** 20:.0f} MiB)",
                   "launch": "hip-graph" if use_graph else "eager"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity,
        "offline": {"what": "quantize_weight_dint4 + pack_dint4 (tiled), once per weight matrix",
                    "ms": round(offline_ms, 4),
                    "GBps": round((N * K * 2 + N * K + N * K + N * K // 2) / (offline_ms * 1e-3) / 1e9, 1)},
        "decode_other_shapes": decode_side, "prefill": prefill, "c4_layer_sweep": c4_sweep, "c2_17_to_128_tokens": mid_tokens,
        "asymmetric_activations": {"what": "w4a8_gemm_asym (token zero-point taken out of the int32 "
                                           "accumulators), same shapes and protocol as the lists above",
                                   "shapes": asym_side},
        "quantizers": quant_side, "value_cache": value_side, "aqas_search": search_side,
        "ceilings": ceilings,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
