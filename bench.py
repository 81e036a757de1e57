#!/usr/bin/env python3
"""Benchmark of the HAGO quantized-operator hot path on one MI355X.

Headline (the JSON line's `value`): int8 TOP/s of the BERT-base dense stack
(BASELINE config 5: M = 32 x 128 = 4096 rows through 768->2304, 768->768,
768->3072, 3072->768), each layer one `hago_qdense` launch with int32
accumulation, zero-point correction and the fused per-channel requantize.
One step = the four launches; inputs are resident in HBM before timing.

The same line carries
  roofline     -- the int8-MFMA GEMM kernel: algorithmic ops / average launch
                  time (HIP events on the launch stream) against 5.0 POP/s;
  cpu_baseline -- the CPU oracle timed on a bounded sample of the same stack;
  ops          -- the other operators of the path (simquant, depthwise,
                  pointwise, standalone requantize, the conv configs and
                  batch-scaled variants), each with its own bound.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # dense int8 MFMA, MI355X published (5.0 POP/s)
PEAK_HBM_GBS = 8000.0     # HBM3E, MI355X published
RAMP_MS = 150.0           # untimed load before the warm-up steps (clock ramp of an idle board)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--ramp-ms", type=float, default=RAMP_MS,
                    help="untimed load before the warm-up steps (clock ramp of an idle board)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-ops", action="store_true")
    ap.add_argument("--only", default="", help="comma list of extra-op names to time (default all)")
    ap.add_argument("--gemm", default="", help="M,N,K: only time hago_qdense on this shape (uniform random "
                    "uint8 activations and int8 weights) and print its line; for counter runs")
    ap.add_argument("--phase-stamps", action="store_true",
                    help="development: load libhago_phase.so (python -m paper_2103_14949_amd.build "
                         "--phase-timing) and print, per config 5 layer, where a workgroup's time goes")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run plain copies of known size (for scaling rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); "
                 "use --gpus 1")

    import torch
    import paper_2103_14949_amd as hago
    from paper_2103_14949_amd import datagen

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.phase_stamps:
        from paper_2103_14949_amd import binding, build as hip_build
        if not os.path.exists(hip_build.PHASE_LIB):
            sys.exit(f"bench.py: {hip_build.PHASE_LIB} is missing: python -m paper_2103_14949_amd.build --phase-timing")
        binding._LIB_PATH = hip_build.PHASE_LIB
    hago.lib()  # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def to_dev(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    def rq_of(mult, shift, out_u8=False, z_out=0, clip=None, rounding=0):
        q = hago.QType(hago.U8 if out_u8 else hago.I8, 8, not out_u8, z_out)
        lo, hi = clip if clip else (None, None)
        return hago.Requant(to_dev(mult), to_dev(shift), q, lo, hi, rounding=rounding)

    def event_times_ms(fn, iters, warmup, reps=5):
        """Milliseconds per call of fn over `iters` back-to-back calls (HIP events on the launch
        stream, so launch latency is amortised as in steady-state inference), `reps` repetitions."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        out = []
        for _ in range(reps):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / iters)
        return out

    def event_time_ms(fn, iters, warmup):
        """Median of five repetitions."""
        return float(np.median(event_times_ms(fn, iters, warmup)))

    if args.gemm:
        Mg, Ng, Kg = (int(v) for v in args.gemm.split(","))
        rng = np.random.default_rng(7)
        a = to_dev(rng.integers(0, 256, (Mg, Kg), dtype=np.uint8))
        w = to_dev(rng.integers(-127, 128, (Ng, Kg), dtype=np.int8))
        rq = rq_of(rng.integers(2 ** 30, 2 ** 31, Ng, dtype=np.int64).astype(np.int32),
                   np.full(Ng, 12, dtype=np.int32))
        out = torch.empty((Mg, Ng), dtype=torch.int8, device=dev)
        f = hago.qdense(a, hago.QType(hago.U8, 8, False, 121), w, hago.QType(hago.I8), None, hago.I32,
                        rq, out=out, prepare=True)
        ms = event_time_ms(f, args.steps, args.warmup)
        ops_g = 2.0 * Mg * Ng * Kg
        print(json.dumps({"gemm": [Mg, Ng, Kg], "us": round(ms * 1e3, 2),
                          "tops": round(ops_g / (ms * 1e-3) / 1e12, 1),
                          "frac_mfma": round(ops_g / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)}), flush=True)
        return

    if args.pmc_calibration:
        # 256 MiB device-to-device copies: 256 MiB fetched and 256 MiB written per kernel
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ headline: config 5
    M = 4096
    layers = []
    for idx, (K, N) in enumerate(datagen.BERT_LAYERS):
        c = datagen.config5_layer(idx, M)
        layers.append(dict(
            K=K, N=N, host=c, a=to_dev(c["a"]), w=to_dev(c["w"]), bias=to_dev(c["bias"]),
            a_t=hago.QType(hago.U8, 8, False, c["z_a"]), w_t=hago.QType(hago.I8),
            rq=rq_of(c["mult"], c["shift"]),
            out=torch.empty((M, N), dtype=torch.int8, device=dev), ops=2.0 * M * N * K))
    total_ops = sum(l["ops"] for l in layers)

    # every launch is marshalled once; the timed loop only re-issues the calls
    for l in layers:
        l["call"] = hago.qdense(l["a"], l["a_t"], l["w"], l["w_t"], l["bias"], hago.I32, l["rq"],
                                out=l["out"], prepare=True)
    calls = [l["call"] for l in layers]

    def run_layer(l):
        l["call"]()

    def step():
        for c in calls:
            c()

    if args.phase_stamps:
        print(json.dumps(phase_stamps(torch, hago, layers, event_times_ms)))
        return

    # An idle board needs about 50 ms of load before its clocks settle (the first 200 steps after
    # idling run 8-13 % slower than the steady state): the stack runs untimed for RAMP_MS before the
    # W warm-up steps, so that the timed steps see the state a busy server is in.
    t_ramp = time.perf_counter()
    while (time.perf_counter() - t_ramp) * 1e3 < args.ramp_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / args.steps
    value_tops = total_ops * args.steps / (wall_ms * 1e-3) / 1e12
    # dominant kernel: the int8 MFMA GEMM; four launches per step
    avg_launch_ms = ev_ms / (args.steps * len(layers))
    achieved = total_ops * args.steps / (ev_ms * 1e-3) / 1e12
    step_reps = [ev_ms / args.steps] + event_times_ms(step, args.steps, 0, reps=4)
    per_layer = []
    for l in layers:
        reps = event_times_ms(lambda: run_layer(l), args.steps, 5)
        ms = float(np.median(reps))
        per_layer.append({"K": l["K"], "N": l["N"], "us": round(ms * 1e3, 3), "us_min": round(min(reps) * 1e3, 3),
                          "tops": round(l["ops"] / (ms * 1e-3) / 1e12, 1),
                          "frac": round(l["ops"] / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)})
    log("config 5 layers:", per_layer)

    # measured ceilings of this machine, same run: the matrix pipe alone on real data, and a streaming copy
    ceilings = measured_ceilings(torch, hago, event_times_ms, dev)
    log("measured ceilings:", ceilings)

    # HBM bytes per launch cannot be counted from inside this process: the figure is the one the
    # committed rocprofv3 --pmc summary of this same command ends with (null if it is absent).
    traffic, traffic_src = None, None
    prof = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        "qgemm_dma_config5_hbm_traffic.md")
    if os.path.exists(prof):
        meta = {}
        for line in open(prof):
            for key in ("traffic_bytes_per_launch", "kernel", "commit"):
                if line.startswith(key + ":"):
                    meta[key] = line.split(":", 1)[1].strip()
        if "traffic_bytes_per_launch" in meta:
            traffic = int(meta["traffic_bytes_per_launch"])
            traffic_src = {"file": "profiles/qgemm_dma_config5_hbm_traffic.md (FETCH_SIZE x2 + WRITE_SIZE, KiB)",
                           "kernel": meta.get("kernel"), "commit": meta.get("commit")}
    roofline = {"bound": "mfma", "traffic_source": traffic_src, "kernel": "qgemm_dma_kernel (int8 MFMA 32x32x32, fused requantize)",
                "achieved": round(achieved, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(achieved / PEAK_INT8_TOPS, 4), "traffic": traffic,
                "avg_launch_us": round(avg_launch_ms * 1e3, 3), "launches_per_step": len(layers),
                "ops_per_step": total_ops,
                "step_us_median_of_5": round(float(np.median(step_reps)) * 1e3, 3),
                "step_us_min_of_5": round(min(step_reps) * 1e3, 3),
                "measured_peak": ceilings.get("mfma_int8_tops"),
                "frac_of_measured_peak": (round(achieved / ceilings["mfma_int8_tops"], 4)
                                          if ceilings.get("mfma_int8_tops") else None),
                "per_layer": per_layer}

    # ------------------------------------------------------------------ other operators
    ops = {}
    if not args.no_extra_ops:
        only = set(filter(None, args.only.split(",")))
        ops = extra_ops(torch, hago, datagen, to_dev, rq_of, event_times_ms, only, ceilings)

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        cpu, parity = cpu_baseline(datagen, layers, torch)

    out = {
        "metric": "int8 TOPS (qdense + fused requantize, BERT-base dense stack)",
        "value": round(value_tops, 2), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_ramp_ms": args.ramp_ms, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "config5: BERT-base dense stack, M=4096 (batch 32 x seq 128), "
                               "u8 x i8 -> i32, per-channel requantize to i8; 4 launches/step",
                   "M": M, "layers_KN": [list(x) for x in datagen.BERT_LAYERS]},
        "roofline": roofline, "cpu_baseline": cpu, "parity_checked": parity, "ceilings": ceilings, "ops": ops,
    }
    print(json.dumps(out), flush=True)


def measured_ceilings(torch, hago, event_times_ms, dev):
    """The chip's own ceilings in this run: matrix instructions only (random operands: the clock under
    matrix-core load depends on the data), and streaming copies of the sizes the HBM-bound lines move,
    over rotating buffers larger than the last-level cache."""
    res = {}
    operands = torch.randint(-128, 128, (8192,), dtype=torch.int8, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    wgs, iters = 256 * 2, 2000      # two workgroups of four wavefronts per CU
    ms = float(np.median(event_times_ms(lambda: hago.probe_mfma_i8(operands, sink, wgs, iters), 5, 2)))
    res["mfma_int8_tops"] = round(2.0 * 32 ** 3 * 16 * iters * wgs / (ms * 1e-3) / 1e12, 1)
    res["mfma_note"] = "v_mfma_i32_32x32x32_i8 only, random operands, 8 wavefronts per CU, %.2f ms" % ms
    for name, nbytes in (("copy_58MB_gbs", 32 * 144 * 3136 * 4), ("copy_14MB_gbs", 32 * 144 * 3136)):
        n = max(2, int(np.ceil(640e6 / (2 * nbytes))))
        srcs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(n)]
        dsts = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(n)]
        state = {"i": 0}

        def run():
            i = state["i"] % n
            hago.probe_copy(srcs[i], dsts[i])
            state["i"] += 1
        ms = float(np.median(event_times_ms(run, 40, 4)))
        res[name] = round(2.0 * nbytes / (ms * 1e-3) / 1e9, 1)
        del srcs, dsts
    res["copy_note"] = "hago_probe_copy (128-bit nontemporal loads/stores), read + written bytes, rotating buffers"
    return res


def phase_stamps(torch, hago, layers, event_times_ms):
    """Per layer of the stack: back-to-back launch time, and the mean over its workgroups of the time
    between the phase timestamps the development build's GEMM kernel writes (100 MHz wall clock)."""
    import ctypes as C
    L = hago.lib()
    L.hago_debug_set_stamp_buffer.argtypes = [C.c_void_p, C.c_int]
    L.hago_debug_set_stamp_buffer.restype = None
    names = ["setup", "prologue_issue", "first_stage_wait", "main_loop", "drain_and_channel_terms",
             "requantize_to_lds", "copy_out"]
    nslots = 8192
    out = []
    for l in layers:
        L.hago_debug_set_stamp_buffer(None, 0)
        us = float(np.median(event_times_ms(l["call"], 100, 20))) * 1e3
        buf = torch.zeros(nslots * 8, dtype=torch.int64, device=l["a"].device)
        L.hago_debug_set_stamp_buffer(buf.data_ptr(), 0)
        for _ in range(5):
            l["call"]()
        torch.cuda.synchronize()
        L.hago_debug_set_stamp_buffer(None, 0)
        h = buf.cpu().numpy().reshape(nslots, 8)
        h = h[h[:, 0] != 0]
        # slot 7: entry, slots 0..6: end of each phase
        t = np.concatenate([h[:, 7:8], h[:, 0:7]], axis=1).astype(np.float64)
        ph = np.diff(t, axis=1).mean(axis=0) * 0.01
        rec = {"K": l["K"], "N": l["N"], "workgroups": int(len(h)), "us_per_launch_back_to_back": round(us, 2),
               "first_entry_to_last_end_us": round(float(h[:, 6].max() - h[:, 7].min()) * 0.01, 2),
               "entry_spread_us": round(float(h[:, 7].max() - h[:, 7].min()) * 0.01, 2),
               "end_spread_us": round(float(h[:, 6].max() - h[:, 6].min()) * 0.01, 2),
               "phase_us": {n: round(float(v), 2) for n, v in zip(names, ph)}}
        rec["main_loop_share_of_workgroup_time"] = round(float(ph[3] / ph.sum()), 3)
        out.append(rec)
    return out


def cpu_baseline(datagen, layers, torch):
    """The oracle as it stands on a bounded sample: one whole step on every core (all 4096 rows of the
    four layers, 58 GOP: about a second on 16 cores), and 256 rows of each layer on one thread.  The
    all-core results are also compared with what the GPU left in the layers' output buffers."""
    from oracle import hago_ref as ref
    ref.build()
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    threads = max(1, min(threads, os.cpu_count() or 1))
    rows = 4096
    ops = 0.0
    parity = True
    t0 = time.perf_counter()
    results = []
    for l in layers:
        c = l["host"]
        rq = ref.Requant(c["mult"], c["shift"], out_dtype=ref.I8)
        results.append(ref.qdense_threaded(c["a"][:rows], c["z_a"], c["w"], c["bias"], ref.I32, rq, threads=threads))
        ops += 2.0 * rows * l["N"] * l["K"]
    dt = time.perf_counter() - t0
    torch.cuda.synchronize()
    for l, want in zip(layers, results):
        parity = parity and bool(np.array_equal(l["out"].cpu().numpy(), want))
    log(f"cpu oracle: {ops / 1e9:.2f} GOP in {dt:.2f} s on {threads} threads; GPU outputs equal: {parity}")
    rows1, ops1 = 256, 0.0
    t0 = time.perf_counter()
    for l in layers:
        c = l["host"]
        rq = ref.Requant(c["mult"], c["shift"], out_dtype=ref.I8)
        ref.qdense(c["a"][:rows1], c["z_a"], c["w"], c["bias"], ref.I32, rq)
        ops1 += 2.0 * rows1 * l["N"] * l["K"]
    dt1 = time.perf_counter() - t0
    log(f"cpu oracle, one thread: {ops1 / 1e9:.2f} GOP in {dt1:.2f} s")
    return {"value": round(ops / dt / 1e12, 5), "unit": "TOP/s", "cores": threads, "kind": "oracle",
            "sample": f"all {rows} rows of each of the 4 layers, one step ({ops / 1e9:.1f} GOP), "
                      f"row slices on {threads} threads, {dt:.2f} s wall",
            "single_thread": {"value": round(ops1 / dt1 / 1e12, 5), "unit": "TOP/s", "cores": 1,
                              "sample": f"the first {rows1} rows of each layer ({ops1 / 1e9:.2f} GOP), {dt1:.2f} s wall"}}, parity


def extra_ops(torch, hago, datagen, to_dev, rq_of, event_times_ms, only, ceilings):
    """Timings of the remaining operators.  HBM-bound operators rotate over buffer sets that
    together exceed the 256 MB last-level cache, so the figure is an HBM rate."""
    dev = "cuda:0"
    res = {}

    def want(name):
        return not only or name in only

    def event_time_ms(fn, iters, warmup):
        """All five repetitions (record() reports their median and minimum)."""
        return event_times_ms(fn, iters, warmup)

    def record(name, reps, ops=None, bytes_=None, bound=None, note=None, warm=None):
        ms = float(np.median(reps))
        r = {"us": round(ms * 1e3, 3), "us_min": round(min(reps) * 1e3, 3)}
        if ops is not None:
            r["tops"] = round(ops / (ms * 1e-3) / 1e12, 3)
            r["frac_mfma"] = round(r["tops"] / PEAK_INT8_TOPS, 4)
        if bytes_ is not None:
            r["gbs"] = round(bytes_ / (ms * 1e-3) / 1e9, 1)
            r["frac_hbm"] = round(r["gbs"] / PEAK_HBM_GBS, 4)
            ref_copy = ceilings.get("copy_58MB_gbs" if bytes_ > 50e6 else "copy_14MB_gbs")
            if ref_copy:
                r["frac_of_measured_copy"] = round(r["gbs"] / ref_copy, 4)
        if warm is not None:   # the same call on ONE buffer set (served from the last-level cache where it fits)
            wms = float(np.median(event_times_ms(warm, 40, 4)))
            r["us_cache_warm"] = round(wms * 1e3, 3)
        r["bound"] = bound
        if note:
            r["note"] = note
        res[name] = r
        log(name, r)

    def rotating(make_call, nbytes_per_set, min_total=640e6):
        """Prepared calls over enough distinct buffer sets to exceed the last-level cache."""
        n = max(2, int(np.ceil(min_total / nbytes_per_set)))
        calls = [make_call(i) for i in range(n)]
        state = {"i": 0}

        def run():
            calls[state["i"] % n]()
            state["i"] += 1
        run.warm = calls[0]
        return run

    # ---- simquant, config 4 tensor
    if want("simquant_c4"):
        c = datagen.config4_simquant()
        x0 = to_dev(c["x"].reshape(32, 144, -1))
        scale, zp = to_dev(c["scale"]), to_dev(c["zp"])
        q = hago.QType(hago.I8)
        nb = x0.numel() * 8
        f = rotating(lambda i: hago.simquant(x0.clone(), scale, zp, q, out=torch.empty_like(x0),
                                             prepare=True), nb)
        record("simquant_c4", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
               note="fp32 [32,144,56,56], per-channel, 8 B/elem")
        del f

    # ---- eight search candidates in one launch (Sec. 6.3)
    if want("simquant_batched8_c4"):
        c = datagen.config4_simquant()
        x0 = to_dev(c["x"].reshape(32, 144, -1))
        bits = [8, 8, 7, 7, 6, 6, 5, 4]
        lo = [-(1 << (b - 1)) for b in bits]
        hi = [(1 << (b - 1)) - 1 for b in bits]
        scales = to_dev(np.stack([c["scale"] * (128.0 / (1 << (b - 1))) for b in bits]).astype(np.float32))
        zps = to_dev(np.zeros((8, 144), np.int32))
        nb = x0.numel() * 4 * 9
        f = rotating(lambda i: hago.simquant_batched(x0.clone(), scales, zps, hago.QType(hago.I8), lo, hi,
                                                     prepare=True), nb)
        record("simquant_batched8_c4", event_time_ms(f, 30, 4), warm=f.warm, bytes_=nb, bound="hbm",
               note="fp32 [32,144,56,56], 8 candidates in one launch, 4 + 32 B/elem "
                    "(8 separate simquant launches move 64 B/elem)")
        del f

    # ---- quantize / dequantize of the same tensor (int8 codes)
    if want("quantize_c4") or want("dequantize_c4") or want("simquant_codes_c4"):
        c = datagen.config4_simquant()
        x0 = to_dev(c["x"].reshape(32, 144, -1))
        scale, zp = to_dev(c["scale"]), to_dev(c["zp"])
        q = hago.QType(hago.I8)
        nb = x0.numel() * 5
        if want("quantize_c4"):
            f = rotating(lambda i: hago.quantize(x0.clone(), scale, zp, q, prepare=True), nb)
            record("quantize_c4", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
                   note="fp32 [32,144,56,56] -> int8 codes, 5 B/elem")
            del f
        if want("simquant_codes_c4"):
            f = rotating(lambda i: hago.simquant_codes(x0.clone(), scale, zp, q, prepare=True), x0.numel() * 9)
            record("simquant_codes_c4", event_time_ms(f, 60, 6), warm=f.warm, bytes_=x0.numel() * 9, bound="hbm",
                   note="fp32 [32,144,56,56] -> fp32 + int8 codes in one pass, 9 B/elem")
            del f
        if want("dequantize_c4"):
            codes0 = hago.quantize(x0, scale, zp, q)
            f = rotating(lambda i: hago.dequantize(codes0.clone(), q, scale, zp, prepare=True), nb)
            record("dequantize_c4", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
                   note="int8 codes [32,144,56,56] -> fp32, 5 B/elem")
            del f

    # ---- max-abs calibration of the same tensor (Eq. 2)
    if want("absmax_c4"):
        c = datagen.config4_simquant()
        x0 = to_dev(c["x"].reshape(32, 144, -1))
        nb = x0.numel() * 4
        f = rotating(lambda i: hago.absmax(x0.clone(), True, prepare=True), nb)
        record("absmax_c4", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
               note="fp32 [32,144,56,56] -> 144 thresholds, 4 B/elem (zero fill + reduction, two launches)")
        del f

    # ---- depthwise + pointwise, config 4
    c4 = datagen.config4()
    a_t, w_t = hago.QType(hago.I8, 8, True, 0), hago.QType(hago.I8)
    if want("depthwise_c4"):
        a0 = to_dev(c4["a"])
        w, rq = to_dev(c4["w_dw"]), rq_of(c4["mult_dw"], c4["shift_dw"])
        nb = a0.numel() * 2
        f = rotating(lambda i: hago.qconv2d(a0.clone(), a_t, w, w_t, None, hago.NCHW, (1, 1), (1, 1),
                                            144, hago.I32, rq, out=torch.empty_like(a0),
                                            prepare=True), nb)
        record("depthwise_c4", event_time_ms(f, 100, 10), warm=f.warm, ops=2.0 * a0.numel() * 9, bytes_=nb,
               bound="hbm", note="i8 [32,144,56,56] 3x3, 2 B/output")
        del f
    if want("pointwise_c4"):
        a0 = to_dev(c4["a"])  # same distribution as the depthwise output
        w, rq = to_dev(c4["w_pw"]), rq_of(c4["mult_pw"], c4["shift_pw"])
        o_shape = (32, 24, 56, 56)
        nb = a0.numel() + 32 * 24 * 56 * 56
        f = rotating(lambda i: hago.qconv2d(a0.clone(), a_t, w, w_t, None, hago.NCHW, (1, 1), (0, 0),
                                            1, hago.I32, rq,
                                            out=torch.empty(o_shape, dtype=torch.int8, device=dev),
                                            prepare=True), nb)
        record("pointwise_c4", event_time_ms(f, 100, 10), warm=f.warm, ops=2.0 * 32 * 56 * 56 * 24 * 144,
               bytes_=nb, bound="hbm", note="1x1 conv 144->24 on MFMA, 168 B/pixel")
        del f

    # ---- the same depthwise layer at stride 2 (a downsampling layer of the same network)
    if want("depthwise_c4_s2"):
        a0 = to_dev(c4["a"])
        w, rq = to_dev(c4["w_dw"]), rq_of(c4["mult_dw"], c4["shift_dw"])
        o_shape = (32, 144, 28, 28)
        nb = a0.numel() + 32 * 144 * 28 * 28
        f = rotating(lambda i: hago.qconv2d(a0.clone(), hago.QType(hago.I8), w, hago.QType(hago.I8), None, hago.NCHW,
                                            (2, 2), (1, 1), 144, hago.I32, rq,
                                            out=torch.empty(o_shape, dtype=torch.int8, device=dev),
                                            prepare=True), nb)
        record("depthwise_c4_s2", event_time_ms(f, 100, 10), warm=f.warm, ops=2.0 * 32 * 144 * 28 * 28 * 9,
               bytes_=nb, bound="hbm", note="i8 [32,144,56,56] 3x3 stride 2, 1.25 B/input")
        del f

    # ---- standalone requantize
    if want("requantize_i32"):
        acc0 = torch.randint(-2 ** 20, 2 ** 20, (32, 144, 3136), dtype=torch.int32, device=dev)
        rq = rq_of(c4["mult_dw"], c4["shift_dw"])
        nb = acc0.numel() * 5
        f = rotating(lambda i: hago.requantize(acc0.clone(), rq,
                                               out=torch.empty(acc0.shape, dtype=torch.int8, device=dev),
                                               prepare=True), nb)
        record("requantize_i32", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
               note="i32 [32,144,3136] -> i8, 5 B/elem")
        del f

    # ---- the second tie rule (halves away from zero) runs through the general code paths
    if want("requantize_i32_half_away"):
        acc0 = torch.randint(-2 ** 20, 2 ** 20, (32, 144, 3136), dtype=torch.int32, device=dev)
        rq = rq_of(c4["mult_dw"], c4["shift_dw"], rounding=hago.ROUND_HALF_AWAY)
        nb = acc0.numel() * 5
        f = rotating(lambda i: hago.requantize(acc0.clone(), rq,
                                               out=torch.empty(acc0.shape, dtype=torch.int8, device=dev),
                                               prepare=True), nb)
        record("requantize_i32_half_away", event_time_ms(f, 60, 6), warm=f.warm, bytes_=nb, bound="hbm",
               note="i32 [32,144,3136] -> i8, 5 B/elem, ties away from zero")
        del f
    if want("dense_c5_ffn1_half_away"):
        c = datagen.config5_layer(2, 4096)
        rq = rq_of(c["mult"], c["shift"], rounding=hago.ROUND_HALF_AWAY)
        f = hago.qdense(to_dev(c["a"]), hago.QType(hago.U8, 8, False, c["z_a"]), to_dev(c["w"]),
                        hago.QType(hago.I8), to_dev(c["bias"]), hago.I32, rq, prepare=True)
        record("dense_c5_ffn1_half_away", event_time_ms(f, 100, 10), ops=2.0 * 4096 * 3072 * 768,
               bound="mfma", note="config 5 layer 768 -> 3072 with ties away from zero (straight-line epilogue, not the LDS-staged one)")
        del f

    # ---- config 1 (as specified and scaled)
    for name, Mrows in (("dense_c1", 64), ("dense_c1_M8192", 8192)):
        if not want(name):
            continue
        c = datagen.config1(M=Mrows)
        a, w = to_dev(c["a"]), to_dev(c["w"])
        rq = rq_of(c["mult"], c["shift"])
        out = torch.empty((Mrows, 128), dtype=torch.int8, device=dev)
        at = hago.QType(hago.U8, 8, False, 128)

        f = hago.qdense(a, at, w, w_t, None, hago.I32, rq, out=out, prepare=True)
        record(name, event_time_ms(f, 200, 20), ops=2.0 * Mrows * 128 * 256,
               bound="latency" if Mrows == 64 else "hbm",
               note="u8 [M,256] x i8 [128,256]" + (" (scaled batch)" if Mrows != 64 else ""))

    # ---- config 2 (as specified and scaled)
    for name, B in (("conv_c2", 1), ("conv_c2_B64", 64), ("conv_c2_B256", 256)):
        if not want(name):
            continue
        c = datagen.config2(B=B)
        a, w = to_dev(c["a"]), to_dev(c["w"])
        rq = rq_of(c["mult"], c["shift"], True, 0, (0, 255))
        out = torch.empty((B, 64, 56, 56), dtype=torch.uint8, device=dev)
        at = hago.QType(hago.U8, 8, False, 0)

        # hago_qconv2d, no scratch memory: one launch straight from the NCHW tensor
        f = hago.qconv2d(a, at, w, w_t, None, hago.NCHW, (1, 1), (1, 1), 1, hago.I32, rq, out=out, prepare=True)
        record(name, event_time_ms(f, 100, 10), ops=2.0 * B * 3136 * 64 * 576,
               bound="latency" if B == 1 else "mfma",
               note="3x3 conv 64->64 @56x56 NCHW, one launch" + (" (scaled batch)" if B != 1 else ""))
        # beside it: both operands rewritten into a workspace, then the streaming implicit GEMM
        ws = torch.empty(hago.qconv2d_workspace_bytes(a.shape, w.shape, hago.NCHW, (1, 1), (1, 1)),
                         dtype=torch.uint8, device=dev)
        f = hago.qconv2d(a, at, w, w_t, None, hago.NCHW, (1, 1), (1, 1), 1, hago.I32, rq, out=out,
                         prepare=True, workspace=ws)
        hago.set_test_hook(hago.HOOK_GEMM_PATH, 2)
        try:
            record(name + "_via_workspace", event_time_ms(f, 100, 10), ops=2.0 * B * 3136 * 64 * 576,
                   bound="latency" if B == 1 else "mfma", note="the same through hago_qconv2d_ws's two-launch path")
        finally:
            hago.set_test_hook(hago.HOOK_GEMM_PATH, 0)

    # ---- config 3 (int16 accumulation; as specified and scaled)
    for name, B in (("conv_c3_acc16", 8), ("conv_c3_acc16_B64", 64), ("conv_c3_acc16_B256", 256)):
        if not want(name):
            continue
        c = datagen.config3(B=B)
        a, w = to_dev(c["a"]), to_dev(c["w"])
        out = torch.empty((B, 128, 28, 28), dtype=torch.int16, device=dev)
        at, wt = hago.QType(hago.I8, 4, False, 0), hago.QType(hago.I8, 4, True, 0)

        f = hago.qconv2d(a, at, w, wt, None, hago.NCHW, (1, 1), (1, 1), 1, hago.I16, None, out=out, prepare=True)
        record(name, event_time_ms(f, 100, 10), ops=2.0 * B * 784 * 128 * 1152, bound="mfma",
               note="3x3 conv 128->128 @28x28, raw int16 out, one launch" + (" (scaled batch)" if B != 8 else ""))
        ws = torch.empty(hago.qconv2d_workspace_bytes(a.shape, w.shape, hago.NCHW, (1, 1), (1, 1)),
                         dtype=torch.uint8, device=dev)
        f = hago.qconv2d(a, at, w, wt, None, hago.NCHW, (1, 1), (1, 1), 1, hago.I16, None, out=out,
                         prepare=True, workspace=ws)
        hago.set_test_hook(hago.HOOK_GEMM_PATH, 2)
        try:
            record(name + "_via_workspace", event_time_ms(f, 100, 10), ops=2.0 * B * 784 * 128 * 1152, bound="mfma",
                   note="the same through hago_qconv2d_ws's two-launch path")
        finally:
            hago.set_test_hook(hago.HOOK_GEMM_PATH, 0)
    return res


if __name__ == "__main__":
    main()
