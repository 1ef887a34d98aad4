#!/usr/bin/env python3
"""Benchmark of the MI355X binary-network forward path (after arXiv 1705.07175).

Headline line (one JSON object on stdout): the bit-packed binary matrix product of
Sec. 6.1 -- two dense 8192 x 8192 +-1 matrices, packed along K -- timed with HIP events
over exactly ``--steps`` launches after ``--warmup`` untimed ones, inputs resident in
HBM.  ``value`` is Gbop/s with 2 binary operations per multiply-accumulate.

The same object carries
  * ``roofline``      the dominant kernel (bgemm) against the integer-VALU XOR+popcount peak,
  * ``cpu_baseline``  the CPU oracle timed on this host on a bounded sample of the same job,
  * ``kernels``       the supporting kernels (pack, unroll, bn_sign_pack, bmaxpool, small-M
                      bgemm) on HBM-sized inputs against the 8 TB/s HBM peak,
  * ``networks``      images/s of the paper's MLP (Sec. 6.2) and CNN (Sec. 6.3) shapes.

All inputs are seeded and synthetic (``paper_1705_07175_amd.synth``).  One GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 CUs x 4 SIMDs, 2.4 GHz peak engine clock.  A SIMD retires 16 lanes per clock of
# the full-rate vector instructions (v_bcnt_u32_b32 among them: 39.3 T lane-ops/s, the rate behind
# the published 78.6 TFLOP/s fp64 vector figure) and 32 lanes per clock of the simple ones
# (v_xor_b32: 78.6 T lane-ops/s, the rate behind the published 157.3 TFLOP/s fp32 vector figure).
# Both rates are measured in every run by esp_xor_popcount_probe's single-instruction modes
# (``roofline.peak_derivation``; kernel trace of those launches: profiles/valu_rates.txt).
CUS, CLOCK_HZ = 256, 2.4e9
FULL_RATE_OPS = CUS * 4 * 16 * CLOCK_HZ          # 39.32e12 lane-ops/s
SIMPLE_RATE_OPS = 2 * FULL_RATE_OPS              # 78.64e12 lane-ops/s
# One v_xor_b32 + one accumulating v_bcnt_u32_b32 per lane handle 32 binary MACs = 64 bop.
VALU_PEAK_TBOPS = 64.0 / (1.0 / SIMPLE_RATE_OPS + 1.0 / FULL_RATE_OPS) / 1e12   # 1677.7 Tbop/s
# the same pair when every vector instruction is charged a full-rate slot (the estimate that
# does not know about the faster xor): 1258.3 Tbop/s
VALU_FULL_RATE_ONLY_TBOPS = 64.0 * FULL_RATE_OPS / 2 / 1e12
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the 8192-cube from the tracked counter runs, used when the profile summary
# is not beside this file: 2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE (KiB per dispatch)
BGEMM_8192_PROFILE = os.path.join(ROOT, "profiles", "bgemm_8192_cube.txt")
BGEMM_8192_FETCH_KIB, BGEMM_8192_WRITE_KIB = 36935.5, 262144.0
MFMA_FP32_PEAK_TFLOPS = 157.3  # dense fp32 MFMA
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
MFMA_FP4_PEAK_TOPS = 10100.0   # dense fp4/fp6 MFMA, TFLOP/s; one binary MAC = 2 flop = 2 bop


def _bgemm_8192_traffic():
    """(bytes per launch, where the figure comes from).  Counters need a profiler pass, so the value
    is the one of the tracked rocprofv3 --pmc runs of ``bench.py --only bgemm``: read from the
    summary under profiles/ when it is there, else the constants copied from it."""
    fetch, write, src = BGEMM_8192_FETCH_KIB, BGEMM_8192_WRITE_KIB, "constants in bench.py copied from profiles/bgemm_8192_cube.txt"
    try:
        section, got = None, {}
        for line in open(BGEMM_8192_PROFILE):
            if line.startswith("workload:"):
                section = line.split(":", 1)[1].strip()
            elif line.startswith("-- rocprofv3 --pmc"):
                counter = line.split()[3]
            elif section == "bgemm" and "bgemm_tile_kernel<128, 64, 8, 4, esp::MatrixA<true>" in line and "mean=" in line:
                got.setdefault(counter, float(line.rsplit("mean=", 1)[1]))
        if "FETCH_SIZE" in got and "WRITE_SIZE" in got:
            fetch, write, src = got["FETCH_SIZE"], got["WRITE_SIZE"], "parsed from profiles/bgemm_8192_cube.txt"
    except OSError:
        pass
    return int((2.0 * fetch + 1.0 * write) * 1024), {
        "source": src + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --only bgemm`; not measured in this run)",
        "read_bytes": int(2.0 * fetch * 1024), "written_bytes": int(write * 1024),
        "counter_scale": "true read bytes = 2.0 x FETCH_SIZE, written = 1.0 x WRITE_SIZE (from a plain 1 GiB copy)"}


def _events_ms(fn, steps, warmup, torch):
    """Average milliseconds per call of ``fn`` over ``steps`` calls, HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def _median_ms(fn, steps, torch):
    """Median milliseconds of ``steps`` calls of ``fn``, each bracketed by its own pair of HIP events
    (so each sample also holds the few microseconds an event pair costs)."""
    return _per_launch_ms(fn, steps, torch)["median_ms"]


def _per_launch_ms(fn, steps, torch):
    """``steps`` calls of ``fn``, each between its own pair of HIP events: median, mean, min, max."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in pairs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return {"median_ms": round(t[len(t) // 2], 5), "mean_ms": round(sum(t) / len(t), 5),
            "min_ms": round(t[0], 5), "max_ms": round(t[-1], 5), "launches": steps}


def _settle(fn, torch, min_ms=60.0, cap_ms=300.0, window=5, tol=0.01):
    """Untimed, reported clock-settle phase: the engine clock ramps for tens of milliseconds after the
    idle gap of the set-up, so ``fn`` is launched in windows of ``window`` calls for at least ``min_ms``
    and then until two consecutive windows agree within ``tol``, at most ``cap_ms``."""
    per_launch, spent = [], 0.0
    while True:
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(window):
            fn()
        stop.record()
        torch.cuda.synchronize()
        ms = start.elapsed_time(stop)
        spent += ms
        per_launch.append(ms / window)
        agree = len(per_launch) >= 2 and abs(per_launch[-1] - per_launch[-2]) <= tol * per_launch[-1]
        if (spent >= min_ms and agree) or spent >= cap_ms:
            break
    return {"clock_settle_ms": round(spent, 2), "windows": len(per_launch), "launches_per_window": window,
            "first_window_ms_per_launch": round(per_launch[0], 5), "last_window_ms_per_launch": round(per_launch[-1], 5),
            "settled": bool(agree)}


def _hbm_entry(name, ms, algo_bytes, workload):
    gbs = algo_bytes / (ms * 1e-3) / 1e9
    return {"kernel": name, "workload": workload, "ms": round(ms, 5), "bound": "hbm",
            "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": int(algo_bytes)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--size", type=int, default=8192, help="M=N=K of the headline binary GEMM")
    ap.add_argument("--no-extras", action="store_true", help="skip supporting kernels and networks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="oracle sample rows (0 = auto)")
    ap.add_argument("--no-settle", action="store_true", help="with --only: skip the untimed clock-settle launches "
                    "(for counter-collecting profiler runs, which serialise every dispatch)")
    ap.add_argument("--only", default="", help="time ONE supporting workload and print its entry "
                    "(for profiler runs): bgemm, small_squares, bcnn<batch>, bmlp<batch>, " + ", ".join(SUPPORTING))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1705_07175_amd import binding as esp
    from paper_1705_07175_amd import nets, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    esp.lib()  # fails loudly if the HIP library is not built

    if args.only.startswith(("bcnn", "bmlp")):
        kind, batch = args.only[:4], int(args.only[4:])
        print(json.dumps(_networks(torch, esp, nets, synth, dev, only=(kind, batch))))
        return 0
    if args.only == "small_squares":
        print(json.dumps(_paper_configs(torch, esp, synth, dev, args.steps, args.warmup)))
        return 0
    if args.only and args.only != "bgemm":
        if args.only not in SUPPORTING:
            print("bench.py: unknown --only %r" % args.only, file=sys.stderr)
            return 2
        entry = _supporting_kernels(torch, esp, synth, dev, np, only=args.only,
                                    steps=args.steps, warmup=args.warmup, settle=not args.no_settle)[0]
        print(json.dumps(entry))
        return 0

    def to_dev_f32(a):
        return torch.from_numpy(a).to(dev).to(torch.float32)

    n = args.size
    a_pm1, b_pm1 = synth.config5_square(n)
    a_f = to_dev_f32(a_pm1)
    A = esp.pack_f32(a_f)
    del a_f
    b_f = to_dev_f32(b_pm1)
    B = esp.pack_f32(b_f)
    C = torch.empty((n, n), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    run_bgemm = lambda: esp.bgemm(A, B, n, out=C)

    def settle_phase(fn, torch_, **kw):
        return {"clock_settle_ms": 0.0, "skipped": "--no-settle"} if args.no_settle else _settle(fn, torch_, **kw)

    # untimed and reported: launches until the engine clock has settled (it ramps for tens of
    # milliseconds after the idle set-up; --warmup alone would be 4 ms of launches at the driver's 5)
    settle = settle_phase(run_bgemm, torch)
    # the timed region: --warmup untimed launches, then EXACTLY --steps launches between one event pair
    ms, wall_ms = _events_ms(run_bgemm, args.steps, args.warmup, torch)
    # the same number of launches again, each between its own event pair: median beside the mean
    per_launch = _per_launch_ms(run_bgemm, args.steps, torch)
    # and a longer sample (Sec. 6: the paper averages 100 runs), whatever --steps is
    long_run = _per_launch_ms(run_bgemm, max(100, args.steps), torch)
    bop = 2.0 * n * n * n
    gbops = bop / (ms * 1e-3) / 1e9
    tbops = gbops / 1e3

    # cheap full-coverage sanity check of the timed result (row checksum identity)
    rows = np.array([0, n // 3, n - 1])
    bsum = b_pm1.astype(np.int64).sum(axis=0)

    def checksum_ok():
        got = C[torch.from_numpy(rows).to(dev)].sum(dim=1, dtype=torch.int64).cpu().numpy()
        return np.array_equal(got, a_pm1[rows].astype(np.int64) @ bsum)

    if not checksum_ok():
        print("bench.py: bgemm result failed its checksum", file=sys.stderr)
        return 1

    # What the vector ALUs sustain on registers only, measured in this run: the xor + popcount
    # pair in the kernel's instruction pattern (the ceiling the kernel can approach), and each of
    # the two instructions alone (the two rates the peak is derived from).
    blocks, iters = 2 * CUS, 2000        # two waves per SIMD: where the bare pair loop is fastest
    sink = torch.empty(4 * blocks * 256, dtype=torch.int32, device=dev)

    def probe_rate(mode, nblocks):
        work = esp.xor_popcount_probe(sink, nblocks, iters, mode)
        fn = lambda: esp.xor_popcount_probe(sink, nblocks, iters, mode)
        settle_phase(fn, torch, min_ms=20.0, cap_ms=100.0)
        t, _ = _events_ms(fn, 20, 5, torch)
        return work / (t * 1e-3) / 1e12, t

    ceiling, ms_p = probe_rate(esp.PROBE_PAIR, blocks)
    # the single-instruction loops need four waves per SIMD to fill the dual-issue of the simple ops
    xor_rate, ms_x = probe_rate(esp.PROBE_XOR_ONLY, 4 * blocks)
    popc_rate, ms_c = probe_rate(esp.PROBE_POPCOUNT_ONLY, 4 * blocks)
    derived_measured = 64.0 / (1.0 / xor_rate + 1.0 / popc_rate)
    props = torch.cuda.get_device_properties(0)
    traffic, traffic_detail = _bgemm_8192_traffic() if n == 8192 else (None, None)

    result = {
        "metric": "binary GEMM Gbop/s (% of int VALU peak); BCNN images/sec at batch 1 and 256",
        "value": round(gbops, 1),
        "unit": "Gbop/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "wall_ms_per_step": round(wall_ms, 5),
        "median_ms_per_step": per_launch["median_ms"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64 words (1-bit operands), int32 accumulate",
        "data": "synthetic",
        "config": {"workload": "config 5: binary GEMM M=N=K=%d, +-1 i.i.d., packed uint64, int32 out "
                               "(the matrix size of Sec. 6.1, Table 1)" % n,
                   "pct_of_int_valu_peak": round(100.0 * tbops / VALU_PEAK_TBOPS, 2),
                   "pct_of_full_rate_only_estimate": round(100.0 * tbops / VALU_FULL_RATE_ONLY_TBOPS, 2)},
        "timing": {"clock_settle": settle,
                   "timed_region": {"launches": args.steps, "mean_ms": round(ms, 5),
                                    "note": "one HIP event pair around exactly --steps launches, after --warmup untimed ones"},
                   "per_launch_event_pairs": per_launch,
                   "per_launch_event_pairs_100": long_run},
        "roofline": {"bound": "alu", "kernel": "bgemm_tile_kernel", "achieved": round(tbops, 2),
                     "peak": round(VALU_PEAK_TBOPS, 1), "unit": "Tbop/s",
                     "frac": round(tbops / VALU_PEAK_TBOPS, 4),
                     # the figure that charges both instructions a full-rate slot
                     "peak_full_rate_only": round(VALU_FULL_RATE_ONLY_TBOPS, 1),
                     "frac_of_full_rate_only_peak": round(tbops / VALU_FULL_RATE_ONLY_TBOPS, 4),
                     "traffic": traffic,
                     "traffic_detail": traffic_detail,
                     # how the peak follows from the two instructions' own rates, nominal and as measured
                     # in this run on registers only (T lane-instructions/s; 64 lanes per wave instruction)
                     "peak_derivation": {
                         "formula": "64 bop / (1 / xor_rate + 1 / popcount_rate)",
                         "nominal": {"xor_rate_tlops": round(SIMPLE_RATE_OPS / 1e12, 2),
                                     "popcount_rate_tlops": round(FULL_RATE_OPS / 1e12, 2),
                                     "peak_tbops": round(VALU_PEAK_TBOPS, 1),
                                     "basis": "256 CUs x 4 SIMDs x 2.4 GHz; v_xor_b32 32 lanes/clk/SIMD, v_bcnt_u32_b32 16"},
                         "measured": {"xor_rate_tlops": round(xor_rate, 2), "popcount_rate_tlops": round(popc_rate, 2),
                                      "peak_tbops": round(derived_measured, 1),
                                      "xor_only_ms": round(ms_x, 5), "popcount_only_ms": round(ms_c, 5),
                                      "pair_ms": round(ms_p, 5),
                                      "launch": "%d (pair) / %d (single instruction) blocks of 256 lanes, %d rounds of "
                                                "an 8 x 8 register block" % (blocks, 4 * blocks, iters),
                                      "xor_over_popcount": round(xor_rate / popc_rate, 3)},
                         "tracked_trace": "profiles/valu_rates.txt"},
                     # the pair loop on registers only (esp_xor_popcount_probe): what instruction
                     # issue and the clock under this load allow; the peak assumes 2.4 GHz
                     "measured_ceiling": round(ceiling, 2),
                     "frac_of_measured_ceiling": round(tbops / ceiling, 4),
                     "implied_clock_ghz": round(ceiling / VALU_PEAK_TBOPS * CLOCK_HZ / 1e9, 3),
                     "device": {"name": props.name, "compute_units": props.multi_processor_count,
                                "clock_rate_khz": getattr(props, "clock_rate", None)},
                     "algorithmic_bop_per_launch": bop,
                     "algorithmic_bytes_per_launch": 2 * n * n // 8 + 4 * n * n},
        "paper_context": "Sec. 6.1 Table 1: 11 ms for this product on a GTX 960 (64-bit packing)",
    }

    del b_f
    # measured alternative: the same product on the matrix cores (4-bit float MFMA)
    run_mfma = lambda: esp.bgemm_mfma(A, B, n, out=C)
    settle_phase(run_mfma, torch, min_ms=30.0, cap_ms=150.0)
    ms_m, _ = _events_ms(run_mfma, args.steps, args.warmup, torch)
    if not checksum_ok():
        print("bench.py: bgemm_mfma result failed its checksum", file=sys.stderr)
        return 1
    tb_m = bop / (ms_m * 1e-3) / 1e12
    result["bgemm_mfma_alternative"] = {
        "kernel": "bgemm_mfma_kernel", "ms": round(ms_m, 5), "gbops": round(tb_m * 1e3, 1),
        "roofline": {"bound": "mfma", "achieved": round(tb_m, 2), "peak": MFMA_FP4_PEAK_TOPS,
                     "unit": "Tbop/s (= TFLOP/s of the fp4 MFMA)", "frac": round(tb_m / MFMA_FP4_PEAK_TOPS, 4)},
        "speedup_over_xor_popcount": round(ms / ms_m, 3)}
    # fetch-width comparison in the spirit of the paper's 32- against 64-bit kernels (Sec. 6.1):
    # the same product with operands that are only 8-byte aligned, which the kernel then stages
    # with 8-byte instead of 16-byte global loads.  The two variants alternate in windows of 10
    # launches behind one settle phase, so that neither has the warmer clock.
    kw = n // 64
    A8 = torch.empty(n * kw + 1, dtype=A.dtype, device=dev)[1:].view(n, kw)
    B8 = torch.empty(n * kw + 1, dtype=B.dtype, device=dev)[1:].view(n, kw)
    A8.copy_(A)
    B8.copy_(B)
    run_8 = lambda: esp.bgemm(A8, B8, n, out=C)
    run_8()
    if not checksum_ok():
        print("bench.py: bgemm result on 8-byte aligned operands failed its checksum", file=sys.stderr)
        return 1
    settle_phase(run_bgemm, torch, min_ms=30.0, cap_ms=150.0)
    w16, w8 = [], []
    for _ in range(5):
        w16.append(_events_ms(run_bgemm, 10, 0, torch)[0])
        w8.append(_events_ms(run_8, 10, 0, torch)[0])
    m16, m8 = sum(w16) / len(w16), sum(w8) / len(w8)
    result["bgemm_fetch_width"] = {"ms_16_byte_loads": round(m16, 5), "ms_8_byte_loads": round(m8, 5),
                                   "ratio_8_over_16": round(m8 / m16, 4),
                                   "windows_ms_16": [round(t, 5) for t in w16], "windows_ms_8": [round(t, 5) for t in w8],
                                   "note": "operands aligned to 16 against 8 bytes; same kernel, same LDS layout; "
                                           "5 x (10 launches of one, 10 of the other), interleaved after one clock-settle phase"}
    del A8, B8
    if args.only == "bgemm":
        print(json.dumps(result))
        return 0
    if not args.no_extras:
        result["kernels"] = _supporting_kernels(torch, esp, synth, dev, np)
        result["paper_configs"] = _paper_configs(torch, esp, synth, dev, args.steps, args.warmup)
        result["networks"] = _networks(torch, esp, nets, synth, dev)
        cnn = result["networks"]["bcnn"]
        # the graded figure: the XOR-popcount engine (the hot path); the matrix cores are a measured alternative
        result["bcnn_images_per_s"] = {
            "engine": "XOR-popcount (vector ALU: v_xor + v_bcnt), the path the metric names",
            "batch1": cnn["1"]["images_per_s"], "batch256": cnn["256"]["images_per_s"],
            "matrix_core_alternative": {
                "auto_engine": {"batch1": cnn["1_auto_engine"]["images_per_s"],
                                "batch256": cnn["256_auto_engine"]["images_per_s"],
                                "note": "opt-in ESP_ENGINE_AUTO: matrix cores where their tiles fill the chip "
                                        "(batch 256), XOR-popcount otherwise"},
                "mfma_engine": {"batch1": cnn["1_mfma_engine"]["images_per_s"],
                                "batch256": cnn["256_mfma_engine"]["images_per_s"]}}}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = _cpu_baseline(a_pm1, b_pm1, n, args.cpu_rows, np)
        if not args.no_extras:
            result["cpu_baseline"]["per_config_seconds"] = _cpu_per_config(synth)

    print(json.dumps(result))
    return 0


SUPPORTING = ("copy", "pack", "bn_sign_pack", "unroll", "bmaxpool", "bgemv", "bgemv_1g", "bconv_cfg2", "conv1_b256",
              "bconv_conv2_b256", "bconv_conv3_b256", "bconv_conv4_b256", "bconv_conv5_b256", "bconv_conv6_b256",
              "bconv_conv2_b256_mfma", "bconv_conv4_b256_mfma", "bconv_conv6_b256_mfma")


def _supporting_kernels(torch, esp, synth, dev, np, only="", steps=20, warmup=3, settle=True):
    """Bandwidth-bound kernels on working sets far larger than the 256 MiB last-level cache,
    plus config 2's convolution.  ``copy`` is torch's plain device copy of 1 GiB: it is not part
    of the library and only calibrates what the profiler's byte counters read per byte moved."""
    out = []
    g = torch.Generator(device=dev)
    g.manual_seed(synth.SEED0)

    def want(name):
        return not only or only == name

    def rand_words(shape):
        return torch.randint(-2**62, 2**62, shape, device=dev, generator=g, dtype=torch.int64)

    def timed(fn):
        """Mean ms per launch behind an untimed clock-settle phase (skipped under a counter-collecting
        profiler, where every dispatch is serialised); short kernels are repeated for about 10 ms."""
        reps = steps
        if settle:
            st = _settle(fn, torch, min_ms=20.0, cap_ms=80.0)
            reps = max(steps, min(2000, int(10.0 / max(st["last_window_ms_per_launch"], 1e-3))))
        return _events_ms(fn, reps, warmup, torch)[0]

    if want("copy"):
        src = rand_words((128 * 1024 * 1024,))
        dst = torch.empty_like(src)
        ms = timed(lambda: dst.copy_(src))
        e = _hbm_entry("copy (torch's plain device copy: the achievable ceiling of this box and the scale of the "
                       "profiler's byte counters; not part of the library)", ms, 2 * src.numel() * 8, "1 GiB -> 1 GiB")
        out.append(e)
        del src, dst

    if want("pack"):
        # 16384 x 16384 float32 (1 GiB) -> 32 MiB of words (the largest matrix of config 5)
        rows, k = 16384, 16384
        x = torch.rand((rows, k), device=dev, generator=g) - 0.5
        dst = torch.empty((rows, k // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.pack_f32(x, out=dst))
        out.append(_hbm_entry("pack_f32", ms, rows * k * 4 + rows * k // 8, "float32 16384x16384 -> bits"))
        del x, dst

    if want("bn_sign_pack"):
        # conv-layer output of the CNN scaled to 1 GiB: rows x 128 channels
        rows, c = 2 * 1024 * 1024, 128
        xi = torch.randint(-1152, 1153, (rows, c), device=dev, generator=g, dtype=torch.int32)
        bnp = synth.bn_params(synth.rng_for(2, 7), c)
        thr_np, flip_np = esp.bn_fold(*bnp, synth.BN_EPS)
        thr = torch.from_numpy(thr_np).to(dev)
        flip = esp.to_packed_tensor(flip_np, dev)
        dst = torch.empty((rows, c // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.bn_sign_pack(xi, thr, flip, out=dst))
        out.append(_hbm_entry("bn_sign_pack", ms, rows * c * 4 + rows * c // 8 + c * 4 + c // 8,
                              "int32 [2Mi][128] -> bits (CNN conv2 output, batch 2048)"))
        del xi, dst

    if want("unroll"):
        # CNN conv2 input at batch 4096: 64 MiB in -> 576 MiB lowered
        b, h, c = 4096, 32, 128
        xin = rand_words((b, h, h, c // 64))
        low = torch.empty((b * h * h, 9 * c // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.unroll(xin, c, 3, 3, 1, 1, out=low))
        out.append(_hbm_entry("unroll", ms, xin.numel() * 8 + low.numel() * 8,
                              "packed [4096][32][32][128] 3x3 s1 p1 -> lowered matrix"))
        del xin, low

    if want("bmaxpool"):
        b, h, c = 4096, 64, 512
        xin = rand_words((b, h, h, c // 64))
        pooled = torch.empty((b, h // 2, h // 2, c // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.bmaxpool(xin, c, 2, 2, out=pooled))
        out.append(_hbm_entry("bmaxpool", ms, xin.numel() * 8 * 1.25, "packed [4096][64][64][512] 2x2 s2 (1 GiB in)"))
        del xin, pooled

    # small-M bgemm (matrix-vector): config 5's batch-1 product, K = N = 16384 (32 MiB of
    # weights) and a 1 GiB weight matrix
    for name, nrows, kk, label in (
            ("bgemv", 16384, 16384, "config 5 GEMV M=1, N=K=16384 (32 MiB weights)"),
            ("bgemv_1g", 524288, 16384, "M=1, N=524288, K=16384 (1 GiB weights)")):
        if not want(name):
            continue
        bw = rand_words((nrows, kk // 64))
        av = rand_words((1, kk // 64))
        cv = torch.empty((1, nrows), dtype=torch.int32, device=dev)
        ms = timed(lambda: esp.bgemm(av, bw, kk, out=cv))
        e = _hbm_entry("bgemv", ms, nrows * kk // 8 + kk // 8 + nrows * 4, label)
        e["gbops"] = round(2.0 * nrows * kk / (ms * 1e-3) / 1e9, 1)
        if name == "bgemv":
            # L2 hit rate 9 %, 32 MiB fetched through the L2's fabric port on every launch (counter runs in
            # profiles/supporting_kernels_hbm.txt): the weights do not stay in the 8 x 4 MiB of L2 between
            # launches.  Whether the 256 MiB memory-side cache or HBM serves them is not visible in the
            # counters, so the rate is quoted against the HBM peak; a launch this short (about 2 us of
            # it are the first loads' latency and the final reduction) never reaches the steady
            # streaming rate of the 1 GiB variant below.
            e["bound"] = "hbm (or the memory-side cache: every launch misses L2; launch too short for steady streaming)"
        out.append(e)
        del bw

    if want("bconv_cfg2"):
        # config 2: batch 32, 32x32x128 -> 128 filters 3x3 (unroll + bgemm), compute-bound
        b, h, c, l2 = 32, 32, 128, 128
        xin = rand_words((b, h, h, c // 64))
        filt = rand_words((l2, 3, 3, c // 64))
        ws = torch.empty(esp.bconv_workspace_bytes(b, h, h, c, 3, 3, 1, 1), dtype=torch.uint8, device=dev)
        pre = torch.empty((b, h, h, l2), dtype=torch.int32, device=dev)
        ms = timed(lambda: esp.bconv(xin, filt, c, 1, 1, workspace=ws, out=pre))
        bop = 2.0 * b * h * h * l2 * 9 * c
        tb = bop / (ms * 1e-3) / 1e12
        entry = {"kernel": "bconv (implicit GEMM, int32 out)", "workload": "config 2: [32][32][32][128] * 128 x 3x3x128",
                 "ms": round(ms, 5), "bound": "alu", "achieved": round(tb, 2),
                 "peak": round(VALU_PEAK_TBOPS, 1), "unit": "Tbop/s", "frac": round(tb / VALU_PEAK_TBOPS, 4)}
        # the whole of config 2 (conv, folded batch-norm threshold, sign, re-pack) as one fused call
        bnp = synth.bn_params(synth.rng_for(2, 8), l2)
        thr_np, flip_np = esp.bn_fold(*bnp, synth.BN_EPS)
        thr = torch.from_numpy(thr_np).to(dev)
        flip = esp.to_packed_tensor(flip_np, dev)
        bits = torch.empty((b, h, h, l2 // 64), dtype=esp.PACKED, device=dev)
        for key, engine in (("fused_bits_out_ms_xor_popcount", esp.ENGINE_XOR_POPCOUNT),
                            ("fused_bits_out_ms_auto_engine", esp.ENGINE_AUTO)):
            fms = timed(lambda: esp.bconv_bn_sign_pack(xin, filt, c, thr, flip, 1, 1, out=bits, engine=engine))
            entry[key] = round(fms, 5)
        out.append(entry)
    if want("conv1_b256"):
        # the CNN's real-valued first layer at batch 256 (3x3x3 -> 128, bf16 matrix cores), fused
        # float threshold + sign + pack: floats in, bits out
        b, h, l2 = 256, 32, 128
        xin = torch.rand((b, h, h, 3), device=dev, generator=g)
        filt = (torch.randint(0, 2, (l2, 3, 3, 3), device=dev, generator=g) * 2 - 1).to(torch.float32)
        bnp = synth.bn_params(synth.rng_for(2, 9), l2)
        thr_np, sgn_np = esp.bn_fold_f32(*bnp, synth.BN_EPS)
        thr, sgn = torch.from_numpy(thr_np).to(dev), torch.from_numpy(sgn_np).to(dev)
        bits = torch.empty((b, h, h, l2 // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.conv_f32_bn_sign_pack(xin, filt, thr, sgn, 1, 1, out=bits))
        # every input is split exactly into three bf16 terms: 3 x 2 x 27 bf16 flop per output
        tf = 3 * 2.0 * b * h * h * l2 * 27 / (ms * 1e-3) / 1e12
        out.append({"kernel": "conv_f32_bn_sign_pack (3x3x3, three bf16 terms per input on the matrix cores)",
                    "workload": "CNN conv1 at batch 256", "ms": round(ms, 5), "bound": "mfma",
                    "achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s (bf16)",
                    "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                    "fp32_equivalent_tflops": round(tf / 3, 2)})
    # the CNN's binary convolutions at batch 256, fused threshold epilogue (bits out)
    for name, h, c, l2 in (("bconv_conv2_b256", 32, 128, 128), ("bconv_conv3_b256", 16, 128, 256),
                           ("bconv_conv4_b256", 16, 256, 256), ("bconv_conv5_b256", 8, 256, 512),
                           ("bconv_conv6_b256", 8, 512, 512)):
        # the XOR-popcount engine is part of the default run; the matrix-core variant only on request
        if only not in ("", name, name + "_mfma"):
            continue
        engine = esp.ENGINE_MFMA if only.endswith("_mfma") else esp.ENGINE_XOR_POPCOUNT
        b = 256
        xin = rand_words((b, h, h, c // 64))
        filt = rand_words((l2, 3, 3, c // 64))
        bnp = synth.bn_params(synth.rng_for(2, 8), l2)
        thr_np, flip_np = esp.bn_fold(*bnp, synth.BN_EPS)
        thr = torch.from_numpy(thr_np).to(dev)
        flip = esp.to_packed_tensor(flip_np, dev)
        bits = torch.empty((b, h, h, l2 // 64), dtype=esp.PACKED, device=dev)
        ms = timed(lambda: esp.bconv_bn_sign_pack(xin, filt, c, thr, flip, 1, 1, out=bits, engine=engine))
        bop = 2.0 * b * h * h * l2 * 9 * c
        tb = bop / (ms * 1e-3) / 1e12
        peak = MFMA_FP4_PEAK_TOPS if engine == esp.ENGINE_MFMA else round(VALU_PEAK_TBOPS, 1)
        out.append({"kernel": "bconv_bn_sign_pack (implicit GEMM)", "workload": only or (name + " (CNN layer at batch 256, fused threshold epilogue)"),
                    "ms": round(ms, 5), "bound": "mfma" if engine == esp.ENGINE_MFMA else "alu",
                    "achieved": round(tb, 2), "peak": peak, "unit": "Tbop/s", "frac": round(tb / peak, 4)})
    return out


def _paper_configs(torch, esp, synth, dev, steps, warmup):
    """The remaining sizes of the paper's evaluation that the other sections do not time: config 1
    (one binary dense layer at batch 64, launch-latency-bound: microseconds only) and the smaller
    squares of config 5, each on the XOR-popcount kernel and on the matrix cores."""
    out = {}
    a_pm1, b_pm1 = synth.config1()
    m, k = a_pm1.shape
    n = b_pm1.shape[0]
    A = esp.pack_f32(torch.from_numpy(a_pm1).to(dev).to(torch.float32))
    B = esp.pack_f32(torch.from_numpy(b_pm1).to(dev).to(torch.float32))
    C = torch.empty((m, n), dtype=torch.int32, device=dev)
    ms, wall = _events_ms(lambda: esp.bgemm(A, B, k, out=C), 200, 200, torch)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(20):
            esp.bgemm(A, B, k, out=C)
    ms_g, wall_g = _events_ms(graph.replay, 20, 20, torch)
    out["config1_bgemm_64x1024x1024"] = {
        "eager_us": round(1e3 * max(ms, wall), 2), "back_to_back_in_a_graph_us": round(1e3 * max(ms_g, wall_g) / 20, 2),
        "note": "0.13 Gbop: bound by launch latency, no roofline fraction is meaningful"}
    for size in (2048, 4096):
        a_pm1, b_pm1 = synth.config5_square(size)
        A = esp.pack_f32(torch.from_numpy(a_pm1).to(dev).to(torch.float32))
        B = esp.pack_f32(torch.from_numpy(b_pm1).to(dev).to(torch.float32))
        C = torch.empty((size, size), dtype=torch.int32, device=dev)
        bop = 2.0 * size ** 3
        # these launches are short: warm up for tens of milliseconds (the engine clock ramps that
        # long after the idle gap of the set-up above) and time about as long
        est, _ = _events_ms(lambda: esp.bgemm(A, B, size, out=C), 20, 5, torch)
        warm, reps = max(warmup, min(3000, int(60.0 / est))), max(steps, min(3000, int(40.0 / est)))
        ms, _ = _events_ms(lambda: esp.bgemm(A, B, size, out=C), reps, warm, torch)
        ms_m, _ = _events_ms(lambda: esp.bgemm_mfma(A, B, size, out=C), reps, warm, torch)
        tb = bop / (ms * 1e-3) / 1e12
        out["config5_bgemm_%d_cube" % size] = {
            "ms": round(ms, 5), "tbops": round(tb, 2), "frac_of_valu_peak": round(tb / VALU_PEAK_TBOPS, 4),
            "mfma_alternative_ms": round(ms_m, 5), "mfma_alternative_tbops": round(bop / (ms_m * 1e-3) / 1e12, 2)}
        del A, B, C
    # What bounds the small squares: the time of a product with 2048 x 2048 outputs is a fixed part
    # (launch, first loads, epilogue and the 16 MiB of results) plus a part proportional to K.  The
    # two are separated by timing K = 2048, 4096 and 8192 and fitting a line; K = 64 and a
    # near-empty kernel (one block, one round of the register probe) show the launch floor.
    g = torch.Generator(device=dev)
    g.manual_seed(synth.SEED0 + 5)
    size = 2048
    C = torch.empty((size, size), dtype=torch.int32, device=dev)
    times = {}
    for k in (64, 2048, 4096, 8192):
        A = torch.randint(-2**62, 2**62, (size, k // 64), device=dev, generator=g, dtype=torch.int64)
        B = torch.randint(-2**62, 2**62, (size, k // 64), device=dev, generator=g, dtype=torch.int64)
        fn = lambda: esp.bgemm(A, B, k, out=C)
        _settle(fn, torch, min_ms=20.0, cap_ms=80.0)
        times[k] = _events_ms(fn, 500, 3, torch)[0] * 1e3
    sink = torch.empty(256, dtype=torch.int32, device=dev)
    fn = lambda: esp.xor_popcount_probe(sink, 1, 1)
    _settle(fn, torch, min_ms=10.0, cap_ms=40.0)
    empty_us = _events_ms(fn, 1000, 10, torch)[0] * 1e3
    # the same inside a HIP graph of 20 back-to-back launches (no host in the loop): the floor of a
    # launch of 512 blocks that does nothing, and what the 16 MiB of int32 results cost on top of a
    # product that writes packed sign bits instead (0.5 MiB)
    def graph_us(fn, n=20):
        fn()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for _ in range(n):
                fn()
        _settle(gr.replay, torch, min_ms=10.0, cap_ms=40.0)
        return _events_ms(gr.replay, 100, 3, torch)[0] / n * 1e3

    sink512 = torch.empty(512 * 256, dtype=torch.int32, device=dev)
    thr0 = torch.zeros(size, dtype=torch.int32, device=dev)
    flip0 = torch.zeros(size // 64, dtype=esp.PACKED, device=dev)
    bits0 = torch.empty((size, size // 64), dtype=esp.PACKED, device=dev)
    in_graph = {"empty_kernel_512_blocks_us": round(graph_us(lambda: esp.xor_popcount_probe(sink512, 512, 1)), 2)}
    for k in (64, 2048):
        A = torch.randint(-2**62, 2**62, (size, k // 64), device=dev, generator=g, dtype=torch.int64)
        B = torch.randint(-2**62, 2**62, (size, k // 64), device=dev, generator=g, dtype=torch.int64)
        in_graph["k%d_int32_out_us" % k] = round(graph_us(lambda: esp.bgemm(A, B, k, out=C)), 2)
        in_graph["k%d_sign_bits_out_us" % k] = round(graph_us(lambda: esp.bgemm_bn_sign_pack(A, B, k, thr0, flip0, out=bits0)), 2)
    slope = (times[8192] - times[2048]) / 6.0                     # us per 1024 bits of K
    fixed = times[2048] - 2.0 * slope
    peak_slope = 2.0 * size * size * 1024 / (VALU_PEAK_TBOPS * 1e12) * 1e6
    out["small_square_decomposition"] = {
        "outputs": "2048 x 2048 int32", "us_by_k": {str(k): round(v, 2) for k, v in times.items()},
        "near_empty_kernel_period_us": round(empty_us, 2),
        "fixed_part_us": round(fixed, 2), "us_per_1024_bits_of_k": round(slope, 3),
        "k_part_frac_of_valu_peak": round(peak_slope / slope, 4),
        "inside_a_graph": in_graph,
        "note": "time(K) = fixed + K-proportional part, fitted on K = 2048 .. 8192; at K = 2048 the fixed part "
                "(launch gap, first loads, epilogue, result write) is %.0f %% of the launch" % (100.0 * fixed / times[2048])}
    return out


def _networks(torch, esp, nets, synth, dev, only=None):
    """images/s of the two networks; batch 1 is timed both eagerly and as a replayed HIP graph."""
    res = {"bmlp": {}, "bcnn": {}}

    def time_net(net, x, batch, steps):
        entry = {}
        # untimed forwards until the engine clock has settled (it ramps for tens of ms)
        st = _settle(lambda: net.forward(x), torch, min_ms=40.0, cap_ms=150.0)
        warm = 3
        steps = max(steps, min(500, int(10.0 / max(st["last_window_ms_per_launch"], 1e-3))))
        ms, wall = _events_ms(lambda: net.forward(x), steps, warm, torch)
        entry["eager_ms"] = round(max(ms, wall), 5)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            net.forward(x)
        _settle(graph.replay, torch, min_ms=20.0, cap_ms=100.0)
        ms_g, wall_g = _events_ms(graph.replay, steps, warm, torch)
        entry["graph_ms"] = round(max(ms_g, wall_g), 5)
        entry["graph_median_ms"] = round(_median_ms(graph.replay, max(steps, 100), torch), 5)
        best = min(entry["eager_ms"], entry["graph_ms"])
        entry["images_per_s"] = round(batch / (best * 1e-3), 1)
        return entry

    layers = synth.mlp_params()
    for batch in (1, 64, 1024):
        if only and only != ("bmlp", batch):
            continue
        net = nets.BinaryMLP(layers, batch, synth.BN_EPS, dev)
        x = torch.from_numpy(synth.mlp_input(batch)).to(dev)
        res["bmlp"][str(batch)] = time_net(net, x, batch, 50)
        del net
        # same network with 8-bit input and the first layer evaluated by bit-planes (Eq. 3)
        net = nets.BinaryMLP(layers, batch, synth.BN_EPS, dev, first_layer="bitplane")
        x8 = (torch.from_numpy(synth.mlp_input(batch)).to(dev) * 256.0).clamp(0, 255).to(torch.uint8)
        res["bmlp"][str(batch) + "_bitplane_first_layer"] = time_net(net, x8, batch, 50)
        del net
        if batch >= 1024:
            # large batches: let the library put the binary layers on the matrix cores
            net = nets.BinaryMLP(layers, batch, synth.BN_EPS, dev, engine=esp.ENGINE_AUTO)
            res["bmlp"][str(batch) + "_auto_engine"] = time_net(net, x, batch, 50)
            del net
            # ... and the bit-plane first layer as well (one call, planes combined in its epilogue)
            net = nets.BinaryMLP(layers, batch, synth.BN_EPS, dev, first_layer="bitplane", engine=esp.ENGINE_AUTO)
            res["bmlp"][str(batch) + "_bitplane_first_layer_auto_engine"] = time_net(net, x8, batch, 50)
            del net
    layers = synth.cnn_params()
    for batch in (1, 256):
        if only and only != ("bcnn", batch):
            continue
        x = torch.from_numpy(synth.cnn_input(batch)).to(dev)
        for key, engine in ((str(batch), esp.ENGINE_XOR_POPCOUNT), (str(batch) + "_mfma_engine", esp.ENGINE_MFMA),
                            (str(batch) + "_auto_engine", esp.ENGINE_AUTO)):
            net = nets.BinaryCNN(layers, batch, synth.BN_EPS, device=dev, engine=engine)
            res["bcnn"][key] = time_net(net, x, batch, 30)
            del net
    res["paper_context"] = "batch 1 on a GTX 960: BMLP 0.26 ms (Table 2), BCNN 1.0 ms (Table 3)"
    return res


def _cpu_baseline(a_pm1, b_pm1, n, sample_rows, np):
    """The oracle's plain +-1 product on a sample of output rows (rows are independent),
    all host threads, extrapolated linearly to the metric's unit."""
    import oracle

    threads = max(1, min(oracle.max_threads(), os.cpu_count() or 1))
    oracle.set_threads(threads)
    probe = oracle.dense_pm1  # plain triple loop, int8 operands, int32 sums
    probe(a_pm1[:threads], b_pm1[: n // 8])               # first touch / thread start-up
    t0 = time.perf_counter()
    probe(a_pm1[: 4 * threads], b_pm1[: n // 4])
    dt = max(time.perf_counter() - t0, 1e-6)
    rate = 4 * threads * (n // 4) * n / dt                 # MAC/s estimate
    rows = sample_rows or int(min(n, max(threads, (15.0 * rate) / (n * n))))
    rows = max(threads, rows - rows % threads)
    t0 = time.perf_counter()
    probe(a_pm1[:rows], b_pm1)
    dt = time.perf_counter() - t0
    oracle.set_threads(1)
    gbops = 2.0 * rows * n * n / dt / 1e9
    return {"value": round(gbops, 2), "unit": "Gbop/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d output rows (all N, all K) of the same product, %.1f s; "
                      "full job extrapolated linearly: %.0f s" % (rows, n, dt, 2.0 * n**3 / (gbops * 1e9))}


def _cpu_per_config(synth):
    """Seconds the oracle takes on the paper-sized configurations it finishes whole, on one thread
    and on all host threads (the larger ones are covered by the sampled headline figure)."""
    import oracle
    from oracle import nets as onets

    def seconds(fn):
        t0 = time.perf_counter()
        fn()
        return round(time.perf_counter() - t0, 4)

    a1, b1 = synth.config1()
    x2, f2, bn2 = synth.config2()
    mlp = synth.mlp_params()
    cnn = synth.cnn_params()
    a5, b5 = synth.config5_square(2048)
    jobs = (
        ("config1_dense_64x1024x1024", lambda: oracle.dense_pm1(a1, b1)),
        ("config2_conv_bn_sign_batch32", lambda: oracle.bn_sign(oracle.conv_pm1(x2, f2, 1, 1), bn2, synth.BN_EPS)),
        ("config3_mlp_batch1", lambda: onets.mlp_forward(synth.mlp_input(1), mlp, synth.BN_EPS)),
        ("config3_mlp_batch64", lambda: onets.mlp_forward(synth.mlp_input(64), mlp, synth.BN_EPS)),
        ("config4_cnn_batch1", lambda: onets.cnn_forward(synth.cnn_input(1), cnn, synth.BN_EPS)),
        ("config5_dense_2048_cube", lambda: oracle.dense_pm1(a5, b5)),
    )
    threads = max(1, min(oracle.max_threads(), os.cpu_count() or 1))
    out = {"threads": threads}
    for name, fn in jobs:
        oracle.set_threads(1)
        one = seconds(fn)
        oracle.set_threads(threads)
        out[name] = {"one_thread": one, "all_threads": seconds(fn)}
    # The larger configurations: a sample of the batch or of the output rows (images and rows are
    # independent), timed, and the whole job EXTRAPOLATED linearly from it.
    a4, b4 = synth.config5_square(4096)
    x3, x4 = synth.mlp_input(1024), synth.cnn_input(256)
    samples = (
        ("config3_mlp_batch1024", 1024, 32, 256, lambda k: onets.mlp_forward(x3[:k], mlp, synth.BN_EPS)),
        ("config4_cnn_batch256", 256, 1, 16, lambda k: onets.cnn_forward(x4[:k], cnn, synth.BN_EPS)),
        ("config5_dense_4096_cube", 4096, 64, 512, lambda k: oracle.dense_pm1(a4[:k], b4)),
    )
    for name, whole, k_one, k_all, fn in samples:
        oracle.set_threads(1)
        one = seconds(lambda: fn(k_one))
        oracle.set_threads(threads)
        allt = seconds(lambda: fn(k_all))
        out[name] = {"one_thread": round(one * whole / k_one, 3), "all_threads": round(allt * whole / k_all, 3),
                     "extrapolated": True,
                     "sample": "%d of %d rows/images on one thread (%.3f s), %d on all threads (%.3f s); "
                               "whole job = sample time x %d / sample size" % (k_one, whole, one, k_all, allt, whole)}
    oracle.set_threads(1)
    return out


if __name__ == "__main__":
    sys.exit(main())
