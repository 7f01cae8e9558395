#!/usr/bin/env python3
"""Throughput of the contraction on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3] [--no-tune] [--no-cpu]

One "step" is one call of the library on one batch of synthetic input: shape split,
tile-config selection, operand staging, MFMA inner product and epilogue.  The default
workload is the fp32 GEMM M=N=K=4096 (entries N(0,1)/64, seed 2); inputs are resident in
HBM before the timed region.  Prints ONE JSON line on stdout; everything else goes to
stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published dense peaks of the part (TFLOP/s), by the arithmetic type of the contraction
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_HBM_GBS = 8000.0
METRIC = "TFLOP/s and % of MI355X matrix peak, fp32 GEMM 4096^3 (1 GPU)"

# HBM bytes per launch of the dominant kernel, from two `rocprofv3 --pmc` passes
# (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch) scaled by what the same counters read
# for a plain 256 MiB device copy in the same run; the summaries are under profiles/.
# An entry is reported only while the kernel sources still hash to the value it was taken
# with and the launch uses the same tile config; otherwise `traffic` is null.
TRAFFIC = {
    1: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 16, "bn": 16, "bk": 64, "wm": 16, "wn": 16, "vec": 4, "sched": 1, "split_k": 1, "split_tail": 0, "mfma": 1}, "bytes": 2981485, "source": "profiles/gemm_f32_256.txt"}],
    2: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 64, "bn": 64, "bk": 64, "wm": 32, "wn": 32, "vec": 4, "raster": 0, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 42108508, "source": "profiles/gemm_f32_transA_1024.txt"},
        {"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 64, "bn": 64, "bk": 64, "wm": 32, "wn": 32, "vec": 4, "raster": 1, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 29527140, "source": "profiles/gemm_f32_transA_1024.txt"}],
    3: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 256, "bn": 256, "bk": 16, "wm": 128, "wn": 64, "vec": 4, "raster": 0, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 719853268, "source": "profiles/gemm_f32_4096.txt"},
        {"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 256, "bn": 256, "bk": 16, "wm": 128, "wn": 64, "vec": 4, "raster": 1, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 470069052, "source": "profiles/gemm_f32_4096.txt"}],
    4: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 112, "bn": 64, "bk": 64, "wm": 112, "wn": 16, "vec": 4, "raster": 1, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 1}, "bytes": 14324840, "source": "profiles/conv2d_f32_8x56x56x64.txt"},
        {"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 112, "bn": 64, "bk": 64, "wm": 112, "wn": 16, "vec": 4, "raster": 0, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 1}, "bytes": 20517259, "source": "profiles/conv2d_f32_8x56x56x64.txt"}],
    5: [{"kernel_hash": "1dda433397d07fd1", "tile": {"bm": 256, "bn": 256, "bk": 32, "wm": 128, "wn": 64, "vec": 8, "raster": 1, "sched": 5, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 1887849981, "source": "profiles/gemm_bf16_8192_negate.txt"},
        {"kernel_hash": "1dda433397d07fd1", "tile": {"bm": 256, "bn": 256, "bk": 32, "wm": 128, "wn": 64, "vec": 8, "raster": 0, "sched": 5, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 1880683579, "source": "profiles/gemm_bf16_8192_negate.txt"}],
    6: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 64, "bn": 64, "bk": 32, "wm": 32, "wn": 32, "vec": 4, "sched": 4, "split_k": 5, "split_tail": 0, "mfma": 0}, "bytes": 91766100, "source": "profiles/gemm_f32_batched_196x256x2305.txt"}],
    7: [{"kernel_hash": "ad97f1a93881e1ca", "tile": {}, "bytes": 1073704569, "source": "profiles/reduce_sum_f32_1gib.txt"}],
    8: [{"kernel_hash": "1dda433397d07fd1", "tile": {"bm": 64, "bn": 64, "bk": 64, "wm": 32, "wn": 32, "vec": 8, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 15995806, "source": "profiles/conv2d_bf16_8x56x56x64.txt"}],
    9: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 256, "bn": 256, "bk": 16, "wm": 128, "wn": 64, "vec": 4, "raster": 0, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 671356715, "source": "profiles/gemm_f32_both_transposed_4096.txt"},
        {"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 256, "bn": 256, "bk": 16, "wm": 128, "wn": 64, "vec": 4, "raster": 1, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 0}, "bytes": 470040369, "source": "profiles/gemm_f32_both_transposed_4096.txt"}],
    10: [{"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 112, "bn": 64, "bk": 64, "wm": 112, "wn": 16, "vec": 4, "raster": 0, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 1}, "bytes": 27123352, "source": "profiles/conv2d_f32_window_accumulate.txt"},
        {"kernel_hash": "3c08264ebc31e41c", "tile": {"bm": 112, "bn": 64, "bk": 64, "wm": 112, "wn": 16, "vec": 4, "raster": 1, "sched": 4, "split_k": 1, "split_tail": 0, "mfma": 1}, "bytes": 20930914, "source": "profiles/conv2d_f32_window_accumulate.txt"}],
    11: [{"kernel_hash": "ad97f1a93881e1ca", "tile": {}, "bytes": 805369830, "source": "profiles/reduce_sum_f32_view_of_short_rows.txt"}],
}


def kernel_hash(dtype: str, op: str = "") -> str:
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2409_03864_amd", "csrc")
    # the sources a kernel is built from: both element types share one skeleton
    h.update(dtype.encode() if op != "reduce_sum" else b"")
    for f in ("tsg_internal.h",) + (("reduce.hip",) if op == "reduce_sum" else ("gemm_kernel.h", "gemm_elem.h")):
        with open(os.path.join(csrc, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def traffic_bytes(k: int, dtype: str, tile: dict, op: str = ""):
    """(bytes per launch, the summary under profiles/ they were taken from), or (None, None)."""
    for e in TRAFFIC.get(k, ()):
        if e["kernel_hash"] == kernel_hash(dtype, op) and all(tile.get(key) == val for key, val in e["tile"].items()):
            return e["bytes"], e.get("source")
    return None, None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def workload_flops(c) -> int:
    """Algorithmic flop count: 2 per multiply-add; convolution taps that fall in the zero
    padding are not work.  The reduce does one add per element."""
    if c["op"] == "reduce_sum":
        return c["rows"] * c["cols"]
    if c["op"] != "conv2d_nhwc":
        return 2 * c.get("B", 1) * c["M"] * c["N"] * c["K"]

    def valid(L, Kk, s, p):
        Lo = (L + 2 * p - Kk) // s + 1
        return sum(1 for o in range(Lo) for t in range(Kk) if 0 <= o * s + t - p < L)

    return (2 * c["N"] * valid(c["H"], c["KH"], c["stride"], c["pad"]) *
            valid(c["W"], c["KW"], c["stride"], c["pad"]) * c["Cin"] * c["Cout"])


def describe(k, c) -> str:
    if c["op"] == "reduce_sum":
        return "cfg%d: %s full additive reduce of a %d x %d %s, %s entries, seed %d" % (
            k, c["dtype"], c["rows"], c["cols"], "view with row pitch %d" % c["ld"] if "ld" in c else "tensor",
            c["dist"], c["seed"])
    if c["op"] == "conv2d_nhwc":
        return ("cfg%d: %s conv2d NHWC N=%d H=W=%d Cin=%d Cout=%d %dx%d stride %d pad %d, seed %d%s"
                % (k, c["dtype"], c["N"], c["H"], c["Cin"], c["Cout"], c["KH"], c["KW"], c["stride"], c["pad"],
                   c["seed"], ", added into the interior of a tensor with a ring of %d pixels" % c["window_ring"]
                   if c.get("window_ring") else ""))
    return "cfg%d: %s %s %sM=%d N=%d K=%d, %s entries, seed %d%s" % (
        k, c["dtype"], c["op"], "batch=%d " % c["B"] if "B" in c else "", c["M"], c["N"], c["K"], c["dist"], c["seed"],
        ", negate fused" if "negate" in c["flags"] else "")


def result_record(k, c, mnk, steps, warmup, wall_s, kernel_ms_avg, tile, alternative, tuned, graph, cpu, search):
    """The one JSON object of a run: a couple of kilobytes at most, so that a harness which
    keeps only the tail of stdout still holds all of it.  The tuner's evaluated points are not
    part of it (they go to stderr and, with --tuner-log, to a file)."""
    M, N, K = mnk
    flops = workload_flops(c)
    hbm_bound = c["op"] == "reduce_sum"
    step_s = wall_s / steps
    if hbm_bound:
        # bound by HBM: algorithmic bytes = every element read once (the 4-byte result is noise)
        work, unit, peak, scale = c["rows"] * c["cols"] * 4, "GB/s", PEAK_HBM_GBS, 1e9
    else:
        work, unit, peak, scale = flops, "TFLOP/s", PEAK_TFLOPS[c["dtype"]], 1e12
    value = work / step_s / scale
    achieved = work / (kernel_ms_avg * 1e-3) / scale
    traffic, source = traffic_bytes(k, c["dtype"], {} if hbm_bound else tile, c["op"])
    roofline = {"bound": "hbm" if hbm_bound else "mfma", "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": traffic,
                # `traffic` is not measured by this run: it is the stored figure of two counter passes over
                # this kernel (file named here), reported only while sources and tile config still match
                "traffic_source": source,
                # HBM rate those bytes amount to at this run's launch time
                "hbm_gbs": None if traffic is None else traffic / (kernel_ms_avg * 1e-3) / 1e9,
                "kernel_ms_avg": kernel_ms_avg, "kernel_hash": kernel_hash(c["dtype"], c["op"])}
    out = {
        "metric": METRIC if k == 3 else ("GB/s and % of MI355X HBM peak, " if hbm_bound else
                                         "TFLOP/s and % of MI355X matrix peak, ") + describe(k, c),
        "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": step_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c["dtype"], "data": "synthetic",
        "pct_of_peak": 100.0 * value / peak,
        "config": {"workload": describe(k, c), "M": M, "N": N, "K": K, "flops_per_step": flops,
                   "tile_config": tile, "alternative": alternative, "tuned": tuned, "hip_graph": graph},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if search is not None:
        out["search"] = search
    return out


# Products the cost model's constants were NOT fitted on (they were fitted on workloads 1 - 6)
HELD_OUT = [(512, 512, 512, False), (768, 768, 768, False), (1536, 1536, 1536, False), (2048, 2048, 2048, False),
            (3072, 1024, 4096, False), (1000, 1000, 1000, False), (2048, 2048, 2048, True), (384, 8192, 640, False)]


def search_report(tsg, torch, dev) -> int:
    """For each held-out shape: exhaustive search in cost-model order (the reference), then what a
    budget of 8 timed points finds in cost-model order and in the model-based order.  One JSON
    line per shape: rank of the model's first pick among all timed points, its time over the best,
    Spearman rank correlation of predicted and measured times, evaluations until within 1 % of the
    best in both orders."""
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    tsg.workspace_set(ws)
    for M, N, K, trans in HELD_OUT:
        import synth
        a, b = synth.gemm_inputs(M, N, K, seed=100, dist="uniform", trans_a=trans)
        A, B = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
        C = torch.zeros((M, N), dtype=torch.float32, device=dev)
        lda = M if trans else K
        iters = 5 if 2.0 * M * N * K >= 1e10 else 30

        def tune(budget, order):
            tsg.tune_cache_clear()
            tsg.search_set(budget, order)
            best, ms, recs = tsg.autotune_gemm(tsg.F32, trans, M, N, K, A, lda, B, N, C, N, iters=iters, log_cap=4096)
            return ms, [r for r in recs if r.ms >= 0]

        best_ms, timed = tune(0, 1)
        ranked = sorted(r.ms for r in timed)
        first = timed[0].ms
        # Spearman correlation of the two orders over the timed points
        n = len(timed)
        by_pred = sorted(range(n), key=lambda i: timed[i].predicted_ms)
        by_meas = sorted(range(n), key=lambda i: timed[i].ms)
        rp, rm = [0] * n, [0] * n
        for rank, i in enumerate(by_pred):
            rp[i] = rank
        for rank, i in enumerate(by_meas):
            rm[i] = rank
        rho = 1.0 - 6.0 * sum((a - b) ** 2 for a, b in zip(rp, rm)) / (n * (n * n - 1.0))
        reach1 = next(i + 1 for i, r in enumerate(timed) if r.best_ms <= best_ms * 1.01)
        ms_b1, t1 = tune(8, 1)
        ms_b2, t2 = tune(8, 2)
        full2_ms, timed2 = tune(0, 2)
        reach2 = next(i + 1 for i, r in enumerate(timed2) if r.best_ms <= full2_ms * 1.01)   # (of its own final best, like reach1)
        print(json.dumps({"probe": "search_report", "shape": [M, N, K], "trans_a": trans, "timed_points": n,
                          "best_ms": round(best_ms, 5), "model_first_pick_ms": round(first, 5),
                          "first_pick_over_best": round(first / best_ms, 4),
                          "first_pick_rank": 1 + sum(1 for v in ranked if v < first),
                          "spearman_pred_vs_measured": round(rho, 3),
                          "evals_to_1pct_model_order": reach1, "evals_to_1pct_adaptive_order": reach2,
                          "budget8_model_order_over_best": round(ms_b1 / best_ms, 4),
                          "budget8_adaptive_order_over_best": round(ms_b2 / best_ms, 4)}), flush=True)
    tsg.search_set(0, 1)
    tsg.tune_cache_clear()
    tsg.workspace_set(None)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 100, or as many as make the timed region last 0.2 s)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default: a tenth of --steps)")
    ap.add_argument("--workload", type=int, default=3, choices=list(range(1, 12)))
    ap.add_argument("--no-tune", action="store_true", help="use the shape heuristic instead of the tuner")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--graph", action="store_true",
                    help="record the K steps once into a HIP graph and time one replay (launch-bound workloads)")
    ap.add_argument("--evals", type=int, default=0, help="tuner budget: timed points, in cost-model order (0 = all)")
    ap.add_argument("--tuner-log", default="", metavar="PATH",
                    help="write the tuner's evaluated points (time, prediction, best so far) to this JSON file")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the product the oracle is timed on")
    ap.add_argument("--pin", default="", help="bm,bn,bk,wm,wn,vec,raster,sched[,split_k[,split_tail[,mfma]]]: pin this tile config instead of tuning")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="instead of a workload, run the register-only MFMA loops (practical ceiling of the matrix "
                         "pipes per dtype, block shape and operand values) and print one line per loop")
    ap.add_argument("--search-report", action="store_true",
                    help="instead of a workload, tune fp32 products of shapes the cost model was not fitted on and "
                         "print, per shape, how the model's order compares with the measured one")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one plain device copy of this many MiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this library runs on ONE GPU; --gpus %d is not supported "
            "(rows of C are independent, so more GPUs would each take a panel of A with no exchange)." % args.gpus)
        return 2

    import numpy as np
    import torch

    import synth
    import paper_2409_03864_amd as tsg

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.mfma_ceiling:
        sink = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        for dtype, name, peak in ((tsg.F32, "f32", PEAK_TFLOPS["f32"]), (tsg.BF16_F32ACC, "bf16", PEAK_TFLOPS["bf16"])):
            for mfma, shape in ((0, "32x32x2" if dtype == tsg.F32 else "32x32x16"),
                                (1, "16x16x4" if dtype == tsg.F32 else "16x16x32")):
                for rnd in (0, 1):
                    for wps in (1, 2):
                        best, sustained = tsg.mfma_ceiling(dtype, mfma, rnd, wps, 20, sink)
                        # at full issue a CU retires 256 fp32 / 4096 bf16 flop per cycle: the rate is a clock
                        ghz = sustained * 1e12 / (256 * (256 if dtype == tsg.F32 else 4096)) / 1e9
                        print(json.dumps({"probe": "mfma_ceiling", "dtype": name, "mfma": shape,
                                          "operands": "N(0,1)/90.5" if rnd else "constant 0.5", "waves_per_simd": wps,
                                          "tflops_best": round(best, 1), "tflops_sustained": round(sustained, 1),
                                          "frac_of_peak": round(sustained / peak, 4),
                                          "effective_ghz": round(ghz, 3)}), flush=True)
        print(json.dumps({"probe": "launch_floor", "launches": 20000,
                          "us_per_launch": round(tsg.launch_floor(20000), 3)}), flush=True)
        return 0

    if args.search_report:
        return search_report(tsg, torch, dev)

    k = args.workload
    t0 = time.time()
    c, a, b = synth.config_inputs(k)
    log("inputs generated in %.1f s: %s" % (time.time() - t0, describe(k, c)))
    dt = tsg.F32 if c["dtype"] == "f32" else tsg.BF16_F32ACC
    flags = (tsg.NEGATE if "negate" in c["flags"] else 0) | (tsg.ACCUMULATE if "accumulate" in c["flags"] else 0)

    def up(x):
        x = np.ascontiguousarray(x)
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).to(dev)

    dA = up(a)
    dB = up(b) if b is not None else None
    # device memory for the split of the k loop (used by shapes whose tiles cannot fill the chip)
    workspace = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    tsg.workspace_set(workspace)
    # raw addresses and the stream handle are taken once: the timed loop then costs one
    # foreign call per step, which matters for the kernels that run a few microseconds
    st = torch.cuda.current_stream().cuda_stream
    pA = dA.data_ptr()
    pB = dB.data_ptr() if dB is not None else 0
    if c["op"] == "reduce_sum":
        M, N, K = c["rows"], c["cols"], 1
        op = None
        dC = torch.zeros((1,), dtype=torch.float32, device=dev)
        pC = dC.data_ptr()

        ld = c.get("ld", N)

        def step():
            tsg.reduce_sum(dt, M, N, pA, ld, pC, flags, st)

        args.no_tune = True      # one kernel form, nothing to search
    elif c["op"] == "conv2d_nhwc":
        Ho = (c["H"] + 2 * c["pad"] - c["KH"]) // c["stride"] + 1
        dC = torch.zeros((c["N"], Ho, Ho, c["Cout"]), dtype=torch.float32, device=dev)
        geom = (c["N"], c["H"], c["W"], c["Cin"], c["Cout"], c["KH"], c["KW"], c["stride"], c["stride"],
                c["pad"], c["pad"])
        op = tsg.OP_CONV2D_NHWC
        M, N, K = c["N"] * Ho * Ho, c["Cout"], c["KH"] * c["KW"] * c["Cin"]

        pC = dC.data_ptr()
        ring = c.get("window_ring", 0)
        if ring:
            # y is the interior of a larger tensor: the call adds into it in place
            big = torch.zeros((c["N"], Ho + 2 * ring, Ho + 2 * ring, c["Cout"]), dtype=torch.float32, device=dev)
            sw_ = c["Cout"]
            sh_ = (Ho + 2 * ring) * sw_
            sn_ = (Ho + 2 * ring) * sh_
            pW = big.data_ptr() + 4 * (ring * sh_ + ring * sw_)

            def step():
                tsg.conv2d_nhwc_window(dt, *geom, pA, pB, pW, sn_, sh_, sw_, flags, st)
        else:
            def step():
                tsg.conv2d_nhwc(dt, *geom, pA, pB, pC, flags, st)

        def tune():   # the window only changes where the epilogue writes: the layer's tuning serves both
            return tsg.autotune_conv2d_nhwc(dt, *geom, dA, dB, dC, flags, iters=tune_iters)
    elif c["op"] == "gemm_batched":
        nb, M, N, K = c["B"], c["M"], c["N"], c["K"]
        op = tsg.OP_GEMM
        dC = torch.zeros((nb, M, N), dtype=torch.float32, device=dev)

        pC = dC.data_ptr()

        def step():
            tsg.gemm_batched(dt, False, nb, M, N, K, pA, K, M * K, pB, N, K * N, pC, N, M * N, flags, st)

        def tune():
            return tsg.autotune_gemm_batched(dt, False, nb, M, N, K, dA, K, M * K, dB, N, K * N, dC, N, M * N,
                                             flags, iters=tune_iters)
    elif c["op"] == "gemm_trans":
        M, N, K = c["M"], c["N"], c["K"]
        op = tsg.OP_GEMM_TRANSA
        dC = torch.zeros((M, N), dtype=torch.float32, device=dev)
        pC = dC.data_ptr()

        def step():
            tsg.gemm_trans(dt, True, True, 1, M, N, K, pA, M, 0, pB, K, 0, pC, N, 0, flags, st)

        def tune():
            return tsg.autotune_gemm_trans(dt, True, True, 1, M, N, K, dA, M, 0, dB, K, 0, dC, N, 0, flags,
                                           iters=tune_iters)
    else:
        M, N, K = c["M"], c["N"], c["K"]
        trans = c["op"] == "gemm_transA"
        op = tsg.OP_GEMM_TRANSA if trans else tsg.OP_GEMM
        dC = torch.zeros((M, N), dtype=torch.float32, device=dev)
        lda = M if trans else K
        fn = tsg.gemm_transA if trans else tsg.gemm

        pC = dC.data_ptr()

        def step():
            fn(dt, M, N, K, pA, lda, pB, N, pC, N, flags, st)

        def tune():
            return tsg.autotune_gemm(dt, trans, M, N, K, dA, lda, dB, N, dC, N, flags, iters=tune_iters)

    if args.copy_calibration:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)            # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        log("copy calibration: one device copy of %d MiB (reads and writes that many bytes)" % args.copy_calibration)
        del src, dst

    # enough back-to-back calls per timed batch that a batch lasts about a millisecond
    tune_iters = 5 if workload_flops(c) >= 1e11 else 50
    tuner_log = None
    search = None
    if args.pin:
        v = [int(t) for t in args.pin.split(",")]
        tsg.tile_config_set(op, dt, tsg.TileConfig(bm=v[0], bn=v[1], bk=v[2], wm=v[3], wn=v[4], vec=v[5], raster=v[6], sched=v[7],
                                                   split_k=(v[8] if len(v) > 8 else 1),
                                                   split_tail=(v[9] if len(v) > 9 else 0),
                                                   mfma=(v[10] if len(v) > 10 else 0)))
        args.no_tune = True
    if not args.no_tune:
        tsg.search_set(args.evals, True)
        best, best_ms, recs = tune()
        tuner_log = [dict(r.config.as_dict(), ms=round(r.ms, 5), predicted_ms=round(r.predicted_ms, 5),
                          best_so_far_ms=round(r.best_ms, 5)) for r in recs]
        timed = [r for r in recs if r.ms >= 0]
        # the first timed point is the cost model's pick, i.e. what a call without tuning uses
        # how many points, in the cost model's order, it took to get within 1 % of the final best
        reach = next(i + 1 for i, r in enumerate(timed) if r.best_ms <= best_ms * 1.01)
        search = {"evaluations": len(timed), "default_ms": timed[0].ms, "best_ms": best_ms,
                  "speedup_vs_default": timed[0].ms / best_ms, "evaluations_to_within_1pct": reach}
        for r in recs:
            log("  tuner: %s -> %.4f ms (best so far %.4f)" % (r.config, r.ms, r.best_ms))
        log("tuner picked %s at %.4f ms" % (best, best_ms))

    # A step of the small workloads takes tens of microseconds, and the first few milliseconds
    # after an idle period run at a lower clock: unless the caller fixes the count, time enough
    # steps for 0.2 s
    for _ in range(20):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        step()
    torch.cuda.synchronize()
    est = (time.perf_counter() - t0) / 20
    if args.steps is None:
        args.steps = max(100, min(1000 if args.graph else 20000, int(0.2 / est)))
    if args.warmup is None:
        args.warmup = max(10, args.steps // 10)
    # The tuner's report above left the GPU idle for a while.  Whatever W is, bring the clock back up
    # first with 0.1 s of untimed steps, and go into the W warmup steps without a gap.
    for _ in range(max(1, min(5000, int(0.1 / est)))):
        step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # whole-step wall clock, and device time of the K launches between two events recorded
    # on the stream the kernels are launched on
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    if args.graph:
        # the library only enqueues kernels on the stream it is given, so a call can be recorded;
        # the K steps become one graph and the timed region is one replay of it
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        st = side.cuda_stream
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(args.steps):
                    step()
            graph.replay()            # untimed first replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(side):
            e0.record()
            graph.replay()
            e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        e0.record()
        for _ in range(args.steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    li = tsg.last_launch()
    avg_kern_ms = e0.elapsed_time(e1) / args.steps

    flops = workload_flops(c)
    ms_per_step = wall * 1e3 / args.steps
    hbm_bound = c["op"] == "reduce_sum"
    if hbm_bound:
        # bound by HBM: algorithmic bytes = every element read once (the 4-byte result is noise)
        nbytes = c["rows"] * c["cols"] * 4
        unit, peak = "GB/s", PEAK_HBM_GBS
        value = nbytes / (wall / args.steps) / 1e9
        achieved = nbytes / (avg_kern_ms * 1e-3) / 1e9
    else:
        unit, peak = "TFLOP/s", PEAK_TFLOPS[c["dtype"]]
        value = flops / (wall / args.steps) / 1e12
        achieved = flops / (avg_kern_ms * 1e-3) / 1e12
    log("step %.4f ms wall, %.4f ms per launch between stream events: %.2f %s = %.1f%% of %.1f"
        % (ms_per_step, avg_kern_ms, achieved, unit, 100 * achieved / peak, peak))

    cpu = None
    if not args.no_cpu:
        import oracle
        if c["op"] == "reduce_sum":
            sub = np.ascontiguousarray(a[:min(M, 65536), :N])
            t0 = time.perf_counter()
            oracle.reduce_sum(sub)
            dtc = time.perf_counter() - t0
            cpu = {"value": sub.size * 4 / dtc / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                   "sample": "rows 0..%d (%d elements, fp64 sum)" % (sub.shape[0] - 1, sub.size),
                   "seconds": round(dtc, 3)}
        elif c["op"] == "conv2d_nhwc":
            t0 = time.perf_counter()
            oracle.conv2d_nhwc(a, b, stride=(c["stride"],) * 2, pad=(c["pad"],) * 2, with_s=False)
            dtc = time.perf_counter() - t0
            sflops, sample = flops, "the whole layer, all %d images (direct convolution)" % c["N"]
        else:
            rows = min(args.cpu_rows, M)
            a0, b0 = (a[0], b[0]) if c["op"] == "gemm_batched" else (a, b)
            ta, tb = c["op"] in ("gemm_transA", "gemm_trans"), c["op"] == "gemm_trans"
            sub = np.ascontiguousarray(a0[:, :rows] if ta else a0[:rows])
            t0 = time.perf_counter()
            oracle.gemm(sub, b0, trans_a=ta, trans_b=tb, with_s=False)
            dtc = time.perf_counter() - t0
            sflops, sample = 2 * rows * N * K, "rows 0..%d of C%s (%d x %d x %d triple loop)" % (
                rows - 1, " of batch 0" if c["op"] == "gemm_batched" else "", rows, N, K)
        if cpu is None:
            cpu = {"value": sflops / dtc / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
                   "sample": sample, "seconds": round(dtc, 3)}
        log("cpu oracle: %s in %.2f s on %d threads = %.4f %s" % (cpu["sample"], dtc, cpu["cores"], cpu["value"],
                                                                  cpu["unit"]))

    out = result_record(k, c, (M, N, K), args.steps, args.warmup, wall, avg_kern_ms,
                        None if hbm_bound else li.config.as_dict(), None if hbm_bound else int(li.alternative),
                        not args.no_tune, bool(args.graph), cpu, search)
    if tuner_log is not None and args.tuner_log:
        # the evaluated points with the best-so-far time after each (the curve of Fig. 11)
        with open(args.tuner_log, "w") as fh:
            json.dump({"workload": describe(k, c), "points": tuner_log}, fh)
        log("tuner log: %d points written to %s" % (len(tuner_log), args.tuner_log))
    sys.stderr.flush()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
