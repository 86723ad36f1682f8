#!/usr/bin/env python3
"""Benchmark of the BiQGEMM lookup-table multiply on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one biq_gemm call (tables built in LDS, keys streamed, partials reduced, alpha
applied) on one batch of synthetic input already resident in HBM.  The headline workload is
the batch-1 GEMV configuration (m = n = 2048, q = 2, mu = 8); consecutive steps use different
packed weight matrices (more than 512 MiB in rotation) so that keys come from HBM, not from a
cache.  The roofline object is measured on the same kernel with the same n, q, mu and batch
but m scaled until the keys are 512 MiB per call: at the literal size a call moves 1 MiB and
is bounded by launch latency, not by any memory system.  One JSON line is printed at the end.
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

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(msg: str) -> None:
    print("[bench] " + msg, file=sys.stderr, flush=True)


class Problem:
    """Device buffers of one workload; `copies` packed weight matrices used in rotation."""

    def __init__(self, biq, torch, w, copies: int, real_first: bool = True, plan=None, x_values: str = "fp32"):
        self.w = w
        dev = torch.device("cuda:0")
        self.key_bytes_padded = biq.biq_packed_bytes(w.m, w.n, w.q)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        # iid uniform bytes are iid uniform +-1 signs, 8 per byte
        self.K = torch.randint(0, 256, (copies, self.key_bytes_padded), dtype=torch.uint8, device=dev,
                               generator=gen)
        if real_first:
            from paper_2005_09904_amd.workloads import make_inputs

            B, alpha, X = make_inputs(w)
            self.host = (B, alpha, X)
            Bd = torch.from_numpy(B).to(dev)
            biq.biq_pack(Bd, self.K[0], w.m, w.n, w.q, w.mu)
            del Bd
            self.alpha = torch.from_numpy(alpha).to(dev)
            self.X = torch.from_numpy(X).to(dev)
        else:
            self.host = None
            self.alpha = torch.rand((w.q, w.m), device=dev, generator=gen) * 0.95 + 0.05
            self.X = torch.randn((w.batch, w.n), device=dev, generator=gen)
        if x_values == "fp16":      # fp32 inputs whose values came from half-precision arithmetic
            self.X = self.X.half().float()
        elif x_values == "bf16":
            self.X = self.X.bfloat16().float()
        self.Y = torch.zeros((w.batch, w.m), dtype=torch.float32, device=dev)
        ws_bytes = biq.biq_workspace_bytes(w.m, w.n, w.q, w.batch, w.mu)
        if plan is not None:
            ws_bytes = max(ws_bytes, biq.biq_plan_workspace_bytes(
                biq.biq_plan_check(w.m, w.n, w.q, w.batch, w.mu, plan), w.m, w.batch))
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.copies = copies
        self.biq = biq
        self.calls = 0
        # one marshalled call per key matrix in the rotation: a step is then one C-ABI call
        self.prepared = [biq.PreparedGemm(self.K[i], self.alpha, self.X, self.Y, w.m, w.n, w.q, w.batch,
                                          w.mu, workspace=self.ws, plan=plan) for i in range(copies)]

    def step(self):
        self.prepared[self.calls % self.copies]()
        self.calls += 1

    def touch_all(self, torch):
        """One untimed call on every key matrix of the rotation (first use of a buffer is not what
        a step is meant to measure), then back to the start of the rotation."""
        for call in self.prepared:
            call()
        torch.cuda.synchronize()
        self.calls = 0


class Timing:
    """Per-call times over the timed regions of one workload: every region is exactly `steps`
    calls between two HIP events on the stream the kernels run on, with a synchronisation on both
    sides.  median / min / mean are over the regions' (event time / steps); `wall` is the host
    clock around the first region / steps (it includes the cost of the synchronisation itself)."""

    def __init__(self, per_region, wall):
        self.regions = len(per_region)
        self.median = float(sorted(per_region)[len(per_region) // 2])
        self.min = float(min(per_region))
        self.mean = float(sum(per_region) / len(per_region))
        self.wall = wall

    def as_dict(self):
        return {"median_us": self.median * 1e6, "min_us": self.min * 1e6, "mean_us": self.mean * 1e6,
                "wall_us_first_region": self.wall * 1e6, "regions": self.regions}


def time_steps(torch, prob: Problem, steps: int, warmup: int, regions: int = 9) -> Timing:
    """`warmup` untimed calls, then `regions` timed regions of exactly `steps` calls each.  One
    region is what the command line asks for; the repetitions give the median and the minimum."""
    for _ in range(warmup):
        prob.step()
    torch.cuda.synchronize()
    per_region = []
    wall = None
    for _ in range(regions):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            prob.step()
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if wall is None:
            wall = (t1 - t0) / steps
        per_region.append(e0.elapsed_time(e1) * 1e-3 / steps)
    return Timing(per_region, wall)


def summarize(w, t: Timing):
    """Rates of one workload from the median per-call time (min and mean beside it)."""
    sec = t.median
    row = {
        "workload": w.name,
        "m": w.m, "n": w.n, "q": w.q, "batch": w.batch, "mu": w.mu,
        "us_per_call": sec * 1e6,
        "min_us_per_call": t.min * 1e6,
        "mean_us_per_call": t.mean * 1e6,
        "wall_us_per_call_first_region": t.wall * 1e6,
        "timed_regions": t.regions,
        "algorithmic_bytes": w.algorithmic_bytes,
        "achieved_GBps": w.algorithmic_bytes / sec / 1e9,
        "hbm_frac": w.algorithmic_bytes / sec / 1e9 / HBM_PEAK_GBPS,
        "weight_GBps": w.key_bytes / sec / 1e9,
        "effective_GOPS": w.dense_equiv_ops / sec / 1e9,
        "lookups_per_s": w.lookups / sec,
    }
    return row


def read_profiled_traffic(algorithmic_bytes: int):
    """HBM bytes per launch of the roofline kernel from the committed counter summary
    (profiles/gemv8_q2_hbm_regime_counters.md: two rocprofv3 --pmc runs, scaled by a copy of known
    size), with the commit it was profiled at.  None if the summary is missing or is for another
    workload: the figure is a profile's, not something this run measures."""
    import re

    path = os.path.join(ROOT, "profiles", "gemv8_q2_hbm_regime_counters.md")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m_traffic = re.search(r"traffic_bytes_per_launch:\s*(\d+)", text)
    m_algo = re.search(r"algorithmic_bytes_per_launch:\s*(\d+)", text)
    m_commit = re.search(r"profiled_at_commit:\s*([0-9a-f]{7,40})", text)
    if not (m_traffic and m_algo) or int(m_algo.group(1)) != algorithmic_bytes:
        return None, None
    return float(m_traffic.group(1)), (m_commit.group(1) if m_commit else None)


def cpu_baseline(w, host_inputs, budget_s: float = 8.0):
    """The oracle as it stands, single thread, fp64, timed on this host on the whole headline
    workload: its lookup-table path (Algorithm 2) and its dense definition (Eq. 2)."""
    import numpy as np
    import oracle

    B, alpha, X = host_inputs
    keys = oracle.pack_keys(B, w.mu)

    def median_time(fn):
        t0 = time.perf_counter()
        fn()
        first = time.perf_counter() - t0
        reps = int(max(3, min(200, budget_s / max(first, 1e-6))))
        times = []
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            times.append(time.perf_counter() - t0)
        return float(np.median(times)), reps

    lut_s, lut_reps = median_time(lambda: oracle.gemm_lut(keys, alpha, X, w.mu))
    dense_s, dense_reps = median_time(lambda: oracle.gemm_dense(B, alpha, X))
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {
        "value": w.algorithmic_bytes / lut_s / 1e9,
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "whole %s workload: oracle gemm_lut (Algorithm 2, fp64), median of %d calls; "
                  "oracle gemm_dense (Eq. 2, fp64) beside it, median of %d calls" % (w.name, lut_reps, dense_reps),
        "us_per_call": lut_s * 1e6,
        "gemm_lut_us_per_call": lut_s * 1e6,
        "gemm_dense_us_per_call": dense_s * 1e6,
        "gemm_dense_GBps": w.algorithmic_bytes / dense_s / 1e9,
        "host_cpu": cpu_model,
        "host_cores_total": os.cpu_count(),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--only", choices=["all", "headline", "roofline", "copy"], default="all",
                    help="restrict the run to one timed region (used for profiling); 'copy' runs a "
                         "plain 512 MiB device copy, the calibration kernel for HBM byte counters")
    ap.add_argument("--workload", default=None,
                    help="time only this named configuration (for profiling), e.g. cfg4_sq4096_q3_b32")
    ap.add_argument("--mu", type=int, default=0, help="with --workload: LUT-unit to use instead of the workload's")
    ap.add_argument("--m", type=int, default=0, help="with --workload: number of output rows instead of the workload's "
                                                     "(the batch-1 bandwidth family scales m)")
    ap.add_argument("--batch", type=int, default=0, help="with --workload: number of input vectors instead of the workload's")
    ap.add_argument("--plan", choices=["default", "lut", "mfma2"], default="default",
                    help="with --workload: the library's plan, its choice among the lookup-table kernels only, or "
                         "the matrix-core kernel with two input terms (on request only: plan.input_terms = 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        return 2

    import torch

    import paper_2005_09904_amd as biq
    from dataclasses import replace

    from paper_2005_09904_amd.workloads import CONFIGS, Workload

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    biq.load_library()  # raises if libbiq.so is missing: there is no fallback
    torch.cuda.set_device(0)

    if args.only == "copy":
        # calibration for rocprofv3 FETCH_SIZE / WRITE_SIZE: reads and writes exactly 512 MiB
        src = torch.randint(0, 256, (512 * 1024 * 1024,), dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": src.numel(), "copies": 10}))
        return 0

    if args.workload:
        w = CONFIGS[args.workload]
        if args.mu:
            w = w.with_mu(args.mu)
        if args.m:
            w = w.scaled_m(args.m)
        if args.batch:
            w = replace(w, batch=args.batch, name="%s_b%d" % (w.name, args.batch))
        plan = (biq.biq_plan_get_lut(w.m, w.n, w.q, w.batch, w.mu) if args.plan == "lut" else
                biq.biq_plan_get_mfma(w.m, w.n, w.q, w.batch, w.mu, 2) if args.plan == "mfma2" else None)
        copies = max(1, min(64, (512 * 1024 * 1024) // w.key_bytes + 1))
        p = Problem(biq, torch, w, copies, real_first=False, plan=plan)
        steps = min(args.steps, 200 if w.lookups < 1e9 else 50)
        p.touch_all(torch)
        srow = summarize(w, time_steps(torch, p, steps, 5))
        srow["plan"] = (plan or biq.biq_plan_get(w.m, w.n, w.q, w.batch, w.mu)).as_dict()
        srow["kernel"] = biq.biq_kernel_name(srow["plan"]["kernel"])
        print(json.dumps(srow))
        return 0

    head = CONFIGS["cfg2_gemv2048_q2_b1"]
    out = {}
    extra = []

    # ---- headline: literal GEMV b=1 configuration, keys cold (rotation > 512 MiB) -------------
    head_sum = None
    prob = None
    if args.only in ("all", "headline"):
        copies = (512 * 1024 * 1024) // head.key_bytes + 1
        prob = Problem(biq, torch, head, copies)
        prob.touch_all(torch)
        cold = time_steps(torch, prob, args.steps, args.warmup)
        head_sum = summarize(head, cold)
        head_sum["keys"] = "cold: %d packed matrices in rotation, each used once before the warm-up" % copies
        log("headline %s (cold keys): median %.2f us/call, min %.2f, mean %.2f over %d regions of %d calls; "
            "host clock of the first region %.2f" %
            (head.name, cold.median * 1e6, cold.min * 1e6, cold.mean * 1e6, cold.regions, args.steps, cold.wall * 1e6))
        # same buffers every call: keys served from cache
        warm = Problem(biq, torch, head, 1)
        wt = time_steps(torch, warm, args.steps, args.warmup)
        head_sum["warm_keys"] = wt.as_dict()
        log("headline %s (warm keys): median %.2f us/call, min %.2f" % (head.name, wt.median * 1e6, wt.min * 1e6))
        del warm

    # ---- roofline: same kernel, m scaled until keys are 512 MiB per call ----------------------
    roof = None
    if args.only in ("all", "roofline"):
        big = head.scaled_m(head.m * 512, "cfg2_shape_m1048576_hbm_regime")
        pb = Problem(biq, torch, big, 2, real_first=False)
        rsteps = max(20, min(200, args.steps // 10))
        pb.touch_all(torch)
        rt = time_steps(torch, pb, rsteps, 5)
        launch_s = rt.median
        plan = biq.biq_plan_get(big.m, big.n, big.q, big.batch, big.mu)
        traffic, traffic_commit = read_profiled_traffic(big.algorithmic_bytes)
        roof = {
            "bound": "hbm",
            "achieved": big.algorithmic_bytes / launch_s / 1e9,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": big.algorithmic_bytes / launch_s / 1e9 / HBM_PEAK_GBPS,
            # from profiles/gemv8_q2_hbm_regime_counters.md (rocprofv3 FETCH_SIZE / WRITE_SIZE scaled
            # by a copy of known size), not measured in this run
            "traffic": traffic,
            "traffic_source": ("profiles/gemv8_q2_hbm_regime_counters.md @ %s" % traffic_commit) if traffic else None,
            "kernel": biq.biq_kernel_name(plan.kernel),
            "workload": big.name,
            "algorithmic_bytes_per_launch": big.algorithmic_bytes,
            "launch_us": launch_s * 1e6,
            "launch_us_min": rt.min * 1e6,
            "launch_us_mean": rt.mean * 1e6,
            "launches_timed": rsteps,
        }
        log("roofline %s: %.1f us/launch, %.0f GB/s (%.1f%% of HBM peak)" %
            (big.name, roof["launch_us"], roof["achieved"], 100 * roof["frac"]))
        del pb
        torch.cuda.empty_cache()
        if head_sum is not None:
            roof["literal_headline"] = {
                "workload": head.name,
                "achieved": head_sum["achieved_GBps"],
                "frac": head_sum["hbm_frac"],
                "launch_us": head_sum["us_per_call"],
                "note": "1 MiB of keys per call: bounded by launch latency, not by HBM",
            }

    # ---- the other configurations (context rows) ------------------------------------------------
    if args.only == "all":
        LDS_PEAK_GBPS = 256 * 128 * 2.4  # 256 CUs x 128 B/clk x 2.4 GHz
        rows = [CONFIGS[k] for k in ["cfg1_fc512_b1", "cfg3_lstm4096x1024_q3_b8", "cfg4_sq4096_q3_b32",
                                     "cfg5_ffn_up_q2_b128", "cfg5_ffn_down_q2_b128"]]
        rows += [CONFIGS["cfg5_ffn_up_q2_b128"].with_mu(6), CONFIGS["cfg5_ffn_up_q2_b128"].with_mu(4)]
        MFMA_F16_PEAK_TFLOPS = 2500.0
        for w in rows:
            default = biq.biq_plan_get(w.m, w.n, w.q, w.batch, w.mu)
            lut = biq.biq_plan_get_lut(w.m, w.n, w.q, w.batch, w.mu)
            # the library's choice first; where that is the unpack + MFMA kernel (exact input
            # split), the lookup-table kernel on the same inputs as a second row and the two-term
            # variant of the matrix-core kernel, which only an explicit plan selects, as a third
            plans = [(None, "fp32")]
            if default.kernel != lut.kernel:
                plans += [(lut, "fp32"), (biq.biq_plan_get_mfma(w.m, w.n, w.q, w.batch, w.mu, 2), "fp32")]
                if w.mu == 8:
                    # the library's plan again on fp32 inputs that hold fp16 / bf16 values (activations
                    # computed in half precision): the exact split has zero third (and second) terms
                    # there and the kernel skips them
                    plans += [(None, "fp16"), (None, "bf16"),
                              (biq.biq_plan_get_mfma(w.m, w.n, w.q, w.batch, w.mu, 2), "fp16")]
            for plan, x_values in plans:
                kname = biq.biq_kernel_name((plan or default).kernel)
                terms = (plan or default).input_terms
                copies = max(1, min(64, (512 * 1024 * 1024) // w.key_bytes + 1))
                p = Problem(biq, torch, w, copies, real_first=False, plan=plan, x_values=x_values)
                steps = 200 if w.lookups < 1e9 else 20
                p.touch_all(torch)
                t = time_steps(torch, p, steps, 5)
                s = summarize(w, t)
                s["input_values"] = x_values
                s["key_copies_in_rotation"] = copies
                s["kernel"] = kname
                s["default_plan"] = plan is None
                if kname == "unpack_mfma":
                    # dense contraction: 2 flop per weight and input vector, times the 16-bit
                    # terms of x (3 bf16: exact; 2 fp16: on request), on columns padded to the
                    # 32-wide MFMA tile
                    padded = -(-w.batch // 32) * 32
                    s["input_terms"] = terms
                    s["mfma_TFLOPs"] = 2.0 * terms * w.q * w.m * w.n * padded / t.median / 1e12
                    s["mfma_frac"] = s["mfma_TFLOPs"] / MFMA_F16_PEAK_TFLOPS
                    if terms == 2 and x_values == "fp32":
                        kname = "unpack_mfma, 2 input terms"
                    elif x_values != "fp32":
                        kname = "unpack_mfma%s, %s-valued inputs" % (", 2 input terms" if terms == 2 else "", x_values)
                        del s["mfma_TFLOPs"], s["mfma_frac"]    # fewer terms are executed than counted above
                elif w.batch > 1:
                    # batched table lookups are bounded by gathers from LDS (4 bytes per lookup)
                    s["lds_gather_GBps"] = 4.0 * w.lookups / t.median / 1e9
                    s["lds_frac"] = s["lds_gather_GBps"] / LDS_PEAK_GBPS
                extra.append(s)
                log("%s [%s]: %.2f us/call, %.1f GB/s, %.0f GOPS" % (w.name, kname, s["us_per_call"],
                                                                   s["achieved_GBps"], s["effective_GOPS"]))
                del p
                torch.cuda.empty_cache()
        # the paper's own GPU grid (Table IV: square matrices, one bit-plane, mu = 8), with the
        # run times it prints for a V100 beside ours: another machine, context only
        PAPER_V100_US = {(512, 1): 4, (512, 32): 11, (512, 128): 30, (512, 256): 58,
                         (1024, 1): 4, (1024, 32): 20, (1024, 128): 70, (1024, 256): 135,
                         (2048, 1): 5, (2048, 32): 47, (2048, 128): 175, (2048, 256): 330,
                         (4096, 1): 7, (4096, 32): 130, (4096, 128): 528, (4096, 256): 1005}
        grid = []
        for (nn, bb), v100 in PAPER_V100_US.items():
            w = Workload("table4_%d_b%d" % (nn, bb), nn, nn, 1, bb, 8, "uniform")
            default = biq.biq_plan_get(nn, nn, 1, bb, 8)
            lut = biq.biq_plan_get_lut(nn, nn, 1, bb, 8)
            row = {"n": nn, "batch": bb, "paper_v100_us": v100}
            for tag, plan in (("us", None), ("lut_us", lut if default.kernel != lut.kernel else None)):
                if tag == "lut_us" and plan is None:
                    continue
                copies = max(2, min(64, (256 * 1024 * 1024) // w.key_bytes + 1))
                p = Problem(biq, torch, w, copies, real_first=False, plan=plan)
                steps = 200 if bb <= 32 else 50
                p.touch_all(torch)
                row[tag] = time_steps(torch, p, steps, 5).median * 1e6
                row["kernel" if tag == "us" else "lut_kernel"] = biq.biq_kernel_name((plan or default).kernel)
                del p
                torch.cuda.empty_cache()
            grid.append(row)
            log("table IV %4d^2 b=%-3d: %7.2f us [%s]%s   (paper, V100: %d us)" %
                (nn, bb, row["us"], row["kernel"],
                 "  tables only: %.2f us" % row["lut_us"] if "lut_us" in row else "", v100))
        out["paper_table4_grid"] = grid
        # quantiser front end (Eq. 1, greedy): fp32 W -> packed signs + scales, HBM bound
        quant = []
        for (m, n, q) in [(4096, 4096, 3), (16384, 4096, 2), (4096, 16384, 2)]:
            Wd = torch.randn((m, n), device="cuda")
            Kq = torch.empty(biq.biq_packed_bytes(m, n, q), dtype=torch.uint8, device="cuda")
            aq = torch.empty((q, m), device="cuda")
            for _ in range(3):
                biq.biq_quantize(Wd, Kq, aq, m, n, q)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 20
            for _ in range(reps):
                biq.biq_quantize(Wd, Kq, aq, m, n, q)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            nbytes = 4 * m * n + q * m * n // 8 + 4 * q * m
            quant.append({"m": m, "n": n, "q": q, "us_per_call": dt * 1e6, "algorithmic_bytes": nbytes,
                          "achieved_GBps": nbytes / dt / 1e9, "hbm_frac": nbytes / dt / 1e9 / HBM_PEAK_GBPS})
            log("quantize %dx%d q=%d: %.1f us, %.0f GB/s (%.1f%% of HBM peak)" %
                (m, n, q, dt * 1e6, nbytes / dt / 1e9, 100 * nbytes / dt / 1e9 / HBM_PEAK_GBPS))
            del Wd, Kq, aq
            torch.cuda.empty_cache()
        out["quantize"] = quant
        # key packing (a1): int8 signs -> bit stream, HBM read bound (1 byte in, 1 bit out per weight)
        packs = []
        for (m, n, q) in [(4096, 4096, 3), (16384, 4096, 2)]:
            Bd = (torch.randint(0, 2, (q, m, n), dtype=torch.int8, device="cuda") * 2 - 1)
            Kp = torch.empty(biq.biq_packed_bytes(m, n, q), dtype=torch.uint8, device="cuda")
            for _ in range(3):
                biq.biq_pack(Bd, Kp, m, n, q, 8)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 20
            for _ in range(reps):
                biq.biq_pack(Bd, Kp, m, n, q, 8)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            nbytes = q * m * n + q * m * n // 8
            packs.append({"m": m, "n": n, "q": q, "us_per_call": dt * 1e6, "algorithmic_bytes": nbytes,
                          "achieved_GBps": nbytes / dt / 1e9, "hbm_frac": nbytes / dt / 1e9 / HBM_PEAK_GBPS})
            log("pack %dx%d q=%d: %.1f us, %.0f GB/s (%.1f%% of HBM peak)" %
                (m, n, q, dt * 1e6, nbytes / dt / 1e9, 100 * nbytes / dt / 1e9 / HBM_PEAK_GBPS))
            del Bd, Kp
            torch.cuda.empty_cache()
        out["pack"] = packs
        # tables to device memory (biq_build_lut, the unfused a2 step): HBM write bound
        luts = []
        for (n, b, mu) in [(4096, 32, 8), (4096, 128, 8), (4096, 128, 4)]:
            Xd = torch.randn((b, n), device="cuda")
            nbytes = biq.biq_lut_bytes(n, b, mu)
            Ld = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
            for _ in range(3):
                biq.biq_build_lut(Xd, Ld, n, b, mu)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 50
            for _ in range(reps):
                biq.biq_build_lut(Xd, Ld, n, b, mu)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            luts.append({"n": n, "batch": b, "mu": mu, "us_per_call": dt * 1e6, "lut_bytes": nbytes,
                         "achieved_GBps": (nbytes + 4 * n * b) / dt / 1e9,
                         "hbm_frac": (nbytes + 4 * n * b) / dt / 1e9 / HBM_PEAK_GBPS})
            log("build_lut n=%d b=%d mu=%d: %.1f us, %.0f GB/s written" % (n, b, mu, dt * 1e6, nbytes / dt / 1e9))
            del Xd, Ld
            torch.cuda.empty_cache()
        out["build_lut"] = luts
        # Table build methods (end of Sec. III-B): every entry from pair sums (table_fill 0, the default)
        # against the order of Algorithm 1 (table_fill 1), on launches that are all table build: 8 rows
        # per workgroup, 16 and 32 tiles per workgroup; the slope is the cost of one more 128 KiB tile.
        fill = {}
        for tf in (0, 1):
            per = {}
            for tiles in (16, 32):
                w = Workload("table_fill_%d_tiles_%d" % (tf, tiles), 2048, 1024 * tiles, 1, 1, 8, "uniform")
                plan = biq.BiqPlan()
                plan.kernel, plan.threads, plan.chunks_per_tile, plan.batch_tile = 1, 1024, 128, 1
                plan.tiles_per_split, plan.rows_per_wg, plan.table_fill = tiles, 8, tf
                p = Problem(biq, torch, w, 2, real_first=False, plan=biq.biq_plan_check(w.m, w.n, 1, 1, 8, plan))
                per[tiles] = time_steps(torch, p, 100, 10).median * 1e6
                del p
            fill["algorithm1_order" if tf else "pair_sums"] = {
                "us_16_tiles": per[16], "us_32_tiles": per[32], "us_per_tile": (per[32] - per[16]) / 16}
            log("table fill %s: %.2f us per 128 KiB tile (16 tiles %.1f us, 32 tiles %.1f us)" %
                ("Algorithm 1 order" if tf else "pair sums", (per[32] - per[16]) / 16, per[16], per[32]))
        out["table_fill_study"] = fill
        # LUT-unit sweep on the FFN up-projection with the lookup-table kernels only, one and 128 input
        # vectors: what mu costs on this chip (Sec. IV-A's rule counts operations, not table bytes)
        sweep = []
        for bb in (1, 128):
            for mu in (4, 6, 8, 9, 10):
                w = replace(CONFIGS["cfg5_ffn_up_q2_b128"], batch=bb, mu=mu, name="cfg5_ffn_up_q2_b%d_mu%d" % (bb, mu))
                plan = biq.biq_plan_get_lut(w.m, w.n, w.q, w.batch, w.mu)
                p = Problem(biq, torch, w, 4, real_first=False, plan=plan)
                t = time_steps(torch, p, 20, 3, regions=5)
                sweep.append({"batch": bb, "mu": mu, "kernel": biq.biq_kernel_name(plan.kernel),
                              "us_per_call": t.median * 1e6})
                log("mu sweep batch %d mu %d [%s]: %.1f us" % (bb, mu, sweep[-1]["kernel"], t.median * 1e6))
                del p
                torch.cuda.empty_cache()
        out["mu_sweep_lut_kernels"] = sweep
        # small layers that do not depend on each other, L = 8 per dispatch (grouped launch) against the
        # same 8 as separate calls; and the LSTM cell step with its update fused (cfg 3's shape)
        class Calls:
            def __init__(self, fns):
                self.fns = fns

            def step(self):
                for fn in self.fns:
                    fn()

        grouped = []
        for name in ["cfg1_fc512_b1", "cfg2_gemv2048_q2_b1", "cfg3_lstm4096x1024_q3_b8"]:
            w = CONFIGS[name]
            L = 8
            probs = [Problem(biq, torch, replace(w, seed=w.seed + 1000 * i), 1, real_first=False) for i in range(L)]
            group = biq.PreparedGroup([(p.K[0], p.alpha, p.X, p.Y, w.m, w.n, w.q, w.batch) for p in probs], w.mu)
            tg = time_steps(torch, Calls([group]), 200, 20)
            ts = time_steps(torch, Calls([p.prepared[0] for p in probs]), 200, 20)
            grouped.append({"workload": w.name, "layers_per_dispatch": L,
                            "grouped_us_per_layer": tg.median * 1e6 / L, "grouped_us_per_call": tg.median * 1e6,
                            "separate_us_per_layer": ts.median * 1e6 / L})
            log("grouped %s x %d: %.2f us per layer in one dispatch, %.2f us per layer as separate calls" %
                (w.name, L, tg.median * 1e6 / L, ts.median * 1e6 / L))
            del probs, group
            torch.cuda.empty_cache()
        out["grouped_launch"] = grouped
        w = CONFIGS["cfg3_lstm4096x1024_q3_b8"]
        hid = w.m // 4
        pl = Problem(biq, torch, w, 1, real_first=False)
        bias = torch.zeros(w.m, device="cuda")
        cprev = torch.randn((w.batch, hid), device="cuda")
        hout, cout = torch.empty_like(cprev), torch.empty_like(cprev)
        tl = time_steps(torch, Calls([biq.PreparedLstmCell(pl.K[0], pl.alpha, bias, pl.X, cprev, hout, cout, hid,
                                                           w.n, w.q, w.batch, w.mu)]), 200, 20)
        tgm = time_steps(torch, pl, 200, 20)
        out["lstm_cell"] = {"hidden": hid, "n": w.n, "q": w.q, "batch": w.batch,
                            "fused_cell_us_per_step": tl.median * 1e6, "biq_gemm_alone_us": tgm.median * 1e6}
        log("lstm cell step (hidden %d, n %d, q %d, batch %d): %.2f us fused; biq_gemm alone %.2f us" %
            (hid, w.n, w.q, w.batch, tl.median * 1e6, tgm.median * 1e6))
        del pl
        torch.cuda.empty_cache()
        # the same small calls as nodes of a HIP graph: 16 consecutive calls (16 key matrices) captured
        # once and replayed, against the same 16 calls issued one by one (the library allocates nothing
        # and records no memset nodes, so its calls can be captured)
        replay = []
        side = torch.cuda.Stream()
        for name in ["cfg1_fc512_b1", "cfg2_gemv2048_q2_b1", "cfg3_lstm4096x1024_q3_b8", "cfg4_sq4096_q3_b32"]:
            w = CONFIGS[name]
            L = 16
            with torch.cuda.stream(side):
                pr = Problem(biq, torch, w, L, real_first=False)
                te = time_steps(torch, Calls(pr.prepared), 20, 3, regions=5)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    for call in pr.prepared:
                        call()
                tr = time_steps(torch, Calls([graph.replay]), 20, 3, regions=5)
            replay.append({"workload": w.name, "calls_per_graph": L, "eager_us_per_call": te.median * 1e6 / L,
                           "graph_replay_us_per_call": tr.median * 1e6 / L})
            log("hip graph %s: %.2f us per call replayed (%d calls per graph), %.2f us issued one by one" %
                (w.name, tr.median * 1e6 / L, L, te.median * 1e6 / L))
            del graph, pr
            torch.cuda.empty_cache()
        out["hip_graph_replay"] = replay
        # the batch-1 bandwidth family: cfg 2's shape with m scaled by powers of two (the launch-latency
        # knee), and the FFN matrices of cfg 5 with one input vector; cold keys, median per call
        fam = []
        family = [head.scaled_m(head.m << k) for k in range(0, 10)]
        family += [replace(CONFIGS["cfg5_ffn_up_q2_b128"], batch=1, name="cfg5_ffn_up_q2_b1"),
                   replace(CONFIGS["cfg5_ffn_down_q2_b128"], batch=1, name="cfg5_ffn_down_q2_b1")]
        for w in family:
            copies = max(2, min(64, (512 * 1024 * 1024) // w.key_bytes + 1))
            p = Problem(biq, torch, w, copies, real_first=False)
            steps = 200 if w.key_bytes < (64 << 20) else 30
            p.touch_all(torch)
            t = time_steps(torch, p, steps, 5)
            s = summarize(w, t)
            plan = biq.biq_plan_get(w.m, w.n, w.q, w.batch, w.mu)
            fam.append({"workload": w.name, "m": w.m, "n": w.n, "key_bytes": w.key_bytes, "us_per_call": s["us_per_call"],
                        "min_us_per_call": s["min_us_per_call"], "achieved_GBps": s["achieved_GBps"],
                        "hbm_frac": s["hbm_frac"], "kernel": biq.biq_kernel_name(plan.kernel),
                        "dispatches": 2 if plan.chunk_splits > 1 else 1})
            log("family %s: %.2f us/call (min %.2f), %.0f GB/s = %.1f%% of HBM peak [%s]" %
                (w.name, s["us_per_call"], s["min_us_per_call"], s["achieved_GBps"], 100 * s["hbm_frac"],
                 fam[-1]["kernel"]))
            del p
            torch.cuda.empty_cache()
        out["gemv_b1_family"] = fam

    cpu = None
    if not args.no_cpu_baseline and prob is not None and prob.host is not None:
        cpu = cpu_baseline(head, prob.host)
        log("cpu oracle on 1 core (%s): gemm_lut %.0f us/call, gemm_dense %.0f us/call" %
            (cpu["host_cpu"], cpu["gemm_lut_us_per_call"], cpu["gemm_dense_us_per_call"]))

    value = head_sum["achieved_GBps"] if head_sum else (roof["achieved"] if roof else None)
    ms_per_step = head_sum["us_per_call"] / 1e3 if head_sum else (roof["launch_us"] / 1e3 if roof else None)
    line = {
        "metric": "biq_gemm achieved HBM GB/s (algorithmic bytes / median time per call), GEMV b=1",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": head.name,
            "m": head.m, "n": head.n, "q": head.q, "batch": head.batch, "mu": head.mu,
            "keys": "cold: %d packed matrices in rotation" % (prob.copies if prob else 0),
            "timing": "9 regions of exactly `steps` calls each, every region between two HIP events and two "
                      "synchronisations; ms_per_step and value are the median over the regions, min / mean / "
                      "host clock of the first region are in `headline`",
        },
        "headline": head_sum,
        "roofline": roof,
        "cpu_baseline": cpu,
        "workloads": extra,
    }
    line.update(out)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
