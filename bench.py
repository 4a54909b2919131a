#!/usr/bin/env python3
"""Benchmark of the LiquidQuant W4A8 GEMM on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-curve] [--no-cpu]

A step is one pass of the whole hot path (load packed W4 + group parameters, unpack,
LiquidQuant dequantisation, INT8 MFMA, per-token x per-channel scaling, FP16 store) over
one batch of synthetic activations, with every input already resident in HBM.  Weights
rotate through enough distinct copies (> 512 MB in total) that the 256 MB Infinity Cache
cannot serve them.  The headline workload is the compute-bound end of the metric's M
range (prefill, M=4096, N=K=8192, group 64); the same JSON line carries the TOPS-vs-M
curve (M = 1..4096), the HBM-bound point (70B up-projection at M=16), the roofline of
the dominant kernel and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, published
PEAK_INT8_TOPS = 5033.0   # dense INT8 MFMA: 256 CU x 4 SIMD x 2048 ops/clk x 2.4 GHz
ROTATE_BYTES = 512 << 20
# HBM-side bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE counter runs of this file
# (scaled by what the same counters read for a plain 1 GiB copy, --copy-ref); the commands
# and raw figures are in profiles/.  Counters cannot be read from inside a timed run, so
# the figure is carried here per (workload, kernel) and is null for anything not profiled.
MEASURED_TRAFFIC_BYTES = {
    ("prefill_M4096_N8192_K8192", "duo_m128"): 477.6e6,
    ("l70b_up_M16_N28672_K8192", "stream16_f2_w4"): 123.3e6,
}


def algorithmic_bytes(M, N, K, g):
    """Bytes the method must move once: packed codes + group parameters + X + Y + scales."""
    return N * K // 2 + 2 * N * K // g + M * K + 2 * M * N + 4 * N + 4 * M


def algorithmic_ops(M, N, K):
    return 2 * M * N * K


class DeviceProblem:
    """Packed weights of one shape in `copies` distinct device buffers + activations."""

    def __init__(self, shape, Ms, torch, api, WL):
        self.shape = shape
        N, K, g = shape.N, shape.K, shape.group
        rng = np.random.Generator(np.random.PCG64(shape.seed))
        W = WL.make_weights(N, K, shape.sigma_w, rng=rng)
        self.packed, self.gparams, self.w_scales = api.liquidquant_pack_weights(W, g)
        del W
        per_copy = self.packed.nbytes + self.gparams.nbytes
        self.copies = max(1, math.ceil(ROTATE_BYTES / per_copy))
        dev = "cuda:0"
        hp, hg = torch.from_numpy(self.packed), torch.from_numpy(self.gparams)
        self.d_packed = [hp.to(dev) for _ in range(self.copies)]
        self.d_gparams = [hg.to(dev) for _ in range(self.copies)]
        self.d_w_scales = torch.from_numpy(self.w_scales).to(dev)
        self.X, self.sx, self.dX, self.dsx, self.dY = {}, {}, {}, {}, {}
        for M in Ms:
            X, sx = WL.make_activations(M, K, shape.outlier_frac, seed=shape.seed + 1000 + M)
            self.X[M], self.sx[M] = X, sx
            self.dX[M] = torch.from_numpy(X).to(dev)
            self.dsx[M] = torch.from_numpy(sx).to(dev)
            self.dY[M] = torch.empty((M, N), dtype=torch.float16, device=dev)

    def launch(self, M, i, api, stream, variant=-1):
        c = i % self.copies
        s = self.shape
        if variant < 0:
            api.w4a8_gemm(self.dX[M], self.dsx[M], self.d_packed[c], self.d_gparams[c], self.d_w_scales,
                          s.N, s.K, s.group, out=self.dY[M], stream=stream.cuda_stream)
        else:
            api.w4a8_gemm_variant(variant, self.dX[M], self.dsx[M], self.d_packed[c], self.d_gparams[c],
                                  self.d_w_scales, s.N, s.K, s.group, want_acc=False, out_y=self.dY[M],
                                  stream=stream.cuda_stream)


def time_steps(prob, M, steps, warmup, torch, api, stream, variant=-1, graph=False):
    """Average milliseconds per launch over `steps` back-to-back launches (HIP events on
    the launch stream), after `warmup` untimed ones.  With graph=True the `steps` launches
    are captured once into a HIP graph and replayed, which takes the Python/ctypes launch
    cost (about 9 us per call) out of the measurement of kernels shorter than that."""
    with torch.cuda.stream(stream):
        for i in range(warmup):
            prob.launch(M, i, api, stream, variant)
        stream.synchronize()
        g = None
        if graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(steps):
                    prob.launch(M, warmup + i, api, stream, variant)
            g.replay()  # untimed first replay
            stream.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        if g is not None:
            g.replay()
        else:
            for i in range(steps):
                prob.launch(M, warmup + i, api, stream, variant)
        e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def point(prob, M, ms, api):
    s = prob.shape
    t = ms * 1e-3
    ops, byt = algorithmic_ops(M, s.N, s.K), algorithmic_bytes(M, s.N, s.K, s.group)
    t_mem, t_mma = byt / (PEAK_HBM_GBS * 1e9), ops / (PEAK_INT8_TOPS * 1e12)
    return {
        "M": M, "N": s.N, "K": s.K, "group": s.group, "us": round(ms * 1e3, 3),
        "tops": round(ops / t / 1e12, 3), "gbs": round(byt / t / 1e9, 1),
        "bound": "hbm" if t_mem >= t_mma else "mfma",
        "frac_of_roofline": round(max(t_mem, t_mma) / t, 4),
        "variant": api.w4a8_variant_name(api.w4a8_select_variant(M, s.N, s.K, s.group)),
    }


def cpu_baseline(prob, M, budget_s=15.0):
    """The C oracle (as it stands) on a bounded row sample of the same workload."""
    from oracle import c_oracle
    from oracle import lqq_oracle as O
    from paper_2509_01229_amd import api

    s = prob.shape
    codes, s_u8, a = api.liquidquant_unpack_weights(prob.packed, prob.gparams, s.N, s.K, s.group)
    canon = O.pack_canonical(codes)
    del codes
    X, sx = prob.X[M], prob.sx[M]
    t0 = time.perf_counter()
    c_oracle.w4a8_gemm(X[:1], sx[:1], canon, s_u8, a, prob.w_scales, s.group)
    t_one = time.perf_counter() - t0                       # dominated by the dequantisation
    t0 = time.perf_counter()
    c_oracle.w4a8_gemm(X[:3], sx[:3], canon, s_u8, a, prob.w_scales, s.group)
    t_three = time.perf_counter() - t0
    per_row = max((t_three - t_one) / 2, 1e-6)
    rows = int(max(1, min(M, (budget_s - t_one) / per_row)))
    t0 = time.perf_counter()
    c_oracle.w4a8_gemm(X[:rows], sx[:rows], canon, s_u8, a, prob.w_scales, s.group)
    dt = time.perf_counter() - t0
    return {
        "value": round(algorithmic_ops(rows, s.N, s.K) / dt / 1e12, 6), "unit": "TOPS",
        "cores": c_oracle.threads(), "kind": "oracle",
        "sample": f"rows 0..{rows} of X (of M={M}), all N={s.N} K={s.K}; one full dequantisation "
                  f"included; {dt:.1f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="prefill_M4096_N8192_K8192")
    ap.add_argument("--variant", type=int, default=-1, help="force a kernel variant (tuning)")
    ap.add_argument("--no-curve", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--copy-ref", action="store_true",
                    help="only run a plain device-to-device copy of 1 GiB five times (reference "
                         "for scaling the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path has no collective); use --gpus 1")

    import torch

    from paper_2509_01229_amd import api
    from paper_2509_01229_amd import workloads as WL

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.copy_ref:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_ref_bytes_read": 1 << 30, "copy_ref_bytes_written": 1 << 30, "copies": 5}))
        return
    api.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    head = WL.by_name(args.workload)
    curve_Ms = [] if args.no_curve else [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096]
    Ms = sorted(set(curve_Ms + [head.M]))
    prob = DeviceProblem(head, Ms, torch, api, WL)

    # Untimed pre-warm of about 0.2 s so that the timed steps run at settled clocks, then the
    # W warm-up steps and the K timed steps of the contract.
    t_end = time.perf_counter() + 0.2
    while time.perf_counter() < t_end:
        time_steps(prob, head.M, 10, 0, torch, api, stream, args.variant)
    ms = time_steps(prob, head.M, args.steps, args.warmup, torch, api, stream, args.variant)
    hp = point(prob, head.M, ms, api)
    ops = algorithmic_ops(head.M, head.N, head.K)
    byt = algorithmic_bytes(head.M, head.N, head.K, head.group)
    if hp["bound"] == "mfma":
        roof = {"bound": "mfma", "achieved": round(ops / (ms * 1e-3) / 1e12, 2), "peak": PEAK_INT8_TOPS,
                "unit": "TOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": round(byt / (ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["kernel"] = hp["variant"]
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get((head.name, hp["variant"]))
    roof["algorithmic_bytes"] = byt

    out = {
        "metric": "W4A8 GEMM TOPS and % of HBM / int8-MFMA roofline vs M (1..4096)",
        "value": hp["tops"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 x uint4->int8, int32 accumulate, fp16 out", "data": "synthetic",
        "config": {"workload": head.name, "M": head.M, "N": head.N, "K": head.K, "group": head.group,
                   "weight_copies_rotated": prob.copies},
        "roofline": roof,
    }

    if not args.no_curve:
        curve = []
        for M in curve_Ms:
            steps = max(20, min(200, int(0.05 / max(1e-6, 1e-3 * ms * M / head.M + 5e-6))))
            curve.append(point(prob, M, time_steps(prob, M, steps, 5, torch, api, stream, graph=M <= 8), api))
        out["curve_N8192_K8192"] = curve
        del prob.d_packed[1:], prob.d_gparams[1:]
        torch.cuda.empty_cache()
        # decode shapes (N = K = 4096) and the HBM-bound 70B point
        extra = []
        for name_Ms in ((WL.DECODE, (1, 4, 16)), (WL.LAYERS_70B[:1], (16,))):
            shp = name_Ms[0][0]
            p2 = DeviceProblem(shp, list(name_Ms[1]), torch, api, WL)
            for M in name_Ms[1]:
                extra.append(point(p2, M, time_steps(p2, M, 200, 20, torch, api, stream, graph=shp.N * shp.K < (1 << 26)), api))
            del p2
            torch.cuda.empty_cache()
        out["memory_bound_points"] = extra
        hb = extra[-1]
        out["roofline_hbm"] = {"bound": "hbm", "achieved": hb["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": round(hb["gbs"] / PEAK_HBM_GBS, 4),
                               "traffic": MEASURED_TRAFFIC_BYTES.get((shp.name, hb["variant"])),
                               "algorithmic_bytes": algorithmic_bytes(hb["M"], hb["N"], hb["K"], hb["group"]),
                               "kernel": hb["variant"],
                               "workload": f"l70b_up M=16 N={hb['N']} K={hb['K']} group {hb['group']}"}

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(prob, head.M)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
