#!/usr/bin/env python3
"""Benchmark of the quantised matmul hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-legs]

The metric has two legs: packed-weight HBM GB/s for decode-sized M (<= 16) and effective
TFLOP/s for prefill-sized M (>= 1024).  The headline (`value`, `ms_per_step`, `roofline`) is
the decode leg on the W3A16 decode configuration (uint3 weights, K=4096, N=14336, group 128,
fp16): one step = qgemm at M=1, M=4 and M=16.  The default run also measures, and reports
under `legs` in the same JSON line, a decode problem of more than 100 MB (signed 4-bit sweep
cell, K=8192, N=28672, M=16) and the prefill leg (uint6, K=8192, N=57344, M=4096, bf16), each
with its own `roofline` block.

Protocol: inputs are seeded, synthetic and resident in HBM before anything is timed; every
call streams a different resident copy of the packed weight (and of its scales and
zero-points), more copies than the last-level cache holds, so that no call finds its weights
in a cache (the paper clears L2 before each run; rotation does the same without a second
kernel inside the timed region).  After ~0.25 s of untimed calls (clock settling) and W
warm-up steps, exactly K steps run between two events on the launch stream: `ms_per_step`,
`value` and `roofline.achieved` come from that region (average launch duration).  Then every
case is launched >= 50 times more, each launch between its own pair of events, and the
MEDIAN of those is reported beside the average (the paper's protocol: 50 runs, median).

Other workloads (for the result tables): cfg1, cfg2_M<m>, cfg3_i<k>[_M<m>], cfg4_f<bits>_M<m>,
cfg5_u<k>_M<m> [--layout 1], sweep_{u,i,f}<bits>[_M<m>], dense_<path>_... see cases_for().
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16/bf16
# plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE counter
# runs of this same command, scaled by what the counters read for a plain copy of known size.
# These are CARRIED OVER from the committed profile summaries, not measured in this run.
MEASURED_TRAFFIC = {
    "cfg2": (24.63e6, "profiles/decode_kernel_cfg2_w3a16.txt"),
    "cfg3_i4": (125.9e6, "profiles/decode_kernel_cfg3_i2_i4_counters.txt"),
    "cfg5_u6_M4096": (3.845e9, "profiles/large_kernel_cfg5_u6_M4096.txt"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-legs", action="store_true", help="headline workload only")
    ap.add_argument("--copies", type=int, default=0, help="resident weight copies to rotate through")
    ap.add_argument("--layout", type=int, default=0, help="device layout of the packed weight (0 or 1)")
    ap.add_argument("--entry", default="qgemm", choices=["qgemm", "qgemm_noalloc"])
    ap.add_argument("--path", type=int, default=0,
                    help="force a path of qgemm (qgemm_tuning.h): 1 streaming, 2 tiled, 4 de-quantise first + 16-bit matmul, "
                         "5 matrix-vector kernel (M <= 4)")
    return ap.parse_args()


DEFAULT_LEGS = ["cfg3_i4", "cfg5_u6_M4096"]


def cases_for(name):
    from paper_2504_12984_amd import workloads as WL
    if name == "cfg1":
        return [WL.cfg1()]
    if name == "cfg2":
        return [WL.cfg2(1), WL.cfg2(4), WL.cfg2(16)]
    if name.startswith("cfg2_M"):
        m = int(name[6:])
        return [WL.cfg2(m) if m in (1, 4, 16) else WL.shrink(WL.cfg2(16), M=m, name=name)]
    if name.startswith("cfg3_i"):
        if "_M" in name:                              # cfg3 recipe at another M (tables only)
            bits, m = name[6:].split("_M")
            return [WL.shrink(WL.cfg3(int(bits)), M=int(m), name=f"cfg3_i{bits}_M{m}")]
        return [WL.cfg3(int(name[6:]))]
    if name.startswith("cfg4_f"):
        bits, m = name[6:].split("_M")
        return [WL.cfg4(int(bits), int(m))]
    if name.startswith("cfg5_u"):
        bits, m = name[6:].split("_M")
        return [WL.cfg5(int(bits), int(m))]
    if name.startswith("a8_i"):                          # int8 activations on the signed sweep's recipe: a8_i4, a8_i4_M64
        rest = name[4:]
        bits, m = rest.split("_M") if "_M" in rest else (rest, "16")
        return [WL.shrink(WL.cfg3(int(bits)), M=int(m), a8=True, name=name)]
    if name.startswith("mx_f") or name.startswith("mxsweep_f"):     # block-scaled e2m1 / e4m3: mx_f4_M1 (K = N = 8192), mxsweep_f8_M16 / _M4096 (N = 57344)
        big = name.startswith("mxsweep")
        bits, m = name.split("_f")[1].split("_M")
        e, mm = {4: (2, 1), 8: (4, 3)}[int(bits)]
        return [WL.Case(name, int(m), 8192, 57344 if big else 8192, WL.KIND_FLOAT, int(bits), e, mm, group=32,
                        act="bf16", scale_dtype="e8m0", zero=None, seed=700 + int(bits))]
    if name.startswith("codebook_"):                     # codebook lookup on the type sweep's shape: codebook_4, codebook_4_M1
        rest = name[9:]
        bits, m = rest.split("_M") if "_M" in rest else (rest, "16")
        return [WL.codebook(int(bits), int(m))]
    if name.startswith("sweep_"):                        # sweep_u4, sweep_i7, sweep_f6 (M = 16), sweep_u4_M8192
        kind = {"u": WL.KIND_UINT, "i": WL.KIND_INT, "f": WL.KIND_FLOAT}[name[6]]
        rest = name[7:]
        if "_M" in rest:
            bits, m = rest.split("_M")
            return [WL.sweep(kind, int(bits), int(m))]
        return [WL.sweep(kind, int(rest))]
    raise SystemExit(f"unknown workload {name}")


def algorithmic_bytes(c):
    """Bytes one call must move: packed W once, scales, zero-points, A, C."""
    P = c.K * c.N * c.bits // 8
    G = c.K // c.group
    S = G * c.N * (1 if c.scale_dtype == "e8m0" else 2)
    Z = G * c.N if c.zero is not None else 0
    a_bytes = c.M * c.K + c.M * 4 if c.a8 else c.M * c.K * 2            # int8 rows + one fp32 scale per row
    return P, P + S + Z + a_bytes + c.M * c.N * 2


def decode_lane_ops_per_element(c):
    """Vector-ALU lane-operations per weight element that unpack + de-quantise needs at the
    least under the bit-exact contract (one instruction handles the two elements of a
    register): fp16 route -- extract, exact subtract (or exact re-bias multiply), rounding
    multiply = 3 per pair; bf16 route -- extract, two mixed-precision fused multiply-adds,
    one packed convert = 4 per pair; floats with a hardware convert save the middle step
    (2 / 3 per pair)."""
    from paper_2504_12984_amd import workloads as WL
    if c.a8:
        # int8 activations: a shift and a mask per register of four codes, + 3 per accumulator
        # and scale group for the zero-point / convert / scale step (16 accumulators per 64 x 128)
        return 2 / 4.0 + 3 * 16 / (64.0 * min(c.group, 128))
    if c.scale_dtype == "e8m0":
        return 1 / 2.0            # one scaled hardware convert per pair of codes
    if c.kind == WL.KIND_CODEBOOK:
        # index extract + address, the LDS read aside, + the rounding multiply: per pair of codes up to
        # 4 bits (one read returns both levels), per code above (+ one merge of the two halves)
        return (3 if c.bits <= 4 else 6) / 2.0 if c.act == "f16" else (7 if c.bits <= 4 else 9) / 2.0
    hw = c.kind == WL.KIND_FLOAT and (c.ebits, c.mbits) in ((2, 1), (3, 2), (4, 3))
    per_pair = (2 if hw else 3) if c.act == "f16" else (3 if hw else 4)
    return per_pair / 2.0


def cpu_baseline(case, budget_s=20.0):
    """Time the oracle, as it stands, on a column sample of the same workload."""
    import numpy as np
    import psutil
    from oracle import qgemm_oracle as O
    from paper_2504_12984_amd import workloads as WL
    inp = WL.make_inputs(case)
    stream = O.pack_canonical(inp["codes"], case.bits)
    A = inp["A"].double().numpy()
    S = inp["scales"].double().numpy()
    proc = psutil.Process()
    cols_done, t_used, cpu_used = 0, 0.0, 0.0
    block = 1024
    while t_used < budget_s and (cols_done < case.N or t_used < 0.5 * budget_s):
        start = cols_done % case.N                    # small workloads: go round again until the budget is half used
        cols = np.arange(start, min(case.N, start + block))
        c0 = proc.cpu_times()
        t0 = time.perf_counter()
        if case.kind == WL.KIND_CODEBOOK:
            O.qgemm_codebook_from_stream(A, stream, case.bits, inp["codebook"].double().numpy(), S, case.group,
                                         case.K, case.N, case.act, cols=cols)
        else:
            O.qgemm_from_stream(A, stream, case.kind, case.bits, case.ebits, case.mbits, S, inp["zeros"],
                                case.group, case.K, case.N, case.act, cols=cols)
        t_used += time.perf_counter() - t0
        c1 = proc.cpu_times()
        cpu_used += (c1.user + c1.system) - (c0.user + c0.system)
        cols_done += cols.size
    frac = cols_done / case.N
    return frac, t_used, cpu_used / max(t_used, 1e-9)


class Leg:
    """One workload resident on the GPU: weight copies, bound calls, timing."""

    def __init__(self, name, layout=0, copies=0, entry="qgemm"):
        import torch
        from paper_2504_12984_amd import binding as B
        from paper_2504_12984_amd import workloads as WL
        self.name, self.layout = name, layout
        self.cases = cases_for(name)
        c0 = self.c0 = self.cases[0]
        self.wt = B.WType(c0.kind, c0.bits, c0.ebits, c0.mbits)
        self.P, _ = algorithmic_bytes(c0)
        dev = "cuda:0"
        inp0 = WL.make_inputs(c0)
        codes = torch.from_numpy(inp0["codes"]).to(dev)
        if c0.a8:
            layout = self.layout = B.QG_LAYOUT_TILE128x64_I8
        packed0 = B.repack(B.qg_pack_codes(codes, c0.bits), self.wt, c0.K, c0.N, layout=layout)
        del codes
        self.copies = copies or int(min(64, max(3, -(-(3 << 29) // self.P))))     # ~1.5 GB of packed weights
        self.packed = [packed0] + [packed0.clone() for _ in range(self.copies - 1)]
        self.scales = [inp0["scales"].to(dev).clone() for _ in range(self.copies)]
        self.zeros = [None if inp0["zeros"] is None else torch.from_numpy(inp0["zeros"]).to(dev).clone()
                      for _ in range(self.copies)]
        inps = [WL.make_inputs(c) if i else inp0 for i, c in enumerate(self.cases)]
        self.As = [x["A"].to(dev) for x in inps]
        self.a_scales = [x["a_scale"].to(dev) if c.a8 else None for x, c in zip(inps, self.cases)]
        inp_table = inp0.get("codebook")
        del inp0, inps
        out_dt = {"f16": torch.float16, "bf16": torch.bfloat16}
        self.Cs = [torch.empty((c.M, c.N), dtype=out_dt[c.act], device=dev) for c in self.cases]
        torch.cuda.synchronize()
        # arguments marshalled once per (case, weight copy): the timed loop is foreign calls only
        self.table = None
        if c0.kind == WL.KIND_CODEBOOK:
            table = self.table = inp_table.to(dev)
            self.calls = [[B.BoundQgemmCodebook(A, self.packed[i], table, self.scales[i], c.bits, c.group, c.N, C)
                           for i in range(self.copies)] for c, A, C in zip(self.cases, self.As, self.Cs)]
        elif c0.a8:
            self.calls = [[B.BoundQgemmA8(A, a_s, self.packed[i], self.scales[i], self.zeros[i], self.wt, c.group, c.N, C)
                           for i in range(self.copies)] for c, A, a_s, C in zip(self.cases, self.As, self.a_scales, self.Cs)]
        else:
            self.calls = [[B.BoundQgemm(A, self.packed[i], self.scales[i], self.zeros[i], self.wt, c.group, c.N, C,
                                        layout=layout, entry=entry)
                           for i in range(self.copies)] for c, A, C in zip(self.cases, self.As, self.Cs)]
        self.rot = 0
        self.small = all(c.M <= 64 for c in self.cases)

    def step(self):
        for per_copy in self.calls:
            per_copy[self.rot % self.copies]()
            self.rot += 1

    def settle(self, seconds=0.25):
        # The GPU's clocks take a few thousand short launches to settle after start-up.
        import torch
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < seconds:
            for _ in range(10 if self.small else 1):
                self.step()
            torch.cuda.synchronize()

    def timed_region(self, steps, warmup):
        import torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            self.step()
        ev1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return ev0.elapsed_time(ev1) / steps, wall_ms / steps

    def per_launch_medians(self, launches=50):
        """Each launch between its own pair of events on the launch stream; median per case, in ms."""
        import torch
        out = []
        for per_copy in self.calls:
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
            for e0, e1 in evs:
                e0.record()
                per_copy[self.rot % self.copies]()
                self.rot += 1
                e1.record()
            torch.cuda.synchronize()
            out.append(statistics.median(e0.elapsed_time(e1) for e0, e1 in evs))
        return out

    def empirical_ceiling(self):
        """Same protocol (back-to-back launches, events): a kernel that only reads the same packed
        weights (decode) or a register-resident matrix-instruction loop (prefill)."""
        import torch
        from paper_2504_12984_amd import binding as B
        sink = torch.zeros(4096, dtype=torch.float32, device="cuda:0")

        def gpu_time_ms(fn, reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        if self.small:
            probes = [B.qg_probe_stream_read(self.packed[i], sink) for i in range(self.copies)]
            for i in range(min(self.copies, 5)):
                probes[i]()
            torch.cuda.synchronize()
            t = gpu_time_ms(lambda i: probes[i % self.copies](), 200)
            return {"what": "kernel that only reads the packed weight of one launch, rotating the same copies",
                    "us": round(t * 1e3, 3), "gbps": round(self.P / (t * 1e-3) / 1e9, 1)}
        is_bf16 = self.c0.act == "bf16"
        emp = {"what": "register-resident 32x32x16 matrix-instruction loop, 1 wavefront per SIMD"}
        for label, rnd in (("constant_operands", False), ("random_operands", True)):
            B.qg_probe_mfma(is_bf16, rnd, 2000, 1, sink)
            torch.cuda.synchronize()
            fl = [0.0]

            def run(i, rnd=rnd):
                fl[0] = B.qg_probe_mfma(is_bf16, rnd, 20000, 1, sink)
            t = gpu_time_ms(run, 5)
            emp[label + "_tflops"] = round(fl[0] / (t * 1e-3) / 1e12, 1)
        return emp

    def report(self, steps, warmup, ceilings=True):
        """Measure and return (ms_per_step, wall_ms_per_step, metric, unit, value, roofline, extra)."""
        self.settle()
        ms_per_step, wall_ms = self.timed_region(steps, warmup)
        medians = self.per_launch_medians(50)
        cases, launches = self.cases, len(self.cases)
        launch_ms = ms_per_step / launches
        flops_step = sum(2.0 * c.M * c.N * c.K for c in cases)
        alg_bytes = sum(algorithmic_bytes(c)[1] for c in cases) / launches
        gbs_packed = launches * self.P / (ms_per_step * 1e-3) / 1e9
        tflops = flops_step / (ms_per_step * 1e-3) / 1e12
        emp = self.empirical_ceiling() if ceilings else None
        med_us = [round(m * 1e3, 3) for m in medians]
        if self.small:
            metric, unit, value = "packed_weight_hbm_gbps", "GB/s", gbs_packed
            ach = alg_bytes / (launch_ms * 1e-3) / 1e9
            traffic = MEASURED_TRAFFIC.get(self.name)
            lane_ops = sum(c.K * c.N * decode_lane_ops_per_element(c) for c in cases) / launches
            valu = lane_ops / (launch_ms * 1e-3) / 1e12
            roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": traffic[0] if traffic else None,
                    "traffic_source": (f"carried over from {traffic[1]} (counter run of this command), "
                                       "not measured in this run") if traffic else None,
                    "kernel": "qg::a8_kernel" if self.c0.a8 else "qg::decode_kernel", "avg_launch_us": round(launch_ms * 1e3, 3),
                    "median_launch_us_per_case": med_us,
                    "algorithmic_bytes_per_launch": int(alg_bytes),
                    "secondary": {"bound": "valu", "lane_ops": int(lane_ops), "achieved": round(valu, 2),
                                  "peak": round(VALU_PEAK_TLANEOPS, 1), "unit": "T lane-ops/s",
                                  "frac": round(valu / VALU_PEAK_TLANEOPS, 4),
                                  "what": "least unpack + de-quantise vector work of the bit-exact contract "
                                          "(lane-operations per launch) over the plain vector-ALU peak"}}
            if emp:
                roof["empirical_ceiling"] = emp
                roof["frac_of_empirical"] = round(gbs_packed / emp["gbps"], 4)
        else:
            metric, unit, value = "effective_tflops", "TFLOP/s", tflops
            roof = {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / MFMA_PEAK_TFLOPS, 4),
                    "traffic": MEASURED_TRAFFIC[self.name][0] if self.name in MEASURED_TRAFFIC and self.layout == 0 else None,
                    "traffic_source": (f"carried over from {MEASURED_TRAFFIC[self.name][1]} (counter run of this command), "
                                       "not measured in this run") if self.name in MEASURED_TRAFFIC and self.layout == 0 else None,
                    "kernel": "qg::large32_kernel" if self.layout == 1 else "qg::large_kernel",
                    "avg_launch_us": round(launch_ms * 1e3, 3), "median_launch_us_per_case": med_us,
                    "algorithmic_flops_per_launch": flops_step / launches}
            if emp:
                roof["empirical_ceiling"] = emp
                roof["frac_of_empirical"] = round(tflops / emp["random_operands_tflops"], 4)
        extra = {"packed_gbps": round(gbs_packed, 1), "tflops": round(tflops, 3),
                 "host_wall_ms_per_step": round(wall_ms, 5)}
        return ms_per_step, metric, unit, value, roof, extra

    def config(self):
        c0 = self.c0
        return {"workload": self.name, "cases": [c.name for c in self.cases], "weight": c0.wname,
                "K": c0.K, "N": c0.N, "group": c0.group, "M": [c.M for c in self.cases],
                "launches_per_step": len(self.cases), "weight_copies_rotated": self.copies, "layout": self.layout,
                "packed_bytes": self.P}

    def vendor_dense_gemm_tflops(self):
        # context, not a target: the vendor library's dense bf16/fp16 GEMM on the same shape and
        # the same activations, weights already de-quantised (it reads 16 bits per weight)
        import torch
        from paper_2504_12984_amd import binding as B
        c0 = self.c0
        if self.table is not None:
            Wd = B.qdequant_codebook(self.packed[0], self.table, self.scales[0], c0.bits, self.As[0].dtype, c0.group, c0.K, c0.N)
        else:
            Wd = B.qdequant(self.packed[0], self.scales[0], self.zeros[0], self.wt, self.As[0].dtype, c0.group, c0.K, c0.N,
                            layout=self.layout)
        Cd = torch.empty_like(self.Cs[0])
        for _ in range(3):
            torch.matmul(self.As[0], Wd, out=Cd)
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(10):
            torch.matmul(self.As[0], Wd, out=Cd)
        d1.record()
        torch.cuda.synchronize()
        return round(2.0 * c0.M * c0.N * c0.K / (d0.elapsed_time(d1) / 10 * 1e-3) / 1e12, 1)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        raise SystemExit(2)
    import torch

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    if args.path:
        from paper_2504_12984_amd import binding as B
        B.qg_set_knob(0, args.path)
    head = Leg(args.workload, layout=args.layout, copies=args.copies, entry=args.entry)
    ms_per_step, metric, unit, value, roof, extra = head.report(args.steps, args.warmup)
    c0 = head.c0
    out = {
        "metric": metric, "value": round(value, 2), "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i8" if c0.a8 else ("bf16" if c0.act == "bf16" else "f16"), "data": "synthetic",
        "config": head.config(), "roofline": roof, "extra": extra,
    }
    if args.entry != "qgemm":
        out["config"]["entry"] = args.entry
    if args.path:
        out["config"]["forced_path"] = args.path
    if not head.small:
        out["extra"]["vendor_dense_gemm_tflops"] = head.vendor_dense_gemm_tflops()
    cpu_case = head.cases[-1]
    small = head.small
    del head
    torch.cuda.empty_cache()

    # ---- the other legs of the metric (default run only) ------------------------------------
    if args.workload == "cfg2" and not args.no_legs:
        legs = []
        for name in DEFAULT_LEGS:
            leg = Leg(name, layout=args.layout)
            n_steps = 100 if leg.small else 50
            l_ms, l_metric, l_unit, l_value, l_roof, l_extra = leg.report(n_steps, 5)
            legs.append({"metric": l_metric, "value": round(l_value, 2), "unit": l_unit, "steps": n_steps,
                         "warmup": 5, "ms_per_step": round(l_ms, 5),
                         "dtype": "bf16" if leg.c0.act == "bf16" else "f16", "config": leg.config(),
                         "roofline": l_roof, "extra": l_extra})
            del leg
            torch.cuda.empty_cache()
        out["legs"] = legs

    if not args.no_cpu:
        frac, t_used, busy = cpu_baseline(cpu_case)
        Pb = cpu_case.K * cpu_case.N * cpu_case.bits // 8
        if small:
            v, u = Pb * frac / t_used / 1e9, "GB/s"
        else:
            v, u = 2.0 * cpu_case.M * cpu_case.N * cpu_case.K * frac / t_used / 1e12, "TFLOP/s"
        out["cpu_baseline"] = {"value": round(v, 6), "unit": u, "cores": max(1, round(busy)), "kind": "oracle",
                               "host_cpus": os.cpu_count(), "cpu_time_over_wall_time": round(busy, 2),
                               "sample": f"{cpu_case.name}: {frac:.2f} passes over the N columns in blocks of 1024, "
                                         f"all M rows, {t_used:.1f} s (unpack+dequant+round+fp64 GEMM); "
                                         f"cores = CPU time / wall time of the NumPy oracle's threads, "
                                         f"host_cpus = os.cpu_count()"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
