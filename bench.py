#!/usr/bin/env python3
"""Benchmark of the AdaHOP per-GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg4-up|cfg1|cfg0]

A step is one pass of the whole path (FOID -> residual masking -> IHT -> MX quantise -> MXFP4 GEMM
-> BF16 outlier GEMM -> sum) over every GEMM of the workload, operands resident in HBM.  Prints one
JSON line: the effective TFLOP/s of the step (sum of 2MNK over the GEMMs / time), the roofline of
the dominant kernel (the block-scaled FP4 GEMM) measured with HIP events on the launch stream, and
the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import sys
import time

import numpy as np

MXFP4_PEAK_TFLOPS = 10066.0   # MI355X dense FP4 matrix-core peak: 256 CU x 16384 flop/clk x 2.4 GHz
BF16_PEAK_TFLOPS = 2516.0

# HBM bytes per launch of the FP4 GEMM kernel, by (M, N, K): rocprofv3 FETCH_SIZE + WRITE_SIZE (KiB per
# dispatch), each scaled by what the same counter reads for a plain 1 GiB copy (--copy-calibration);
# the runs and the scaling are in profiles/gemm_mx_16384x28672x8192_counters.txt.
GEMM_HBM_TRAFFIC_BYTES = {(16384, 28672, 8192): 4.99e9, (8192, 8192, 2048): 3.57e8}
GEMM_HBM_TRAFFIC_SOURCE = {(16384, 28672, 8192): "profiles/gemm_mx_16384x28672x8192_counters.txt",
                           (8192, 8192, 2048): "profiles/gemm_mx_dual_8192x8192x2048_counters.txt"}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="cfg4", choices=["cfg4", "cfg4-up", "cfg3", "cfg1", "cfg0", "paper-table3"])
    p.add_argument("--k-pct", type=float, default=1.0, help="extraction count as %% of the extracted dim (cfg4)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-extras", action="store_true", help="skip the k-sweep / BF16 / per-stage extras")
    p.add_argument("--no-other-workloads", action="store_true",
                   help="skip the one-line summaries of configs[1], configs[3] and the latency-table shapes")
    p.add_argument("--dominant-kernel-only", action="store_true",
                   help="profiling aid: time only the FP4 GEMM of the largest product (the roofline object); the "
                        "whole-step figures of the JSON line are then absent")
    p.add_argument("--quantizer-only", action="store_true",
                   help="profiling aid: time only the IHT + MXFP4 quantiser on the largest product's B operand, read "
                        "K-contiguous and K-strided, with the workload's transform block and with block 32")
    p.add_argument("--copy-calibration", action="store_true",
                   help="also run one plain 1 GiB device-to-device copy (reference reading for rocprofv3's "
                        "FETCH_SIZE / WRITE_SIZE counters)")
    return p.parse_args()


def build_workload(name, k_pct):
    from paper_2604_02525_amd import inputs
    I = inputs
    if name == "cfg0":
        return "configs[0]: M=N=K=256, IHT block 32", I.config0()
    if name == "cfg1":
        return "configs[1]: fwd X[8192,2048] W[8192,2048], IHT block 128", I.config1()
    if name == "cfg3":
        return ("configs[3]: LLaMA-7B-shaped layer at T=8192 (QKV, O, gate, up, down; fwd+dgrad+wgrad, 15 GEMMs), IHT block "
                "128, seeded per-GEMM strategy table, k = 1 % of the extracted dim"), I.config3()
    if name == "paper-table3":
        return ("the two GEMMs of the paper's kernel latency table: (14336,4096,32768) and (4096,4096,32768) weight "
                "gradients, IHT block 32, OE-col with rank 64"), I.paper_latency_shapes()
    which = ("up",) if name == "cfg4-up" else ("up", "down")
    # fwd: activation channel outliers are K-channels of A; dgrad: gradient token rows are rows of A;
    # wgrad: gradient token rows are K-channels of A = G_Y^T.
    strategies = (I.IHT_OE_K, I.IHT_OE_ROW, I.IHT_OE_K) if k_pct > 0 else (I.IHT, I.IHT, I.IHT)
    desc = (f"configs[4]: T=16384, {'+'.join(which)} 8192<->28672, fwd+dgrad+wgrad, IHT block 256, "
            f"fwd/wgrad OE-K, dgrad OE-row, k={k_pct}% of the extracted dim")
    return desc, I.config4(which=which, strategies=strategies, k_pct=k_pct)


class Prepared:
    """Device operands, output and workspace of one GEMM, allocated once outside the timed region."""

    def __init__(self, ah, torch, g, cache):
        def dev(op):
            key = id(op.bits)
            if key not in cache:
                cache[key] = torch.from_numpy(op.bits.view(np.int16)).cuda()
            return ah.Operand(cache[key], op.k_contig)
        self.g = g
        self.A, self.B = dev(g.A), dev(g.B)
        self.M, self.N, self.K = g.shape
        self.flops = 2.0 * self.M * self.N * self.K
        self.C = torch.empty((self.M, self.N), dtype=torch.float32, device="cuda")
        self.idx = torch.zeros(max(g.k, 1), dtype=torch.int32, device="cuda")

    def workspace(self, ah, torch, pool):
        need = ah.adahop_gemm_workspace_bytes(self.M, self.N, self.K, self.g.strategy, self.g.k)
        if pool.get("ws") is None or pool["ws"].numel() < need:
            pool["ws"] = torch.empty(need, dtype=torch.uint8, device="cuda")
        return pool["ws"]


def run_gemm(ah, p, ws, strategy=None, k=None):
    import ctypes as C
    s = p.g.strategy if strategy is None else strategy
    kk = p.g.k if k is None else k
    rc = ah.lib().adahop_gemm(C.byref(p.A.c()), C.byref(p.B.c()), p.C.data_ptr(), p.C.stride(0), s, p.g.iht_block, kk,
                              p.idx.data_ptr(), 0, ws.data_ptr(), ws.numel(), ah._stream(None))
    if rc != 0:
        raise ah.AdahopError(rc, "adahop_gemm")


def time_ms(torch, fn, iters, warmup=1):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def bf16_views(torch, p):
    a16, b16 = p.A.tensor.view(torch.bfloat16), p.B.tensor.view(torch.bfloat16)
    return (a16 if p.A.k_contig else a16.t()), (b16.t() if p.B.k_contig else b16)


def stage_times(ah, torch, inputs, p, ws, iters=5):
    """Per-stage times of one product, each stage bracketed by its own events (so the stages do not overlap and the
    sum exceeds the fused call slightly): FOID, quantise A, quantise B, K-channel gathers + MXFP4 product (+ the BF16
    row / column product), and the MXFP4 kernel alone on the packed operands."""
    g = p.g
    oe = g.strategy in (inputs.IHT_OE_ROW, inputs.IHT_OE_COL, inputs.IHT_OE_K) and g.k > 0
    scored, axis = {inputs.IHT_OE_ROW: (p.A, 0), inputs.IHT_OE_COL: (p.B, 0), inputs.IHT_OE_K: (p.A, 1)}.get(g.strategy, (p.A, 0))
    dim = scored.outer if axis == 0 else scored.K
    idx = torch.zeros(max(g.k, 1), dtype=torch.int32, device="cuda")
    mask = torch.empty(max(dim, 8), dtype=torch.uint8, device="cuda")
    scores = torch.empty(max(dim, 8), dtype=torch.float32, device="cuda")
    ac = torch.empty((p.M, p.K // 2), dtype=torch.uint8, device="cuda")
    asc = torch.empty((p.M, p.K // 32), dtype=torch.uint8, device="cuda")
    bc = torch.empty((p.N, p.K // 2), dtype=torch.uint8, device="cuda")
    bsc = torch.empty((p.N, p.K // 32), dtype=torch.uint8, device="cuda")
    gws = torch.empty(ah.adahop_gemm_mx_workspace_bytes(p.M, p.N, p.K), dtype=torch.uint8, device="cuda")
    import ctypes as C
    L, st = ah.lib(), ah._stream(None)

    def foid():
        if oe:
            rc = L.adahop_foid_topk(C.byref(scored.c()), axis, g.k, idx.data_ptr(), mask.data_ptr(), scores.data_ptr(), st)
            assert rc == 0

    stages = [
        ("foid_topk", foid),
        ("quantize_a", lambda: ah.adahop_pack_operand(p.A, 0, g.strategy, g.iht_block, g.k if oe else 0, idx, ac, asc)),
        ("quantize_b", lambda: ah.adahop_pack_operand(p.B, 1, g.strategy, g.iht_block, g.k if oe else 0, idx, bc, bsc)),
        ("product_with_outlier_part", lambda: ah.adahop_gemm(p.A, p.B, g.strategy, g.iht_block, g.k, idx=idx if oe else None,
                                                             Cout=p.C, workspace=ws, a_packed=(ac, asc), b_packed=(bc, bsc))),
        ("mxfp4_kernel_alone", lambda: ah.adahop_gemm_mx(ac, asc, bc, bsc, p.C, gws)),
    ]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(iters)]
    for fn in [f for _, f in stages]:
        fn()
    torch.cuda.synchronize()
    for it in range(iters):
        ev[it][0].record()
        for si, (_, fn) in enumerate(stages):
            fn()
            ev[it][si + 1].record()
    torch.cuda.synchronize()
    out = {name: sum(ev[it][si].elapsed_time(ev[it][si + 1]) for it in range(iters)) / iters
           for si, (name, _) in enumerate(stages)}
    out["outlier_part_ms"] = out["product_with_outlier_part"] - out["mxfp4_kernel_alone"]
    return {"name": g.name, "strategy": inputs.STRATEGY_NAMES[g.strategy], "k": g.k, "ms": out}


def workload_summary(ah, torch, inputs, name, k_pct=1.0):
    """One line for another workload: step time of the whole path, the same with pure IHT, hipBLASLt BF16."""
    desc, gemms = build_workload(name, k_pct)
    cache, pool = {}, {}
    prepared = [Prepared(ah, torch, g, cache) for g in gemms]
    for p in prepared:
        p.workspace(ah, torch, pool)
    ws = pool["ws"]
    flops = sum(p.flops for p in prepared)

    def step():
        for p in prepared:
            run_gemm(ah, p, ws)

    def step_iht():
        for p in prepared:
            run_gemm(ah, p, ws, strategy=inputs.IHT if p.g.strategy != inputs.NONE else inputs.NONE, k=0)

    def step_bf16():
        for p in prepared:
            am, bm = bf16_views(torch, p)
            torch.matmul(am, bm)

    t, t_iht, t_bf = time_ms(torch, step, 5, 2), time_ms(torch, step_iht, 5, 2), time_ms(torch, step_bf16, 3, 1)
    worst = None
    oe = [p for p in prepared if p.g.k > 0]
    if oe and len(prepared) > 1:
        per = []
        for p in oe:
            a = time_ms(torch, lambda: run_gemm(ah, p, ws), 5)
            b = time_ms(torch, lambda: run_gemm(ah, p, ws, strategy=inputs.IHT, k=0), 5)
            per.append((100.0 * (a - b) / b, p.g.name))
        worst = {"pct": max(per)[0], "gemm": max(per)[1], "mean_pct": sum(x for x, _ in per) / len(per)}
    stages = [stage_times(ah, torch, inputs, p, ws) for p in prepared] if name == "paper-table3" else None
    out = {"workload": desc, "gemms": len(prepared), "step_ms": t, "tflops": flops / t / 1e9,
           "pct_mxfp4_peak": 100.0 * flops / t / 1e9 / MXFP4_PEAK_TFLOPS, "step_ms_iht_only": t_iht,
           "tflops_iht_only": flops / t_iht / 1e9, "step_ms_bf16_hipblaslt": t_bf, "speedup_vs_bf16": t_bf / t}
    if stages:
        out["per_stage_ms"] = stages
    if worst:
        out["oe_overhead_pct_worst"] = worst
    elif oe:
        out["oe_overhead_pct"] = 100.0 * (t - t_iht) / t_iht
    del prepared, cache, pool, ws
    torch.cuda.empty_cache()
    return out


def cpu_baseline(workload_gemms):
    """The oracle, as it stands, on a bounded slab of the first GEMM of the workload."""
    from oracle import reference as orc
    g = workload_gemms[0]
    M, N, K = g.shape
    ms, ns = min(M, 4096), min(N, 8192)
    a = g.A.bits[:ms] if g.A.k_contig else g.A.bits[:, :ms]
    b = g.B.bits[:ns] if g.B.k_contig else g.B.bits[:, :ns]
    k = min(g.k, {2: ms, 3: ns, 4: K}.get(g.strategy, 0))
    t0 = time.perf_counter()
    orc.adahop_gemm(a, g.A.k_contig, b, g.B.k_contig, g.strategy, g.iht_block, k)
    dt = time.perf_counter() - t0
    return {"value": 2.0 * ms * ns * K / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"whole path of {g.name} cropped to M={ms}, N={ns}, K={K} ({dt:.1f} s)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported", file=sys.stderr)
        return 2
    import torch
    from paper_2604_02525_amd import binding as ah, inputs
    ah.lib()
    torch.cuda.set_device(0)

    desc, gemms = build_workload(args.workload, args.k_pct)
    cache, pool = {}, {}
    prepared = [Prepared(ah, torch, g, cache) for g in gemms]
    for p in prepared:
        p.workspace(ah, torch, pool)
    ws = pool["ws"]
    total_flops = sum(p.flops for p in prepared)

    def step():
        for p in prepared:
            run_gemm(ah, p, ws)

    if args.quantizer_only:
        big = max(prepared, key=lambda p: p.flops)
        res = []
        for op in (big.B, ah.Operand(big.B.tensor, not big.B.k_contig)):
            codes = torch.empty((op.outer, op.K // 2), dtype=torch.uint8, device="cuda")
            scales = torch.empty((op.outer, op.K // 32), dtype=torch.uint8, device="cuda")
            for b in sorted({big.g.iht_block, 32}, reverse=True):
                ms = time_ms(torch, lambda: ah.adahop_iht_quantize(op, b, None, None, codes, scales), max(5, args.steps), 2)
                res.append({"outer": op.outer, "K": op.K, "k_contig": bool(op.k_contig), "iht_block": b, "ms": ms,
                            "GBps": 2.53125 * op.outer * op.K / (ms * 1e-3) / 1e9})
        out = {"metric": "IHT + MXFP4 quantiser, algorithmic GB/s (2.53125 B per element)", "unit": "GB/s", "peak_GBps": 8000.0,
               "n_gpus": 1, "data": "synthetic", "config": {"workload": desc}, "runs": res}
        if args.copy_calibration:
            src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            out["copy_calibration_bytes"] = src.numel() * 4
        print(json.dumps(out))
        return 0

    if args.dominant_kernel_only:
        wall_ms = ms_per_step = value = None
    else:
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ms_per_step = max(e0.elapsed_time(e1) / args.steps, 0.0)
        value = total_flops / (ms_per_step * 1e-3) / 1e12

    # Dominant kernel: the FP4 GEMM alone on the largest GEMM's quantised operands.
    big = max(prepared, key=lambda p: p.flops)
    run_gemm(ah, big, ws, strategy=inputs.IHT, k=0)
    L = ah.adahop_gemm_workspace_layout(big.M, big.N, big.K, inputs.IHT, 0)
    view = lambda off, n: ws[off:off + n]
    ac, asc = view(L.a_codes, big.M * big.K // 2), view(L.a_scales, big.M * big.K // 32)
    bc, bsc = view(L.b_codes, big.N * big.K // 2), view(L.b_scales, big.N * big.K // 32)
    ac, asc = ac.view(big.M, -1), asc.view(big.M, -1)
    bc, bsc = bc.view(big.N, -1), bsc.view(big.N, -1)
    gemm_ws = torch.empty(ah.adahop_gemm_mx_workspace_bytes(big.M, big.N, big.K), dtype=torch.uint8, device="cuda")
    gemm_ms = time_ms(torch, lambda: ah.adahop_gemm_mx(ac, asc, bc, bsc, big.C, gemm_ws), max(5, args.steps))
    achieved = big.flops / (gemm_ms * 1e-3) / 1e12
    # The same launch as it runs inside a step: right after the two quantisers that produce its operands (which
    # leave the packed operands, not C, in the caches, and the chip in the state a bandwidth-bound kernel leaves it).
    iters = max(5, args.steps)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for it in range(iters + 1):
        ah.adahop_iht_quantize(big.A, big.g.iht_block, None, None, ac, asc)
        ah.adahop_iht_quantize(big.B, big.g.iht_block, None, None, bc, bsc)
        if it:
            ev[it - 1][0].record()
        ah.adahop_gemm_mx(ac, asc, bc, bsc, big.C, gemm_ws)
        if it:
            ev[it - 1][1].record()
    torch.cuda.synchronize()
    in_step_ms = sum(a.elapsed_time(b) for a, b in ev) / iters
    in_step = big.flops / (in_step_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "mxfp4 gemm", "achieved": achieved, "peak": MXFP4_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MXFP4_PEAK_TFLOPS,
                "traffic": GEMM_HBM_TRAFFIC_BYTES.get((big.M, big.N, big.K)),
                "traffic_source": (GEMM_HBM_TRAFFIC_SOURCE[(big.M, big.N, big.K)] + " (rocprofv3 --pmc runs; not measured in "
                                   "this run)") if (big.M, big.N, big.K) in GEMM_HBM_TRAFFIC_SOURCE else None,
                "shape": [big.M, big.N, big.K], "ms": gemm_ms, "timing": "back to back, operands warm",
                "in_step_ms": in_step_ms, "in_step_achieved": in_step, "in_step_frac": in_step / MXFP4_PEAK_TFLOPS}

    out = {"metric": "effective TFLOP/s of IHT+MXFP4(+OE) GEMM vs BF16 GEMM; % MXFP4 MFMA peak",
           "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "mxfp4 (e2m1 x e8m0) with fp32 accumulate; bf16 outlier path", "data": "synthetic",
           "config": {"workload": desc, "gemms": [p.g.name for p in prepared], "flops_per_step": total_flops},
           "pct_mxfp4_peak": None if value is None else 100.0 * value / MXFP4_PEAK_TFLOPS,
           "wall_ms_per_step": wall_ms, "roofline": roofline}

    if not args.no_extras and not args.dominant_kernel_only:
        extras = {}
        # per-GEMM pipeline time and the same GEMM with pure IHT (no extraction)
        per = []
        for p in prepared:
            t_cfg = time_ms(torch, lambda: run_gemm(ah, p, ws), 5)
            t_iht = time_ms(torch, lambda: run_gemm(ah, p, ws, strategy=inputs.IHT, k=0), 5)
            am, bm = bf16_views(torch, p)
            t_bf16 = time_ms(torch, lambda: torch.matmul(am, bm), 5)
            # the same with an fp32 result, as this path delivers it (torch exposes no bf16-in / fp32-out GEMM:
            # the conversion is a second pass over C)
            t_bf16_f32 = time_ms(torch, lambda: p.C.copy_(torch.matmul(am, bm)), 3)
            per.append({"name": p.g.name, "shape": [p.M, p.N, p.K], "strategy": inputs.STRATEGY_NAMES[p.g.strategy],
                        "k": p.g.k, "ms": t_cfg, "tflops": p.flops / t_cfg / 1e9, "ms_iht_only": t_iht,
                        "tflops_iht_only": p.flops / t_iht / 1e9, "oe_overhead_pct": 100.0 * (t_cfg - t_iht) / t_iht,
                        "ms_bf16_hipblaslt": t_bf16, "tflops_bf16_hipblaslt": p.flops / t_bf16 / 1e9,
                        "ms_bf16_hipblaslt_fp32_result": t_bf16_f32,
                        "speedup_vs_bf16": t_bf16 / t_cfg})
        extras["per_gemm"] = per
        t_iht_total = sum(x["ms_iht_only"] for x in per)
        extras["iht_only_tflops"] = total_flops / t_iht_total / 1e9
        extras["iht_only_pct_mxfp4_peak"] = 100.0 * extras["iht_only_tflops"] / MXFP4_PEAK_TFLOPS
        extras["bf16_hipblaslt_tflops"] = total_flops / sum(x["ms_bf16_hipblaslt"] for x in per) / 1e9
        # bf16 C (what the paper's kernels emit): the FP4 GEMM alone on the largest shape, and the whole step
        c16 = torch.empty((big.M, big.N), dtype=torch.bfloat16, device="cuda")
        g16_ms = time_ms(torch, lambda: ah.adahop_gemm_mx(ac, asc, bc, bsc, c16, gemm_ws), max(5, args.steps))

        def step_ex(c_bf16, packed_b):
            for p in prepared:
                cb = c16.view(-1)[:p.M * p.N].view(p.M, p.N) if c_bf16 else p.C
                ah.adahop_gemm(p.A, p.B, p.g.strategy, p.g.iht_block, p.g.k, Cout=cb, workspace=ws,
                               b_packed=packed_b.get(p.g.name), c_bf16=bool(c_bf16))
        s16_ms = time_ms(torch, lambda: step_ex(1, {}), 3)
        extras["bf16_output"] = {"gemm_ms": g16_ms, "gemm_tflops": big.flops / g16_ms / 1e9, "step_ms": s16_ms,
                                 "step_tflops": total_flops / s16_ms / 1e9}
        # quantise-once reuse: operands whose residual does not depend on the extracted indices (here the
        # weight of every product that extracts rows of A or nothing) packed outside the timed region
        packed_b = {}
        for p in prepared:
            if p.g.strategy in (inputs.IHT, inputs.IHT_OE_ROW):
                packed_b[p.g.name] = ah.adahop_pack_operand(p.B, 1, p.g.strategy, p.g.iht_block)
        if packed_b:
            r_ms = time_ms(torch, lambda: step_ex(0, packed_b), 3)
            extras["b_operand_packed_once"] = {"gemms": sorted(packed_b), "step_ms": r_ms,
                                               "step_tflops": total_flops / r_ms / 1e9}
        del packed_b, c16
        # the comparison strategy of Eq. 6 on the largest product: outer transforms (block 128) + rotations of C
        if big.M % 128 == 0 and big.N % 128 == 0:
            def run_oht():
                ah.adahop_gemm(big.A, big.B, inputs.OHT, 128, Cout=big.C, workspace=ws)
            t_oht = time_ms(torch, run_oht, 5)
            t_inv = time_ms(torch, lambda: ah.adahop_oht_inverse(big.C, 128), 5)
            qa = torch.empty((big.A.outer, big.K // 2), dtype=torch.uint8, device="cuda")
            qs = torch.empty((big.A.outer, big.K // 32), dtype=torch.uint8, device="cuda")
            t_q = time_ms(torch, lambda: ah.adahop_oht_quantize(big.A, 128, qa, qs), 5)
            extras["oht_comparison"] = {"shape": [big.M, big.N, big.K], "block": 128, "pipeline_ms": t_oht,
                                        "tflops": big.flops / t_oht / 1e9, "inverse_rotations_ms": t_inv,
                                        "inverse_GBps": 8.0 * big.M * big.N / (t_inv * 1e-3) / 1e9,
                                        "quantize_a_ms": t_q,
                                        "quantize_a_GBps": 2.53125 * big.A.outer * big.K / (t_q * 1e-3) / 1e9}
            del qa, qs
        # launch-bound case (configs[0]: 256^3, IHT block 32): the same call eager and replayed from a HIP graph
        g0 = inputs.config0()[0]
        p0 = Prepared(ah, torch, g0, cache)
        ws0 = torch.empty(ah.adahop_gemm_workspace_bytes(p0.M, p0.N, p0.K, g0.strategy, g0.k), dtype=torch.uint8, device="cuda")
        run_gemm(ah, p0, ws0)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                run_gemm(ah, p0, ws0)
        torch.cuda.synchronize()
        extras["launch_bound_256cubed_us"] = {"eager": 1e3 * time_ms(torch, lambda: run_gemm(ah, p0, ws0), 200, warmup=20),
                                              "graph_replay": 1e3 * time_ms(torch, graph.replay, 200, warmup=20)}
        # what the matrix cores sustain with no memory traffic at all (register-only loop, 256 workgroups)
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        probe = {}
        for name, rnd in (("constant_operands", 0), ("random_operands", 1)):
            flop = ah.adahop_probe_mfma_rate(rnd, 256, 4000, sink)
            p_ms = time_ms(torch, lambda: ah.adahop_probe_mfma_rate(rnd, 256, 4000, sink), 3)
            probe[name] = flop / p_ms / 1e9
        for idle in (1, 2):   # idle stretches between the instructions: the clock rises, the rate falls by less than the duty
            flop = ah.adahop_probe_mfma_rate(1, 256, 4000, sink, idle_sleeps=idle)
            p_ms = time_ms(torch, lambda: ah.adahop_probe_mfma_rate(1, 256, 4000, sink, idle_sleeps=idle), 3)
            probe[f"random_operands_idle{idle}"] = flop / p_ms / 1e9
        extras["mfma_only_tflops"] = probe
        # quantiser bandwidth on the largest operand of the largest GEMM (2 + 1/2 + 1/32 bytes / element)
        qx = big.B if big.N >= big.M else big.A
        codes = torch.empty((qx.outer, qx.K // 2), dtype=torch.uint8, device="cuda")
        scales = torch.empty((qx.outer, qx.K // 32), dtype=torch.uint8, device="cuda")
        q_ms = time_ms(torch, lambda: ah.adahop_iht_quantize(qx, big.g.iht_block, None, None, codes, scales), 10)
        extras["iht_quantize"] = {"outer": qx.outer, "K": qx.K, "k_contig": qx.k_contig, "ms": q_ms,
                                  "GBps": 2.53125 * qx.outer * qx.K / (q_ms * 1e-3) / 1e9, "peak_GBps": 8000.0}
        q_sr = time_ms(torch, lambda: ah.adahop_iht_quantize(qx, big.g.iht_block, None, None, codes, scales, sr_seed=1), 10)
        extras["iht_quantize_stochastic_rounding"] = {"ms": q_sr, "GBps": 2.53125 * qx.outer * qx.K / (q_sr * 1e-3) / 1e9}
        # the same operand read K-strided (as the weight-gradient and dgrad products see their operands)
        qs = ah.Operand(qx.tensor, not qx.k_contig)
        cs = torch.empty((qs.outer, qs.K // 2), dtype=torch.uint8, device="cuda")
        ss = torch.empty((qs.outer, qs.K // 32), dtype=torch.uint8, device="cuda")
        qs_ms = time_ms(torch, lambda: ah.adahop_iht_quantize(qs, big.g.iht_block, None, None, cs, ss), 10)
        extras["iht_quantize_k_strided"] = {"outer": qs.outer, "K": qs.K, "k_contig": qs.k_contig, "ms": qs_ms,
                                            "GBps": 2.53125 * qs.outer * qs.K / (qs_ms * 1e-3) / 1e9, "peak_GBps": 8000.0}
        del codes, scales, cs, ss
        # the calibration-phase detector (App. A) on the same operand, both layouts: reads the operand once
        det = {}
        for name_, op_ in (("k_contig", qx), ("k_strided", qs)):
            dws = torch.empty(max(int(ah.lib().adahop_detect_pattern_workspace_bytes(__import__("ctypes").byref(op_.c()))), 256),
                              dtype=torch.uint8, device="cuda")
            d_ms = time_ms(torch, lambda: ah.adahop_detect_pattern(op_, 2.0, dws), 10)
            det[name_] = {"ms": d_ms, "GBps": 2.0 * op_.outer * op_.K / (d_ms * 1e-3) / 1e9}
        extras["detect_pattern"] = {"outer": qx.outer, "K": qx.K, "peak_GBps": 8000.0, **det}
        # the BF16 row / column product alone (gather, skinny product, slice reduction): bound by reading the long
        # operand once; and FOID (scores + top-k) alone
        rowp = next((p for p in prepared if p.g.strategy in (inputs.IHT_OE_ROW, inputs.IHT_OE_COL) and p.g.k > 0), None)
        if rowp is not None:
            kind = rowp.g.strategy
            long_op, dim = (rowp.B, rowp.M) if kind == inputs.IHT_OE_ROW else (rowp.A, rowp.N)
            scored = rowp.A if kind == inputs.IHT_OE_ROW else rowp.B
            sel = torch.randperm(dim, device="cuda")[:rowp.g.k].to(torch.int32)
            gws = torch.empty(ah.adahop_oe_gather_bytes(rowp.M, rowp.N, rowp.K, kind, rowp.g.k), dtype=torch.uint8, device="cuda")
            oe_ms = time_ms(torch, lambda: ah.adahop_oe_gemm_bf16(rowp.A, rowp.B, kind, sel, rowp.C, gws), 10)
            lbytes = 2.0 * long_op.outer * long_op.K
            extras["oe_row_col_product"] = {"gemm": rowp.g.name, "k": rowp.g.k, "long_operand": [long_op.outer, long_op.K],
                                            "long_operand_k_contig": bool(long_op.k_contig), "ms": oe_ms,
                                            "GBps": lbytes / (oe_ms * 1e-3) / 1e9, "peak_GBps": 8000.0,
                                            "tflops_bf16": 2.0 * rowp.g.k * long_op.outer * long_op.K / oe_ms / 1e9}
            mask = torch.empty(dim, dtype=torch.uint8, device="cuda")
            scores = torch.empty(dim, dtype=torch.float32, device="cuda")
            import ctypes as C
            f_ms = time_ms(torch, lambda: ah.lib().adahop_foid_topk(C.byref(scored.c()), 0, rowp.g.k, sel.data_ptr(),
                                                                    mask.data_ptr(), scores.data_ptr(), ah._stream(None)), 10)
            extras["foid_topk"] = {"dim": dim, "k": rowp.g.k, "ms": f_ms}
            del gws, mask, scores, sel
        if args.workload.startswith("cfg4"):
            # extraction-count sweep of configs[4]: K-channels on the up-projection forward, rows on its dgrad
            sweep = []
            for p in prepared[:2]:
                dim = p.K if p.g.strategy == inputs.IHT_OE_K else p.M
                # the pure-IHT reference is timed before and after the sweep (the smaller counts): the first timing
                # after a change of shape runs into the clock ramp of the power management
                base = lambda: run_gemm(ah, p, ws, strategy=inputs.IHT, k=0)
                t0 = time_ms(torch, base, 5, warmup=3)
                points = []
                for pc in (0.0, 0.25, 1.0, 2.0):
                    k = inputs.pct(pc, dim)
                    if k > p.idx.numel():
                        p.idx = torch.zeros(k, dtype=torch.int32, device="cuda")
                    need = ah.adahop_gemm_workspace_bytes(p.M, p.N, p.K, p.g.strategy, k)
                    if ws.numel() < need:
                        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
                    points.append((pc, k, time_ms(torch, lambda: run_gemm(ah, p, ws, k=k), 5, warmup=2)))
                t0 = min(t0, time_ms(torch, base, 5, warmup=2))
                for pc, k, t in points:
                    sweep.append({"name": p.g.name, "strategy": inputs.STRATEGY_NAMES[p.g.strategy], "k_pct": pc, "k": k,
                                  "ms": t, "ms_iht_only": t0, "oe_overhead_pct": 100.0 * (t - t0) / t0})
            extras["cfg4_k_sweep"] = sweep
            extras["per_stage_ms"] = [stage_times(ah, torch, inputs, p, ws) for p in prepared]
        elif args.workload == "paper-table3":
            # the stages of the paper's kernel latency table (right): FOID | IHT and quantise | fused product with the
            # BF16 outlier part and its scatter
            extras["per_stage_ms"] = [stage_times(ah, torch, inputs, p, ws) for p in prepared]
        out["extras"] = extras
        if args.workload == "cfg4" and not args.no_other_workloads:
            del prepared, cache, pool, ws, big, ac, asc, bc, bsc, gemm_ws
            torch.cuda.empty_cache()
            extras["other_workloads"] = {n: workload_summary(ah, torch, inputs, n) for n in ("cfg1", "cfg3", "paper-table3")}

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = src.numel() * 4
        del src, dst

    if not args.no_cpu_baseline and not args.dominant_kernel_only:
        out["cpu_baseline"] = cpu_baseline(gemms)

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
