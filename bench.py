#!/usr/bin/env python3
"""Benchmark of the QLoRA linear hot path on one MI355X.

A step is one forward + backward pass (Y, then dX, dL1, dL2) through the seven linears of one
LLaMA-65B-shaped decoder block (q/k/v/o 8192x8192, gate/up 8192x22016, down 22016x8192) at 4096
tokens with LoRA r = 64, alpha = 16 on every linear; the weights are NF4 + Double Quantization,
quantised by this library before the timed region and resident in HBM.  Successive steps cycle
through a pool of differently-seeded blocks so weights are not served from cache.

Prints ONE JSON line: the metric is fwd+bwd TFLOP/s (algorithmic FLOPs 4*M*h*o + 6*M*r*(h+o) per
linear); `roofline` is the main MFMA GEMM kernel against the bf16 dense peak, timed with HIP events
around every launch inside the timed region; `cpu_baseline` is the fp64 CPU oracle on a bounded
sample of the same workload.  The other rows of the path (quantise, standalone dequant, few-token
GEMV), the 7B- and 13B-shaped blocks and the main GEMM per shape are measured after the timed region
and reported in `extra`.
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

PEAK_BF16_TFLOPS = 2516.6      # 256 CU x 2.4 GHz x 4096 FLOP/clk/CU (dense)
PEAK_HBM_GBS = 8000.0
SECTIONS = ("plain", "quantize", "dequant", "types", "dropout", "configs", "gemv", "gemm_shapes", "adam", "stacked",
            "fused_bwd", "mfma_ceiling", "hbm_ceiling")


def _ensure_built():
    from paper_2305_14314_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)


def _time_ms(torch, fn, iters, warmup=2):
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


def _time_graph_ms(torch, fn, calls, replays=3):
    """ms per fn() with `calls` invocations captured into one HIP graph, so that the timed region holds GPU
    work only (eager launches of ~20 us kernels from Python are bound by the host)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(calls):
            fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * calls)


def _read_traffic():
    """HBM bytes per GEMM launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "gemm_nt_llama65b_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(seconds_target=16.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload: forward and input-gradient
    rows of the 8192 x 8192 linear (fp64, OpenMP), and quantise + doubleDequant of one 8192 x 22016 tensor."""
    import oracle
    from paper_2305_14314_amd import synth
    h = o = 8192
    r, s = 64, 0.25
    W = synth.normal_f32((h, o), synth.SIGMA_W, synth.tensor_seed(3, 0, "W"))
    q = oracle.nf4_quantize(W)
    What = oracle.nf4_dequant(q)
    rows = 256
    X = synth.normal_bf16((rows, h), 1.0, synth.tensor_seed(3, 0, "X"))
    dY = synth.normal_bf16((rows, o), 1.0, synth.tensor_seed(3, 0, "dY"))
    L1 = synth.normal_bf16((h, r), 0.01, synth.tensor_seed(3, 0, "L1"))
    L2 = synth.normal_bf16((r, o), 0.01, synth.tensor_seed(3, 0, "L2"))
    flops, secs, reps = 0.0, 0.0, 0
    while secs < seconds_target and reps < 16:
        t0 = time.perf_counter()
        oracle.linear_fwd(X, What, L1, L2, s)
        oracle.linear_bwd_dx(dY, What, L1, L2, s)
        secs += time.perf_counter() - t0
        flops += 2 * (2.0 * rows * h * o + 2.0 * rows * r * (h + o))
        reps += 1
    del W, q, What
    Wg = synth.normal_f32((8192, 22016), synth.SIGMA_W, synth.tensor_seed(3, 4, "W"))
    t0 = time.perf_counter()
    qg = oracle.nf4_quantize(Wg)
    t_q = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.nf4_dequant(qg)
    t_d = time.perf_counter() - t0
    el = Wg.size
    return {"value": flops / secs * 1e-12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{reps} x (Y and dX for {rows} token rows of the 8192x8192 linear, r=64), fp64 loops, "
                      f"{secs:.1f} s",
            "quantize_dequant_8192x22016": {"quantize_s": round(t_q, 3), "dequant_s": round(t_d, 3),
                                            "quantize_GBps": round(el * 4.5159 / t_q * 1e-9, 3),
                                            "dequant_GBps": round(el * 2.5159 / t_d * 1e-9, 3)}}


class Block:
    """Resident operands of one workload (a decoder block's seven linears at M tokens) and its fwd+bwd step."""

    def __init__(self, torch, ql, synth, cfg_index, pool_blocks, dev, time_quant=False):
        cfg = synth.CONFIGS[cfg_index]
        self.torch, self.ql = torch, ql
        self.M, self.r = cfg["M"], cfg["r"]
        self.s = cfg["alpha"] / self.r
        self.linears = cfg["linears"]
        M, r, linears = self.M, self.r, self.linears
        widths = sorted({w for hw in linears for w in hw})
        # weights are drawn on the device, one tensor at a time, quantised into preallocated buffers and discarded;
        # the quantise row is timed here: HIP events around the calls of a block, back to back on the stream
        self.pool = [[ql.nf4_alloc(h, o, dev) for h, o in linears] for _ in range(pool_blocks)]
        self.t_quant_ms, self.quant_elems = 0.0, 0
        scratch = torch.empty(max(ql.qlora_nf4_sizes(h, o)[3] for h, o in linears), dtype=torch.uint8, device=dev)
        for b in range(pool_blocks):
            Ws = [synth.normal_f32_device((h, o), synth.SIGMA_W, synth.tensor_seed(cfg_index, li, "W") + b, dev)
                  for li, (h, o) in enumerate(linears)]
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for li in range(len(linears)):
                ql.qlora_nf4_quantize(Ws[li], scratch=scratch, out=self.pool[b][li])
            e1.record()
            torch.cuda.synchronize()
            if b > 0 and time_quant:                            # the first block warms up
                self.t_quant_ms += e0.elapsed_time(e1)
                self.quant_elems += sum(h * o for h, o in linears)
            del Ws
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.BASE_SEED + (0 if cfg_index == 3 else cfg_index))
        self.rnd = lambda *shape, sd=1.0: (torch.randn(*shape, device=dev, dtype=torch.float32, generator=gen) * sd).to(
            torch.bfloat16)
        rnd = self.rnd
        empty = lambda *shape: torch.empty(*shape, device=dev, dtype=torch.bfloat16)
        self.X = {w: rnd(M, w) for w in widths}
        self.dY = {w: rnd(M, w) for w in widths}
        self.L1 = [rnd(h, r, sd=cfg["sigma_l"]) for h, o in linears]
        self.L2 = [rnd(r, o, sd=cfg["sigma_l"]) for h, o in linears]
        self.Y = {w: empty(M, w) for w in widths}
        self.dX = {w: empty(M, w) for w in widths}
        self.T = [empty(M, 2 * r) for _ in linears]
        self.dL1 = [torch.empty_like(a) for a in self.L1]
        self.dL2 = [torch.empty_like(a) for a in self.L2]
        ws_bytes = max(max(ql.qlora_linear_fwd_sizes(M, h, o, r), ql.qlora_linear_bwd_sizes(M, h, o, r)) for h, o in linears)
        self.ws = ql.workspace_alloc(ws_bytes, dev)
        self.flops_step = sum(4.0 * M * h * o + 6.0 * M * r * (h + o) for h, o in linears)

    def step(self, k):
        ql, s = self.ql, self.s
        block = self.pool[k % len(self.pool)]
        for li, (h, o) in enumerate(self.linears):
            ql.qlora_linear_fwd(self.X[h], block[li], self.L1[li], self.L2[li], s, Y=self.Y[o], T_save=self.T[li],
                                workspace=self.ws)
        for li in reversed(range(len(self.linears))):
            h, o = self.linears[li]
            ql.qlora_linear_bwd(self.dY[o], self.X[h], block[li], self.L1[li], self.L2[li], s, T_saved=self.T[li],
                                dX=self.dX[h], dL1=self.dL1[li], dL2=self.dL2[li], workspace=self.ws)

    def timed_steps(self, steps, warmup, first=0):
        """(ms per step from the host clock, GEMM ms, launches, FLOPs from HIP events around every main-GEMM launch)"""
        torch, ql = self.torch, self.ql
        for k in range(warmup):
            self.step(first + k)
        torch.cuda.synchronize()
        ql.qlora_profile_gemm(True)
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(first + warmup + k)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ql.qlora_profile_gemm(False)
        gemm_ms, launches, gemm_flops = ql.qlora_profile_gemm_read()
        return (t1 - t0) * 1e3 / steps, gemm_ms, launches, gemm_flops


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--pool-blocks", type=int, default=80, help="differently-seeded weight blocks resident in HBM")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--sections", default="all",
                    help="comma-separated parts of `extra` to run, of " + ",".join(SECTIONS) + " (default all); "
                         "profiling runs name the part whose kernels they want")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 512 MiB device copy, the known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build is single-GPU; --gpus must be 1 (tokens would shard across GPUs with one "
                         "sum of the adapter gradients per step; that path is not built)\n")
        sys.exit(2)
    want = lambda name: not args.no_extra and (args.sections == "all" or name in args.sections.split(","))

    _ensure_built()
    import torch
    import paper_2305_14314_amd as ql
    from paper_2305_14314_amd import synth

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    B = Block(torch, ql, synth, 3, args.pool_blocks, dev, time_quant=True)
    M, r, s, linears, pool = B.M, B.r, B.s, B.linears, B.pool
    d, ffn = 8192, 22016
    X, dY, L1, L2, Y, dX, T, ws = B.X, B.dY, B.L1, B.L2, B.Y, B.dX, B.T, B.ws
    flops_step = B.flops_step

    if args.pmc_calibration:
        src = torch.empty(512 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step, gemm_ms, gemm_launches, gemm_flops = B.timed_steps(args.steps, args.warmup)
    tflops = flops_step / (ms_per_step * 1e-3) * 1e-12
    achieved = gemm_flops / (gemm_ms * 1e-3) * 1e-12 if gemm_ms > 0 else 0.0
    out = {
        "metric": "QLoRA linear fwd+bwd TFLOP/s (% bf16 MFMA peak); 4-bit GEMV HBM GB/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[3]: LLaMA-65B-shaped block, 7 linears (4x 8192x8192, 2x 8192x22016, "
                               "1x 22016x8192), NF4+DQ weights, LoRA r=64 alpha=16, 4096 tokens bf16, fwd+bwd",
                   "tokens": M, "r": r, "pool_blocks": len(pool), "flops_per_step": flops_step,
                   "pct_of_bf16_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2)},
        "roofline": {"bound": "mfma", "kernel": "gemm_nt_kernel", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": _read_traffic(),
                     "traffic_source": "profiles/gemm_nt_llama65b_pmc.txt (rocprofv3 --pmc runs of this command, "
                                       "committed; not measured in this run)",
                     "launches": gemm_launches,
                     "avg_launch_ms": round(gemm_ms / max(1, gemm_launches), 5),
                     "flops_per_launch": gemm_flops / max(1, gemm_launches)},
    }

    extra = {}
    if want("plain"):
        # the same steps without the HIP events around the GEMM launches: each recorded event is a marker of its own
        # on the stream and costs a bubble of 4-5 us before and after the kernel it brackets (28 per step)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            B.step(args.warmup + args.steps + k)
        torch.cuda.synchronize()
        ms_plain = (time.perf_counter() - t0) * 1e3 / args.steps
        extra["step_without_gemm_events"] = {"ms_per_step": round(ms_plain, 4),
                                             "TFLOPs": round(flops_step / (ms_plain * 1e-3) * 1e-12, 2)}
    if want("quantize") and B.quant_elems:
        gbs_q = B.quant_elems * 4.5159 / (B.t_quant_ms * 1e-3) * 1e-9
        extra["quantize"] = {"GBps": round(gbs_q, 1), "frac_hbm": round(gbs_q / PEAK_HBM_GBS, 4),
                             "elements": B.quant_elems, "ms": round(B.t_quant_ms, 3), "bytes_per_element": 4.5159}
    if want("dequant"):
        # standalone doubleDequant over the pool (cold weights): 0.5159 B read + 2 B written per element
        outb = torch.empty(ffn * d, dtype=torch.bfloat16, device=dev)
        k = [0]

        def deq():
            blk = pool[k[0] % len(pool)]
            k[0] += 1
            for Wq in blk:
                ql.qlora_nf4_dequant(Wq, out=outb[:Wq.rows * Wq.cols].view(Wq.rows, Wq.cols))
        t = _time_ms(torch, deq, max(4, len(pool)))
        el = sum(h * o for h, o in linears)
        extra["dequant"] = {"GBps": round(el * 2.5159 / (t * 1e-3) * 1e-9, 1),
                            "frac_hbm": round(el * 2.5159 / (t * 1e-3) * 1e-9 / PEAK_HBM_GBS, 4),
                            "bytes_per_element": 2.5159}
        del outb
    if want("stacked"):
        # the layers of a block that read one input, forward only: one call per layer against one stacked call
        # (one matrix product over all outputs, adapters block-diagonal in the second contraction segment)
        st = {}
        for name, idx in (("qkv", [0, 1, 2]), ("gate_up", [4, 5])):
            n = len(idx)
            outs = [linears[i][1] for i in idx]
            Ys = [torch.empty((M, o_), dtype=torch.bfloat16, device=dev) for o_ in outs]
            Yst = torch.empty((M, sum(outs)), dtype=torch.bfloat16, device=dev)
            ws_st = ql.workspace_alloc(ql.qlora_linear_fwd_stacked_sizes(M, d, outs, [r] * n), dev)
            k = [0]

            def separate():
                blk = pool[k[0] % len(pool)]
                k[0] += 1
                for j, i in enumerate(idx):
                    ql.qlora_linear_fwd(X[d], blk[i], L1[i], L2[i], s, Y=Ys[j], workspace=ws)

            def stacked():
                blk = pool[k[0] % len(pool)]
                k[0] += 1
                ql.qlora_linear_fwd_stacked(X[d], [blk[i] for i in idx], [L1[i] for i in idx],
                                            [L2[i] for i in idx], [s] * n, Y=Yst, workspace=ws_st)
            t_sep = _time_ms(torch, separate, 12)
            t_st = _time_ms(torch, stacked, 12)
            st[name] = {"separate_us": round(t_sep * 1e3, 1), "stacked_us": round(t_st * 1e3, 1),
                        "stacked_over_separate": round(t_st / t_sep, 4)}
            del Ys, Yst, ws_st
            # backward (input gradient and adapter gradients): one call per layer, whose input gradients a block then
            # has to add up (two or one elementwise sums of M x h), against one stacked call that writes the sum
            dYst = B.rnd(M, sum(outs))
            dYs = [dYst[:, j * outs[0]:(j + 1) * outs[0]].contiguous() for j in range(n)]
            dXs = [torch.empty((M, d), dtype=torch.bfloat16, device=dev) for _ in range(n)]
            dXst = torch.empty((M, d), dtype=torch.bfloat16, device=dev)
            ws_sb = ql.workspace_alloc(ql.qlora_linear_bwd_stacked_sizes(M, d, outs, [r] * n), dev)

            def separate_bwd(add=True):
                blk = pool[k[0] % len(pool)]
                k[0] += 1
                for j, i in enumerate(idx):
                    ql.qlora_linear_bwd(dYs[j], X[d], blk[i], L1[i], L2[i], s, T_saved=T[i], dX=dXs[j], dL1=B.dL1[i],
                                        dL2=B.dL2[i], workspace=ws)
                if add:
                    for j in range(1, n):
                        dXs[0].add_(dXs[j])

            def stacked_bwd():
                blk = pool[k[0] % len(pool)]
                k[0] += 1
                ql.qlora_linear_bwd_stacked(dYst, X[d], [blk[i] for i in idx], [L1[i] for i in idx], [L2[i] for i in idx],
                                            [s] * n, T_saveds=[T[i] for i in idx], dX=dXst, workspace=ws_sb,
                                            dL1s=[B.dL1[i] for i in idx], dL2s=[B.dL2[i] for i in idx])
            t_sep = _time_ms(torch, separate_bwd, 12)
            t_sep0 = _time_ms(torch, lambda: separate_bwd(False), 12)
            t_st = _time_ms(torch, stacked_bwd, 12)
            st[name + "_bwd"] = {"separate_with_sums_us": round(t_sep * 1e3, 1), "separate_without_sums_us": round(t_sep0 * 1e3, 1),
                                 "stacked_us": round(t_st * 1e3, 1), "stacked_over_separate_with_sums": round(t_st / t_sep, 4)}
            del dYst, dYs, dXs, dXst, ws_sb
        extra["stacked"] = st
    if want("mfma_ceiling"):
        # what the matrix cores sustain on this board under its power limit: a register-only loop of the GEMM's MFMA on
        # Gaussian operands, one wave per SIMD, without LDS traffic, with the fragment reads of the GEMM's wave tile, and
        # with those and the LDS writes of its operand tiles (everything the GEMM does except fetching the tiles)
        outp = torch.empty(256 * 256, dtype=torch.float32, device=dev)
        cz = {}
        modes = (("registers_only", 0), ("with_fragment_reads", 1), ("with_fragment_reads_and_tile_writes", 2))
        for name, reads in modes + modes:
            fl = [0.0]

            def probe():
                fl[0] = ql.qlora_mfma_probe(reads, 200000, out=outp)   # ~25 ms a call: long enough for the power limit to act
            t = _time_ms(torch, probe, 3)
            cz[name + "_TFLOPs"] = max(cz.get(name + "_TFLOPs", 0.0), round(fl[0] / (t * 1e-3) * 1e-12, 1))
        cz["gemm_over_ceiling_with_reads_and_writes"] = round(achieved / cz["with_fragment_reads_and_tile_writes_TFLOPs"], 4)
        cz["note"] = ("16x16x32 bf16 MFMAs on N(0,1) operands in registers, 256 CUs x 4 waves; the board's power limit sets "
                      "these rates, and they depend on the operand values")
        extra["mfma_ceiling"] = cz
        del outp
    if want("hbm_ceiling"):
        # what plain streams reach on this board: 1 GiB read, written, and copied, by the library's probe kernel
        a_ = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        b_ = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        hz = {}
        for name, mode, nbuf in (("read", 0, 1), ("write", 1, 1), ("copy_read_plus_write", 2, 2)):
            best = 0.0
            for wgs in (4, 8, 16):
                t = _time_ms(torch, lambda: ql.qlora_hbm_probe(mode, a_ if mode != 1 else None, b_ if mode != 0 else None,
                                                                 sink, wgs), 6)
                best = max(best, nbuf * (1 << 30) / (t * 1e-3) * 1e-9)
            hz[name + "_GBps"] = round(best, 1)
            hz[name + "_frac_hbm"] = round(best / PEAK_HBM_GBS, 4)
        hz["note"] = "16-byte accesses, four in flight per lane, 4 / 8 / 16 workgroups of 256 threads per CU (best of the three)"
        extra["hbm_ceiling"] = hz
        del a_, b_, sink
    if want("fused_bwd"):
        # the input gradient of one layer in its two forms: dequantise into the workspace, then multiply (what the step
        # runs), against the product that decodes the weight's tiles itself (the bf16 weight is never in HBM)
        fb = {}
        for i in (0, 6):                                       # a square layer and the down projection
            h_, o_ = linears[i]
            dX_ = torch.empty((M, h_), dtype=torch.bfloat16, device=dev)
            k = [0]

            def dx_only():
                blk = pool[k[0] % len(pool)]
                k[0] += 1
                ql.qlora_linear_bwd(dY[o_], None, blk[i], L1[i], L2[i], s, dX=dX_, need_dL=False, workspace=ws)
            t = {}
            for mode in (0, 1, 0, 1):
                prev = ql.qlora_bwd_fused_dequant(mode)
                tm = _time_ms(torch, dx_only, 8)
                ql.qlora_bwd_fused_dequant(prev)
                t[mode] = min(t.get(mode, tm), tm)
            fb[f"{h_}x{o_}"] = {"dequant_then_gemm_us": round(t[0] * 1e3, 1), "fused_us": round(t[1] * 1e3, 1),
                               "fused_over_two_kernels": round(t[1] / t[0], 4)}
            del dX_
        extra["fused_bwd"] = fb
    if want("adam"):
        # optimizer step on the adapters of 8 blocks (80 M parameters in one flat buffer): global-norm pass over the
        # gradient, then Adam with clipping, the bf16 copy and the cleared gradient: 4 + 34 bytes per parameter
        n_par = 8 * sum(h * r + r * o for h, o in linears)
        pa = [torch.zeros(n_par, dtype=torch.float32, device=dev) for _ in range(3)]
        ga = torch.randn(n_par, dtype=torch.float32, device=dev) * 1e-3
        pb = torch.empty(n_par, dtype=torch.bfloat16, device=dev)
        acc = torch.zeros(1, dtype=torch.float64, device=dev)
        tstep = [0]

        def adam():
            tstep[0] += 1
            acc.zero_()
            ql.qlora_grad_sqnorm(ga, acc)
            ql.qlora_adam_step(pa[0], pa[1], pa[2], ga, tstep[0], 1e-4, 0.9, 0.999, 1e-8, grad_scale=1.0 / 16,
                               max_grad_norm=0.3, sqnorm=acc, param_bf16=pb, zero_grad=True)
        t = _time_ms(torch, adam, 10)
        extra["adam"] = {"params": n_par, "us": round(t * 1e3, 1), "bytes_per_param": 38,
                         "GBps": round(n_par * 38 / (t * 1e-3) * 1e-9, 1),
                         "frac_hbm": round(n_par * 38 / (t * 1e-3) * 1e-9 / PEAK_HBM_GBS, 4)}
        del pa, ga, pb
    if want("types"):
        # the data types of the paper's comparison (Section 4) on one 8192 x 8192 N(0, 0.02) tensor: round-trip error
        # of quantise + doubleDequant in units of sigma (NF4 is the smallest), and the rate of the quantise pass
        # when the decision thresholds arrive at run time
        Wn = synth.normal_f32_device((d, d), synth.SIGMA_W, 424242)
        types = {}
        for name, dt in (("nf4", ql.NF4), ("fp4_e2m1", ql.FP4_E2M1), ("fp4_e3m0", ql.FP4_E3M0), ("int4", ql.INT4),
                         ("nf3", ql.NF3), ("nf2", ql.NF2)):
            Wq_t = ql.qlora_quantize_4bit(Wn, dt)
            err = (ql.qlora_nf4_dequant(Wq_t).float() - Wn).abs().mean().item() / synth.SIGMA_W
            t = _time_ms(torch, lambda: ql.qlora_quantize_4bit(Wn, dt, out=Wq_t), 5)
            types[name] = {"mean_abs_err_over_sigma": round(err, 4),
                           "quantize_GBps": round(d * d * 4.5159 / (t * 1e-3) * 1e-9, 1)}
            del Wq_t
        Wq_t = ql.qlora_nf4_quantize(Wn, dq_blocksize=0)                 # NF4 without Double Quantization: 4.5 bit
        types["nf4_without_dq"] = {
            "mean_abs_err_over_sigma": round((ql.qlora_nf4_dequant(Wq_t).float() - Wn).abs().mean().item() / synth.SIGMA_W, 4),
            "bits_per_param": Wq_t.nbytes * 8 / (d * d)}
        del Wq_t
        Wq_t = ql.qlora_quantize_int8(Wn)                                # Eq. 1 / Eq. 2 as printed: 8-bit integers
        t = _time_ms(torch, lambda: ql.qlora_quantize_int8(Wn, out=Wq_t), 5, warmup=1)
        Wd_t = torch.empty((d, d), dtype=torch.bfloat16, device=dev)
        t2 = _time_ms(torch, lambda: ql.qlora_nf4_dequant(Wq_t, out=Wd_t), 5, warmup=1)
        types["int8"] = {
            "mean_abs_err_over_sigma": round((ql.qlora_nf4_dequant(Wq_t).float() - Wn).abs().mean().item() / synth.SIGMA_W, 5),
            "bits_per_param": round(Wq_t.nbytes * 8 / (d * d), 4),
            "quantize_GBps": round(d * d * (4 + 1.0159) / (t * 1e-3) * 1e-9, 1),
            "dequant_GBps": round(d * d * (1.0159 + 2) / (t2 * 1e-3) * 1e-9, 1)}
        del Wq_t, Wd_t
        del Wn
        extra["data_types"] = types
    if want("dropout"):
        # the training-loop variants of the same step (same pool, same shapes): LoRA dropout at the rate the paper
        # uses for 65B (seeded keep-masks, one per input width) and adapter gradients accumulated in fp32
        p_drop = 0.05
        gen_m = torch.Generator(device=dev)
        gen_m.manual_seed(synth.BASE_SEED + 1)
        masks = {w: ql.pack_keep_mask(torch.rand(M, w, device=dev, generator=gen_m) >= p_drop) for w in (d, ffn)}
        ws_drop = ql.workspace_alloc(max(max(ql.qlora_linear_dropout_sizes(M, h, o, r)) for h, o in linears), dev)
        a1 = [torch.zeros(h, r, dtype=torch.float32, device=dev) for h, o in linears]
        a2 = [torch.zeros(r, o, dtype=torch.float32, device=dev) for h, o in linears]
        kd = [0]

        def step_dropout():
            block = pool[kd[0] % len(pool)]
            kd[0] += 1
            for li, (h, o) in enumerate(linears):
                ql.qlora_linear_fwd_dropout(X[h], block[li], L1[li], L2[li], s, masks[h], p_drop, Y=Y[o], T_save=T[li],
                                            workspace=ws_drop)
            for li in reversed(range(len(linears))):
                h, o = linears[li]
                ql.qlora_linear_bwd_dropout(dY[o], X[h], block[li], L1[li], L2[li], s, masks[h], p_drop, T_saved=T[li],
                                            dX=dX[h], dL1_acc=a1[li], dL2_acc=a2[li], workspace=ws_drop)
        t = _time_ms(torch, step_dropout, 5, warmup=1)
        extra["step_with_dropout_and_fp32_accumulation"] = {
            "ms_per_step": round(t, 4), "TFLOPs": round(flops_step / (t * 1e-3) * 1e-12, 2), "p": p_drop}
        del masks, ws_drop, a1, a2
    if want("gemv"):
        # few-token regime (workload configs[4]): forward and input gradient at 1, 4, 16 tokens
        gemv = {}
        rnd = B.rnd
        for m in cfg_few_tokens():
            Xs = {d: rnd(m, d), ffn: rnd(m, ffn)}
            Ys = {d: torch.empty(m, d, device=dev, dtype=torch.bfloat16),
                  ffn: torch.empty(m, ffn, device=dev, dtype=torch.bfloat16)}
            hs, os_ = [h for h, o in linears], [o for h, o in linears]
            wsz = max(max(ql.qlora_linear_fwd_sizes(m, h, o, r), ql.qlora_linear_bwd_sizes(m, h, o, r))
                      for h, o in linears)
            wsz = max(wsz, ql.qlora_linear_fwd_multi_sizes(m, d, [d] * 3, [r] * 3),
                      ql.qlora_linear_fwd_multi_sizes(m, d, [ffn] * 2, [r] * 2),
                      ql.qlora_linear_list_sizes(m, hs, os_, [r] * 7, False),
                      ql.qlora_linear_list_sizes(m, hs, os_, [r] * 7, True))
            wss = ws[:wsz]
            kk = [0]
            Yqkv = [torch.empty(m, d, device=dev, dtype=torch.bfloat16) for _ in range(3)]
            Ygu = [torch.empty(m, ffn, device=dev, dtype=torch.bfloat16) for _ in range(2)]
            Yl = [torch.empty(m, o, device=dev, dtype=torch.bfloat16) for h, o in linears]
            dXl = [torch.empty(m, h, device=dev, dtype=torch.bfloat16) for h, o in linears]
            Xl = [Xs[h] for h, o in linears]
            dYl = [Xs[o] for h, o in linears]

            def next_block():
                blk = pool[kk[0] % len(pool)]
                kk[0] += 1
                return blk

            def few_fwd_grouped():
                # the layers of a block that read the same input in one launch each: q/k/v, then o, gate/up, down
                blk = next_block()
                ql.qlora_linear_fwd_multi(Xs[d], blk[0:3], L1[0:3], L2[0:3], [s] * 3, Ys=Yqkv, workspace=wss)
                ql.qlora_linear_fwd(Xs[d], blk[3], L1[3], L2[3], s, Y=Ys[d], workspace=wss)
                ql.qlora_linear_fwd_multi(Xs[d], blk[4:6], L1[4:6], L2[4:6], [s] * 2, Ys=Ygu, workspace=wss)
                ql.qlora_linear_fwd(Xs[ffn], blk[6], L1[6], L2[6], s, Y=Ys[d], workspace=wss)

            def few_fwd():
                blk = next_block()
                for li, (h, o) in enumerate(linears):
                    ql.qlora_linear_fwd(Xs[h], blk[li], L1[li], L2[li], s, Y=Ys[o], workspace=wss)

            def few_bwd():
                blk = next_block()
                for li, (h, o) in enumerate(linears):
                    ql.qlora_linear_bwd(Xs[o], None, blk[li], L1[li], L2[li], s, dX=Ys[h], need_dL=False,
                                        workspace=wss)

            def few_fwd_list():                              # the block's seven linears as one persistent launch
                ql.qlora_linear_fwd_list(Xl, next_block(), L1, L2, [s] * 7, Ys=Yl, workspace=wss)

            def few_bwd_list():
                ql.qlora_linear_bwd_list(dYl, next_block(), L1, L2, [s] * 7, dXs=dXl, workspace=wss)

            bytes_block = sum(h * o * 0.51587 for h, o in linears)
            gbs = lambda t_ms: bytes_block / (t_ms * 1e-3) * 1e-9
            tfe = _time_ms(torch, few_fwd, 2 * len(pool))
            tbe = _time_ms(torch, few_bwd, 2 * len(pool))
            res = {}
            for name, fn in (("single", few_fwd), ("single_bwd", few_bwd), ("grouped", few_fwd_grouped),
                             ("list", few_fwd_list), ("list_bwd", few_bwd_list)):
                kk[0] = 0
                res[name] = _time_graph_ms(torch, fn, len(pool))
            # the headline few-token figures are the list launches: one call per block and direction
            gemv[f"tokens_{m}"] = {"fwd_GBps": round(gbs(res["list"]), 1), "bwd_dx_GBps": round(gbs(res["list_bwd"]), 1),
                                   "fwd_frac_hbm": round(gbs(res["list"]) / PEAK_HBM_GBS, 4),
                                   "bwd_dx_frac_hbm": round(gbs(res["list_bwd"]) / PEAK_HBM_GBS, 4),
                                   "fwd_us_per_block": round(res["list"] * 1e3, 2),
                                   "bwd_us_per_block": round(res["list_bwd"] * 1e3, 2),
                                   "fwd_single_calls_GBps": round(gbs(res["single"]), 1),
                                   "fwd_single_calls_frac_hbm": round(gbs(res["single"]) / PEAK_HBM_GBS, 4),
                                   "bwd_dx_single_calls_GBps": round(gbs(res["single_bwd"]), 1),
                                   "bwd_dx_single_calls_frac_hbm": round(gbs(res["single_bwd"]) / PEAK_HBM_GBS, 4),
                                   "fwd_single_us_per_linear": round(res["single"] * 1e3 / 7, 2),
                                   "bwd_single_us_per_linear": round(res["single_bwd"] * 1e3 / 7, 2),
                                   "fwd_grouped_GBps": round(gbs(res["grouped"]), 1),
                                   "fwd_grouped_frac_hbm": round(gbs(res["grouped"]) / PEAK_HBM_GBS, 4),
                                   "fwd_grouped_us_per_block": round(res["grouped"] * 1e3, 2),
                                   "fwd_eager_GBps": round(gbs(tfe), 1), "bwd_dx_eager_GBps": round(gbs(tbe), 1)}
        extra["gemv"] = {"bytes_per_weight": 0.51587, "note": "packed + 8-bit constants + c1 traffic only; weights "
                         "cycle through the resident pool; one pass over the pool captured in a HIP graph (the eager "
                         "figures include Python launch cost); fwd / bwd_dx: the seven linears of a block as ONE "
                         "launch (qlora_linear_fwd_list / _bwd_list, every layer with its own input); single_calls: "
                         "seven launches; grouped: q/k/v and gate/up, which read the same input, as one launch each "
                         "(4 launches per block)", **gemv}
    if want("gemm_shapes"):
        # the main GEMM alone, per shape (dX = dY What^T, no adapter), beside torch.matmul on the same operands
        # (the vendor GEMM library, for context: same shape, same data, same NT layout)
        by_shape = {}
        for (h, o) in sorted(set(linears)):
            Wq = pool[0][linears.index((h, o))]
            Wd = ql.qlora_nf4_dequant(Wq)
            bwd = lambda: ql.qlora_linear_bwd(dY[o], None, Wq, None, None, s, dX=dX[h], need_dL=False, workspace=ws)
            for _ in range(2):
                bwd()
            torch.cuda.synchronize()
            ql.qlora_profile_gemm(True)
            ql.qlora_profile_gemm_read()
            for _ in range(8):
                bwd()
            torch.cuda.synchronize()
            ql.qlora_profile_gemm(False)
            g_ms, g_n, g_fl = ql.qlora_profile_gemm_read()
            t_lib = _time_ms(torch, lambda: torch.matmul(dY[o], Wd.t(), out=dX[h]), 8)
            by_shape[f"M{M}_N{h}_K{o}"] = {"gemm_nt_TFLOPs": round(g_fl / (g_ms * 1e-3) * 1e-12, 1),
                                           "torch_matmul_TFLOPs": round(2.0 * M * h * o / (t_lib * 1e-3) * 1e-12, 1)}
            del Wd
        extra["gemm_by_shape"] = by_shape
    if want("configs"):
        # the 7B- and 13B-shaped blocks at 8192 tokens (workloads configs[1], configs[2]): the same fwd + bwd step
        cfgs = {}
        for ci in (1, 2):
            Bc = Block(torch, ql, synth, ci, min(8, args.pool_blocks), dev)
            ms, g_ms, g_n, g_fl = Bc.timed_steps(max(4, args.steps // 2), 2)
            tf = Bc.flops_step / (ms * 1e-3) * 1e-12
            cfgs[synth.CONFIGS[ci]["name"]] = {
                "tokens": Bc.M, "ms_per_step": round(ms, 4), "TFLOPs": round(tf, 2),
                "pct_of_bf16_peak": round(100.0 * tf / PEAK_BF16_TFLOPS, 2), "flops_per_step": Bc.flops_step,
                "gemm_TFLOPs": round(g_fl / (g_ms * 1e-3) * 1e-12, 2) if g_ms > 0 else None,
                "gemm_frac": round(g_fl / (g_ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4) if g_ms > 0 else None}
            del Bc
            torch.cuda.empty_cache()
        extra["other_configs"] = cfgs
    out["extra"] = extra

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


def cfg_few_tokens():
    from paper_2305_14314_amd import synth
    return synth.CONFIGS[4]["M"]


if __name__ == "__main__":
    main()
