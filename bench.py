#!/usr/bin/env python3
"""Benchmark of the SPION sparse-attention path on one MI355X.

A step is one forward + backward pass of the block-sparse attention (SDDMM, row softmax, SpMM and
their gradients) of every layer of the workload, each with the pattern that spion_pattern produced
for it; pattern generation happens once per layer in the method and is timed separately.  Inputs
are synthetic (seeded) and already resident in HBM.  The step rotates through several buffer sets,
together larger than the 256 MB Infinity Cache, so that every step streams its tensors from HBM
("cold", the headline); the same loop on one buffer set ("warm") is reported next to it.

Default workload: cfg4_bf16_L4096 (B=4, H=4, L=4096, d=64, bf16, block 64, ~8 % of the blocks kept),
the configuration the metric is quoted on; after it the default run also times the 4-layer stack of
configuration 5 (`stack`: per-layer times and their imbalance).  `--workload cfg5` makes the stack
the headline instead; any other workload name runs that workload alone.

Prints ONE JSON line: metric / value / ms_per_step for the whole step; `roofline` (achieved
algorithmic GB/s of the longest phase against the HBM peak, with measured traffic when a profile is
on file) and `roofline_mfma`; `path` (whole-step fractions, warm timing); `layers` (per-layer phase
times: forward call, backward call, and each side of the backward launched alone); `pattern`
(spion_pattern timing, and its convolution + pooling stage alone); `stack`; `density_sweep` (the
same step on random block masks of 2-30 % density, made by the no-fill variant of spion_pattern);
`producers` (score-map mean and Frobenius distance); `ceilings` (what a plain copy and a library bf16
GEMM reach on this GPU); `streaming_floor` (the time a plain device copy needs for each phase's
algorithmic bytes at this size); `cpu_baseline` (the CPU oracle).
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

PHASES = ("fwd", "bwd")          # the two library calls of a step
DEFAULT_WORKLOAD = "cfg4_bf16_L4096"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    help="a workload name from spion_inputs.WORKLOADS, or cfg5 for the 4-layer stack")
    ap.add_argument("--variant", default="density", choices=("density", "one_minus_target"),
                    help="which quantiles the workloads use (see spion_inputs)")
    ap.add_argument("--sets", type=int, default=0,
                    help="rotating buffer sets per layer (0: enough to exceed the Infinity Cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stack", action="store_true", help="skip the 4-layer stack after the default workload")
    ap.add_argument("--stack-steps", type=int, default=40)
    ap.add_argument("--pattern-iters", type=int, default=20)
    ap.add_argument("--preroll-ms", type=float, default=300.0,
                    help="untimed steps run for this long before the warm-up steps")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the density sweep, the producer kernels and the measured ceilings")
    return ap.parse_args()


def read_traffic(workload: str, phase: str):
    """HBM bytes per call of `phase` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    recorded in profiles/traffic_<workload>.txt (lines "phase fetch_bytes write_bytes"); None if
    no such measurement is on file."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload)
    try:
        with open(path) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) == 3 and parts[0] == phase:
                    return int(float(parts[1]) + float(parts[2]))
    except OSError:
        pass
    return None


def event_ms(torch, fn, iters, warmup=3):
    """Mean milliseconds per call of fn(), timed with events on the current stream."""
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


class Bench:
    """Buffers, patterns and timing loops of one workload (one or several layers)."""

    def __init__(self, sp, acc, si, torch, dev, layers, n_sets, pattern_iters, flush):
        self.sp, self.acc, self.torch, self.dev = sp, acc, torch, dev
        w0 = layers[0]
        self.w0 = w0
        self.tdt = torch.float32 if w0.dtype == "f32" else torch.bfloat16
        self.esz = 4 if w0.dtype == "f32" else 2
        self.code = sp.binding._dtype_code(self.tdt)
        self.BH = w0.B * w0.H
        self.n_sets = n_sets
        self.layers = []
        flush_words = flush.view(torch.int32)
        flush_sink = torch.zeros((), dtype=torch.int32, device=dev)
        for w in layers:
            ly = type("Layer", (), {})()
            ly.w = w
            ly.Q, ly.K, ly.V, ly.dO = si.make_qkv_do(w)
            ly.A = si.make_score_map(w, ly.Q, ly.K)
            A_dev = torch.from_numpy(ly.A).to(dev)
            ly.pat = sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value)
            ws_pat = torch.empty(sp.spion_pattern_workspace_bytes(w.L, w.block), dtype=torch.uint8, device=dev)

            def timed_pattern(flags, ly=ly, w=w, A_dev=A_dev, ws_pat=ws_pat):
                ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(pattern_iters)]
                ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(pattern_iters)]
                scratch = sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value, flags=flags,
                                              sync=False, workspace=ws_pat)
                for i in range(pattern_iters):
                    # evict A^s from the caches by READING another 512 MB (a write pass would leave the
                    # Infinity Cache full of dirty lines whose write-back then competes with the call)
                    flush_sink.copy_(flush_words.max())
                    ev0[i].record()
                    sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value, flags=flags,
                                        sync=False, out=scratch, workspace=ws_pat)
                    ev1[i].record()
                torch.cuda.synchronize()
                ms = sorted(a.elapsed_time(b) for a, b in zip(ev0, ev1))
                return ms[len(ms) // 2]

            ly.pattern_ms = timed_pattern(0)
            ly.pool_ms = timed_pattern(sp.SPION_PATTERN_POOL_ONLY)
            ly.nnzb = ly.pat.nnzb
            ly.density = ly.nnzb / float(w.nb * w.nb)
            ly.sets = []
            for _ in range(n_sets):
                q, k, v, do = [torch.from_numpy(t).to(dev).to(self.tdt).view(w.B, w.H, w.L, w.d).contiguous()
                               for t in (ly.Q, ly.K, ly.V, ly.dO)]
                s = dict(q=q, k=k, v=v, do=do, O=torch.empty_like(q), dQ=torch.empty_like(q),
                         dK=torch.empty_like(q), dV=torch.empty_like(q),
                         LSE=torch.empty((w.B, w.H, w.L), dtype=torch.float32, device=dev))
                nbytes = sp.spion_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.block, self.code, ly.nnzb, True)
                s["ws"] = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
                ly.sets.append(s)
            self.layers.append(ly)

    def fwd(self, ly, s):
        w = ly.w
        self.sp.spion_attn_fwd(s["q"], s["k"], s["v"], s["O"], s["LSE"], ly.pat.row_ptr, ly.pat.col_idx,
                               ly.nnzb, w.B, w.H, w.L, w.d, w.block, self.code)

    def bwd(self, ly, s, flags=0):
        w = ly.w
        self.sp.spion_attn_bwd(s["q"], s["k"], s["v"], s["O"], s["do"], s["LSE"], s["dQ"], s["dK"], s["dV"],
                               ly.pat.row_ptr, ly.pat.col_idx, ly.pat.col_ptr, ly.pat.row_idx, ly.pat.bsr_pos,
                               ly.nnzb, w.B, w.H, w.L, w.d, w.block, self.code, flags=flags, workspace=s["ws"])

    def run(self, n_steps, rotate):
        for i in range(n_steps):
            for ly in self.layers:
                self.fwd(ly, ly.sets[i % self.n_sets if rotate else 0])
            for ly in reversed(self.layers):
                self.bwd(ly, ly.sets[i % self.n_sets if rotate else 0])

    def timed(self, n_steps, rotate):
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(n_steps, rotate)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n_steps

    def step_times(self, steps, warmup, preroll_ms):
        """ms per step: cold (rotating buffer sets) and warm (one buffer set)."""
        # untimed pre-roll: clocks, page tables and TLBs of all buffer sets settle (a few hundred steps
        # measure ~3 % faster than the first ones on this GPU); then the W warm-up steps, then K timed
        t_end = time.perf_counter() + preroll_ms * 1e-3
        while time.perf_counter() < t_end:
            self.run(max(1, 50 // len(self.layers)), True)
            self.torch.cuda.synchronize()
        self.run(warmup, True)
        ms_cold = self.timed(steps, True)
        self.run(warmup, False)
        ms_warm = self.timed(steps, False)
        return ms_cold, ms_warm

    def phase_times(self, steps, warmup):
        """Per layer: duration of each library call of the step, and of each side of the backward
        launched alone.  HIP events on the launch stream (torch's current stream): K calls of one
        phase back to back on the rotating buffer sets between two events, so that the figure is the
        kernels' own duration (what a kernel trace shows) without an event pair per launch."""
        sp, torch = self.sp, self.torch
        phases = {"fwd": lambda ly, s: self.fwd(ly, s), "bwd": lambda ly, s: self.bwd(ly, s),
                  "bwd_query_alone": lambda ly, s: self.bwd(ly, s, sp.SPION_ATTN_BWD_QUERY_SIDE_ONLY),
                  "bwd_key_alone": lambda ly, s: self.bwd(ly, s, sp.SPION_ATTN_BWD_KEY_SIDE_ONLY)}
        out = []
        for ly in self.layers:
            km = {}
            for name, phase in phases.items():
                for i in range(warmup):
                    phase(ly, ly.sets[i % self.n_sets])
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(steps):
                    phase(ly, ly.sets[i % self.n_sets])
                e1.record()
                torch.cuda.synchronize()
                km[name] = e0.elapsed_time(e1) / steps
            fl = self.acc.useful_flops(ly.nnzb, ly.w.block, ly.w.d, self.BH, products=6)
            tot = km["fwd"] + km["bwd"]
            out.append({"layer": ly.w.layer, "nnzb": ly.nnzb, "block_density": round(ly.density, 5),
                        "kernel_ms": {k: round(v, 5) for k, v in km.items()},
                        "ms": round(tot, 5), "tflops": round(fl / (tot * 1e-3) / 1e12, 3),
                        "pattern_ms": round(ly.pattern_ms, 5), "useful_flop": fl})
        return out


def extras(sp, acc, torch, dev, w, tdt, code, BH, esz):
    """Side measurements at the workload's shape: throughput against block density, the two
    reductions that feed the pattern generator, and what plain library kernels reach on this GPU."""
    out = {}
    L, bs, d, nb = w.L, w.block, w.d, w.nb
    # density sweep: the top (density) fraction of the blocks of a random map, no fill, diagonal forced
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    A = torch.rand((L, L), generator=gen, device=dev, dtype=torch.float32)
    q, k, v, do = [torch.randn((w.B, w.H, L, d), generator=gen, device=dev, dtype=torch.float32).to(tdt)
                   for _ in range(4)]
    O, dQ, dK, dV = [torch.empty_like(q) for _ in range(4)]
    LSE = torch.empty((w.B, w.H, L), dtype=torch.float32, device=dev)
    sweep = []
    for rho in (0.02, 0.05, 0.10, 0.20, 0.30):
        pat = sp.generate_pattern(A, bs, 1, sp.SPION_T_QUANTILE, 1.0 - rho, flags=sp.SPION_PATTERN_NO_FILL)
        ws = torch.empty(max(sp.spion_attn_workspace_bytes(w.B, w.H, L, d, bs, code, pat.nnzb, True), 256),
                         dtype=torch.uint8, device=dev)

        def step():
            sp.spion_attn_fwd(q, k, v, O, LSE, pat.row_ptr, pat.col_idx, pat.nnzb, w.B, w.H, L, d, bs, code)
            sp.spion_attn_bwd(q, k, v, O, do, LSE, dQ, dK, dV, pat.row_ptr, pat.col_idx, pat.col_ptr,
                              pat.row_idx, pat.bsr_pos, pat.nnzb, w.B, w.H, L, d, bs, code, workspace=ws)

        ms = event_ms(torch, step, 30)
        fl = acc.useful_flops(pat.nnzb, bs, d, BH, products=6)
        sweep.append({"block_density": round(pat.nnzb / float(nb * nb), 4), "nnzb": pat.nnzb,
                      "ms": round(ms, 5), "tflops": round(fl / (ms * 1e-3) / 1e12, 2)})
    out["density_sweep"] = {"mask": "random blocks (no-fill variant on a uniform random map), warm buffers",
                            "points": sweep}
    # producers of the pattern input
    n_maps = 16
    maps = torch.rand((n_maps, L, L), generator=gen, device=dev, dtype=torch.float32)
    mean = torch.empty((L, L), dtype=torch.float32, device=dev)
    ms_mean = event_ms(torch, lambda: sp.score_mean(maps, out=mean), 10)
    f_out = torch.empty(3, dtype=torch.float64, device=dev)
    f_ws = torch.empty(sp.spion_frobenius_workspace_bytes(), dtype=torch.uint8, device=dev)
    ms_frob = event_ms(torch, lambda: sp.frobenius_distance(maps[0], maps[1], out=f_out, workspace=f_ws), 10)
    out["producers"] = {
        "score_mean": {"maps": n_maps, "ms": round(ms_mean, 5),
                       "GBps": round((n_maps + 1) * 4 * L * L / (ms_mean * 1e-3) / 1e9, 1)},
        "frobenius_distance": {"ms": round(ms_frob, 5), "GBps": round(2 * 4 * L * L / (ms_frob * 1e-3) / 1e9, 1)}}
    del maps
    # what library kernels reach here: a device copy and a bf16 GEMM (context for the published peaks)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    ms_copy = event_ms(torch, lambda: dst.copy_(src), 10)
    ms_yard = event_ms(torch, lambda: sp.spion_copy_yardstick(src, dst, 1 << 30), 10)
    del src, dst
    a = torch.randn((8192, 8192), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    b = torch.randn((8192, 8192), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    ms_gemm = event_ms(torch, lambda: torch.matmul(a, b), 10)
    out["ceilings"] = {"copy_GBps_read_plus_write": round(2 * (1 << 30) / (ms_copy * 1e-3) / 1e9, 1),
                       "yardstick_copy_GBps_read_plus_write": round(2 * (1 << 30) / (ms_yard * 1e-3) / 1e9, 1),
                       "gemm_bf16_8192_TFLOPs": round(2 * 8192.0 ** 3 / (ms_gemm * 1e-3) / 1e12, 1)}
    # what moving each phase's algorithmic bytes costs at this size: one device copy per phase with the
    # same byte count (half read, half written), source and destination rotating through 1 GiB so
    # that they come from HBM, timed with events like the phases themselves
    pool_a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    pool_b = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    floor = {}
    for k in PHASES:
        half = acc.algorithmic_bytes(k, BH, L, d, esz) // 2 // 256 * 256
        n_slots = (1 << 30) // half
        state = {"i": 0}

        def one(half=half, n_slots=n_slots, state=state):
            o = (state["i"] % n_slots) * half
            pool_b[o:o + half].copy_(pool_a[o:o + half])
            state["i"] += 1

        floor[k + "_us"] = round(event_ms(torch, one, 60) * 1e3, 2)
    floor["step_us"] = round(sum(floor.values()), 2)
    floor["what"] = "device copy of the same byte count per phase (half read, half written), from HBM"
    out["streaming_floor"] = floor
    return out


def main() -> int:
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (every (batch, head) pair is independent "
              "and the path uses no collectives); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2309_12578_amd as sp
    from paper_2309_12578_amd import accounting as acc
    import spion_inputs as si

    sp.load()   # fails loudly when libspion.so has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    stack_layers = [si.workload(5, l, variant=args.variant) for l in range(4)]
    if args.workload == "cfg5":
        layers = stack_layers
        wl_name = "cfg5_4layer_bf16_L4096"
    else:
        layers = [si.workload(args.workload, variant=args.variant)]
        wl_name = layers[0].name
    w0 = layers[0]
    esz = 4 if w0.dtype == "f32" else 2
    set_bytes = 8 * acc.tensor_bytes(w0.B * w0.H, w0.L, w0.d, esz)
    n_sets = args.sets if args.sets > 0 else max(2, -(-400_000_000 // (set_bytes * len(layers))))

    flush = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device=dev)
    bench = Bench(sp, acc, si, torch, dev, layers, n_sets, args.pattern_iters, flush)
    BH, tdt, code = bench.BH, bench.tdt, bench.code

    # one launch of known traffic in the library's own access shapes: the yardstick that scales
    # rocprofv3's FETCH_SIZE / WRITE_SIZE readings (see profiles/) into bytes
    cal_src = torch.empty(64 * 1024 * 1024, dtype=torch.uint8, device=dev).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    flush.fill_(0)
    sp.spion_copy_yardstick(cal_src, cal_dst, cal_src.numel())
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # ---------------------------------------------------------------- headline: cold, rotating sets
    ms_cold, ms_warm = bench.step_times(args.steps, args.warmup, args.preroll_ms)
    per_layer = bench.phase_times(args.steps, args.warmup)

    # ---------------------------------------------------------------- accounting
    flops_step = sum(p["useful_flop"] for p in per_layer)
    tflops = flops_step / (ms_cold * 1e-3) / 1e12
    peak_tf = acc.MI355X_MFMA_TFLOPS[w0.dtype]
    # dominant phase: the one with the largest summed duration over the layers; roofline on the
    # layer where it is longest
    dom = max(PHASES, key=lambda k: sum(p["kernel_ms"][k] for p in per_layer))
    dom_layer = max(per_layer, key=lambda p: p["kernel_ms"][dom])
    dom_ms = dom_layer["kernel_ms"][dom]
    dom_bytes = acc.algorithmic_bytes(dom, BH, w0.L, w0.d, esz)
    dom_gbps = dom_bytes / (dom_ms * 1e-3) / 1e9
    dom_products = 2 if dom == "fwd" else 4
    dom_tflops = acc.useful_flops(dom_layer["nnzb"], w0.block, w0.d, BH, products=dom_products) / (dom_ms * 1e-3) / 1e12
    path_bytes = acc.algorithmic_bytes("path", BH, w0.L, w0.d, esz) * len(layers)
    dom_wl = layers[dom_layer["layer"]].name if len(layers) > 1 else wl_name
    dom_kernels = {"fwd": "attn_fwd_bf16_kernel", "bwd": "attn_bwd_bf16_kernel + attn_bwd_bf16_reduce_kernel"}

    out = {
        "metric": "sparse MHA fwd+bwd useful TFLOP/s (ms per step = ms/layer x layers) at L=%d" % w0.L,
        "value": round(tflops, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_cold, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w0.dtype,
        "data": "synthetic",
        "config": {"workload": wl_name, "variant": args.variant, "layers": len(layers), "B": w0.B, "H": w0.H,
                   "L": w0.L, "d": w0.d, "block": w0.block, "filter": w0.filt,
                   "nnzb": [p["nnzb"] for p in per_layer] if len(per_layer) > 1 else per_layer[0]["nnzb"],
                   "block_density": [p["block_density"] for p in per_layer] if len(per_layer) > 1
                   else per_layer[0]["block_density"],
                   "cache": "cold (rotating %d buffer sets per layer, %.0f MB in total)"
                            % (n_sets, n_sets * len(layers) * set_bytes / 1e6)},
        "roofline": {"kernel": dom, "kernels": dom_kernels[dom] if w0.dtype == "bf16" and w0.block >= 32 else dom,
                     "workload": dom_wl, "bound": "hbm", "achieved": round(dom_gbps, 2),
                     "peak": acc.MI355X_HBM_GBPS, "unit": "GB/s",
                     "frac": round(dom_gbps / acc.MI355X_HBM_GBPS, 5), "traffic": read_traffic(dom_wl, dom),
                     "avg_kernel_ms": round(dom_ms, 5), "algorithmic_bytes": dom_bytes},
        "roofline_mfma": {"kernel": dom, "achieved": round(dom_tflops, 3), "peak": peak_tf,
                          "unit": "TFLOP/s", "frac": round(dom_tflops / peak_tf, 5)},
        "path": {"useful_flop": flops_step, "mfma_frac": round(tflops / peak_tf, 5),
                 "ms_per_layer": round(ms_cold / len(layers), 5),
                 "launches_per_layer_step": 3 if w0.dtype == "bf16" and w0.block >= 32 else 4,
                 "algorithmic_bytes": path_bytes,
                 "hbm_GBps": round(path_bytes / (ms_cold * 1e-3) / 1e9, 2),
                 "hbm_frac": round(path_bytes / (ms_cold * 1e-3) / 1e9 / acc.MI355X_HBM_GBPS, 5),
                 "ms_per_step_warm": round(ms_warm, 5),
                 "tflops_warm": round(flops_step / (ms_warm * 1e-3) / 1e12, 3),
                 "paper_ops_sparse_fwd_per_head": [acc.paper_ops_sparse(w0.L, w0.d, p["nnzb"] * w0.block ** 2)
                                                   for p in per_layer]},
        "layers": [{k: v for k, v in p.items() if k != "useful_flop"} for p in per_layer],
        "pattern": {"ms": round(sum(ly.pattern_ms for ly in bench.layers), 5),
                    "A_s_bytes": 4 * w0.L * w0.L * len(layers),
                    "GBps_whole_call": round(4 * w0.L * w0.L * len(layers)
                                             / (sum(ly.pattern_ms for ly in bench.layers) * 1e-3) / 1e9, 2),
                    "conv_pool_ms": round(sum(ly.pool_ms for ly in bench.layers), 5),
                    "conv_GBps": round(4 * w0.L * w0.L * len(layers)
                                       / (sum(ly.pool_ms for ly in bench.layers) * 1e-3) / 1e9, 2)},
    }

    def imbalance(pl):
        lm = [p["ms"] for p in pl]
        return {"layer_ms_max_over_min": round(max(lm) / min(lm), 3),
                "density_max_over_min": round(max(p["block_density"] for p in pl)
                                              / min(p["block_density"] for p in pl), 3)}

    if len(per_layer) > 1:
        out["imbalance"] = imbalance(per_layer)

    if not args.no_extras:
        out.update(extras(sp, acc, torch, dev, w0, tdt, code, BH, esz))

    # ---------------------------------------------------------------- CPU baseline: the oracle as it is
    ref_fl = None
    if not args.no_cpu_baseline:
        import oracle
        nthr = oracle.threads()
        ly = bench.layers[-1] if len(bench.layers) > 1 else bench.layers[0]
        w = ly.w
        n_heads = min(BH, max(nthr, 1))
        t0 = time.perf_counter()
        ref = oracle.generate_pattern(ly.A, w.block, w.filt, w.thresh_mode, w.thresh_value)
        t_pat = time.perf_counter() - t0
        P = oracle.upsample(ref["fl_out"], w.block)
        reps, t_attn = 0, 0.0
        while reps < 8 and t_attn < 10.0:       # about 10 s of CPU work, whole passes only
            t0 = time.perf_counter()
            oracle.attn_fwd(ly.Q[:n_heads], ly.K[:n_heads], ly.V[:n_heads], P)
            oracle.attn_bwd(ly.Q[:n_heads], ly.K[:n_heads], ly.V[:n_heads], ly.dO[:n_heads], P)
            t_attn += time.perf_counter() - t0
            reps += 1
        cpu_tf = reps * acc.useful_flops(ref["nnzb"], w.block, w.d, n_heads, products=6) / t_attn / 1e12
        out["cpu_baseline"] = {
            "value": round(cpu_tf, 6), "unit": "TFLOP/s", "cores": nthr, "kind": "oracle",
            "sample": "fp64 dense-masked oracle, %d x forward+backward of %d of %d (batch,head) slices of %s "
                      "in %.2f s (useful FLOP of the kept blocks / time); oracle pattern generation %.2f s"
                      % (reps, n_heads, BH, w.name, t_attn, t_pat),
            "pattern_s": round(t_pat, 3)}
        out["pattern"]["mask_matches_oracle"] = bool(
            np.array_equal(ref["fl_out"], ly.pat.fl_out.cpu().numpy()))

    # ---------------------------------------------------------------- the 4-layer stack of configuration 5
    if args.workload == DEFAULT_WORKLOAD and not args.no_stack:
        del bench
        torch.cuda.empty_cache()
        # one buffer set per layer: the four layers' tensors (537 MB) already exceed the Infinity Cache
        stack = Bench(sp, acc, si, torch, dev, stack_layers, 1, max(2, args.pattern_iters // 4), flush)
        s_cold, _ = stack.step_times(args.stack_steps, 5, 100.0)
        s_layers = stack.phase_times(args.stack_steps, 5)
        s_flop = sum(p["useful_flop"] for p in s_layers)
        out["stack"] = {"workload": "cfg5_4layer_bf16_L4096", "B": stack_layers[0].B, "H": stack_layers[0].H,
                        "steps": args.stack_steps, "ms_per_step": round(s_cold, 5),
                        "tflops": round(s_flop / (s_cold * 1e-3) / 1e12, 3),
                        "mfma_frac": round(s_flop / (s_cold * 1e-3) / 1e12 / peak_tf, 5),
                        "layers": [{k: v for k, v in p.items() if k != "useful_flop"} for p in s_layers],
                        "pattern_ms": round(sum(ly.pattern_ms for ly in stack.layers), 5),
                        "imbalance": imbalance(s_layers)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
