#!/usr/bin/env python3
"""Benchmark of the SPION sparse-attention path on one MI355X.

A step is one forward + backward pass of the block-sparse attention of one layer (SDDMM, row
softmax, SpMM and their gradients) on the L = 4096 workload, using the pattern that
spion_pattern produced for that layer; pattern generation happens once per layer in the method and
is timed separately.  Inputs are synthetic (seeded) and already resident in HBM; the step rotates
through several buffer sets larger than the 256 MB Infinity Cache so that every step streams its
tensors from HBM ("cold"); the same loop on a single buffer set ("warm") is reported next to it.

Prints ONE JSON line (see the design doc for the fields).
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


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4_bf16_L4096")
    ap.add_argument("--sets", type=int, default=6, help="rotating buffer sets (cold-cache timing)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pattern-iters", type=int, default=20)
    return ap.parse_args()


def read_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    recorded in profiles/traffic_<workload>.txt (lines "kernel fetch_bytes write_bytes"); None if
    no such measurement is on file."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload)
    try:
        with open(path) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) == 3 and parts[0] == kernel:
                    return int(float(parts[1]) + float(parts[2]))
    except OSError:
        pass
    return None


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
    w = si.workload(args.workload)
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    esz = 4 if w.dtype == "f32" else 2
    BH = w.B * w.H

    # ---------------------------------------------------------------- inputs
    Q, K, V, dO = si.make_qkv_do(w)
    A = si.make_score_map(w, Q, K)
    A_dev = torch.from_numpy(A).to(dev)

    # ---------------------------------------------------------------- pattern (timed separately)
    pat = sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value)
    ws_pat = torch.empty(sp.spion_pattern_workspace_bytes(w.L, w.block), dtype=torch.uint8, device=dev)
    flush = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device=dev)
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.pattern_iters)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.pattern_iters)]
    for i in range(args.pattern_iters):
        flush.fill_(i & 1)          # evict A^s from the caches: the map comes straight from training
        ev0[i].record()
        sp.generate_pattern(A_dev, w.block, w.filt, w.thresh_mode, w.thresh_value, sync=False, out=pat,
                            workspace=ws_pat)
        ev1[i].record()
    torch.cuda.synchronize()
    pat_ms = sorted(a.elapsed_time(b) for a, b in zip(ev0, ev1))
    pattern_ms = pat_ms[len(pat_ms) // 2]
    del flush
    nnzb = pat.nnzb
    density = nnzb / float(w.nb * w.nb)

    # ---------------------------------------------------------------- buffer sets
    def make_set():
        q, k, v, do = [torch.from_numpy(t).to(dev).to(tdt).view(w.B, w.H, w.L, w.d).contiguous()
                       for t in (Q, K, V, dO)]
        s = dict(q=q, k=k, v=v, do=do, O=torch.empty_like(q), dQ=torch.empty_like(q),
                 dK=torch.empty_like(q), dV=torch.empty_like(q),
                 LSE=torch.empty((w.B, w.H, w.L), dtype=torch.float32, device=dev))
        nbytes = sp.spion_attn_workspace_bytes(w.B, w.H, w.L, w.d, w.block, sp.binding._dtype_code(tdt),
                                               nnzb, True)
        s["ws"] = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        return s

    sets = [make_set() for _ in range(max(args.sets, 1))]

    # one plain device copy of known size: the yardstick that scales rocprofv3's FETCH_SIZE /
    # WRITE_SIZE readings (see profiles/) into bytes
    cal_src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst
    code = sp.binding._dtype_code(tdt)

    def fwd(s):
        sp.spion_attn_fwd(s["q"], s["k"], s["v"], s["O"], s["LSE"], pat.row_ptr, pat.col_idx, nnzb,
                          w.B, w.H, w.L, w.d, w.block, code)

    def bwd(s, flags=0):
        sp.spion_attn_bwd(s["q"], s["k"], s["v"], s["O"], s["do"], s["LSE"], s["dQ"], s["dK"], s["dV"],
                          pat.row_ptr, pat.col_idx, pat.col_ptr, pat.row_idx, pat.bsr_pos, nnzb,
                          w.B, w.H, w.L, w.d, w.block, code, flags=flags, workspace=s["ws"])

    def run(n_steps, use_sets):
        for i in range(n_steps):
            s = use_sets[i % len(use_sets)]
            fwd(s)
            bwd(s)

    def timed(n_steps, use_sets):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(n_steps, use_sets)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n_steps

    # ---------------------------------------------------------------- headline: cold, rotating sets
    run(args.warmup, sets)
    ms_cold = timed(args.steps, sets)
    # warm: one buffer set, tensors stay in the Infinity Cache between steps
    run(args.warmup, sets[:1])
    ms_warm = timed(args.steps, sets[:1])

    # ---------------------------------------------------------------- per-kernel durations (events)
    names = ("fwd", "bwd_query", "bwd_key")
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i in range(args.steps):
        s = sets[i % len(sets)]
        evs[i][0].record()
        fwd(s)
        evs[i][1].record()
        bwd(s, sp.SPION_ATTN_BWD_QUERY_SIDE_ONLY)
        evs[i][2].record()
        bwd(s, sp.SPION_ATTN_BWD_KEY_SIDE_ONLY)
        evs[i][3].record()
    torch.cuda.synchronize()
    kern_ms = {n: float(np.mean([e[j].elapsed_time(e[j + 1]) for e in evs])) for j, n in enumerate(names)}

    # ---------------------------------------------------------------- accounting
    flops_step = acc.useful_flops(nnzb, w.block, w.d, BH, products=6)
    tflops = flops_step / (ms_cold * 1e-3) / 1e12
    peak_tf = acc.MI355X_MFMA_TFLOPS[w.dtype]
    dom = max(kern_ms, key=kern_ms.get)
    dom_bytes = acc.algorithmic_bytes(dom, BH, w.L, w.d, esz)
    dom_gbps = dom_bytes / (kern_ms[dom] * 1e-3) / 1e9
    dom_products = {"fwd": 2, "bwd_query": 2, "bwd_key": 2}[dom]
    dom_tflops = acc.useful_flops(nnzb, w.block, w.d, BH, products=dom_products) / (kern_ms[dom] * 1e-3) / 1e12
    path_bytes = acc.algorithmic_bytes("path", BH, w.L, w.d, esz)

    traffic = read_traffic(w.name, dom)

    out = {
        "metric": "sparse MHA fwd+bwd useful TFLOP/s (ms/layer in ms_per_step) at L=%d" % w.L,
        "value": round(tflops, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_cold, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "L": w.L, "d": w.d, "block": w.block,
                   "filter": w.filt, "nnzb": nnzb, "block_density": round(density, 5),
                   "cache": "cold (rotating %d buffer sets, %.0f MB)" % (len(sets), len(sets) * 8 * acc.tensor_bytes(BH, w.L, w.d, esz) / 1e6)},
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": round(dom_gbps, 2),
                     "peak": acc.MI355X_HBM_GBPS, "unit": "GB/s",
                     "frac": round(dom_gbps / acc.MI355X_HBM_GBPS, 5), "traffic": traffic,
                     "avg_kernel_ms": round(kern_ms[dom], 5), "algorithmic_bytes": dom_bytes},
        "roofline_mfma": {"kernel": dom, "achieved": round(dom_tflops, 3), "peak": peak_tf,
                          "unit": "TFLOP/s", "frac": round(dom_tflops / peak_tf, 5)},
        "path": {"useful_flop": flops_step, "mfma_frac": round(tflops / peak_tf, 5),
                 "algorithmic_bytes": path_bytes,
                 "hbm_GBps": round(path_bytes / (ms_cold * 1e-3) / 1e9, 2),
                 "hbm_frac": round(path_bytes / (ms_cold * 1e-3) / 1e9 / acc.MI355X_HBM_GBPS, 5),
                 "ms_per_step_warm": round(ms_warm, 5),
                 "tflops_warm": round(flops_step / (ms_warm * 1e-3) / 1e12, 3),
                 "kernel_ms": {k: round(v, 5) for k, v in kern_ms.items()},
                 "paper_ops_sparse_fwd_per_head": acc.paper_ops_sparse(w.L, w.d, nnzb * w.block * w.block)},
        "pattern": {"ms": round(pattern_ms, 5), "min_ms": round(pat_ms[0], 5),
                    "A_s_bytes": 4 * w.L * w.L,
                    "GBps_whole_call": round(4 * w.L * w.L / (pattern_ms * 1e-3) / 1e9, 2)},
    }

    # ---------------------------------------------------------------- CPU baseline: the oracle as is
    if not args.no_cpu_baseline:
        import oracle
        nthr = oracle.threads()
        n_heads = min(BH, max(nthr, 1))
        t0 = time.perf_counter()
        ref = oracle.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
        t_pat = time.perf_counter() - t0
        P = oracle.upsample(ref["fl_out"], w.block)
        t0 = time.perf_counter()
        oracle.attn_fwd(Q[:n_heads], K[:n_heads], V[:n_heads], P)
        oracle.attn_bwd(Q[:n_heads], K[:n_heads], V[:n_heads], dO[:n_heads], P)
        t_attn = time.perf_counter() - t0
        cpu_tf = acc.useful_flops(ref["nnzb"], w.block, w.d, n_heads, products=6) / t_attn / 1e12
        out["cpu_baseline"] = {
            "value": round(cpu_tf, 6), "unit": "TFLOP/s", "cores": nthr, "kind": "oracle",
            "sample": "fp64 dense-masked oracle, forward+backward of %d of %d (batch,head) slices of %s "
                      "in %.2f s (useful FLOP of the kept blocks / time); oracle pattern generation %.2f s"
                      % (n_heads, BH, w.name, t_attn, t_pat),
            "pattern_s": round(t_pat, 3)}
        out["pattern"]["mask_matches_oracle"] = bool(
            np.array_equal(ref["fl_out"], pat.fl_out.cpu().numpy()))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
