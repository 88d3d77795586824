#!/usr/bin/env python3
"""Benchmark of the MRP chain step on one MI355X.

A "step" is one denoising step's whole chain on one synthetic batch: state 0
(reduce the prior logits, reveal) and K heads (head MLP, shared LM head with
residual add and fused split-vocabulary reduction, merge / reveal / draft
[/ remask]).  Default workload: the SDAR-1.7B-shaped drafting configuration
(d=2048, V=151936, B=32, block 4 -> 128 rows, K=3), whose LM-head kernel is
HBM-bound.  Inputs are seeded and synthetic and resident in HBM before the timed
region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--skip-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16


def traffic_from_profile(cid: int):
    """HBM bytes per LM-head launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    as recorded in the committed counter summary; None if no summary exists."""
    path = os.path.join(ROOT, "profiles", f"lm_head_cfg{cid}_pmc.txt")
    try:
        with open(path) as f:
            m = re.search(r"^TRAFFIC_BYTES_PER_LAUNCH\s*=\s*([0-9.eE+]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="benchmark configuration 0..4")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (row or vocabulary sharding across GPUs is "
              "described in DESIGN.md but not built); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import mrp_inputs as mi
    import paper_2605_18817_amd as mrp

    if not torch.cuda.is_available():
        print("bench.py: no GPU; the MRP chain has no CPU path", file=sys.stderr)
        return 3

    cfg = mi.CONFIGS[args.config]
    d, V, B, L, K, M = cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, cfg.M

    def dev_bits(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()

    # ---- inputs resident in HBM ----
    W = mi.lm_head(cfg)
    E = mi.embedding(cfg)
    heads_h = [mi.head_weights(cfg, k) for k in range(K)]
    ctx = mrp.MrpContext(d, V, M, L)
    E_d = dev_bits(E)
    w_d = dev_bits(W)
    Wp_d = mrp.pack_weight(w_d)
    del w_d
    heads_d = [mrp.Head(mrp.pack_weight(dev_bits(w1)), mrp.pack_weight(dev_bits(w2)), dev_bits(g))
               for (w1, w2, g) in heads_h]
    h_bits = mi.hidden(cfg)
    h_d = dev_bits(h_bits)
    z0 = mi.logits0(cfg)
    z_d = torch.from_numpy(z0).cuda()
    hrun_d = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    io = mrp.StepIO(B, L, K)
    rcfg = mrp.RevealCfg(tau=cfg.tau, tau_remask=cfg.tau_remask, fresh_block=1)
    torch.cuda.synchronize()

    def step():
        ctx.chain_step(B, K, h_d, hrun_d, E_d, Wp_d, heads_d, z_d, rcfg, io)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)      # HIP events around every LM-head kernel, on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    lm_ms = ctx.profile_read()
    ctx.profile_enable(False)
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = M * K * args.steps / elapsed

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- roofline of the dominant kernel (LM head + residual add + fused reduction) ----
    lm_avg_ms = float(np.mean(lm_ms)) if lm_ms else float("nan")
    lm_bytes = 2.0 * V * d + 8.0 * M * V          # stream W_lm once, read + write the logit state
    lm_flops = 2.0 * M * V * d
    mem_time = lm_bytes / (HBM_PEAK_GBS * 1e9)
    mfma_time = lm_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if mem_time >= mfma_time:
        ach = lm_bytes / (lm_avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS}
    else:
        ach = lm_flops / (lm_avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS}
    roof["traffic"] = traffic_from_profile(cfg.cid)
    roof["kernel"] = ("lm_persist_kernel" if M <= 128 and V % 4 == 0 else
                      "tiled_gemm_kernel<EPI_LM>" if M >= 768 and V % 4 == 0 else "stream_gemm_kernel<EPI_LM>")
    roof["kernel_ms"] = lm_avg_ms
    roof["launches"] = len(lm_ms)
    roof["lm_head_share_of_step"] = (lm_avg_ms * K) / ms_per_step

    # ---- the oracle, as it stands, on the host cores (bounded sample of whole sequences) ----
    cpu = None
    if not args.skip_cpu_baseline:
        import oracle as orc
        ns = min(B, max(1, int(os.environ.get("MRP_BENCH_ORACLE_SEQS", "16" if d <= 2048 else "2"))))
        seqs = list(range(ns))
        rows = np.concatenate([np.arange(b * L, (b + 1) * L) for b in seqs])
        oc = orc.make_cfg(d, V, ns, L, K, tau=cfg.tau, tau_remask=cfg.tau_remask)
        zz = z0[rows].astype(np.float64)
        hh = mi.bf16_bits_to_f64(h_bits[rows])
        c0 = time.perf_counter()
        orc.chain_step(oc, E, W, heads_h, zz, hh)
        c1 = time.perf_counter()
        cpu = {"value": len(rows) * K / (c1 - c0), "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
               "sample": f"{ns} of {B} sequences ({len(rows)} rows x {K} heads) of the same workload, "
                         f"{c1 - c0:.1f} s wall, fp64, gcc -O2 -fopenmp"}

    out = {
        "metric": "MRP draft tokens/sec per step (B\u00d7block\u00d7K) on 1 GPU; % HBM/MFMA roofline",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.cid} ({cfg.name}): d={d} V={V} B={B} block={L} rows={M} K={K} "
                               f"tau={cfg.tau}" + (f" tau_remask={cfg.tau_remask}" if cfg.tau_remask >= 0 else ""),
                   "accumulate": "fp32", "logit_state": "fp32"},
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
