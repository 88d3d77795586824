#!/usr/bin/env python3
"""Benchmark of the MRP chain step on one MI355X.

A "step" is one denoising step's whole chain on one synthetic batch: state 0
(reduce the prior logits, reveal) and K heads (head MLP, shared LM head with
residual add and fused split-vocabulary reduction, merge / reveal / draft
[/ remask]).  Default workload: the largest configuration (d=4096, V=151936,
B=256, block 16 -> 4096 rows, K=3, remask on), whose LM-head kernel is MFMA-bound;
the same line carries, in its "config1_hbm_regime" sub-object, the SDAR-1.7B-shaped
drafting configuration (d=2048, B=32, block 4 -> 128 rows), whose LM-head kernel is
HBM-bound.  Inputs are seeded and synthetic and resident in HBM before the timed
region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--skip-cpu-baseline]

Further workloads of the same library, each printing its own JSON line in the same format
(--workload kl_loss | residual_rms | tbody | lm_traffic | library_gemm): the training objective (forward +
gradient), the residual-magnitude reducer, the chain with the transformer head body (--depth D), the bytes of
one LM-head launch moved without arithmetic (the memory system's floor for that kernel's traffic mix), and, as
context only, the vendor library's plain GEMM on the LM head's contraction.
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


def traffic_from_profile(cid, name: str = ""):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), as recorded in the
    committed counter summary (the LM-head kernel of configuration `cid`, or the summary `name`);
    None if no summary exists."""
    path = os.path.join(ROOT, "profiles", name or f"lm_head_cfg{cid}_pmc.txt")
    try:
        with open(path) as f:
            m = re.search(r"^TRAFFIC_BYTES_PER_LAUNCH\s*=\s*([0-9.eE+]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


FP64_VECTOR_PEAK_TFLOPS = 78.6  # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz


def _time_steps(torch, step, warmup, steps):
    """Wall time and HIP-event time (on the launch stream, which is torch's current stream) of `steps` calls."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return time.perf_counter() - t0, e0.elapsed_time(e1) * 1e-3


def _line(metric, value, unit, args, elapsed, dtype, workload, roof, cpu):
    return {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": dtype, "data": "synthetic", "config": {"workload": workload},
            "roofline": roof, "cpu_baseline": cpu}


def bench_kl_loss(args, np, torch, mi, mrp) -> dict:
    """Equation 3 forward + gradient on config-2-sized logits (1024 rows x 151936)."""
    cfg = mi.CONFIGS[args.config if args.config not in (None, 1) else 2]
    M, V = cfg.M, cfg.V
    t = mi.logits0(cfg, step=1)
    s = t + mi.residual(cfg)
    mask = (np.arange(M) % 5 != 2).astype(np.uint8)
    ctx = mrp.MrpContext(256, V, M, cfg.L)
    t_d, s_d, m_d = torch.from_numpy(t).cuda(), torch.from_numpy(s).cuda(), torch.from_numpy(mask).cuda()
    loss = torch.empty((M,), dtype=torch.float32, device="cuda")
    grad = torch.empty((M, V), dtype=torch.float32, device="cuda")
    elapsed, ev = _time_steps(torch, lambda: ctx.kl_loss(M, t_d, s_d, m_d, 1.0 / M, loss, grad), args.warmup, args.steps)
    byt = 20.0 * M * V * (mask.mean())          # masked-out rows are neither read nor re-read (their gradient is written: +4MV)
    byt += 4.0 * M * V * (1 - mask.mean())
    ach = byt / (ev / args.steps) / 1e9
    roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": traffic_from_profile(None, "kl_loss_pmc.txt") if (M, V) == (1024, 151936) else None,
            "kernel": "kl_partial_kernel + kl_finish_kernel + kl_grad_kernel",
            "kernel_ms": 1e3 * ev / args.steps}
    cpu = None
    if not args.skip_cpu_baseline:
        import oracle as orc
        n = M
        c0 = time.perf_counter()
        orc.kl_loss(np.ascontiguousarray(t[:n]), np.ascontiguousarray(s[:n]), np.ascontiguousarray(mask[:n]), 1.0 / M)
        c1 = time.perf_counter()
        cpu = {"value": n / (c1 - c0), "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n} of {M} rows, {c1 - c0:.1f} s wall, fp64, gcc -O2"}
    ctx.close()
    return _line("KL objective (Eq. 3) forward + gradient, rows/s on 1 GPU; % HBM roofline", M * args.steps / elapsed,
                 "rows/s", args, elapsed, "f32", f"{M} rows x V={V} fp32 teacher and student logits, 80% of rows masked in",
                 roof, cpu)


def bench_residual_rms(args, np, torch, mi, mrp) -> dict:
    """Appendix B magnitudes of 8 blocks of 17 logit states (16 x 151936 fp32 each)."""
    nb, S, N = 8, 17, 16 * 151936
    X = np.stack([mi.block_states(2, b, S, N) for b in range(nb)])
    ctx = mrp.MrpContext(256, 4096, 16, 16)
    X_d = torch.from_numpy(X).cuda()
    pair = torch.empty((nb, S, S), dtype=torch.float64, device="cuda")
    delta = torch.empty((S,), dtype=torch.float64, device="cuda")
    elapsed, ev = _time_steps(torch, lambda: ctx.residual_rms(nb, S, N, X_d, False, pair, delta), args.warmup, args.steps)
    # By the published peaks the kernel is HBM-bound: every state is read once (4 S N bytes per block,
    # 165 us at 8 TB/s for this workload) against 442 fp64 flop per entry (109 us at 78.6 TFLOP/s).
    byt = 4.0 * nb * S * N
    flop = (136 + 2 * 153) * float(nb) * N       # per entry: 136 fp64 subtractions, 153 fused multiply-adds
    ach = byt / (ev / args.steps) / 1e9
    roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": traffic_from_profile(None, "residual_rms_pmc.txt"),
            "traffic_source": "profiles/residual_rms_pmc.txt (an earlier run of this command under rocprofv3 --pmc)",
            "kernel": "rms_partial_kernel<17>", "kernel_ms": 1e3 * ev / args.steps,
            "fp64_TFLOPs": flop / (ev / args.steps) / 1e12, "fp64_frac_of_78.6": flop / (ev / args.steps) / 1e12 / FP64_VECTOR_PEAK_TFLOPS}
    cpu = None
    if not args.skip_cpu_baseline:
        import oracle as orc
        n = N
        Xs = np.ascontiguousarray(X[:1, :, :n].astype(np.float64))
        c0 = time.perf_counter()
        orc.residual_rms(Xs)
        c1 = time.perf_counter()
        cpu = {"value": (n / N) / (c1 - c0), "unit": "blocks/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n} of {N} entries of one block's 17 states, {c1 - c0:.1f} s wall, fp64, gcc -O2"}
    ctx.close()
    return _line("residual-magnitude blocks/s (App. B: 17 states of 16 x V logits) on 1 GPU; % HBM roofline",
                 nb * args.steps / elapsed, "blocks/s", args, elapsed, "f64",
                 f"{nb} blocks x 17 states x {N} fp32 entries (random-walk stand-in states)", roof, cpu)


def bench_lm_traffic(args, np, torch, mi, mrp) -> dict:
    """The bytes of one config-1 LM-head launch (packed W_lm streamed once, the 128 x V logit tile read and
    written back) moved by mrp_probe_lm_traffic with no arithmetic at all, in three stages, next to the
    LM-head kernel itself: how much of the kernel's time is the memory system's for this traffic mix."""
    cfg = mi.CONFIGS[1]
    d, V, B, L, K, M = cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, cfg.M
    bits = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    ctx = mrp.MrpContext(d, V, M, L)
    Wp_d = mrp.pack_weight(bits(mi.lm_head(cfg)))
    z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
    z_before = z_d.clone()
    wb, zb = 2.0 * V * d, 4.0 * M * V
    stages = {}
    for mode, name, byt in ((0, "weights", wb), (1, "weights+z_read", wb + zb), (2, "weights+z_read+z_write", wb + 2 * zb)):
        _, ev = _time_steps(torch, lambda: ctx.probe_lm_traffic(mode, M, Wp_d, z_d), args.warmup, args.steps)
        t = ev / args.steps
        stages[name] = {"us": 1e6 * t, "GBps": byt / t / 1e9, "bytes": byt}
    assert torch.equal(z_d, z_before), "the probe must leave the logits unchanged"
    # the kernel itself, in the chain
    E_d = bits(mi.embedding(cfg))
    heads_d = [mrp.Head(mrp.pack_weight(bits(w1), body=True), mrp.pack_weight(bits(w2), body=True), bits(g))
               for (w1, w2, g) in (mi.head_weights(cfg, k) for k in range(K))]
    h_d = bits(mi.hidden(cfg))
    hrun_d = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    io = mrp.StepIO(B, L, K)
    rcfg = mrp.RevealCfg(tau=cfg.tau, fresh_block=1)
    step = lambda: ctx.chain_step(B, K, h_d, hrun_d, E_d, Wp_d, heads_d, z_d, rcfg, io)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    elapsed, _ = _time_steps(torch, step, 0, args.steps)
    lm_avg = float(np.mean(ctx.profile_read())) * 1e-3
    ctx.close()
    full = stages["weights+z_read+z_write"]
    roof = {"bound": "hbm", "achieved": full["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": full["GBps"] / HBM_PEAK_GBS,
            "traffic": None, "kernel": "lm_traffic_kernel<2> (no arithmetic)", "kernel_ms": full["us"] * 1e-3,
            "stages": stages,
            "lm_persist_kernel_us": 1e6 * lm_avg, "lm_persist_GBps": (wb + 2 * zb) / lm_avg / 1e9,
            "lm_persist_over_traffic_floor": 1e6 * lm_avg / full["us"]}
    return _line("bytes of one LM-head launch moved without arithmetic (config 1), GB/s on 1 GPU; % HBM roofline",
                 full["GBps"], "GB/s", args, full["us"] * 1e-6 * args.steps, "u8",
                 f"config 1 LM head: {wb / 1e6:.0f} MB packed W_lm + {zb / 1e6:.0f} MB logit tile read and written back", roof, None)


def bench_library_gemm(args, np, torch, mi, mrp) -> dict:
    """Context only, no part of the path: the vendor library's plain bf16 GEMM (torch.matmul, bf16 output) on the
    LM head's contraction y W_lm^T at configs 2, 3, 4's row counts -- no logit state, no residual add, no
    vocabulary reduction -- next to which the fused LM-head tile kernel can be read."""
    d, V = mi.CONFIGS[4].d, mi.CONFIGS[4].V
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    W = (torch.randn(V, d, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    rows = {}
    for M in (1024, 2048, 4096):
        y = torch.randn(M, d, device="cuda", generator=g).to(torch.bfloat16)
        out = torch.empty(M, V, device="cuda", dtype=torch.bfloat16)
        _, ev = _time_steps(torch, lambda: torch.matmul(y, W.t(), out=out), args.warmup, args.steps)
        t = ev / args.steps
        rows[str(M)] = {"us": 1e6 * t, "TFLOPs": 2.0 * M * V * d / t / 1e12, "frac": 2.0 * M * V * d / t / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        del y, out
    r = rows["4096"]
    roof = {"bound": "mfma", "achieved": r["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": r["frac"],
            "traffic": None, "kernel": "vendor library GEMM (torch.matmul, bf16 in, bf16 out)", "kernel_ms": r["us"] * 1e-3,
            "by_rows": rows}
    return _line("vendor library bf16 GEMM on the LM head's contraction (context, not the path), TFLOP/s on 1 GPU",
                 r["TFLOPs"], "TFLOP/s", args, r["us"] * 1e-6 * args.steps, "bf16",
                 f"y[4096 x {d}] W_lm[{V} x {d}]^T, plain GEMM without logit state or reduction", roof, None)


def bench_tbody(args, np, torch, mi, mrp) -> dict:
    """Config 1 with the transformer head body: D = 3 layers of the backbone family's shape at d = 2048
    (16 query / 8 kv heads of 128, gated MLP 6144), prefix caches of 1024 positions, one module applied K times."""
    cfg = mi.CONFIGS[1]
    d, V, B, L, K, M = cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, cfg.M
    td = mi.TBodyDims(D=args.depth, n_heads=16, n_kv_heads=8, head_dim=128, d_ff=6144, P_max=1024)
    bits = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    w1, _, g = mi.head_weights(cfg, 0)
    layers_h = [mi.tf_layer(cfg, td, 0, l) for l in range(td.D)]
    plen = mi.prefix_lens(cfg, td)
    if args.prefix_len is not None:      # every sequence the same committed prefix (attention time by prefix length)
        plen = np.full_like(plen, min(max(args.prefix_len, 0), td.P_max))
    ctx = mrp.MrpContext(d, V, M, L)
    ctx.tbody_create(td.D, td.n_heads, td.n_kv_heads, td.d_ff, td.P_max, td.rope_theta)
    E_d, Wp_d = bits(E), mrp.pack_weight(bits(W))
    head = mrp.Head(mrp.pack_weight(bits(w1), body=True), None, bits(g))
    pk = lambda a: mrp.pack_weight(bits(a), body=True)
    layers = [mrp.TLayer(pk(l["Wqkv"]), pk(l["Wo"]), pk(l["Wgu"]),
                         pk(l["Wdown"]), bits(l["g1"]), bits(l["g2"]), bits(l["kc"]), bits(l["vc"]))
              for l in layers_h]
    h_bits, z0 = mi.hidden(cfg), mi.logits0(cfg)
    h_d, z_d, plen_d = bits(h_bits), torch.from_numpy(z0).cuda(), torch.from_numpy(plen).cuda()
    hrun_d = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    io = mrp.StepIO(B, L, K)
    rcfg = mrp.RevealCfg(tau=cfg.tau, fresh_block=1)
    step = lambda: ctx.chain_step_tf(B, K, h_d, hrun_d, E_d, Wp_d, [head] * K, layers * K, plen_d, z_d, rcfg, io)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    elapsed, _ = _time_steps(torch, step, 0, args.steps)
    lm_ms = ctx.profile_read()
    lm_avg = float(np.mean(lm_ms))
    ach = (2.0 * V * d + 8.0 * M * V) / (lm_avg * 1e-3) / 1e9
    roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": traffic_from_profile(1), "kernel": "lm_persist_kernel", "kernel_ms": lm_avg,
            "lm_head_share_of_step": lm_avg * K / (1e3 * elapsed / args.steps)}
    cpu = None
    if not args.skip_cpu_baseline:
        import oracle as orc
        seqs = [0, B - 1]
        rows = np.concatenate([np.arange(b * L, (b + 1) * L) for b in seqs])
        oc = orc.make_cfg(d, V, len(seqs), L, K, tau=cfg.tau)
        tc = orc.make_tcfg(td.D, td.n_heads, td.n_kv_heads, td.head_dim, td.d_ff, td.P_max, td.rope_theta)
        sub = [dict(l, kc=np.ascontiguousarray(l["kc"][seqs]), vc=np.ascontiguousarray(l["vc"][seqs])) for l in layers_h]
        c0 = time.perf_counter()
        orc.chain_step(oc, E, W, [(w1, None, g)] * K, z0[rows].astype(np.float64), mi.bf16_bits_to_f64(h_bits[rows]),
                       tbody=orc.TBody(tc, [sub] * K, plen[seqs]))
        c1 = time.perf_counter()
        cpu = {"value": len(rows) * K / (c1 - c0), "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
               "sample": f"sequences 0 and {B - 1} of {B} ({len(rows)} rows x {K} heads), {c1 - c0:.1f} s wall, fp64"}
    ctx.close()
    roof["body_ms_per_head"] = (1e3 * elapsed / args.steps - lm_avg * K) / K      # everything of a head but its LM-head kernel
    return _line(f"MRP draft tokens/sec per step with the transformer head body (D={td.D}) on 1 GPU; % HBM roofline of the LM head",
                 M * K * args.steps / elapsed, "tokens/s", args, elapsed, "bf16",
                 f"config 1 sizes (d={d} V={V} B={B} block={L} K={K}), head body: {td.D} layers, 16/8 heads of 128, d_ff 6144, "
                 + ("prefix lengths uniform in [0, 1024]" if args.prefix_len is None
                    else f"prefix length {int(plen[0])} for every sequence"), roof, cpu)


def host_cpu_info():
    """CPU model and physical core count of the host (from /proc/cpuinfo)."""
    model, cores = "unknown", set()
    try:
        phys = core = None
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.startswith("model name") and model == "unknown":
                    model = ln.split(":", 1)[1].strip()
                elif ln.startswith("physical id"):
                    phys = ln.split(":", 1)[1].strip()
                elif ln.startswith("core id"):
                    core = ln.split(":", 1)[1].strip()
                elif not ln.strip():
                    if phys is not None and core is not None:
                        cores.add((phys, core))
                    phys = core = None
    except OSError:
        pass
    return model, (len(cores) or None)


def run_chain_config(cfg, args, np, torch, mi, mrp) -> dict:
    """Time `args.steps` chain steps of one benchmark configuration (inputs resident in HBM), the
    LM-head kernel bracketed by HIP events on the launch stream, and the oracle on a bounded sample."""
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
    heads_d = [mrp.Head(mrp.pack_weight(dev_bits(w1), body=True), mrp.pack_weight(dev_bits(w2), body=True), dev_bits(g))
               for (w1, w2, g) in heads_h]
    h_bits = mi.hidden(cfg)
    h_d = dev_bits(h_bits)
    ns = min(B, max(1, int(os.environ.get("MRP_BENCH_ORACLE_SEQS", "32" if d <= 2048 else "8"))))
    z0 = mi.logits0(cfg)
    z_d = torch.from_numpy(z0).cuda()
    z0 = np.ascontiguousarray(z0[:ns * L])          # the oracle's sample; the rest of the host copy is dropped
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
        del src, dst

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
    roof["traffic"] = traffic_from_profile(cfg.cid) if cfg == mi.CONFIGS[cfg.cid] else None
    roof["traffic_source"] = (f"profiles/lm_head_cfg{cfg.cid}_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier "
                              "run of this command, scaled by what the counters read for a 1 GiB copy; not measured in this run"
                              if roof["traffic"] is not None else None)
    roof["kernel"] = (("lm_persist_kernel_32rows" if M <= 32 else "lm_persist_kernel_64rows" if M <= 64 else
                       "lm_persist_kernel" if M <= 128 else "lm_persist_kernel_256rows")
                      if M <= 256 and V % 4 == 0 else
                      "lm_persist_kernel_256rows (+ a second launch for the rows beyond 256)" if M <= 512 and V % 4 == 0 else
                      "tiled_gemm_kernel<EPI_LM>" if V % 4 == 0 else "stream_gemm_kernel<EPI_LM>")
    roof["kernel_ms"] = lm_avg_ms
    roof["launches"] = len(lm_ms)
    roof["algorithmic_bytes_per_launch"] = lm_bytes
    roof["flop_per_launch"] = lm_flops
    roof["lm_head_share_of_step"] = (lm_avg_ms * K) / ms_per_step

    # ---- the oracle, as it stands, on the host cores (bounded sample of whole sequences) ----
    cpu = None
    if not args.skip_cpu_baseline:
        import oracle as orc
        rows = np.arange(ns * L)
        oc = orc.make_cfg(d, V, ns, L, K, tau=cfg.tau, tau_remask=cfg.tau_remask)
        zz = z0[rows].astype(np.float64)
        hh = mi.bf16_bits_to_f64(h_bits[rows])
        c0 = time.perf_counter()
        orc.chain_step(oc, E, W, heads_h, zz, hh)
        c1 = time.perf_counter()
        model, phys = host_cpu_info()
        cpu = {"value": len(rows) * K / (c1 - c0), "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
               "physical_cores": phys, "cpu_model": model,
               "sample": f"first {ns} of {B} sequences ({len(rows)} rows x {K} heads) of the same workload, "
                         f"{c1 - c0:.1f} s wall, fp64, gcc -O2 -fopenmp, {orc.threads()} OpenMP threads"}
    ctx.close()
    workload = (f"config {cfg.cid} ({cfg.name}): d={d} V={V} B={B} block={L} rows={M} K={K} "
                f"tau={cfg.tau}" + (f" tau_remask={cfg.tau_remask}" if cfg.tau_remask >= 0 else ""))
    del z_d, Wp_d, E_d, heads_d, h_d, hrun_d, io
    torch.cuda.empty_cache()
    return {"workload": workload, "value": tokens_per_s, "unit": "tokens/s", "ms_per_step": ms_per_step,
            "roofline": roof, "cpu_baseline": cpu}


def chain_line(res: dict, args) -> dict:
    return {
        "metric": "MRP draft tokens/sec per step (B\u00d7block\u00d7K) on 1 GPU; % HBM/MFMA roofline",
        "value": res["value"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": res["workload"],
                   "accumulate": "fp32", "logit_state": "fp32", "lm_head_operands": "bf16",
                   "head_body_operands": "fp32 activations as two fp16 terms, bf16 weights converted to fp16"},
        "roofline": res["roofline"],
        "cpu_baseline": res["cpu_baseline"],
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="chain", choices=["chain", "kl_loss", "residual_rms", "tbody", "lm_traffic", "library_gemm"],
                    help="chain (default): the headline metric; the others time further entry points")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="time one benchmark configuration 0..4 only (default: configuration 4 as the line, "
                         "configuration 1 in its config1_hbm_regime sub-object)")
    ap.add_argument("--batch", type=int, default=None,
                    help="with --config N: override the number of sequences B (e.g. --config 2 --batch 32 times the "
                         "512-row case, the last row count on the persistent LM-head kernel before the tile kernel takes over)")
    ap.add_argument("--depth", type=int, default=3,
                    help="--workload tbody: transformer layers per head (the paper's depth sweep uses 1, 2, 3, 4, 8)")
    ap.add_argument("--prefix-len", type=int, default=None,
                    help="--workload tbody: give every sequence this prefix length (0..1024) instead of the seeded mix")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (sequences would shard by rows, the vocabulary by "
              "columns with one small all-gather per head; neither is built); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import mrp_inputs as mi
    import paper_2605_18817_amd as mrp

    if not torch.cuda.is_available():
        print("bench.py: no GPU; the MRP chain has no CPU path", file=sys.stderr)
        return 3

    if args.workload != "chain":
        fn = {"kl_loss": bench_kl_loss, "residual_rms": bench_residual_rms, "tbody": bench_tbody,
              "lm_traffic": bench_lm_traffic, "library_gemm": bench_library_gemm}[args.workload]
        print(json.dumps(fn(args, np, torch, mi, mrp)))
        return 0

    if args.config is not None:
        cfg = mi.CONFIGS[args.config] if args.batch is None else mi.config(args.config, B=args.batch)
        res = run_chain_config(cfg, args, np, torch, mi, mrp)
        print(json.dumps(chain_line(res, args)))
        return 0
    # default: the largest configuration (MFMA-bound) is the line; the SDAR-1.7B-shaped configuration
    # (HBM-bound LM head) rides along in a sub-object with its own step time, roofline and oracle baseline
    big = run_chain_config(mi.CONFIGS[4], args, np, torch, mi, mrp)
    small = run_chain_config(mi.CONFIGS[1], args, np, torch, mi, mrp)
    out = chain_line(big, args)
    out["config1_hbm_regime"] = {k: small[k] for k in ("workload", "value", "unit", "ms_per_step", "roofline",
                                                          "cpu_baseline")}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
