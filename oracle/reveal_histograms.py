#!/usr/bin/env python3
"""Reveal-count histograms of the benchmark inputs, from the oracle alone (TEST INFRASTRUCTURE).

For each benchmark configuration and for its literal and its straddling input recipe, runs the
oracle's chain step on a sample of whole sequences and prints, per state, how many positions each
sequence revealed (histogram over sequences), how many of those reveals were forced (no position
above the threshold), and how many rows the remask rule took back.  The literal N(0, 2) logits
almost never exceed the reveal threshold, so they exercise the forced branch only; the straddling
variant (spikes U(10, 20) on half the rows) exists so that both sides of every comparison occur.

    python oracle/reveal_histograms.py [--configs 0 1 2 3 4] [--seqs 8]      (prints a markdown table)
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import mrp_inputs as mi   # noqa: E402
import oracle as orc      # noqa: E402


def run(cfg, nseq):
    ns = min(cfg.B, nseq)
    seqs = list(range(ns))
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    heads = [mi.head_weights(cfg, k) for k in range(cfg.K)]
    z0 = mi.logits0(cfg, seqs=seqs).astype(np.float64)
    h = mi.bf16_bits_to_f64(mi.hidden(cfg, seqs=seqs))
    oc = orc.make_cfg(cfg.d, cfg.V, ns, cfg.L, cfg.K, tau=cfg.tau, tau_remask=cfg.tau_remask)
    o = orc.chain_step(oc, E, W, heads, z0, h)
    rows = []
    masked = np.ones(ns * cfg.L, bool)
    for k in range(cfg.K + 1):
        conf = o.conf[k].reshape(ns, cfg.L)
        mk = masked.reshape(ns, cfg.L)
        above = ((conf > cfg.tau) & mk).sum(1)                      # candidates over the threshold
        revealed = np.where(above > 0, above, np.minimum(1, mk.sum(1)))
        forced = int(((above == 0) & (mk.sum(1) > 0)).sum())
        hist = np.bincount(revealed, minlength=cfg.L + 1)
        rem = int(o.remasked[k].sum())
        rows.append((k, hist, forced, rem, float(np.median(o.conf[k])), float(o.conf[k].max())))
        # replay the mask life cycle from the oracle's own outputs
        for b in range(ns):
            idx = np.flatnonzero(mk[b])
            if len(idx) == 0:
                continue
            sel = idx[conf[b, idx] > cfg.tau]
            if len(sel) == 0:
                sel = idx[[np.argmax(conf[b, idx])]]
            masked[b * cfg.L + sel] = False
        masked[o.remasked[k].astype(bool)] = True
    assert np.array_equal(masked, o.masked.astype(bool)), "histogram replay disagrees with the oracle's masks"
    return ns, rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", type=int, nargs="*", default=[0, 1, 2, 3, 4])
    ap.add_argument("--seqs", type=int, default=8)
    args = ap.parse_args()
    print("| config | inputs | sequences | state | reveals per sequence: count x sequences | forced | remasked rows | median conf | max conf |")
    print("|---|---|---|---|---|---|---|---|---|")
    for cid in args.configs:
        for name, cfg in (("literal", mi.config(cid)), ("straddling", mi.straddling(mi.config(cid)))):
            ns, rows = run(cfg, args.seqs)
            for (k, hist, forced, rem, med, mx) in rows:
                h = ", ".join(f"{n}x{int(c)}" for n, c in enumerate(hist) if c)
                print(f"| {cid} | {name} | {ns} of {cfg.B} | {k} | {h} | {forced} | {rem} | {med:.2e} | {mx:.3f} |", flush=True)


if __name__ == "__main__":
    main()
