"""Seeded synthetic inputs for the MRP chain step.

This module only *draws numbers*: it holds none of the method's arithmetic
(no GEMM, no softmax, no reveal rule).  Both the CPU oracle's tests and the
GPU path's tests/bench take their input bytes from here, so that the two
sides see the same bits.

Recipe (shapes follow the five benchmark configurations; the SDAR-shaped
sizes d=2048/4096, V=151936, block 16 or sub-block 4 stand in for the paper's
SDAR-1.7B / SDAR-8B backbones, Section 4.1 "Models"):

* LM head ``W_lm`` and embedding ``E``: bf16 [V, d], N(0, 0.02).
* K distinct heads: ``W1`` bf16 [d, 2d], ``W2`` bf16 [d, d], N(0, 0.02);
  RMSNorm gain ``gamma`` bf16 [d] = 1.0 (a norm gain, not an init-std weight).
* hidden states ``h``: bf16 [M, d], N(0, 1).
* prior logit state ``z0``: fp32 [M, V], N(0, 2); optionally a fraction of the
  rows receives one additive spike at a uniformly drawn vocabulary index.
* stand-in residual ``delta`` for the training objective: fp32 [M, V], N(0, 0.5).
* block states for the residual-magnitude measurement: ``X^(0)`` ~ N(0, 2), then independent
  N(0, 0.4) increments per state (a random walk), fp32 [S, N] per block, optionally rounded to bf16.
* transformer head body: every projection bf16 N(0, 0.02), norm gains 1.0; prefix key/value caches
  bf16 [B, P_max, n_kv, head_dim], N(0, 1); prefix lengths uniform in [0, P_max] with sequence 0 at 0
  and the last sequence at P_max.
* verify logits: fp32 [B, L, V], N(0, 2); a +8 boost is *added by the caller*
  at the drafted (position, token) pairs selected by ``verify_boost_mask``.

"N(0, s)": s is the standard deviation.  Every tensor is drawn in independent
chunks (one chunk = one sequence for per-row tensors, 4096 rows for weights),
each from its own ``numpy.random.SeedSequence([BASE, config, tensor, chunk])``,
so any subset of sequences can be regenerated without drawing the rest and the
result does not depend on the number of worker threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Iterable, Optional, Sequence

import numpy as np

SEED_BASE = 0x4D5250  # "MRP"

# tensor ids (part of the seed)
T_WLM, T_E, T_W1, T_W2, T_H, T_Z, T_SPIKE, T_VERIFY, T_BOOST, T_DELTA, T_STATES, T_TF, T_KV, T_PLEN = range(14)

WEIGHT_CHUNK_ROWS = 4096


@dataclass(frozen=True)
class Config:
    """One benchmark configuration (sizes and thresholds only)."""

    cid: int
    d: int
    V: int
    B: int
    L: int
    K: int
    tau: float
    tau_remask: float = -1.0      # < 0: remask disabled
    spike_frac: float = 0.0       # fraction of rows with one spiked logit
    spike_lo: float = 12.0        # spike height drawn U(spike_lo, spike_hi)
    spike_hi: float = 12.0
    steps: int = 1                # consecutive chain steps with resident z
    name: str = ""

    @property
    def M(self) -> int:
        return self.B * self.L


CONFIGS = {
    0: Config(0, 256, 4096, 1, 4, 3, 0.9, name="tiny"),
    1: Config(1, 2048, 151936, 32, 4, 3, 0.9, spike_frac=0.05, name="sdar1.7b-draft"),
    2: Config(2, 4096, 151936, 64, 16, 3, 0.9, name="sdar8b-draft"),
    3: Config(3, 4096, 151936, 128, 16, 3, 0.9, name="sdar8b-spec-verify"),
    4: Config(4, 4096, 151936, 256, 16, 3, 0.5, tau_remask=0.3, steps=8,
              name="sdar8b-remask"),
}


def config(cid: int, **overrides) -> Config:
    """Configuration ``cid``; keyword overrides build a variant with the same
    seeds (e.g. a smaller ``B`` or ``V`` for a CPU-sized parity case)."""
    return replace(CONFIGS[cid], **overrides)


def straddling(cfg: Config) -> Config:
    """Variant whose spike heights U(10, 20) put confidences on both sides of
    the reveal / remask thresholds (the literal N(0,2) inputs almost never
    exceed confidence 0.5)."""
    return replace(cfg, spike_frac=0.5, spike_lo=10.0, spike_hi=20.0)


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions for input quantisation (round to nearest even)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------
def _rng(cfg_id: int, tensor: int, chunk: int, extra: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([SEED_BASE, cfg_id, tensor, chunk, extra])
    return np.random.Generator(np.random.PCG64(ss))


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _pmap(fn, items):
    items = list(items)
    if len(items) <= 1:
        return [fn(i) for i in items]
    with ThreadPoolExecutor(_workers()) as ex:
        return list(ex.map(fn, items))


def _normal_bf16(cfg_id: int, tensor: int, rows: int, cols: int, std: float, extra: int = 0) -> np.ndarray:
    out = np.empty((rows, cols), dtype=np.uint16)
    nchunk = (rows + WEIGHT_CHUNK_ROWS - 1) // WEIGHT_CHUNK_ROWS

    def one(c):
        r0 = c * WEIGHT_CHUNK_ROWS
        r1 = min(rows, r0 + WEIGHT_CHUNK_ROWS)
        g = _rng(cfg_id, tensor, c, extra)
        x = g.standard_normal((r1 - r0, cols), dtype=np.float32)
        x *= np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(x)

    _pmap(one, range(nchunk))
    return out


def lm_head(cfg: Config) -> np.ndarray:
    """Shared (frozen) LM head ``W_lm``: bf16 bits [V, d]."""
    return _normal_bf16(cfg.cid, T_WLM, cfg.V, cfg.d, 0.02)


def embedding(cfg: Config) -> np.ndarray:
    """Token embedding ``E``: bf16 bits [V, d]."""
    return _normal_bf16(cfg.cid, T_E, cfg.V, cfg.d, 0.02)


def head_weights(cfg: Config, k: int, gamma: str = "ones"):
    """Head ``k`` (0-based): (W1 [d,2d], W2 [d,d], gamma [d]) as bf16 bits.
    ``gamma``: "ones" (benchmark), "normal" (N(0,0.02)) or "zeros"."""
    d = cfg.d
    w1 = _normal_bf16(cfg.cid, T_W1, d, 2 * d, 0.02, extra=k)
    w2 = _normal_bf16(cfg.cid, T_W2, d, d, 0.02, extra=k)
    if gamma == "ones":
        g = f32_to_bf16_bits(np.ones(d, dtype=np.float32))
    elif gamma == "zeros":
        g = np.zeros(d, dtype=np.uint16)
    elif gamma == "normal":
        g = f32_to_bf16_bits(_rng(cfg.cid, T_W2, 1 << 20, k).standard_normal(d, dtype=np.float32)
                             * np.float32(0.02))
    else:
        raise ValueError(gamma)
    return w1, w2, g


def _seqs(cfg: Config, seqs: Optional[Iterable[int]]) -> Sequence[int]:
    s = list(range(cfg.B)) if seqs is None else [int(b) for b in seqs]
    for b in s:
        if not 0 <= b < cfg.B:
            raise IndexError(b)
    return s


def hidden(cfg: Config, step: int = 0, seqs: Optional[Iterable[int]] = None) -> np.ndarray:
    """Backbone hidden states for denoising step ``step``: bf16 bits
    [len(seqs)*L, d], N(0, 1); rows of the listed sequences, in list order."""
    s = _seqs(cfg, seqs)
    out = np.empty((len(s) * cfg.L, cfg.d), dtype=np.uint16)

    def one(j):
        g = _rng(cfg.cid, T_H, s[j], step)
        out[j * cfg.L:(j + 1) * cfg.L] = f32_to_bf16_bits(
            g.standard_normal((cfg.L, cfg.d), dtype=np.float32))

    _pmap(one, range(len(s)))
    return out


def logits0(cfg: Config, seqs: Optional[Iterable[int]] = None, out: Optional[np.ndarray] = None,
            step: int = 0) -> np.ndarray:
    """Prior logit state ``z0``: fp32 [len(seqs)*L, V], N(0, 2) plus spikes.  ``step`` > 0 gives the
    (independent) prior logits a stand-in backbone produces at a later denoising step."""
    s = _seqs(cfg, seqs)
    if out is None:
        out = np.empty((len(s) * cfg.L, cfg.V), dtype=np.float32)

    def one(j):
        b = s[j]
        blk = out[j * cfg.L:(j + 1) * cfg.L]
        g = _rng(cfg.cid, T_Z, b, step)
        g.standard_normal(out=blk, dtype=np.float32)
        blk *= np.float32(2.0)
        if cfg.spike_frac > 0.0:
            gs = _rng(cfg.cid, T_SPIKE, b, step)
            hit = gs.random(cfg.L) < cfg.spike_frac
            idx = gs.integers(0, cfg.V, cfg.L)
            hgt = gs.uniform(cfg.spike_lo, cfg.spike_hi, cfg.L).astype(np.float32)
            for r in range(cfg.L):
                if hit[r]:
                    blk[r, idx[r]] += hgt[r]

    _pmap(one, range(len(s)))
    return out


def residual(cfg: Config, seqs: Optional[Iterable[int]] = None, step: int = 0) -> np.ndarray:
    """Stand-in for a head's predicted logit residual ``delta_t``: fp32 [len(seqs)*L, V], N(0, 0.5)."""
    s = _seqs(cfg, seqs)
    out = np.empty((len(s) * cfg.L, cfg.V), dtype=np.float32)

    def one(j):
        blk = out[j * cfg.L:(j + 1) * cfg.L]
        _rng(cfg.cid, T_DELTA, s[j], step).standard_normal(out=blk, dtype=np.float32)
        blk *= np.float32(0.5)

    _pmap(one, range(len(s)))
    return out


def block_states(cfg_id: int, block: int, S: int, N: int, bf16: bool = False, base_std: float = 2.0,
                 step_std: float = 0.4) -> np.ndarray:
    """Stand-in for the S states a backbone tensor goes through while one block is decoded:
    state 0 ~ N(0, base_std), each later state the previous one plus fresh N(0, step_std) noise.
    fp32 [S, N], or bf16 bits [S, N] (each state rounded after the sum)."""
    g = _rng(cfg_id, T_STATES, block)
    out = np.empty((S, N), dtype=np.float32)
    g.standard_normal(out=out, dtype=np.float32)
    out[0] *= np.float32(base_std)
    out[1:] *= np.float32(step_std)
    np.cumsum(out, axis=0, out=out)
    return f32_to_bf16_bits(out) if bf16 else out


@dataclass(frozen=True)
class TBodyDims:
    """Sizes of the transformer head body (the decoder layer of the backbone's family)."""

    D: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    P_max: int
    rope_theta: float = 1.0e6


def tf_layer(cfg: Config, td: TBodyDims, k: int, l: int, gain: str = "ones") -> dict:
    """Layer ``l`` of head ``k``: bf16 bits of Wqkv [(nh+2nkv)hd, d], Wo [d, nh hd], Wgu [2 d_ff, d],
    Wdown [d, d_ff], the two norm gains [d] and the prefix caches kc, vc [B, P_max, nkv, hd]."""
    d, qd, kvd = cfg.d, td.n_heads * td.head_dim, td.n_kv_heads * td.head_dim
    tag = (k * 64 + l) * 8
    out = {
        "Wqkv": _normal_bf16(cfg.cid, T_TF, qd + 2 * kvd, d, 0.02, extra=tag + 0),
        "Wo": _normal_bf16(cfg.cid, T_TF, d, qd, 0.02, extra=tag + 1),
        "Wgu": _normal_bf16(cfg.cid, T_TF, 2 * td.d_ff, d, 0.02, extra=tag + 2),
        "Wdown": _normal_bf16(cfg.cid, T_TF, d, td.d_ff, 0.02, extra=tag + 3),
    }
    for n, name in enumerate(("g1", "g2")):
        if gain == "ones":
            out[name] = f32_to_bf16_bits(np.ones(d, dtype=np.float32))
        else:
            out[name] = f32_to_bf16_bits(1.0 + 0.1 * _rng(cfg.cid, T_TF, 1 << 20, tag + 4 + n)
                                         .standard_normal(d, dtype=np.float32))
    rows = cfg.B * td.P_max
    cols = td.n_kv_heads * td.head_dim
    shape = (cfg.B, td.P_max, td.n_kv_heads, td.head_dim)
    out["kc"] = _normal_bf16(cfg.cid, T_KV, max(rows, 1), cols, 1.0, extra=tag + 0)[:rows].reshape(shape)
    out["vc"] = _normal_bf16(cfg.cid, T_KV, max(rows, 1), cols, 1.0, extra=tag + 1)[:rows].reshape(shape)
    return out


def prefix_lens(cfg: Config, td: TBodyDims) -> np.ndarray:
    """Committed prefix length per sequence: int32 [B] in [0, P_max]."""
    p = _rng(cfg.cid, T_PLEN, 0).integers(0, td.P_max + 1, cfg.B).astype(np.int32)
    p[0] = 0
    p[-1] = td.P_max
    return p


def verify_logits(cfg: Config, seqs: Optional[Iterable[int]] = None) -> np.ndarray:
    """Synthetic backbone verify logits before boosting: fp32
    [len(seqs), L, V], N(0, 2)."""
    s = _seqs(cfg, seqs)
    out = np.empty((len(s), cfg.L, cfg.V), dtype=np.float32)

    def one(j):
        g = _rng(cfg.cid, T_VERIFY, s[j])
        g.standard_normal(out=out[j], dtype=np.float32)
        out[j] *= np.float32(2.0)

    _pmap(one, range(len(s)))
    return out


def verify_boost_mask(cfg: Config, p: float = 0.7) -> np.ndarray:
    """Bernoulli(p) choice of which (sequence, draft) pairs get the boost:
    bool [B, K]."""
    return _rng(cfg.cid, T_BOOST, 0).random((cfg.B, cfg.K)) < p


def apply_verify_boost(verify: np.ndarray, draft_pos: np.ndarray, draft_tok: np.ndarray,
                       mask: np.ndarray, boost: float = 8.0) -> None:
    """Add ``boost`` in place at verify[b, draft_pos[b,j], draft_tok[b,j]] for
    every (b, j) selected by ``mask`` whose draft exists (pos >= 0)."""
    B, K = draft_pos.shape
    for b in range(B):
        for j in range(K):
            if mask[b, j] and draft_pos[b, j] >= 0:
                verify[b, draft_pos[b, j], draft_tok[b, j]] += np.float32(boost)
