"""Shared machinery of the GPU parity tests: builds a problem from the seeded
generators, runs the HIP path through the C-ABI binding, runs the CPU oracle
(head by head, keeping every intermediate state) and compares the two under the
parity rule:

* logits  |z_gpu - z_orc| <= 2e-2 + 2e-2 |z_orc|  (bf16 inputs, fp32 accumulation), against the
  PLAIN oracle (no intermediate rounded: the definition l <- l + W_lm RMSNorm(u) gamma);
* tokens, masks, drafts, remask flags, accept lengths bit-exact against the oracle run with its
  LM-head operand rounded to bf16 (the precision both sides then take each decision in), except
  - a token may differ where that oracle's top-2 logit gap is below 1e-3,
  - a decision of the state being decided may differ where, among the quantities that decision
    compares, an oracle confidence is within 1e-3 (relative) of its threshold (a still-masked
    candidate against tau; a remask-eligible row against tau_remask) or the two candidates on either
    side of a rank boundary the rule uses (most confident vs runner-up; last selected vs first not
    selected when the set is chosen by rank) are within 1e-3 (relative) of each other;
  once a sequence has used an exemption its later states are not compared (a different
  conditioning token changes the rest of its chain).  Exemptions are counted and the number of
  sequences that may use one is an explicit argument, 0 unless a test says otherwise.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from types import SimpleNamespace
from typing import List, Optional, Sequence

import numpy as np
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp

LOGIT_ATOL = 2e-2
LOGIT_RTOL = 2e-2
GAP_EXEMPT = 1e-3
CONF_EXEMPT = 1e-3
# Engineering bounds well inside the parity rule, against the oracle variant with the bf16 LM-head operand
# (the two sides then differ by fp32 round-off only).  Observed: logits up to 1.8e-3 after one chain step
# and 3.3e-3 after 8 steps on a resident logit state at d = 4096 (24 fp32 accumulations of 4096 terms
# each into logits of magnitude ~10); the bound is about twice the largest value seen.
LOGIT_TIGHT = 8e-3
LSE_ATOL = 2e-3
CONF_RTOL = 4e-3


def dev_bits(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


class Problem:
    """Weights of one configuration on host (for the oracle) and device (packed)."""

    def __init__(self, cfg: mi.Config, gamma: str = "ones", max_rows: Optional[int] = None,
                 share_heads: bool = False):
        self.cfg = cfg
        self.W = mi.lm_head(cfg)
        self.E = mi.embedding(cfg)
        nh = 1 if share_heads else cfg.K
        hs = [mi.head_weights(cfg, k, gamma) for k in range(nh)]
        self.heads = [hs[0]] * cfg.K if share_heads else hs
        self.ctx = mrp.MrpContext(cfg.d, cfg.V, max_rows or cfg.M, cfg.L)
        self.E_d = dev_bits(self.E)
        w_d = dev_bits(self.W)
        self.Wp_d = mrp.pack_weight(w_d)
        del w_d
        dh = []
        for (w1, w2, g) in hs:
            dh.append(mrp.Head(mrp.pack_weight(dev_bits(w1), body=True), mrp.pack_weight(dev_bits(w2), body=True),
                               dev_bits(g)))
        self.heads_d = [dh[0]] * cfg.K if share_heads else dh
        torch.cuda.synchronize()

    def close(self):
        self.ctx.close()


def gpu_chain(prob: Problem, B: int, K: int, z_d: torch.Tensor, h_bits: Optional[np.ndarray],
              rcfg: mrp.RevealCfg, io: Optional[mrp.StepIO] = None, hrun_d: Optional[torch.Tensor] = None,
              heads=None):
    """Run mrp_chain_step; z_d (device fp32 [M][V]) is updated in place."""
    cfg = prob.cfg
    M = B * cfg.L
    io = io or mrp.StepIO(B, cfg.L, K)
    if hrun_d is None:
        hrun_d = torch.zeros((M, cfg.d), dtype=torch.float32, device="cuda")
    h_d = dev_bits(h_bits) if h_bits is not None else None
    prob.ctx.chain_step(B, K, h_d, hrun_d, prob.E_d, prob.Wp_d, heads or prob.heads_d, z_d, rcfg, io)
    torch.cuda.synchronize()
    return io, hrun_d


def io_to_host(io: mrp.StepIO) -> SimpleNamespace:
    return SimpleNamespace(tok=io.tok.cpu().numpy(), conf=io.conf.cpu().numpy(), lse=io.lse.cpu().numpy(),
                           revealed_at=io.revealed_at.cpu().numpy(), masked=io.masked.cpu().numpy(),
                           cond_tok=io.cond_tok.cpu().numpy(), protect_pos=io.protect_pos.cpu().numpy(),
                           draft_pos=io.draft_pos.cpu().numpy(), draft_tok=io.draft_tok.cpu().numpy(),
                           remasked=io.remasked.cpu().numpy(), x_tok=io.x_tok.cpu().numpy())


@dataclass
class OracleRun:
    """Oracle results for a subset of sequences, with the state after every head."""
    out: SimpleNamespace
    snaps: List[SimpleNamespace] = field(default_factory=list)   # snaps[k]: state after state k
    pre0: Optional[SimpleNamespace] = None                       # masks before state 0 decided


def oracle_chain(prob: Problem, z0_rows: np.ndarray, hrun_rows: np.ndarray, rcfg: mrp.RevealCfg, K: int,
                 masked=None, revealed_at=None, cond_tok=None, protect_pos=None, heads=None, x_tok=None,
                 round_y: int = 1, tbody: Optional["orc.TBody"] = None) -> OracleRun:
    """Oracle chain on the given rows (whole sequences), one head per call so that
    every intermediate state is kept.  hrun_rows: float64 [rows][d].  round_y = 1: the oracle's
    bf16-operand variant (decisions are compared against it); 0: the plain definition.  tbody: the K heads'
    transformer layers (then every head is fuse projection + layers; W2 unused)."""
    cfg = prob.cfg
    L = cfg.L
    Bs = z0_rows.shape[0] // L
    M = Bs * L
    heads = heads or prob.heads
    z = np.ascontiguousarray(z0_rows, dtype=np.float64)
    hrun = np.ascontiguousarray(hrun_rows, dtype=np.float64)
    tok = np.full((K + 1, M), -1, np.int32); conf = np.zeros((K + 1, M)); lse = np.zeros((K + 1, M))
    gap = np.full((K + 1, M), np.inf); rem = np.zeros((K + 1, M), np.uint8)
    dpos = np.full((Bs, K + 1), -1, np.int32); dtok = np.full((Bs, K + 1), -1, np.int32)
    snaps = []
    st = dict(masked=masked, revealed_at=revealed_at, cond_tok=cond_tok, protect_pos=protect_pos, x_tok=x_tok)
    ptok = np.ones((K + 1, M))   # probability of the recorded token under each state's logits (remask_mode 1)
    rmode = getattr(rcfg, "remask_mode", 0)

    def mk(Kc, offset, run0, fresh):
        return orc.make_cfg(cfg.d, cfg.V, Bs, L, Kc, tau=rcfg.tau, r_min=rcfg.r_min, max_accept=rcfg.max_accept,
                            carry_hidden=rcfg.carry_hidden, tau_remask=rcfg.tau_remask,
                            head_reveal=rcfg.head_reveal, fresh_block=fresh, state_offset=offset, run_state0=run0,
                            remask_mode=rmode, round_y=round_y)

    def snap(o):
        snaps.append(SimpleNamespace(z=o.z.copy(), hrun=o.hrun.copy(), masked=o.masked.copy(),
                                     revealed_at=o.revealed_at.copy(), cond_tok=o.cond_tok.copy(),
                                     protect_pos=o.protect_pos.copy(), x_tok=o.x_tok.copy()))

    fresh0 = bool(rcfg.run_state0 and rcfg.fresh_block)
    pre0 = SimpleNamespace(
        masked=np.ones(M, np.uint8) if (masked is None or fresh0) else np.array(masked, np.uint8),
        revealed_at=np.full(M, -1, np.int8) if (revealed_at is None or fresh0) else np.array(revealed_at, np.int8),
        protect_pos=np.full(Bs, -1, np.int32) if protect_pos is None else np.array(protect_pos, np.int32))
    off = rcfg.state_offset
    if rcfg.run_state0:
        o = orc.chain_step(mk(0, off, 1, rcfg.fresh_block), prob.E, prob.W, [], z, hrun, **st)
        tok[0], conf[0], lse[0], gap[0], rem[0] = o.tok[0], o.conf[0], o.lse[0], o.gap[0], o.remasked[0]
        dpos[:, 0], dtok[:, 0] = o.draft_pos[:, 0], o.draft_tok[:, 0]
    else:
        o = SimpleNamespace(z=z, hrun=hrun, masked=pre0.masked.copy(), revealed_at=pre0.revealed_at.copy(),
                            cond_tok=np.zeros(Bs, np.int32) if cond_tok is None else np.array(cond_tok, np.int32),
                            protect_pos=pre0.protect_pos.copy(),
                            x_tok=np.full(M, -1, np.int32) if x_tok is None else np.array(x_tok, np.int32))
    snap(o)
    for k in range(1, K + 1):
        tb = None if tbody is None else orc.TBody(tbody.tcfg, [tbody.layers[k - 1]], tbody.prefix_len)
        o = orc.chain_step(mk(1, off + k - 1, 0, 0), prob.E, prob.W, [heads[k - 1]], o.z, o.hrun, masked=o.masked,
                           revealed_at=o.revealed_at, cond_tok=o.cond_tok, protect_pos=o.protect_pos, x_tok=o.x_tok,
                           tbody=tb)
        if rmode == 1:
            ptok[k] = orc.token_prob(o.z, o.lse[1], o.x_tok)
        tok[k], conf[k], lse[k], gap[k], rem[k] = o.tok[1], o.conf[1], o.lse[1], o.gap[1], o.remasked[1]
        dpos[:, k], dtok[:, k] = o.draft_pos[:, 1], o.draft_tok[:, 1]
        snap(o)
    out = SimpleNamespace(z=o.z, hrun=o.hrun, tok=tok, conf=conf, lse=lse, gap=gap, remasked=rem, draft_pos=dpos,
                          draft_tok=dtok, masked=o.masked, revealed_at=o.revealed_at, cond_tok=o.cond_tok,
                          protect_pos=o.protect_pos, x_tok=o.x_tok, ptok=ptok)
    return OracleRun(out, snaps, pre0)


def head_view(run: OracleRun, k: int) -> OracleRun:
    """Head k of a run as a one-head run (slot 0 = state k - 1, slot 1 = state k): what a call with
    K = 1, state_offset = k - 1, run_state0 = 0, fed the run's state k - 1, has to produce."""
    o, s0, s1 = run.out, run.snaps[k - 1], run.snaps[k]
    sl = lambda a: np.stack([a[k - 1], a[k]])
    out = SimpleNamespace(z=s1.z, hrun=s1.hrun, tok=sl(o.tok), conf=sl(o.conf), lse=sl(o.lse), gap=sl(o.gap),
                          remasked=sl(o.remasked), draft_pos=np.ascontiguousarray(o.draft_pos[:, k - 1:k + 1]),
                          draft_tok=np.ascontiguousarray(o.draft_tok[:, k - 1:k + 1]), masked=s1.masked,
                          revealed_at=s1.revealed_at, cond_tok=s1.cond_tok, protect_pos=s1.protect_pos,
                          x_tok=s1.x_tok, ptok=sl(o.ptok))
    pre = SimpleNamespace(masked=s0.masked, revealed_at=s0.revealed_at, protect_pos=s0.protect_pos)
    return OracleRun(out, [s0, s1], pre)


def _decision_fragile(conf, masked_before, ra_before, protect, state, rcfg, reveal_here, ptok=None) -> bool:
    """True when a decision of THIS state of one sequence compares oracle quantities that lie inside
    the exemption band: a still-masked candidate's confidence against tau, the candidates on either
    side of a rank boundary the rule uses against each other, or a remask-eligible row's confidence
    (probability of its recorded token in remask_mode 1) against tau_remask.  conf: this state's
    oracle confidences of the sequence's L rows; masked_before / ra_before: the sequence's masks
    before this state decided; state: the global state index."""
    c = np.asarray(conf, np.float64)
    L = len(c)
    cand = np.flatnonzero(np.asarray(masked_before) != 0)
    if reveal_here and len(cand):
        cc = c[cand]
        if np.any(np.abs(cc - rcfg.tau) < CONF_EXEMPT * max(rcfg.tau, 1e-30)):
            return True
        s = np.sort(cc)[::-1]                       # most confident first
        ns = int(np.sum(s > rcfg.tau))
        bounds = {0}                                # most confident vs runner-up: the draft
        if rcfg.max_accept:
            m = min(max((7 * len(cand)) // 10, 5), L)
            if ns > m:
                ns = m
                bounds.add(m - 1)                   # last kept vs first cut by the cap
        if ns < rcfg.r_min:
            ns = min(rcfg.r_min, len(cand))
            bounds.add(ns - 1)                      # last forced vs first not forced
        for r in bounds:
            if 0 <= r and r + 1 < len(s) and (s[r] - s[r + 1]) < CONF_EXEMPT * s[r]:
                return True
    if rcfg.tau_remask >= 0 and state >= 1:
        ra = np.asarray(ra_before).astype(np.int64)
        elig = (ra >= 0) & (ra <= state - 1)
        if protect is not None and 0 <= protect < L:
            elig[protect] = False
        cr = np.asarray(ptok, np.float64) if (getattr(rcfg, "remask_mode", 0) == 1 and ptok is not None) else c
        if np.any(np.abs(cr[elig] - rcfg.tau_remask) < CONF_EXEMPT * max(rcfg.tau_remask, 1e-30)):
            return True
    return False


def _same_decisions(a: SimpleNamespace, ja: int, b: SimpleNamespace, jb: int, L: int, k: int) -> bool:
    """State k's decisions of sequence ja of run a equal those of sequence jb of run b."""
    ra, rb = slice(ja * L, (ja + 1) * L), slice(jb * L, (jb + 1) * L)
    if a.draft_pos[ja, k] != b.draft_pos[jb, k] or a.draft_tok[ja, k] != b.draft_tok[jb, k]:
        return False
    return bool(np.array_equal(a.remasked[k, ra], b.remasked[k, rb]))


def compare_chain(g: SimpleNamespace, z_g_rows: Optional[np.ndarray], hrun_g_rows: Optional[np.ndarray],
                  orun: OracleRun, seqs: Sequence[int], L: int, K: int, rcfg: mrp.RevealCfg,
                  plain: Optional[OracleRun] = None, max_exempt: int = 0) -> dict:
    """Compare GPU outputs (full batch, indexed by sequence id) with oracle outputs (subset, in list
    order).  z_g_rows / hrun_g_rows: GPU rows of the subset, in list order.  orun: the oracle run with
    the bf16 LM-head operand (decisions, tight logit bound); plain: the plain-definition run of the same
    inputs (the stated logit tolerance).  At most max_exempt sequences may use an exemption."""
    o = orun.out
    stats = dict(seqs=len(seqs), rows=len(seqs) * L, tok_exempt=0, decision_exempt=0, diverged=0,
                 max_logit_err=0.0, max_lse_err=0.0, max_conf_rel=0.0)
    k0 = 0 if rcfg.run_state0 else 1
    off = rcfg.state_offset
    gpu_ok = []
    for jj, b in enumerate(seqs):
        rg = slice(b * L, (b + 1) * L)
        ro = slice(jj * L, (jj + 1) * L)
        diverged = False
        fragile_any = False
        for k in range(k0, K + 1):
            what = f"seq {b} state {k}"
            lse_err = np.abs(g.lse[k, rg] - o.lse[k, ro]).max()
            conf_rel = (np.abs(g.conf[k, rg] - o.conf[k, ro]) / o.conf[k, ro]).max()
            stats["max_lse_err"] = max(stats["max_lse_err"], float(lse_err))
            stats["max_conf_rel"] = max(stats["max_conf_rel"], float(conf_rel))
            assert lse_err <= LSE_ATOL, f"{what}: lse error {lse_err}"
            assert conf_rel <= CONF_RTOL, f"{what}: confidence rel. error {conf_rel}"
            neq = g.tok[k, rg] != o.tok[k, ro]
            if neq.any():
                assert np.all(o.gap[k, ro][neq] < GAP_EXEMPT), \
                    f"{what}: token differs with top-2 gap {o.gap[k, ro][neq]}"
                stats["tok_exempt"] += int(neq.sum())
                diverged = True
                break
            before = orun.pre0 if k == 0 else orun.snaps[k - 1]
            prot = int(before.protect_pos[jj]) if k > 0 else -1
            reveal_here = (k == 0) or bool(rcfg.head_reveal)
            fragile = _decision_fragile(o.conf[k, ro], before.masked[ro], before.revealed_at[ro], prot, off + k, rcfg,
                                        reveal_here, o.ptok[k, ro])
            fragile_any = fragile_any or fragile
            same = (g.draft_pos[b, k] == o.draft_pos[jj, k] and g.draft_tok[b, k] == o.draft_tok[jj, k]
                    and np.array_equal(g.remasked[k, rg], o.remasked[k, ro]))
            if not same:
                assert fragile, (f"{what}: decision differs: draft ({g.draft_pos[b, k]},{g.draft_tok[b, k]}) vs "
                                 f"({o.draft_pos[jj, k]},{o.draft_tok[jj, k]}), conf {o.conf[k, ro]}")
                stats["decision_exempt"] += 1
                diverged = True
                break
        if not diverged:
            same = (np.array_equal(g.masked[rg], o.masked[ro]) and np.array_equal(g.revealed_at[rg], o.revealed_at[ro])
                    and g.cond_tok[b] == o.cond_tok[jj] and g.protect_pos[b] == o.protect_pos[jj]
                    and np.array_equal(g.x_tok[rg], o.x_tok[ro]))
            if not same:
                assert fragile_any, (f"seq {b}: final masks differ: {g.masked[rg]} vs {o.masked[ro]}; "
                                     f"{g.revealed_at[rg]} vs {o.revealed_at[ro]}")
                stats["decision_exempt"] += 1
                diverged = True
        gpu_ok.append(not diverged)
        if diverged:
            stats["diverged"] += 1
            continue
        if z_g_rows is not None:
            zo = o.z[ro]
            err = np.abs(z_g_rows[ro].astype(np.float64) - zo)
            stats["max_logit_err"] = max(stats["max_logit_err"], float(err.max()))
            assert err.max() <= LOGIT_TIGHT, f"seq {b}: logit error {err.max()} above the engineering bound"
        if hrun_g_rows is not None:
            np.testing.assert_allclose(hrun_g_rows[ro], o.hrun[ro], rtol=2e-4, atol=2e-4)
    assert stats["diverged"] <= max_exempt, f"more exempted sequences than the test allows ({max_exempt}): {stats}"

    if plain is not None:
        # The stated tolerance, against the plain definition.  The plain run takes its own decisions; a
        # sequence's state k is comparable while the plain run's decisions of states < k equal the GPU's
        # (the same conditioning tokens went into the heads).
        p = plain.out
        stats.update(plain_states=0, plain_logit_rows=0, plain_skipped_seqs=0, max_logit_err_plain=0.0,
                     max_lse_err_plain=0.0, plain_tok_diff_outside_gap=0, plain_tok_diff_inside_gap=0)
        for jj, b in enumerate(seqs):
            rg = slice(b * L, (b + 1) * L)
            ro = slice(jj * L, (jj + 1) * L)
            inputs_same = True
            for k in range(k0, K + 1):
                if not inputs_same:
                    break
                stats["plain_states"] += 1
                m_p = p.lse[k, ro] + np.log(p.conf[k, ro])               # the row maxima
                tol = LOGIT_ATOL + LOGIT_RTOL * np.abs(m_p)
                lse_err = np.abs(g.lse[k, rg] - p.lse[k, ro])
                stats["max_lse_err_plain"] = max(stats["max_lse_err_plain"], float(lse_err.max()))
                # a log-sum-exp moves by at most the largest logit error of its row
                assert np.all(lse_err <= LOGIT_ATOL + LOGIT_RTOL * np.abs(p.lse[k, ro]) + tol), \
                    f"seq {b} state {k}: lse differs from the plain definition by {lse_err.max()}"
                neq = g.tok[k, rg] != p.tok[k, ro]
                if neq.any():
                    gaps = p.gap[k, ro][neq]
                    # two logits inside the tolerance of each other are the only ones that can swap
                    assert np.all(gaps <= 2 * tol[neq]), f"seq {b} state {k}: token differs from the plain definition with gap {gaps}"
                    stats["plain_tok_diff_outside_gap"] += int(np.sum(gaps >= GAP_EXEMPT))
                    stats["plain_tok_diff_inside_gap"] += int(np.sum(gaps < GAP_EXEMPT))
                same = (g.draft_pos[b, k] == p.draft_pos[jj, k] and g.draft_tok[b, k] == p.draft_tok[jj, k]
                        and np.array_equal(g.remasked[k, rg], p.remasked[k, ro]))
                if k < K and not same:
                    inputs_same = False
            if not inputs_same:
                stats["plain_skipped_seqs"] += 1
                continue
            if z_g_rows is not None:
                zp = p.z[ro]
                err = np.abs(z_g_rows[ro].astype(np.float64) - zp)
                stats["max_logit_err_plain"] = max(stats["max_logit_err_plain"], float(err.max()))
                stats["plain_logit_rows"] += L
                bad = err > LOGIT_ATOL + LOGIT_RTOL * np.abs(zp)
                assert not bad.any(), f"seq {b}: {bad.sum()} logits outside the parity tolerance of the plain definition, max err {err.max()}"
        assert stats["plain_skipped_seqs"] <= max(max_exempt, len(seqs) // 4), \
            f"too few sequences comparable with the plain definition: {stats}"
    return stats
