"""GPU parity of the joint verification's candidate blocks (Figure 1 (d)) and of the device error
word: mrp_build_candidates against the oracle bit for bit, alone and chained
chain step -> candidates -> stand-in backbone -> mrp_verify_accept_joint."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp
from harness import Problem, gpu_chain, io_to_host, oracle_chain

pytestmark = pytest.mark.gpu

MASK = 151935      # stand-in id of the mask token


def _gpu_candidates(ctx, B, L, K, x_t, m_t, dpos, dtok, stride=None):
    stride = stride or K
    ct = torch.full((B, K + 1, L), -5, dtype=torch.int32, device="cuda")
    cm = torch.full((B, K + 1, L), 9, dtype=torch.uint8, device="cuda")
    ctx.build_candidates(B, K, torch.from_numpy(x_t).cuda(), torch.from_numpy(m_t).cuda(), dpos, dtok, stride, MASK, ct, cm)
    torch.cuda.synchronize()
    return ct.cpu().numpy(), cm.cpu().numpy()


@pytest.mark.parametrize("B,L,K", [(1, 1, 1), (37, 16, 3), (300, 7, 16), (5, 64, 4)])
def test_build_candidates_matches_oracle(B, L, K):
    rng = np.random.default_rng(100 * B + L)
    ctx = mrp.MrpContext(256, 4096, B * L, L)
    try:
        m_t = (rng.random((B, L)) < 0.7).astype(np.uint8)
        x_t = rng.integers(0, 4096, (B, L)).astype(np.int32)
        dpos = rng.integers(-1, L, (B, K)).astype(np.int32)      # repeats and unmasked positions included
        dtok = rng.integers(0, 4096, (B, K)).astype(np.int32)
        want_t, want_m = orc.build_candidates(x_t, m_t, dpos, dtok, MASK)
        got_t, got_m = _gpu_candidates(ctx, B, L, K, x_t, m_t, torch.from_numpy(dpos).cuda(), torch.from_numpy(dtok).cuda())
        np.testing.assert_array_equal(got_t, want_t)
        np.testing.assert_array_equal(got_m, want_m)
        assert ctx.poll_error() == 0
        # K = 0: the block itself
        t0, m0 = _gpu_candidates(ctx, B, L, 0, x_t, m_t, torch.from_numpy(dpos).cuda(), torch.from_numpy(dtok).cuda(), stride=K)
        np.testing.assert_array_equal(t0[:, 0], np.where(m_t == 1, MASK, x_t))
        np.testing.assert_array_equal(m0[:, 0], m_t)
        # a draft position beyond the block is skipped (as the oracle does) and reported once polled
        bad = dpos.copy(); bad[B // 2, K - 1] = L + 3
        want_t, want_m = orc.build_candidates(x_t, m_t, bad, dtok, MASK)
        got_t, got_m = _gpu_candidates(ctx, B, L, K, x_t, m_t, torch.from_numpy(bad).cuda(), torch.from_numpy(dtok).cuda())
        np.testing.assert_array_equal(got_t, want_t)
        np.testing.assert_array_equal(got_m, want_m)
        assert ctx.poll_error() == 2 and "draft position" in ctx.last_error()
        assert ctx.poll_error() == 0                              # cleared by the poll
        # argument errors, before any launch
        z = torch.zeros(4, dtype=torch.int32, device="cuda")
        assert ctx.build_candidates(B, K, None, z, z, z, K, MASK, z, z, check=False) == -1
        assert ctx.build_candidates(B, K, z, z, z, z, K - 1, MASK, z, z, check=False) == -2
        assert ctx.build_candidates(B + 1, K, z, z, z, z, K, MASK, z, z, check=False) == -2
        assert ctx.build_candidates(0, K, z, z, z, z, K, MASK, z, z) == 0
    finally:
        ctx.close()


def _standin_backbone(cfg, cand_tok, cand_masked, dpos, dtok, agree):
    """Synthetic verifier logits [B][K+1][L][V] that depend on the candidates' contents: N(0, 2), plus +12 at
    one token per (candidate, position) -- a hash of the candidate's tokens, or, where `agree` says so, the
    draft the chain made at that position (so that some drafts are accepted)."""
    B, K1, L = cand_tok.shape
    V = cfg.V
    # (one seeded chunk per (sequence, candidate): the generator draws per sequence of a batch of B * (K + 1))
    ver = mi.verify_logits(mi.config(cfg.cid, d=cfg.d, V=V, B=B * K1, L=L)).reshape(B, K1, L, V)
    h = (cand_tok.astype(np.int64) * (np.arange(L) + 3)).sum(-1)                   # [B][K+1]
    for b in range(B):
        for k in range(K1):
            for p in range(L):
                t = int((h[b, k] * 2654435761 + 7919 * p) % V)
                if k < K1 - 1 and dpos[b, k] == p and agree[b, k]:
                    t = int(dtok[b, k])
                ver[b, k, p, t] += 12.0
    return ver


def test_chain_candidates_joint_verify_end_to_end():
    """Speculative mode end to end on a small case: static r = 1 drafting (Algorithm 3), candidate blocks
    from the chain's state, a stand-in backbone that reads the candidates, joint verification; every
    stage equals the oracle's."""
    cfg = mi.straddling(mi.config(0, d=256, V=4100, B=11, L=8))
    K = cfg.K
    rcfg = mrp.RevealCfg(tau=1.0, r_min=1)
    prob = Problem(cfg)
    try:
        z0, h = mi.logits0(cfg), mi.hidden(cfg)
        z_d = torch.from_numpy(z0).cuda()
        io, _ = gpu_chain(prob, cfg.B, K, z_d, h, rcfg)
        g = io_to_host(io)
        o = oracle_chain(prob, z0, mi.bf16_bits_to_f64(h), rcfg, K).out
        np.testing.assert_array_equal(g.draft_pos, o.draft_pos)
        np.testing.assert_array_equal(g.draft_tok, o.draft_tok)
        np.testing.assert_array_equal(g.revealed_at, o.revealed_at)

        def block_before_drafting(ra, x_tok):
            m_t = (ra != 0).astype(np.uint8).reshape(cfg.B, cfg.L)        # only the backbone's own reveal is in x_t
            return np.where(m_t == 1, -1, x_tok.reshape(cfg.B, cfg.L)).astype(np.int32), m_t

        x_t, m_t = block_before_drafting(g.revealed_at, g.x_tok)
        # the drafts are read in place from the chain's [B][K+1] arrays (column 0 is the backbone's reveal)
        got_t, got_m = _gpu_candidates(prob.ctx, cfg.B, cfg.L, K, x_t, m_t, io.draft_pos.view(-1)[1:],
                                       io.draft_tok.view(-1)[1:], stride=K + 1)
        xo, mo = block_before_drafting(o.revealed_at, o.x_tok)
        dpos, dtok = np.ascontiguousarray(o.draft_pos[:, 1:]), np.ascontiguousarray(o.draft_tok[:, 1:])
        want_t, want_m = orc.build_candidates(xo, mo, dpos, dtok, MASK)
        np.testing.assert_array_equal(got_t, want_t)
        np.testing.assert_array_equal(got_m, want_m)
        assert (dpos >= 0).all() and want_m[:, K].sum() == cfg.B * (cfg.L - 1 - K)
        agree = np.random.default_rng(9).random((cfg.B, K)) < 0.7
        ver = _standin_backbone(cfg, got_t, got_m, dpos, dtok, agree)
        match = torch.zeros((cfg.B, K), dtype=torch.uint8, device="cuda")
        alen = torch.zeros(cfg.B, dtype=torch.int32, device="cuda"); corr = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
        prob.ctx.verify_accept_joint(cfg.B, K, torch.from_numpy(ver).cuda(), io.draft_pos.view(-1)[1:],
                                     io.draft_tok.view(-1)[1:], K + 1, match, alen, corr)
        torch.cuda.synchronize()
        m_o, a_o, c_o = orc.verify_accept_joint(_standin_backbone(cfg, want_t, want_m, dpos, dtok, agree), dpos, dtok)
        np.testing.assert_array_equal(match.cpu().numpy(), m_o)
        np.testing.assert_array_equal(alen.cpu().numpy(), a_o)
        np.testing.assert_array_equal(corr.cpu().numpy(), c_o)
        assert 0 < a_o.sum() < cfg.B * K
        assert prob.ctx.poll_error() == 0
    finally:
        prob.close()


def test_error_word_reports_clamped_conditioning_token():
    """A conditioning token outside the vocabulary (caller error on a resumed call) is clamped by the
    gather and reported by mrp_poll_error, instead of passing silently."""
    cfg = mi.config(0, B=3, L=4, K=1)
    prob = Problem(cfg)
    try:
        z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
        io = mrp.StepIO(cfg.B, cfg.L, 1)
        io.cond_tok.copy_(torch.tensor([5, cfg.V + 10, 7], dtype=torch.int32))
        hrun = torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")
        r = mrp.RevealCfg(tau=0.9, fresh_block=0, state_offset=0, run_state0=0)
        gpu_chain(prob, cfg.B, 1, z_d, mi.hidden(cfg), r, io=io, hrun_d=hrun)
        assert prob.ctx.poll_error() == 1 and "cond_tok" in prob.ctx.last_error()
        io.cond_tok.copy_(torch.tensor([5, 6, 7], dtype=torch.int32))
        gpu_chain(prob, cfg.B, 1, z_d, mi.hidden(cfg), r, io=io, hrun_d=hrun)
        assert prob.ctx.poll_error() == 0
    finally:
        prob.close()
