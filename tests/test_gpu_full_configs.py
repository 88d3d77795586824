"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
the GPU runs the whole batch, the oracle a seeded sample of whole sequences (sequences
are independent), compared element by element under the same parity rule; the verify
stage is compared exactly on the full batch (the oracle's argmax over the drafted rows is
cheap)."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp
from harness import Problem, compare_chain, gpu_chain, io_to_host, oracle_chain

pytestmark = pytest.mark.gpu


def _sample_rows(cfg, seqs):
    return np.concatenate([np.arange(b * cfg.L, (b + 1) * cfg.L) for b in seqs])


def _run_full(cfg, rcfg, seqs, steps=1):
    prob = Problem(cfg)
    try:
        z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
        rows = _sample_rows(cfg, seqs)
        z_o = z_d[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
        io = mrp.StepIO(cfg.B, cfg.L, cfg.K)
        o_state = dict(masked=None, revealed_at=None, cond_tok=None, protect_pos=None, x_tok=None)
        x_out_d = torch.full((cfg.M,), -1, dtype=torch.int32, device="cuda")
        n_masked_d = torch.empty((cfg.B,), dtype=torch.int32, device="cuda")
        x_out_o = np.full(len(rows), -1, np.int32)
        all_stats = []
        for step in range(steps):
            h = mi.hidden(cfg, step=step)
            r = mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=1 if step == 0 else 0)
            io, hrun_d = gpu_chain(prob, cfg.B, cfg.K, z_d, h, r, io=io)
            g = io_to_host(io)
            o = oracle_chain(prob, z_o, mi.bf16_bits_to_f64(h[rows]), r, cfg.K, **o_state)
            zg = z_d[torch.from_numpy(rows).cuda()].cpu().numpy()
            stats = compare_chain(g, zg, hrun_d.cpu().numpy()[rows], o.out, seqs, cfg.L, cfg.K, r,
                                  max_exempt_frac=0.5)
            all_stats.append(stats)
            print(f"\n[config {cfg.cid} step {step}: rows={cfg.M} sample={len(rows)}] {stats}", flush=True)
            if step + 1 < steps:
                # between denoising steps the caller commits what stayed revealed; z stays resident
                prob.ctx.commit(cfg.B, io.x_tok, io.revealed_at, io.masked, x_out_d, n_masked_d)
                x_out_o, ra, n_o = orc.commit(len(seqs), cfg.L, o.out.x_tok, o.out.revealed_at, o.out.masked, x_out_o)
                if not stats["diverged"]:
                    np.testing.assert_array_equal(x_out_d.cpu().numpy()[rows], x_out_o)
                    np.testing.assert_array_equal(n_masked_d.cpu().numpy()[list(seqs)], n_o)
                o_state = dict(masked=o.out.masked, revealed_at=ra, cond_tok=o.out.cond_tok,
                               protect_pos=o.out.protect_pos, x_tok=o.out.x_tok)
                z_o = o.out.z
                if stats["diverged"]:
                    break   # an exempted decision changes the sequence's later inputs: stop comparing
        return prob, io, g, all_stats
    except Exception:
        prob.close()
        raise


@pytest.mark.timeout(600)
def test_config1_full_batch():
    cfg = mi.config(1)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=[0, 7, 19, 31])
    prob.close()


@pytest.mark.timeout(900)
def test_config2_full_batch():
    cfg = mi.config(2)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=[5, 63])
    prob.close()


@pytest.mark.timeout(900)
def test_config3_draft_then_verify():
    cfg = mi.config(3)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=[100])
    try:
        # synthetic backbone verify logits: N(0,2), +8 at the drafted (position, token) on a Bernoulli(0.7) subset
        K = cfg.K
        dpos = np.ascontiguousarray(g.draft_pos[:, 1:])          # the K drafts are states 1..K
        dtok = np.ascontiguousarray(g.draft_tok[:, 1:])
        assert (dpos >= 0).all()
        verify = mi.verify_logits(cfg)
        mi.apply_verify_boost(verify, dpos, dtok, mi.verify_boost_mask(cfg))
        v_d = torch.from_numpy(verify).cuda()
        match = torch.zeros((cfg.B, K), dtype=torch.uint8, device="cuda")
        alen = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
        corr = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
        # the drafts are read in place from the chain's [B][K+1] arrays (column 0 is the backbone's reveal)
        prob.ctx.verify_accept(cfg.B, K, v_d, io.draft_pos.view(-1)[1:], io.draft_tok.view(-1)[1:], K + 1,
                               match, alen, corr)
        torch.cuda.synchronize()
        m_o, a_o, c_o = orc.verify_accept(verify, dpos, dtok)
        np.testing.assert_array_equal(match.cpu().numpy(), m_o)
        np.testing.assert_array_equal(alen.cpu().numpy(), a_o)
        np.testing.assert_array_equal(corr.cpu().numpy(), c_o)
        # sanity of the synthetic recipe: a boosted draft wins only if it beats the row maximum
        print(f"\n[config 3 verify] mean accept_len {a_o.mean():.3f}, per-draft match {m_o.mean():.3f}")
        assert 0.1 < m_o.mean() < 0.7 and a_o.max() <= K
    finally:
        prob.close()


@pytest.mark.timeout(1100)
def test_config4_resident_logits_remask():
    cfg = mi.config(4)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau, tau_remask=cfg.tau_remask), seqs=[77],
                                   steps=cfg.steps)
    prob.close()
    assert len(stats) >= 1
