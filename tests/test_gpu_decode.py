"""GPU parity of the decode loop around the chain: recorded tokens, the committed-token remask
variant, mrp_commit, and whole-block decoding against a seeded stand-in backbone."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp
from harness import (CONF_EXEMPT, GAP_EXEMPT, Problem, compare_chain, dev_bits, gpu_chain, io_to_host, oracle_chain)

pytestmark = pytest.mark.gpu


def test_committed_token_remask_mode():
    # remask compares the probability of the token revealed at the row (not the row's top-1)
    cfg = mi.straddling(mi.config(0, d=256, V=4100, B=12, L=8))
    rcfg = mrp.RevealCfg(tau=0.3, tau_remask=0.8, remask_mode=1)
    prob = Problem(cfg)
    try:
        z0 = mi.logits0(cfg); h = mi.hidden(cfg)
        z_d = torch.from_numpy(z0).cuda()
        io, hrun_d = gpu_chain(prob, cfg.B, cfg.K, z_d, h, rcfg)
        g = io_to_host(io)
        o = oracle_chain(prob, z0, mi.bf16_bits_to_f64(h), rcfg, cfg.K)
        stats = compare_chain(g, z_d.cpu().numpy(), hrun_d.cpu().numpy(), o, list(range(cfg.B)), cfg.L, cfg.K, rcfg)
        print(f"\n[committed-token remask] {stats} remasked={int(o.out.remasked.sum())}")
        assert o.out.remasked.sum() > 0
        # A crafted resume state in which the two rules must differ: every row was "revealed" at state
        # 0 with a recorded token that is NOT its argmax, so confident rows survive the top-1 rule
        # and fall to the committed-token rule.
        M = cfg.M
        s0 = o.snaps[0]
        x_bad = ((o.out.tok[0] + 17) % cfg.V).astype(np.int32)
        ra = np.zeros(M, np.int8); mk = np.zeros(M, np.uint8)
        outs = {}
        for mode in (0, 1):
            r1 = mrp.RevealCfg(tau=0.3, tau_remask=0.5, remask_mode=mode, fresh_block=0, state_offset=0, run_state0=0)
            io1 = mrp.StepIO(cfg.B, cfg.L, 1)
            io1.masked.copy_(torch.from_numpy(mk)); io1.revealed_at.copy_(torch.from_numpy(ra))
            io1.cond_tok.copy_(torch.from_numpy(s0.cond_tok)); io1.protect_pos.fill_(-1)
            io1.x_tok.copy_(torch.from_numpy(x_bad))
            z1 = torch.from_numpy(s0.z.astype(np.float32)).cuda()
            hr1 = torch.from_numpy(s0.hrun.astype(np.float32)).cuda()
            io1, hr1 = gpu_chain(prob, cfg.B, 1, z1, None, r1, io=io1, hrun_d=hr1, heads=prob.heads_d[:1])
            g1 = io_to_host(io1)
            o1 = oracle_chain(prob, s0.z, s0.hrun, r1, 1, masked=mk, revealed_at=ra, cond_tok=s0.cond_tok,
                              protect_pos=np.full(cfg.B, -1, np.int32), heads=prob.heads[:1], x_tok=x_bad)
            compare_chain(g1, z1.cpu().numpy(), hr1.cpu().numpy(), o1, list(range(cfg.B)), cfg.L, 1, r1)
            outs[mode] = o1.out.remasked[1].astype(bool)
        confident = o1.out.conf[1] >= 0.5
        assert confident.sum() > 0 and not outs[0][confident].any() and outs[1][confident].all()
        # a missing x_tok is an argument error, reported before anything is launched
        io2 = mrp.StepIO(cfg.B, cfg.L, cfg.K); io2.x_tok = None
        rc = prob.ctx.chain_step(cfg.B, cfg.K, dev_bits(h), hrun_d, prob.E_d, prob.Wp_d, prob.heads_d, z_d, rcfg, io2,
                                 check=False)
        assert rc == -1
    finally:
        prob.close()


def test_commit_bit_exact():
    cfg = mi.config(0, B=37, L=16)
    prob = Problem(cfg)
    try:
        rng = np.random.default_rng(11)
        M = cfg.M
        ra = rng.integers(-2, 4, M).astype(np.int8)
        masked = (ra == -1).astype(np.uint8)
        x_tok = rng.integers(0, cfg.V, M).astype(np.int32)
        x_out0 = np.where(ra == -2, rng.integers(0, cfg.V, M), -1).astype(np.int32)
        want_x, want_ra, want_n = orc.commit(cfg.B, cfg.L, x_tok, ra, masked, x_out0)
        ra_d = torch.from_numpy(ra).cuda(); x_out_d = torch.from_numpy(x_out0).cuda()
        n_d = torch.full((cfg.B,), -7, dtype=torch.int32, device="cuda")
        prob.ctx.commit(cfg.B, torch.from_numpy(x_tok).cuda(), ra_d, torch.from_numpy(masked).cuda(), x_out_d, n_d)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(x_out_d.cpu().numpy(), want_x)
        np.testing.assert_array_equal(ra_d.cpu().numpy(), want_ra)
        np.testing.assert_array_equal(n_d.cpu().numpy(), want_n)
        assert prob.ctx.commit(0, ra_d, ra_d, ra_d, x_out_d, n_d) == 0                 # empty batch
        assert prob.ctx.commit(1, None, ra_d, ra_d, x_out_d, n_d, check=False) == -1
    finally:
        prob.close()


def _decode_setup():
    cfg = mi.straddling(mi.config(0, d=256, V=4100, B=10, L=8, K=2))
    return cfg, Problem(cfg)


@pytest.mark.parametrize("rcfg", [
    mrp.RevealCfg(tau=1.0, r_min=1),                                        # Algorithm 2, static r = 1
    mrp.RevealCfg(tau=0.6, tau_remask=0.6, head_reveal=0),                  # Algorithm 4, same threshold
    mrp.RevealCfg(tau=0.5, tau_remask=0.4, max_accept=1, remask_mode=1),    # cap on, committed-token remask
], ids=["static", "alg4", "cap-committed"])
def test_decode_block_teacher_forced(rcfg):
    """Every denoising step of a block decode, the GPU fed the oracle's state of the step before
    (so that an exempted decision cannot hide later errors), including mrp_commit."""
    cfg, prob = _decode_setup()
    try:
        B, L, K, M = cfg.B, cfg.L, cfg.K, cfg.M
        step_cfg = mrp.RevealCfg(**{**rcfg.__dict__, "fresh_block": 0})
        masked = np.ones(M, np.uint8); ra = np.full(M, -1, np.int8); x_out = np.full(M, -1, np.int32)
        steps = 0
        while masked.any():
            assert steps < L
            z0 = mi.logits0(cfg, step=steps); h = mi.hidden(cfg, step=steps)
            io = mrp.StepIO(B, L, K)
            io.masked.copy_(torch.from_numpy(masked)); io.revealed_at.copy_(torch.from_numpy(ra))
            z_d = torch.from_numpy(z0).cuda()
            io, hrun_d = gpu_chain(prob, B, K, z_d, h, step_cfg, io=io)
            g = io_to_host(io)
            o = oracle_chain(prob, z0, mi.bf16_bits_to_f64(h), step_cfg, K, masked=masked, revealed_at=ra)
            stats = compare_chain(g, z_d.cpu().numpy(), hrun_d.cpu().numpy(), o, list(range(B)), L, K, step_cfg)
            # commit on both sides from the ORACLE's end-of-step state
            want_x, want_ra, want_n = orc.commit(B, L, o.out.x_tok, o.out.revealed_at, o.out.masked, x_out)
            ra_d = torch.from_numpy(o.out.revealed_at).cuda(); x_out_d = torch.from_numpy(x_out).cuda()
            n_d = torch.empty((B,), dtype=torch.int32, device="cuda")
            prob.ctx.commit(B, torch.from_numpy(o.out.x_tok).cuda(), ra_d, torch.from_numpy(o.out.masked).cuda(),
                            x_out_d, n_d)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(x_out_d.cpu().numpy(), want_x)
            np.testing.assert_array_equal(ra_d.cpu().numpy(), want_ra)
            np.testing.assert_array_equal(n_d.cpu().numpy(), want_n)
            masked, ra, x_out = o.out.masked, want_ra, want_x
            steps += 1
            print(f"\n[decode step {steps}] {stats} masked left {int(masked.sum())}")
        assert np.all(x_out >= 0)
    finally:
        prob.close()


def test_decode_block_free_running():
    """The binding's decode loop (chain step + commit per denoising step, device-resident state)
    against the oracle's loop: a decoded block may differ only if the oracle's run of that sequence
    contains a decision inside the exemption bands, and at least four in five must be identical."""
    cfg, prob = _decode_setup()
    try:
        B, L, K = cfg.B, cfg.L, cfg.K
        rcfg = mrp.RevealCfg(tau=0.6, tau_remask=0.6, head_reveal=0)

        def backbone_gpu(step, x_out, masked):
            return torch.from_numpy(mi.logits0(cfg, step=step)).cuda(), dev_bits(mi.hidden(cfg, step=step))

        def backbone_cpu(step, x_out, masked):
            return mi.logits0(cfg, step=step).astype(np.float64), mi.bf16_bits_to_f64(mi.hidden(cfg, step=step))

        x_g, steps_g, io = prob.ctx.decode_block(B, K, backbone_gpu, prob.E_d, prob.Wp_d, prob.heads_d, rcfg)
        oc = orc.make_cfg(cfg.d, cfg.V, B, L, K, tau=rcfg.tau, tau_remask=rcfg.tau_remask, head_reveal=0)
        x_o, steps_o, hist = orc.decode_block(oc, prob.E, prob.W, prob.heads, backbone_cpu)
        x_g = x_g.cpu().numpy()
        fragile = np.zeros(B, bool)
        for out in hist:
            for b in range(B):
                rows = slice(b * L, (b + 1) * L)
                for k in range(K + 1):
                    c = out.conf[k, rows]
                    near = lambda t: bool(np.any(np.abs(c - t) < CONF_EXEMPT * t))
                    top2 = np.sort(c)[::-1][:2]
                    if near(rcfg.tau) or near(rcfg.tau_remask) or (len(top2) == 2 and top2[0] - top2[1] < CONF_EXEMPT * top2[0]) \
                            or out.gap[k, rows].min() < GAP_EXEMPT:
                        fragile[b] = True
        same = np.array([np.array_equal(x_g[b * L:(b + 1) * L], x_o[b * L:(b + 1) * L]) for b in range(B)])
        assert np.all(same | fragile), f"decoded blocks differ without a decision inside the exemption bands: {same}"
        assert same.sum() >= (4 * B) // 5
        if same.all():
            assert steps_g == steps_o
        assert np.all(x_g >= 0)
        print(f"\n[free-running decode] steps gpu {steps_g} oracle {steps_o}, identical blocks {int(same.sum())}/{B}")
    finally:
        prob.close()
