"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
the GPU runs the whole batch, the oracle a seeded sample of whole sequences (sequences
are independent) that takes one sequence from EVERY 256-row tile of the batch, so that
every row tile of the tiled GEMM kernels (and every XCD super-block of its tile order)
is compared.  Each configuration is compared twice:

* free-running — one call for the whole chain, as the benchmark launches it — against the
  oracle's run with the bf16 LM-head operand (decisions bit-exact, no exemption allowed on
  these seeded inputs) and against the plain-definition run (logits within the stated
  tolerance);
* teacher-forced — one call per head, the sampled sequences fed the oracle's state of the
  head before — so that a difference in one head cannot hide the next.

The verify stage is compared exactly on the full batch (the oracle's argmax over the
drafted rows is cheap)."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp
from harness import Problem, compare_chain, dev_bits, gpu_chain, head_view, io_to_host, oracle_chain

pytestmark = pytest.mark.gpu

TILE_ROWS = 256


def _sample_rows(cfg, seqs):
    return np.concatenate([np.arange(b * cfg.L, (b + 1) * cfg.L) for b in seqs])


def one_sequence_per_row_tile(cfg, salt=0):
    """One sequence from every 256-row tile of the batch (seeded position inside the tile; the first
    tile takes its first sequence and the last tile its last, so both ends of the batch are in)."""
    per_tile = max(1, TILE_ROWS // cfg.L)
    n_tiles = (cfg.B + per_tile - 1) // per_tile
    rng = np.random.default_rng(1000 * cfg.cid + salt)
    seqs = []
    for t in range(n_tiles):
        lo, hi = t * per_tile, min(cfg.B, (t + 1) * per_tile)
        b = lo if t == 0 else (hi - 1 if t == n_tiles - 1 else int(rng.integers(lo, hi)))
        seqs.append(b)
    return seqs


def _assert_no_exemption(stats, what):
    assert stats["tok_exempt"] == 0 and stats["decision_exempt"] == 0 and stats["diverged"] == 0, \
        f"{what}: an exemption was used on inputs that need none: {stats}"


def _run_full(cfg, rcfg, seqs, steps=1):
    """Free-running chain steps on the whole batch against the oracle on `seqs`.  Every step must be
    compared (no exemption on these inputs), also against the plain definition."""
    prob = Problem(cfg)
    try:
        z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
        rows = _sample_rows(cfg, seqs)
        rows_d = torch.from_numpy(rows).cuda()
        z_o = z_d[rows_d].cpu().numpy().astype(np.float64)
        io = mrp.StepIO(cfg.B, cfg.L, cfg.K)
        o_state = dict(masked=None, revealed_at=None, cond_tok=None, protect_pos=None, x_tok=None)
        x_out_d = torch.full((cfg.M,), -1, dtype=torch.int32, device="cuda")
        n_masked_d = torch.empty((cfg.B,), dtype=torch.int32, device="cuda")
        x_out_o = np.full(len(rows), -1, np.int32)
        all_stats = []
        g = None
        for step in range(steps):
            h = mi.hidden(cfg, step=step)
            r = mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=1 if step == 0 else 0)
            io, hrun_d = gpu_chain(prob, cfg.B, cfg.K, z_d, h, r, io=io)
            g = io_to_host(io)
            hs = mi.bf16_bits_to_f64(h[rows])
            o = oracle_chain(prob, z_o, hs, r, cfg.K, **o_state)
            # The stated logit tolerance is that of one chain step: the plain definition is applied to the
            # same step inputs (on a resident logit state the roundings of the bf16 operand of all earlier
            # steps' heads would otherwise add up, as the square root of their number, in both columns).
            plain = oracle_chain(prob, z_o, hs, r, cfg.K, round_y=0, **o_state)
            zg = z_d[rows_d].cpu().numpy()
            stats = compare_chain(g, zg, hrun_d[rows_d].cpu().numpy(), o, seqs, cfg.L, cfg.K, r, plain=plain)
            _assert_no_exemption(stats, f"config {cfg.cid} step {step}")
            all_stats.append(stats)
            print(f"\n[config {cfg.cid} step {step}: rows={cfg.M} sample={len(rows)} seqs={list(seqs)}] {stats}", flush=True)
            if step + 1 < steps:
                # between denoising steps the caller commits what stayed revealed; z stays resident
                prob.ctx.commit(cfg.B, io.x_tok, io.revealed_at, io.masked, x_out_d, n_masked_d)
                x_out_o, ra, n_o = orc.commit(len(seqs), cfg.L, o.out.x_tok, o.out.revealed_at, o.out.masked, x_out_o)
                np.testing.assert_array_equal(x_out_d.cpu().numpy()[rows], x_out_o)
                np.testing.assert_array_equal(n_masked_d.cpu().numpy()[list(seqs)], n_o)
                o_state = dict(masked=o.out.masked, revealed_at=ra, cond_tok=o.out.cond_tok,
                               protect_pos=o.out.protect_pos, x_tok=o.out.x_tok)
                z_o = o.out.z
        return prob, io, g, all_stats
    except Exception:
        prob.close()
        raise


def _run_teacher_forced(prob, cfg, rcfg, seqs):
    """State 0, then one call per head; before head k the sampled sequences' state (logits, running
    hidden state, masks, conditioning token) is overwritten with the oracle's state k - 1."""
    rows = _sample_rows(cfg, seqs)
    rows_d = torch.from_numpy(rows).cuda()
    seqs_d = torch.from_numpy(np.asarray(seqs)).cuda()
    z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
    h = mi.hidden(cfg)
    full = oracle_chain(prob, z_d[rows_d].cpu().numpy().astype(np.float64), mi.bf16_bits_to_f64(h[rows]),
                        mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=1), cfg.K)
    # state 0 alone
    io0 = mrp.StepIO(cfg.B, cfg.L, 0)
    r0 = mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=1)
    hrun_d = torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")
    h_d = dev_bits(h)
    prob.ctx.chain_step(cfg.B, 0, h_d, hrun_d, prob.E_d, prob.Wp_d, [], z_d, r0, io0)
    torch.cuda.synchronize()
    g = io_to_host(io0)
    io = mrp.StepIO(cfg.B, cfg.L, 1)      # the per-head calls: slot 0 untouched, slot 1 = the head's state
    for name in ("masked", "revealed_at", "cond_tok", "protect_pos", "x_tok"):
        getattr(io, name).copy_(getattr(io0, name))
    o = full.out
    for jj, b in enumerate(seqs):
        rg, ro = slice(b * cfg.L, (b + 1) * cfg.L), slice(jj * cfg.L, (jj + 1) * cfg.L)
        np.testing.assert_array_equal(g.tok[0, rg], o.tok[0, ro])
        np.testing.assert_allclose(g.lse[0, rg], o.lse[0, ro], atol=2e-5)
        np.testing.assert_allclose(g.conf[0, rg], o.conf[0, ro], rtol=1e-4)
        assert g.draft_pos[b, 0] == o.draft_pos[jj, 0] and g.draft_tok[b, 0] == o.draft_tok[jj, 0]
        s0 = full.snaps[0]
        np.testing.assert_array_equal(g.masked[rg], s0.masked[ro])
        np.testing.assert_array_equal(g.revealed_at[rg], s0.revealed_at[ro])
        assert g.cond_tok[b] == s0.cond_tok[jj] and g.protect_pos[b] == s0.protect_pos[jj]
    out = []
    for k in range(1, cfg.K + 1):
        s = full.snaps[k - 1]
        put = lambda dst, src, idx: dst.index_copy_(0, idx, torch.from_numpy(np.ascontiguousarray(src)).cuda())
        put(z_d, s.z.astype(np.float32), rows_d)
        put(io.masked, s.masked, rows_d); put(io.revealed_at, s.revealed_at, rows_d); put(io.x_tok, s.x_tok, rows_d)
        put(io.cond_tok, s.cond_tok, seqs_d); put(io.protect_pos, s.protect_pos, seqs_d)
        if k > 1:
            put(hrun_d, s.hrun.astype(np.float32), rows_d)
        r1 = mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=0, state_offset=k - 1, run_state0=0)
        prob.ctx.chain_step(cfg.B, 1, h_d if k == 1 else None, hrun_d, prob.E_d, prob.Wp_d, prob.heads_d[k - 1:k], z_d,
                            r1, io)
        torch.cuda.synchronize()
        g = io_to_host(io)
        stats = compare_chain(g, z_d[rows_d].cpu().numpy(), hrun_d[rows_d].cpu().numpy(), head_view(full, k), seqs,
                              cfg.L, 1, r1)
        _assert_no_exemption(stats, f"config {cfg.cid} teacher-forced head {k}")
        print(f"\n[config {cfg.cid} teacher-forced head {k}: sample={len(rows)}] {stats}", flush=True)
        out.append(stats)
    return out


@pytest.mark.timeout(600)
def test_config1_full_batch():
    cfg = mi.config(1)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=[0, 7, 19, 31])
    try:
        _run_teacher_forced(prob, cfg, mrp.RevealCfg(tau=cfg.tau), seqs=[3, 12, 28])
    finally:
        prob.close()


@pytest.mark.timeout(900)
def test_config2_full_batch():
    cfg = mi.config(2)
    seqs = one_sequence_per_row_tile(cfg)
    assert len(seqs) == 4
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=seqs)
    try:
        _run_teacher_forced(prob, cfg, mrp.RevealCfg(tau=cfg.tau), seqs=one_sequence_per_row_tile(cfg, salt=1))
    finally:
        prob.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("B", [16, 24, 32])
def test_config2_middle_row_range(B):
    """Between config 1's and config 2's row counts at config 2's width (d = 4096): the LM head runs on the
    persistent kernel's 256-row form, in one launch at 256 rows (B = 16) and in two at 384 and 512 rows
    (B = 24, 32); the head body on the small-row GEMMs with 64-feature tiles.  One sequence from every
    256-row group."""
    cfg = mi.config(2, B=B)
    assert 128 < cfg.M < 768
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=one_sequence_per_row_tile(cfg))
    try:
        _run_teacher_forced(prob, cfg, mrp.RevealCfg(tau=cfg.tau), seqs=one_sequence_per_row_tile(cfg, salt=1))
    finally:
        prob.close()


@pytest.mark.timeout(1100)
def test_config3_draft_then_verify():
    cfg = mi.config(3)
    seqs = one_sequence_per_row_tile(cfg)
    assert len(seqs) == 8
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau), seqs=seqs)
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
        del v_d, verify
        _run_teacher_forced(prob, cfg, mrp.RevealCfg(tau=cfg.tau), seqs=one_sequence_per_row_tile(cfg, salt=1))
    finally:
        prob.close()


@pytest.mark.timeout(1100)
def test_config4_every_row_tile():
    """Step 0 of the largest configuration: one sequence from each of its 16 row tiles, free-running
    (the benchmark's launch) and teacher-forced per head."""
    cfg = mi.config(4)
    seqs = one_sequence_per_row_tile(cfg)
    assert len(seqs) == 16
    rcfg = mrp.RevealCfg(tau=cfg.tau, tau_remask=cfg.tau_remask)
    prob, io, g, stats = _run_full(cfg, rcfg, seqs=seqs)
    try:
        _run_teacher_forced(prob, cfg, rcfg, seqs=one_sequence_per_row_tile(cfg, salt=1))
    finally:
        prob.close()


@pytest.mark.timeout(1100)
def test_config4_resident_logits_remask():
    """The 8 consecutive steps on the resident logit state: every step is compared."""
    cfg = mi.config(4)
    prob, io, g, stats = _run_full(cfg, mrp.RevealCfg(tau=cfg.tau, tau_remask=cfg.tau_remask), seqs=[77, 201],
                                   steps=cfg.steps)
    prob.close()
    assert len(stats) == cfg.steps
    assert all(s["diverged"] == 0 and s["seqs"] == 2 for s in stats)
