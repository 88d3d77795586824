"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element at sizes the oracle finishes in seconds (several tiles, ragged tails,
both activation-tile variants, the scalar vocabulary path)."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import paper_2605_18817_amd as mrp
from harness import (Problem, compare_chain, dev_bits, gpu_chain, io_to_host, oracle_chain)

pytestmark = pytest.mark.gpu


def _free_run(cfg, rcfg, gamma="ones", share_heads=False, seqs=None, max_exempt=0):
    prob = Problem(cfg, gamma=gamma, share_heads=share_heads)
    try:
        z0 = mi.logits0(cfg)
        h = mi.hidden(cfg)
        z_d = torch.from_numpy(z0).cuda()
        io, hrun_d = gpu_chain(prob, cfg.B, cfg.K, z_d, h, rcfg)
        g = io_to_host(io)
        seqs = list(range(cfg.B)) if seqs is None else seqs
        rows = np.concatenate([np.arange(b * cfg.L, (b + 1) * cfg.L) for b in seqs])
        o = oracle_chain(prob, z0[rows], mi.bf16_bits_to_f64(h[rows]), rcfg, cfg.K)
        plain = oracle_chain(prob, z0[rows], mi.bf16_bits_to_f64(h[rows]), rcfg, cfg.K, round_y=0)
        stats = compare_chain(g, z_d.cpu().numpy()[rows], hrun_d.cpu().numpy()[rows], o, seqs, cfg.L, cfg.K,
                              rcfg, plain=plain, max_exempt=max_exempt)
        print(f"\n[{cfg.name or cfg.cid} d={cfg.d} V={cfg.V} M={cfg.M}] {stats}")
        return prob, g, o, stats
    except Exception:
        prob.close()
        raise


def test_pack_weight_layout():
    rng = np.random.default_rng(3)
    for rows, cols in ((32, 16), (70, 48), (129, 256)):
        w = rng.integers(0, 65536, (rows, cols), dtype=np.uint16)
        out = mrp.pack_weight(dev_bits(w)).cpu().numpy().view(np.uint16)
        rpad = (rows + 31) // 32 * 32
        assert out.size == rpad * cols
        wp = np.zeros((rpad, cols), np.uint16); wp[:rows] = w
        # [row block][col block][lane][8] with lane = row % 32 + 32 * ((col % 16) // 8)
        ref = wp.reshape(rpad // 32, 32, cols // 16, 2, 8).transpose(0, 2, 3, 1, 4).reshape(-1)
        np.testing.assert_array_equal(out, ref)


def test_pack_body_weight_converts_to_fp16():
    """Head-body weights: same block layout, every bf16 value as the nearest fp16 (exact in fp16's
    normal range, subnormal below 6.1e-5)."""
    rng = np.random.default_rng(4)
    rows, cols = 70, 48
    vals = rng.normal(0, 0.02, (rows, cols)).astype(np.float32)
    vals[0, :8] = [0.0, 1.0, -2.5, 3e-5, -1e-6, 6.1e-5, 1000.0, -0.0]
    w = mi.f32_to_bf16_bits(vals)
    out = mrp.pack_weight(dev_bits(w), body=True).cpu().numpy().view(np.uint16)
    rpad = (rows + 31) // 32 * 32
    want = np.zeros((rpad, cols), np.uint16)
    want[:rows] = mi.bf16_bits_to_f32(w).astype(np.float16).view(np.uint16)
    ref = want.reshape(rpad // 32, 32, cols // 16, 2, 8).transpose(0, 2, 3, 1, 4).reshape(-1)
    np.testing.assert_array_equal(out, ref)


def test_config0_tiny():
    cfg = mi.config(0)
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=cfg.tau))
    prob.close()
    assert stats["diverged"] == 0


def test_ragged_rows_and_vocab_with_remask():
    # M = 35 (ragged 32-row tile), V = 4100 (ragged 32- and 128-wide vocabulary tiles), d = 384
    cfg = mi.straddling(mi.config(0, d=384, V=4100, B=5, L=7))
    rcfg = mrp.RevealCfg(tau=0.5, tau_remask=0.3)
    prob, g, o, stats = _free_run(cfg, rcfg)
    prob.close()
    assert (o.out.remasked.sum() > 0) and ((o.out.revealed_at == 0).sum() > cfg.B)


def test_scalar_vocab_path_and_max_accept():
    cfg = mi.straddling(mi.config(0, d=128, V=4099, B=3, L=16))
    rcfg = mrp.RevealCfg(tau=0.3, max_accept=1)
    prob, g, o, stats = _free_run(cfg, rcfg)
    prob.close()


@pytest.mark.timeout(600)
def test_maximum_hidden_size_and_block_length():
    """The largest hidden size (d = 8192) and block length (L = 64) the library accepts."""
    cfg = mi.straddling(mi.config(0, d=8192, V=1024, B=2, L=64, K=1))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.9, tau_remask=0.5, max_accept=1))
    prob.close()


def test_block_of_one_position():
    """L = 1: every sequence is a single row; the forced reveal takes it at state 0, later states have
    nothing left to reveal (draft (-1, -1)) and keep the conditioning token."""
    cfg = mi.straddling(mi.config(0, B=9, L=1, K=2))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.9))
    prob.close()
    assert np.all(g.draft_pos[:, 0] == 0) and np.all(g.draft_pos[:, 1:] == -1)
    assert np.all(g.masked == 0)


@pytest.mark.parametrize("B,L", [(12, 64), (40, 7), (112, 7)])
def test_tile_major_partials_with_odd_and_long_blocks(B, L):
    """The GEMM kernels that own whole row tiles write their vocabulary partials tile-major; the merge
    then runs threads over a sequence's rows (block lengths that are not a power of two, and the longest)."""
    cfg = mi.straddling(mi.config(0, d=256, V=4096 + 36, B=B, L=L, K=1))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.9, tau_remask=0.5), seqs=list(range(0, B, max(1, B // 6))))
    prob.close()


def test_many_rows_wide_tile_static_top2():
    # M = 336 > 128 selects the 256-row activation tile (two row groups, the second ragged)
    cfg = mi.straddling(mi.config(0, d=256, V=2048 + 64, B=21, L=16))
    rcfg = mrp.RevealCfg(tau=1.0, r_min=2)           # static decoding: the two most confident per state
    prob, g, o, stats = _free_run(cfg, rcfg)
    prob.close()
    assert np.all((g.masked.reshape(cfg.B, cfg.L) == 0).sum(1) == 2 * (cfg.K + 1))


def test_tiled_path_ragged_tiles():
    # M = 800 >= 768 selects the 256 x 256 tiled kernels: 4 row tiles (the last with 32 rows),
    # V = 1000 -> 4 vocabulary tiles (the last with 232 entries, 8 of them in a partial 32-block)
    cfg = mi.straddling(mi.config(0, d=128, V=1000, B=50, L=16))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.5, tau_remask=0.3))
    prob.close()
    # same row count with a vocabulary that is not a multiple of 4: tiled head GEMMs, scalar LM-head path
    cfg = mi.straddling(mi.config(0, d=256, V=1030, B=48, L=16, K=2))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.5))
    prob.close()


def test_weight_shared_heads_and_alg4_mode():
    # one module applied K times; reveal only at state 0, remask with the same tau (Algorithm 4)
    cfg = mi.straddling(mi.config(0, d=256, V=4096, B=8, L=8, K=2))
    rcfg = mrp.RevealCfg(tau=0.6, tau_remask=0.6, head_reveal=0)
    prob, g, o, stats = _free_run(cfg, rcfg, share_heads=True)
    prob.close()
    assert np.all(g.draft_pos[:, 1:] == -1)


def test_gamma_variants():
    cfg = mi.config(0, B=4, L=4)
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=cfg.tau), gamma="normal")
    prob.close()


def test_zero_residual_bit_exact_and_deterministic():
    cfg = mi.config(0, B=6, L=4, V=4100)
    prob = Problem(cfg, gamma="zeros")
    try:
        z0 = mi.logits0(cfg); h = mi.hidden(cfg)
        z_d = torch.from_numpy(z0).cuda()
        io, _ = gpu_chain(prob, cfg.B, cfg.K, z_d, h, mrp.RevealCfg(tau=cfg.tau))
        g = io_to_host(io)
        np.testing.assert_array_equal(z_d.cpu().numpy(), z0)              # z + 0 == z, bit for bit
        for k in range(1, cfg.K + 1):
            np.testing.assert_array_equal(g.tok[k], g.tok[0])
            np.testing.assert_allclose(g.conf[k], g.conf[0], rtol=1e-5)
    finally:
        prob.close()
    # same inputs twice -> bit-identical outputs (fixed-order split-vocabulary merge)
    cfg = mi.straddling(mi.config(0, d=256, V=8200, B=9, L=16))
    prob = Problem(cfg)
    try:
        z0 = mi.logits0(cfg); h = mi.hidden(cfg)
        outs = []
        for _ in range(2):
            z_d = torch.from_numpy(z0).cuda()
            io, hr = gpu_chain(prob, cfg.B, cfg.K, z_d, h, mrp.RevealCfg(tau=0.5, tau_remask=0.3))
            g = io_to_host(io)
            outs.append((z_d.cpu().numpy(), hr.cpu().numpy(), g))
        np.testing.assert_array_equal(outs[0][0], outs[1][0])
        np.testing.assert_array_equal(outs[0][1], outs[1][1])
        for f in ("tok", "conf", "lse", "masked", "revealed_at", "draft_pos", "draft_tok", "remasked", "cond_tok"):
            np.testing.assert_array_equal(getattr(outs[0][2], f), getattr(outs[1][2], f))
    finally:
        prob.close()


def test_teacher_forced_heads_and_resume():
    """Each head on its own, fed the oracle's previous state (so a flipped decision in one
    head cannot hide errors in the next), and a resumed call equals the tail of a full run."""
    cfg = mi.straddling(mi.config(0, d=256, V=4096, B=6, L=8))
    rcfg = mrp.RevealCfg(tau=0.5, tau_remask=0.3)
    prob = Problem(cfg)
    try:
        z0 = mi.logits0(cfg); h = mi.hidden(cfg)
        seqs = list(range(cfg.B))
        full = oracle_chain(prob, z0, mi.bf16_bits_to_f64(h), rcfg, cfg.K)
        for k in range(1, cfg.K + 1):
            s = full.snaps[k - 1]
            io = mrp.StepIO(cfg.B, cfg.L, 1)
            io.masked.copy_(torch.from_numpy(s.masked)); io.revealed_at.copy_(torch.from_numpy(s.revealed_at))
            io.cond_tok.copy_(torch.from_numpy(s.cond_tok)); io.protect_pos.copy_(torch.from_numpy(s.protect_pos))
            io.x_tok.copy_(torch.from_numpy(s.x_tok))
            z_d = torch.from_numpy(s.z.astype(np.float32)).cuda()
            hrun_d = torch.from_numpy(s.hrun.astype(np.float32)).cuda()
            r1 = mrp.RevealCfg(tau=rcfg.tau, tau_remask=rcfg.tau_remask, fresh_block=0, state_offset=k - 1,
                               run_state0=0)
            io, hrun_d = gpu_chain(prob, cfg.B, 1, z_d, None, r1, io=io, hrun_d=hrun_d, heads=prob.heads_d[k - 1:k])
            g = io_to_host(io)
            o1 = oracle_chain(prob, s.z, s.hrun, r1, 1, masked=s.masked, revealed_at=s.revealed_at,
                              cond_tok=s.cond_tok, protect_pos=s.protect_pos, heads=prob.heads[k - 1:k], x_tok=s.x_tok)
            stats = compare_chain(g, z_d.cpu().numpy(), hrun_d.cpu().numpy(), o1, seqs, cfg.L, 1, r1)
            print(f"\n[teacher-forced head {k}] {stats}")
            np.testing.assert_array_equal(o1.out.tok[1], full.out.tok[k])
    finally:
        prob.close()


def test_sdar_width_vocab_few_rows():
    # real vocabulary and hidden size of the 1.7B-shaped configuration, two sequences
    cfg = mi.config(1, B=2, spike_frac=0.5)
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=cfg.tau))
    prob.close()


def test_empty_batch_and_errors():
    cfg = mi.config(0)
    prob = Problem(cfg)
    try:
        ctx = prob.ctx
        io = mrp.StepIO(1, cfg.L, cfg.K)
        z_d = torch.from_numpy(mi.logits0(cfg)).cuda()
        hrun = torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")
        h_d = dev_bits(mi.hidden(cfg))
        rc = mrp.RevealCfg()
        args = (h_d, hrun, prob.E_d, prob.Wp_d, prob.heads_d, z_d, rc, io)
        assert ctx.chain_step(0, cfg.K, *args) == 0                       # empty batch: nothing to do
        assert ctx.chain_step(2, cfg.K, *args, check=False) == -4          # rows beyond the workspace
        assert "max_rows" in ctx.last_error()
        assert ctx.chain_step(1, 17, *args, check=False) == -2             # too many heads
        assert ctx.chain_step(1, cfg.K, h_d, None, *args[2:], check=False) == -1
        zz = torch.zeros(cfg.M * cfg.V + 4, dtype=torch.float32, device="cuda")[1:]  # misaligned view
        with pytest.raises(mrp.MrpError):
            ctx.chain_step(1, cfg.K, h_d, hrun, prob.E_d, prob.Wp_d, prob.heads_d, zz[:cfg.M * cfg.V], rc, io)
        with pytest.raises(mrp.MrpError):
            mrp.MrpContext(100, 4096, 4, 4)                                # d not a multiple of 128
        with pytest.raises(mrp.MrpError):
            mrp.pack_weight(torch.zeros((4, 10), dtype=torch.int16, device="cuda"))
        torch.cuda.synchronize()
    finally:
        prob.close()


@pytest.mark.parametrize("d,B,L,K", [
    (256, 129, 1, 2),    # one row past the 128-row LM-head form: its 256-row form, small-row head GEMMs (5 row tiles)
    (256, 16, 16, 2),    # 256 rows: the 256-row form filled exactly
    (256, 257, 1, 1),    # two LM-head launches (256 + 1 rows), 9 row tiles: 64-feature tiles
    (256, 32, 16, 1),    # 512 rows: two full LM-head launches
    (256, 513, 1, 1),    # one row past: the tile kernel for the LM head, small-row kernels for the body
    (256, 59, 13, 1),    # 767 rows, the last row count of the small-row head body at this width
    (4096, 25, 8, 2),    # wide model, 200 rows: 64-feature tiles, 7 row tiles, the last ragged
    (4096, 37, 16, 1),   # wide model, 592 rows: tile kernel with k split for the head body (48 tiles x 4 parts)
])
def test_row_counts_where_the_kernels_change(d, B, L, K):
    """Row counts on both sides of every switch between kernel families (LM head: 128 / 256 / 512 rows;
    head body: 768 rows, 512 for d > 2048; 32- against 64-feature tiles), each against the oracle."""
    V = 1028 if d > 256 else 4096 + 36
    cfg = mi.straddling(mi.config(0, d=d, V=V, B=B, L=L, K=K))
    prob, g, o, stats = _free_run(cfg, mrp.RevealCfg(tau=0.9, tau_remask=0.5), seqs=list(range(0, B, max(1, B // 5))))
    prob.close()
