"""The chain step allocates nothing and enqueues only kernels on the caller's stream, so a caller can
record it into a HIP graph.  The graph is replayed several times, with the program's own eager work
and synchronisations between the replays, and every replay is compared bit for bit with the eager
result (the kernels are deterministic)."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import paper_2605_18817_amd as mrp
from harness import Problem, dev_bits, io_to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid,over", [(0, dict(B=4, L=4, K=2)), (0, dict(d=512, V=4096, B=48, L=16, K=1))])
def test_chain_step_in_a_hip_graph_replays_bit_exact(cid, over):
    cfg = mi.straddling(mi.config(cid, **over))
    prob = Problem(cfg)
    try:
        z0_d = torch.from_numpy(mi.logits0(cfg)).cuda()
        h_d = dev_bits(mi.hidden(cfg))
        rcfg = mrp.RevealCfg(tau=0.9, tau_remask=0.5)

        def fresh():
            return z0_d.clone(), torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")

        # eager reference
        z_e, hr_e = fresh()
        io_e = mrp.StepIO(cfg.B, cfg.L, cfg.K)
        prob.ctx.chain_step(cfg.B, cfg.K, h_d, hr_e, prob.E_d, prob.Wp_d, prob.heads_d, z_e, rcfg, io_e)
        torch.cuda.synchronize()
        ref = io_to_host(io_e)

        # record into a graph on a side stream (default priority), static buffers
        z_g, hr_g = fresh()
        io_g = mrp.StepIO(cfg.B, cfg.L, cfg.K)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            prob.ctx.chain_step(cfg.B, cfg.K, h_d, hr_g, prob.E_d, prob.Wp_d, prob.heads_d, z_g, rcfg, io_g)
        torch.cuda.synchronize()

        for rep in range(3):
            z_g.copy_(z0_d)
            hr_g.zero_()
            # unrelated eager work between the replays
            junk = (z0_d[:8] * float(rep + 1)).sum().item()
            assert np.isfinite(junk)
            graph.replay()
            torch.cuda.synchronize()
            got = io_to_host(io_g)
            for name in ("tok", "conf", "lse", "masked", "revealed_at", "cond_tok", "draft_pos", "draft_tok", "remasked",
                         "x_tok"):
                np.testing.assert_array_equal(getattr(got, name), getattr(ref, name), err_msg=f"replay {rep}: {name}")
            assert torch.equal(z_g, z_e) and torch.equal(hr_g, hr_e), f"replay {rep}"
    finally:
        prob.close()
