"""GPU parity of the chain with the transformer head body (Section 3.2; D layers between the fuse
projection and the shared LM head) against the fp64 oracle, free-running over all K heads, under
the same parity rule as the MLP body (tests/harness.py).  Weights, prefix caches and prefix lengths
come from the seeded generators; prefix lengths include 0 and the cache capacity."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp
from harness import compare_chain, dev_bits, io_to_host, oracle_chain

pytestmark = pytest.mark.gpu


class TfProblem:
    def __init__(self, cfg, td, gain="normal", share=False):
        self.cfg, self.td = cfg, td
        self.W, self.E = mi.lm_head(cfg), mi.embedding(cfg)
        nh = 1 if share else cfg.K
        self.heads = [mi.head_weights(cfg, k, "normal" if gain == "normal" else "ones") for k in range(nh)]
        if gain == "normal":   # gains around 1 rather than around 0
            self.heads = [(w1, w2, mi.f32_to_bf16_bits((1.0 + 5 * mi.bf16_bits_to_f32(g)).astype(np.float32)))
                          for (w1, w2, g) in self.heads]
        self.layers = [[mi.tf_layer(cfg, td, k, l, gain=gain) for l in range(td.D)] for k in range(nh)]
        if share:
            self.heads = self.heads * cfg.K
            self.layers = self.layers * cfg.K
        self.plen = mi.prefix_lens(cfg, td)
        self.ctx = mrp.MrpContext(cfg.d, cfg.V, cfg.M, cfg.L)
        self.ctx.tbody_create(td.D, td.n_heads, td.n_kv_heads, td.d_ff, td.P_max, td.rope_theta)
        self.E_d = dev_bits(self.E)
        self.Wp_d = mrp.pack_weight(dev_bits(self.W))
        self.keep = []
        dev_heads, dev_layers = {}, {}
        self.heads_d, self.layers_d = [], []
        for k in range(cfg.K):
            key = id(self.heads[k][0])
            if key not in dev_heads:
                w1, _, g = self.heads[k]
                dev_heads[key] = mrp.Head(mrp.pack_weight(dev_bits(w1), body=True), None, dev_bits(g))
                ls = []
                for lay in self.layers[k]:
                    kc = dev_bits(lay["kc"]) if td.P_max > 0 else None
                    vc = dev_bits(lay["vc"]) if td.P_max > 0 else None
                    pk = lambda a: mrp.pack_weight(dev_bits(a), body=True)
                    ls.append(mrp.TLayer(pk(lay["Wqkv"]), pk(lay["Wo"]), pk(lay["Wgu"]), pk(lay["Wdown"]),
                                         dev_bits(lay["g1"]), dev_bits(lay["g2"]), kc, vc))
                dev_layers[key] = ls
            self.heads_d.append(dev_heads[key])
            self.layers_d += dev_layers[key]
        self.plen_d = torch.from_numpy(self.plen).cuda()
        torch.cuda.synchronize()

    def close(self):
        self.ctx.close()


def _run(cfg, td, rcfg, seqs=None, gain="normal", share=False, max_exempt=0):
    prob = TfProblem(cfg, td, gain=gain, share=share)
    try:
        z0 = mi.logits0(cfg)
        h = mi.hidden(cfg)
        z_d = torch.from_numpy(z0).cuda()
        hrun_d = torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")
        io = mrp.StepIO(cfg.B, cfg.L, cfg.K)
        prob.ctx.chain_step_tf(cfg.B, cfg.K, dev_bits(h), hrun_d, prob.E_d, prob.Wp_d, prob.heads_d, prob.layers_d,
                               prob.plen_d, z_d, rcfg, io)
        torch.cuda.synchronize()
        g = io_to_host(io)
        seqs = list(range(cfg.B)) if seqs is None else list(seqs)
        rows = np.concatenate([np.arange(b * cfg.L, (b + 1) * cfg.L) for b in seqs])
        tc = orc.make_tcfg(td.D, td.n_heads, td.n_kv_heads, td.head_dim, td.d_ff, td.P_max, td.rope_theta)
        sub = [[dict(lay, kc=np.ascontiguousarray(lay["kc"][seqs]), vc=np.ascontiguousarray(lay["vc"][seqs]))
                for lay in ls] for ls in prob.layers]
        tb = orc.TBody(tc, sub, prob.plen[seqs])
        heads = [(w1, None, g_) for (w1, _, g_) in prob.heads]
        o = oracle_chain(prob, z0[rows], mi.bf16_bits_to_f64(h[rows]), rcfg, cfg.K, heads=heads, tbody=tb)
        plain = oracle_chain(prob, z0[rows], mi.bf16_bits_to_f64(h[rows]), rcfg, cfg.K, heads=heads, tbody=tb, round_y=0)
        stats = compare_chain(g, z_d.cpu().numpy()[rows], hrun_d.cpu().numpy()[rows], o, seqs, cfg.L, cfg.K, rcfg,
                              plain=plain, max_exempt=max_exempt)
        print(f"\n[tbody d={cfg.d} M={cfg.M} D={td.D} nh={td.n_heads}/{td.n_kv_heads} P<={td.P_max}] {stats}", flush=True)
        return stats
    finally:
        prob.close()


def test_small_two_heads_two_layers_prefix_over_two_tiles():
    cfg = mi.straddling(mi.config(0, B=4, L=4, K=2))
    td = mi.TBodyDims(D=2, n_heads=2, n_kv_heads=1, head_dim=128, d_ff=384, P_max=200)
    _run(cfg, td, mrp.RevealCfg(tau=0.9))


def test_block_of_16_four_query_heads_per_kv_head():
    cfg = mi.straddling(mi.config(0, d=512, B=3, L=16, K=1))
    td = mi.TBodyDims(D=1, n_heads=4, n_kv_heads=1, head_dim=128, d_ff=640, P_max=300)
    _run(cfg, td, mrp.RevealCfg(tau=0.9, tau_remask=0.5))


@pytest.mark.parametrize("L,P_max", [(8, 260), (16, 400)])
def test_two_kv_heads_prefix_over_several_tiles(L, P_max):
    """16 and 32 query vectors per kv head (the two middle register-tile widths of the attention kernel)."""
    cfg = mi.straddling(mi.config(0, d=512, B=2, L=L, K=1))
    td = mi.TBodyDims(D=1, n_heads=4, n_kv_heads=2, head_dim=128, d_ff=384, P_max=P_max)
    _run(cfg, td, mrp.RevealCfg(tau=0.9))


def test_no_prefix_three_layers_shared_module():
    cfg = mi.straddling(mi.config(0, B=2, L=4, K=3))
    td = mi.TBodyDims(D=3, n_heads=2, n_kv_heads=2, head_dim=128, d_ff=256, P_max=0)
    _run(cfg, td, mrp.RevealCfg(tau=0.9), gain="ones", share=True)


@pytest.mark.parametrize("D", [4, 8])
def test_depth_sweep_four_and_eight_layers(D):
    """The deeper bodies of the depth sweep (Section 4.5 varies D over 1, 2, 3, 4, 8) on a small case."""
    cfg = mi.straddling(mi.config(0, B=3, L=4, K=1))
    td = mi.TBodyDims(D=D, n_heads=2, n_kv_heads=1, head_dim=128, d_ff=256, P_max=70)
    _run(cfg, td, mrp.RevealCfg(tau=0.9, tau_remask=0.5))


def test_many_rows_tiled_gemm_path():
    cfg = mi.config(0, d=512, V=4096, B=48, L=16, K=1)
    td = mi.TBodyDims(D=1, n_heads=4, n_kv_heads=2, head_dim=128, d_ff=512, P_max=64)
    _run(cfg, td, mrp.RevealCfg(tau=0.9), seqs=[0, 1, 17, 47])


def test_160_rows_two_row_groups_of_the_wide_gemm():
    """160 rows: the projections run on the 64-feature x 128-row tiles with a ragged second row group (32 of 128
    rows) and k split over workgroups; 20 (kv head, sequence) pairs share their prefixes between two workgroups."""
    cfg = mi.straddling(mi.config(0, d=512, B=10, L=16, K=2))
    td = mi.TBodyDims(D=2, n_heads=4, n_kv_heads=2, head_dim=128, d_ff=512, P_max=300)
    _run(cfg, td, mrp.RevealCfg(tau=0.9), seqs=[0, 4, 9])


def test_400_rows_four_row_groups_wide_output():
    """400 rows (three whole row groups of 128 and one of 16) with a 3072-feature gate/up projection: 96 tiles of 128
    features, the form of the projection kernel that wide outputs take; sequences from the first, a middle and the
    last row group are compared."""
    cfg = mi.straddling(mi.config(0, d=256, V=4096, B=25, L=16, K=1))
    td = mi.TBodyDims(D=1, n_heads=2, n_kv_heads=1, head_dim=128, d_ff=1536, P_max=40)
    _run(cfg, td, mrp.RevealCfg(tau=0.9), seqs=[0, 11, 24])


def test_long_prefix_shared_by_four_workgroups():
    """Two (kv head, sequence) pairs with a 1024-position cache: four workgroups per pair; sequence 0 has no
    prefix (its three extra workgroups write empty partials), sequence 1 a full one."""
    cfg = mi.straddling(mi.config(0, d=256, B=2, L=8, K=1))
    td = mi.TBodyDims(D=1, n_heads=2, n_kv_heads=1, head_dim=128, d_ff=256, P_max=1024)
    _run(cfg, td, mrp.RevealCfg(tau=0.9))


@pytest.mark.timeout(900)
def test_config1_shape_three_layers():
    """Config 1's sizes with the backbone family's layer shape at that width (16 query / 8 kv heads
    of 128, gated MLP of 6144) and a 1024-position prefix cache; the oracle checks two sequences."""
    cfg = mi.config(1, K=1)
    td = mi.TBodyDims(D=3, n_heads=16, n_kv_heads=8, head_dim=128, d_ff=6144, P_max=1024)
    _run(cfg, td, mrp.RevealCfg(tau=cfg.tau), seqs=[0, 31], gain="ones")


def test_tbody_argument_errors():
    cfg = mi.config(0)
    ctx = mrp.MrpContext(cfg.d, cfg.V, cfg.M, cfg.L)
    try:
        assert ctx.tbody_create(0, 2, 1, 256, 16, check=False) != 0            # no layers
        assert ctx.tbody_create(1, 3, 2, 256, 16, check=False) != 0            # heads not a multiple of kv heads
        assert ctx.tbody_create(1, 2, 1, 200, 16, check=False) != 0            # d_ff not a multiple of 128
        assert ctx.tbody_create(1, 2, 1, 256, 16, head_dim=64, check=False) != 0
        io = mrp.StepIO(cfg.B, cfg.L, 1)
        z = torch.zeros((cfg.M, cfg.V), dtype=torch.float32, device="cuda")
        hr = torch.zeros((cfg.M, cfg.d), dtype=torch.float32, device="cuda")
        w = torch.zeros((cfg.V * cfg.d,), dtype=torch.int16, device="cuda")
        head = mrp.Head(w, None, w)
        lay = mrp.TLayer(w, w, w, w, w, w, w, w)
        plen = torch.zeros((cfg.B,), dtype=torch.int32, device="cuda")
        # the body's workspace was never created
        assert ctx.chain_step_tf(cfg.B, 1, None, hr, w, w, [head], [lay], plen, z, mrp.RevealCfg(), io, check=False) != 0
        assert ctx.tbody_create(1, 2, 1, 256, 16) == 0
        assert ctx.tbody_create(1, 2, 1, 256, 16, check=False) != 0            # only once
        assert ctx.chain_step_tf(cfg.B, 1, None, hr, w, w, [head], [lay], None, z, mrp.RevealCfg(), io, check=False) != 0
        assert ctx.chain_step_tf(cfg.B, 1, None, hr, w, w, [head], [], plen, z, mrp.RevealCfg(), io, check=False) != 0
    finally:
        ctx.close()
    # a block longer than the attention kernel stages is refused
    ctx = mrp.MrpContext(256, 4096, 64, 32)
    try:
        assert ctx.tbody_create(1, 2, 1, 256, 16, check=False) != 0
    finally:
        ctx.close()
