"""GPU parity of the head's training objective (Section 3.3, Equation 3): per-row
KL(softmax(l_{t-1}) || softmax(l_t + delta_t)) and its gradient with respect to the student
logits, through the C-ABI, against the fp64 oracle.

Inputs: teacher = the seeded prior logits of denoising step 1, student = those of step 0 plus a
seeded N(0, 0.5) stand-in residual (a trained head makes the two close; a second case uses
teacher + residual so that the loss is small and cancellation in it is exercised).

Tolerances (fp32 arithmetic with the hardware exponential, |logit| < ~40, V <= 151936):
every exponential carries a relative error of a few 2^-24 plus |x - lse| 2^-24 from its rounded
argument, i.e. < 4e-6 relative; sums of V such terms in a tree keep that relative error.
  loss:  a_T/s_T, lse_T and lse_S are each ~|lse| <= 20 accurate to ~1e-5 absolute, their
         combination to < 1e-4 absolute:  |loss_gpu - loss_orc| <= 1e-4 + 1e-4 |loss_orc|.
  grad:  scale (q - p) with p, q <= 1:    |g_gpu - g_orc| <= scale (2e-5 (p + q) + 1e-12).
"""
import numpy as np
import pytest
import torch
from scipy.special import softmax

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp

pytestmark = pytest.mark.gpu


def _inputs(cfg, seqs, close):
    t = mi.logits0(cfg, seqs, step=1)
    if close:
        s = t + mi.residual(cfg, seqs)
    else:
        s = mi.logits0(cfg, seqs, step=0) + mi.residual(cfg, seqs)
    return t, np.ascontiguousarray(s, dtype=np.float32)


def _check(t, s, mask, scale, loss_g, grad_g, rows=None):
    rows = np.arange(t.shape[0]) if rows is None else rows
    m = None if mask is None else np.ascontiguousarray(mask[rows])
    loss_o, grad_o = orc.kl_loss(np.ascontiguousarray(t[rows]), np.ascontiguousarray(s[rows]), m, scale)
    np.testing.assert_allclose(loss_g[rows], loss_o, rtol=1e-4, atol=1e-4 * abs(scale))
    if grad_g is not None:
        p = softmax(t[rows].astype(np.float64), axis=1)
        q = softmax(s[rows].astype(np.float64), axis=1)
        err = np.abs(grad_g[rows] - grad_o)
        bound = abs(scale) * (2e-5 * (p + q) + 1e-12)
        assert np.all(err <= bound), float((err / bound).max())
        if m is not None:
            assert np.all(grad_g[rows][m == 0] == 0.0) and np.all(loss_g[rows][m == 0] == 0.0)
    return loss_o


@pytest.mark.parametrize("V,M,close", [(4096, 4, False), (4096, 4, True), (5003, 24, False), (8192, 16, True),
                                       (33000, 8, False), (151936, 8, True)])
def test_kl_loss_and_gradient_match_oracle(V, M, close):
    cfg = mi.config(0, V=V, B=M // 4, L=4)
    ctx = mrp.MrpContext(cfg.d, V, M, cfg.L)
    try:
        t, s = _inputs(cfg, None, close)
        mask = (np.arange(M) % 3 != 1).astype(np.uint8)
        t_d, s_d = torch.from_numpy(t).cuda(), torch.from_numpy(s).cuda()
        for mk, scale in ((None, 1.0), (mask, 0.25)):
            loss = torch.full((M,), 7.0, dtype=torch.float32, device="cuda")
            grad = torch.full((M, V), 7.0, dtype=torch.float32, device="cuda")
            mk_d = None if mk is None else torch.from_numpy(mk).cuda()
            ctx.kl_loss(M, t_d, s_d, mk_d, scale, loss, grad)
            torch.cuda.synchronize()
            lo = _check(t, s, mk, scale, loss.cpu().numpy(), grad.cpu().numpy())
            # forward only leaves grad alone and gives the same loss bits
            loss2 = torch.empty_like(loss)
            ctx.kl_loss(M, t_d, s_d, mk_d, scale, loss2, None)
            torch.cuda.synchronize()
            assert torch.equal(loss, loss2)
        print(f"\n[kl V={V} M={M} close={close}] mean loss {lo.mean():.4f}", flush=True)
    finally:
        ctx.close()


def test_kl_loss_zero_when_student_equals_teacher_up_to_a_constant():
    cfg = mi.config(0, V=10000, B=2, L=4)
    ctx = mrp.MrpContext(cfg.d, cfg.V, cfg.M, cfg.L)
    try:
        t = mi.logits0(cfg)
        t_d = torch.from_numpy(t).cuda()
        s_d = t_d + 2.0
        loss = torch.empty((cfg.M,), dtype=torch.float32, device="cuda")
        grad = torch.empty((cfg.M, cfg.V), dtype=torch.float32, device="cuda")
        ctx.kl_loss(cfg.M, t_d, s_d, None, 1.0, loss, grad)
        torch.cuda.synchronize()
        assert loss.abs().max().item() < 1e-4
        assert grad.abs().max().item() < 2e-5
        # row sums of the gradient vanish (both softmaxes sum to one)
        assert grad.double().sum(1).abs().max().item() < 1e-5
    finally:
        ctx.close()


def test_kl_loss_argument_errors():
    cfg = mi.config(0)
    ctx = mrp.MrpContext(cfg.d, cfg.V, cfg.M, cfg.L)
    try:
        t = torch.zeros((cfg.M, cfg.V), dtype=torch.float32, device="cuda")
        loss = torch.zeros((cfg.M,), dtype=torch.float32, device="cuda")
        assert ctx.kl_loss(cfg.M + 1, t, t, None, 1.0, loss, None, check=False) != 0
        assert ctx.kl_loss(cfg.M, None, t, None, 1.0, loss, None, check=False) != 0
        assert ctx.kl_loss(cfg.M, t.view(-1)[1:], t, None, 1.0, loss, None, check=False) != 0   # misaligned
        assert ctx.kl_loss(0, t, t, None, 1.0, loss, None, check=False) == 0
    finally:
        ctx.close()


@pytest.mark.timeout(600)
def test_kl_loss_full_size_sampled_rows():
    """Config 2's row count and vocabulary (the size the throughput figure is quoted on); the
    oracle checks a sample of rows, the rest by invariants that hold at any size."""
    cfg = mi.config(2)
    M, V = cfg.M, cfg.V
    ctx = mrp.MrpContext(256, V, M, cfg.L)
    try:
        t, s = _inputs(cfg, None, True)
        mask = (np.arange(M) % 5 != 2).astype(np.uint8)
        t_d, s_d = torch.from_numpy(t).cuda(), torch.from_numpy(s).cuda()
        loss = torch.empty((M,), dtype=torch.float32, device="cuda")
        grad = torch.empty((M, V), dtype=torch.float32, device="cuda")
        ctx.kl_loss(M, t_d, s_d, torch.from_numpy(mask).cuda(), 1.0 / M, loss, grad)
        torch.cuda.synchronize()
        rows = np.array([0, 1, 2, 517, 1022, 1023])
        loss_h = loss.cpu().numpy()
        _check(t, s, mask, 1.0 / M, loss_h, grad.cpu().numpy(), rows)
        on = mask == 1
        assert np.all(loss_h[on] > 0) and np.all(loss_h[~on] == 0)
        rs = grad.double().sum(1).abs().max().item()
        assert rs < 1e-5 / M * 4, rs
        assert torch.all(grad[torch.from_numpy(~on).cuda()] == 0)
    finally:
        ctx.close()
