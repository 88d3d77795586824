"""GPU parity of the residual-magnitude measurement (Appendix B): pairwise RMS of block-state
differences, the reference magnitudes and the per-r means, through the C-ABI, against the fp64
oracle.  Inputs: the seeded random-walk block states (fp32 for logits, bf16 for hidden states).

Tolerance: both sides form (double)x_u - (double)x_t exactly and square-accumulate in fp64; only
the order of the N <= 2.5e6 additions differs, which moves a sum of positive terms by at most
N 2^-53 < 3e-10 relative (typically 1e-14): rtol 1e-11 on every RMS, zeros exact."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import oracle as orc
import paper_2605_18817_amd as mrp

pytestmark = pytest.mark.gpu
RTOL = 1e-11


def _states(n_blocks, S, N, bf16, cid=0):
    return np.stack([mi.block_states(cid, b, S, N, bf16=bf16) for b in range(n_blocks)])


def _run(ctx, X, bf16):
    nb, S, N = X.shape
    X_d = torch.from_numpy(X.view(np.int16) if bf16 else X).cuda()
    pair = torch.full((nb, S, S), -1.0, dtype=torch.float64, device="cuda")
    delta = torch.full((S,), -1.0, dtype=torch.float64, device="cuda")
    ctx.residual_rms(nb, S, N, X_d, bf16, pair, delta)
    torch.cuda.synchronize()
    return pair.cpu().numpy(), delta.cpu().numpy()


def _oracle(X, bf16):
    Xd = mi.bf16_bits_to_f64(X) if bf16 else X.astype(np.float64)
    return orc.residual_rms(np.ascontiguousarray(Xd))


@pytest.fixture(scope="module")
def ctx():
    c = mrp.MrpContext(256, 4096, 4, 4)
    yield c
    c.close()


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("S,N,nb", [(3, 1, 1), (5, 101, 3), (5, 512, 2), (9, 1000, 2), (17, 513, 1), (17, 5000, 3),
                                    (17, 66666, 2)])
def test_residual_rms_matches_oracle(ctx, S, N, nb, bf16):
    X = _states(nb, S, N, bf16)
    pair_g, delta_g = _run(ctx, X, bf16)
    pair_o, delta_o = _oracle(X, bf16)
    np.testing.assert_allclose(pair_g, pair_o, rtol=RTOL, atol=0)
    np.testing.assert_allclose(delta_g, delta_o, rtol=RTOL, atol=0)
    assert np.all(pair_g[:, np.tri(S, k=-1, dtype=bool)] == 0.0)


def test_residual_rms_is_deterministic_and_sees_sub_ulp_differences(ctx):
    X = _states(2, 17, 40000, False)
    a = _run(ctx, X, False)
    b = _run(ctx, X, False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # bf16 states one ulp apart at 1.0: the residual 2^-7 is recovered exactly
    tiny = np.empty((1, 3, 64), np.uint16)
    tiny[0, 0] = 0x3F80; tiny[0, 1] = 0x3F81; tiny[0, 2] = 0x3F82
    pair, delta = _run(ctx, tiny, True)
    assert pair[0, 0, 1] == 2.0 ** -7 and pair[0, 0, 2] == 2.0 ** -6 and delta[1] == 2.0 ** -7


def test_residual_rms_argument_errors(ctx):
    X = torch.zeros((1, 5, 64), dtype=torch.float32, device="cuda")
    pair = torch.zeros((1, 5, 5), dtype=torch.float64, device="cuda")
    delta = torch.zeros((5,), dtype=torch.float64, device="cuda")
    assert ctx.residual_rms(1, 4, 64, X, False, pair, delta, check=False) != 0      # unsupported state count
    assert ctx.residual_rms(5000, 5, 64, X, False, pair, delta, check=False) != 0   # too many blocks
    assert ctx.residual_rms(1, 5, 0, X, False, pair, delta, check=False) != 0
    assert ctx.residual_rms(1, 5, 64, None, False, pair, delta, check=False) != 0
    assert ctx.residual_rms(0, 5, 64, X, False, pair, delta, check=False) == 0
    with pytest.raises(RuntimeError):
        ctx.residual_rms(1, 4, 64, X, False, pair, delta)


@pytest.mark.timeout(600)
def test_residual_rms_full_size_logits_and_hidden(ctx):
    """The paper's shapes: 17 states of a 16-position block; logits N = 16 x 151936 (fp32, 4
    blocks), hidden states N = 16 x 4096 (bf16, 200 blocks, the paper's minimum count)."""
    for (nb, N, bf16) in ((4, 16 * 151936, False), (200, 16 * 4096, True)):
        X = _states(nb, 17, N, bf16, cid=2)
        pair_g, delta_g = _run(ctx, X, bf16)
        pair_o, delta_o = _oracle(X, bf16)
        np.testing.assert_allclose(pair_g, pair_o, rtol=RTOL, atol=0)
        np.testing.assert_allclose(delta_g, delta_o, rtol=RTOL, atol=0)
        print(f"\n[residual rms nb={nb} N={N} bf16={bf16}] ref {delta_g[0]:.4f} r=1 {delta_g[1]:.4f} "
              f"r=16 {delta_g[16]:.4f}", flush=True)
