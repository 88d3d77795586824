"""Pins for the CPU oracle: each piece is checked against something other than
itself — a library routine, a closed form, an invariant the paper or the
mathematics fixes, or brute force on tiny inputs."""
import itertools
import os

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import mrp_inputs as mi
import oracle as orc

RNG = np.random.default_rng(12345)
HERE = os.path.dirname(os.path.abspath(__file__))


def bits(x):
    return mi.f32_to_bf16_bits(np.asarray(x, np.float32))


def val(b):
    return mi.bf16_bits_to_f64(b)


# ------------------------------------------------------------------ reduction
def test_reduce_matches_library_logsumexp():
    for V in (1, 2, 7, 1000, 4099):
        z = RNG.normal(0, 2, (5, V))
        tok, conf, lse = orc.reduce_rows(z)
        np.testing.assert_allclose(lse, logsumexp(z, axis=1), rtol=1e-13, atol=1e-13)
        np.testing.assert_array_equal(tok, z.argmax(1))
        np.testing.assert_allclose(conf, np.exp(z.max(1) - logsumexp(z, axis=1)), rtol=1e-12)


def test_reduce_closed_forms():
    V = 4096
    # uniform row: conf = 1/V, lowest index wins the tie
    tok, conf, lse = orc.reduce_rows(np.full((1, V), 3.25))
    assert tok[0] == 0 and abs(conf[0] - 1.0 / V) < 1e-15 and abs(lse[0] - (3.25 + np.log(V))) < 1e-12
    # one-hot plus a: conf = e^a / (e^a + V - 1)
    for a, at in ((2.0, 17), (12.0, V - 1), (0.5, 0)):
        z = np.zeros((1, V)); z[0, at] = a
        tok, conf, _ = orc.reduce_rows(z)
        assert tok[0] == at
        assert abs(conf[0] - np.exp(a) / (np.exp(a) + V - 1)) < 1e-14
    # exact tie between two maxima: lowest index
    z = RNG.normal(0, 1, (1, 50)); z[0, 40] = 9.0; z[0, 11] = 9.0
    assert orc.reduce_rows(z)[0][0] == 11


def test_reduce_shift_invariance_and_permutation_equivariance():
    z = RNG.normal(0, 2, (4, 513))
    tok, conf, lse = orc.reduce_rows(z)
    tok2, conf2, lse2 = orc.reduce_rows(z + 7.5)          # normalising constants cancel
    np.testing.assert_array_equal(tok, tok2)
    np.testing.assert_allclose(conf, conf2, rtol=1e-12)
    np.testing.assert_allclose(lse2 - lse, 7.5, rtol=1e-12)
    perm = RNG.permutation(513)
    tok3, conf3, lse3 = orc.reduce_rows(np.ascontiguousarray(z[:, perm]))
    np.testing.assert_array_equal(perm[tok3], tok)
    np.testing.assert_allclose(conf3, conf, rtol=1e-12)
    np.testing.assert_allclose(lse3, lse, rtol=1e-12)


def test_probabilities_sum_to_one():
    z = RNG.normal(0, 2, (6, 4096)); z[2, 5] += 12
    _, conf, lse = orc.reduce_rows(z)
    p = np.exp(z - lse[:, None])
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-12)
    np.testing.assert_allclose(p.max(1), conf, rtol=1e-12)


# ------------------------------------------------------------------ bf16 cast
def test_bf16_round_matches_library_cast():
    x = np.concatenate([RNG.normal(0, 1, 20000), RNG.normal(0, 1e-3, 2000), RNG.normal(0, 300, 2000),
                        # exact ties between neighbouring bf16 values, both parities
                        np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -(2.0 + 2 ** -7), 0.0, 1.0, -0.5])])
    x = x.astype(np.float32).astype(np.float64)            # fp32-representable inputs
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.bf16_round(x), ref)
    # and the generator's own bit-level rounding agrees with the library cast as well
    np.testing.assert_array_equal(val(bits(x)), ref)


# ------------------------------------------------------------------ head body
def _rand_head(d, V, scale=0.2):
    W1 = bits(RNG.normal(0, scale, (d, 2 * d))); W2 = bits(RNG.normal(0, scale, (d, d)))
    g = bits(RNG.normal(1, 0.3, d)); E = bits(RNG.normal(0, 1, (V, d)))
    return W1, W2, g, E


def _numpy_head(W1, W2, g, E, cond_tok, hrun, L, eps=1e-6):
    """Library-matmul statement of the head body (independent of the C code)."""
    M = hrun.shape[0]
    e = val(E)[np.repeat(cond_tok, L)]
    x = np.concatenate([hrun, e], axis=1)                   # h first, then the embedding
    a = x @ val(W1).T
    s = a / (1.0 + np.exp(-a))
    u = s @ val(W2).T
    y = u / np.sqrt((u * u).mean(1, keepdims=True) + eps) * val(g)[None, :]
    return u, y


@pytest.mark.parametrize("d,V,B,L", [(8, 16, 2, 3), (64, 100, 3, 4), (256, 4096, 1, 4)])
def test_head_mlp_matches_library_matmul(d, V, B, L):
    W1, W2, g, E = _rand_head(d, V)
    cfg = orc.make_cfg(d, V, B, L, 1)
    hrun = RNG.normal(0, 1, (B * L, d))
    cond = RNG.integers(0, V, B).astype(np.int32)
    h0 = hrun.copy()
    u, y = orc.head_mlp(cfg, W1, W2, g, E, cond, hrun)
    u_ref, y_ref = _numpy_head(W1, W2, g, E, cond, h0, L)
    np.testing.assert_allclose(u, u_ref, rtol=1e-11, atol=1e-12)
    # the definition: no intermediate is rounded
    np.testing.assert_allclose(y, y_ref, rtol=1e-11, atol=1e-12)
    # the bf16-operand variant: y is the bf16 rounding of the normalised output (within half a
    # bf16 step of it, exactly representable in bf16); nothing upstream of it changes
    cfg_r = orc.make_cfg(d, V, B, L, 1, round_y=1)
    h_r = h0.copy()
    u_r, y_r = orc.head_mlp(cfg_r, W1, W2, g, E, cond, h_r)
    np.testing.assert_array_equal(u_r, u)
    np.testing.assert_array_equal(h_r, hrun)
    assert np.all(np.abs(y_r - y_ref) <= np.abs(y_ref) * 2.0 ** -8 + 1e-30)
    np.testing.assert_array_equal(y_r, val(bits(y_r)))
    assert np.mean(y_r == val(bits(y))) > 0.999            # (a rounding tie may flip under 1e-12 noise)
    np.testing.assert_allclose(hrun, h0 + u_ref, rtol=1e-11, atol=1e-12)      # h <- h + Delta
    cfg2 = orc.make_cfg(d, V, B, L, 1, carry_hidden=0)
    h1 = h0.copy()
    orc.head_mlp(cfg2, W1, W2, g, E, cond, h1)
    np.testing.assert_array_equal(h1, h0)


def test_silu_and_rmsnorm_closed_forms():
    d, V = 16, 4
    eye = np.eye(d)
    W1 = bits(np.concatenate([eye, np.zeros((d, d))], 1)); W2 = bits(eye)
    g = bits(np.ones(d)); E = bits(np.zeros((V, d)))
    cfg = orc.make_cfg(d, V, 1, 2, 1, carry_hidden=0)
    a = RNG.normal(0, 3, d)
    hrun = np.stack([a, -a]); hrun[:, 0] = 0.0
    u, y = orc.head_mlp(cfg, W1, W2, g, E, np.zeros(1, np.int32), hrun)
    assert u[0, 0] == 0.0                                                    # SiLU(0) = 0
    np.testing.assert_allclose(u[0] - u[1], hrun[0], rtol=1e-13, atol=1e-15)   # SiLU(a) - SiLU(-a) = a
    big = np.full((2, d), 40.0)
    u2, _ = orc.head_mlp(cfg, W1, W2, g, E, np.zeros(1, np.int32), big)
    np.testing.assert_allclose(u2, 40.0, rtol=1e-15)                            # SiLU(a) -> a
    # RMSNorm with unit gain: unit RMS up to eps and the bf16 step
    rms = np.sqrt((y * y).mean(1))
    np.testing.assert_allclose(rms, 1.0, atol=4e-3)
    # gain is applied elementwise after normalisation
    g2 = bits(np.linspace(0.5, 2.0, d))
    _, y2 = orc.head_mlp(cfg, W1, W2, g2, E, np.zeros(1, np.int32), hrun)
    np.testing.assert_allclose(y2, y * val(g2)[None, :], rtol=2.0 ** -7, atol=1e-30)


def test_embedding_row_and_concat_order():
    """The embedding half of W1 sees E[cond_tok] of the row's own sequence."""
    d, V, B, L = 8, 5, 2, 2
    W1 = bits(np.concatenate([np.zeros((d, d)), np.eye(d)], 1)); W2 = bits(np.eye(d))
    E = bits(RNG.normal(0, 2, (V, d))); g = bits(np.ones(d))
    cfg = orc.make_cfg(d, V, B, L, 1, carry_hidden=0)
    cond = np.array([3, 1], np.int32)
    u, _ = orc.head_mlp(cfg, W1, W2, g, E, cond, RNG.normal(0, 1, (B * L, d)))
    e = val(E)
    for i in range(B * L):
        ei = e[cond[i // L]]
        np.testing.assert_allclose(u[i], ei / (1 + np.exp(-ei)), rtol=1e-13, atol=1e-15)


def test_lm_head_add_matches_library_matmul():
    for (M, V, d) in ((3, 17, 8), (5, 300, 64)):
        W = bits(RNG.normal(0, 0.05, (V, d)))
        y = val(bits(RNG.normal(0, 1, (M, d))))
        z = RNG.normal(0, 2, (M, V)); z0 = z.copy()
        orc.lm_head_add(W, y, z)
        np.testing.assert_allclose(z, z0 + y @ val(W).T, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ chain
def _tiny_problem(cid=0, **ov):
    cfg = mi.config(cid, **ov)
    return cfg, mi.lm_head(cfg), mi.embedding(cfg), [mi.head_weights(cfg, k) for k in range(cfg.K)], \
        mi.hidden(cfg), mi.logits0(cfg)


def test_zero_residual_leaves_logits_unchanged():
    cfg, W, E, heads, h, z0 = _tiny_problem()
    for variant in ("gamma", "w2"):
        hs = []
        for (w1, w2, g) in heads:
            hs.append((w1, w2, np.zeros_like(g)) if variant == "gamma" else (w1, np.zeros_like(w2), g))
        oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, tau=cfg.tau)
        out = orc.chain_step(oc, E, W, hs, z0, val(h))
        np.testing.assert_array_equal(out.z, z0.astype(np.float64))        # bit for bit
        for k in range(1, cfg.K + 1):
            np.testing.assert_array_equal(out.tok[k], out.tok[0])
            np.testing.assert_array_equal(out.conf[k], out.conf[0])


def test_chain_matches_library_composition_config0():
    """Whole chain on the tiny configuration against a numpy restatement built from
    library matmul / logsumexp (control flow: greedy forced reveal only)."""
    _chain_against_library(round_y=0)


def test_chain_matches_library_composition_config0_bf16_operand():
    """The same with the LM-head operand rounded to bf16 (the variant decisions are compared against)."""
    _chain_against_library(round_y=1)


def _chain_against_library(round_y):
    cfg, W, E, heads, h, z0 = _tiny_problem()
    oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, tau=cfg.tau, round_y=round_y)
    out = orc.chain_step(oc, E, W, heads, z0, val(h), dump_y=True)
    z = z0.astype(np.float64); hrun = val(h)
    masked = np.ones(cfg.M, bool)
    for k in range(cfg.K + 1):
        if k > 0:
            u, y = _numpy_head(*heads[k - 1], E, cond, hrun, cfg.L)
            hrun = hrun + u
            if round_y:
                yq = val(bits(y))
                # identical rounding wherever y is not within 1e-9 (relative) of a rounding tie
                step = 2.0 ** (np.floor(np.log2(np.abs(y) + 1e-300)) - 7)
                frac = np.abs(y) / step % 1.0
                safe = np.abs(frac - 0.5) > 1e-6
                np.testing.assert_array_equal(out.y[k - 1][safe], yq[safe])
                z = z + out.y[k - 1] @ val(W).T
            else:
                np.testing.assert_allclose(out.y[k - 1], y, rtol=1e-10, atol=1e-12)
                z = z + y @ val(W).T
        lse = logsumexp(z, axis=1)
        conf = np.exp(z.max(1) - lse)
        np.testing.assert_array_equal(out.tok[k], z.argmax(1))
        np.testing.assert_allclose(out.conf[k], conf, rtol=1e-9)
        np.testing.assert_allclose(out.lse[k], lse, rtol=1e-11)
        cond = np.empty(cfg.B, np.int32)
        for b in range(cfg.B):
            rows = np.arange(b * cfg.L, (b + 1) * cfg.L)
            cand = rows[masked[rows]]
            sel = cand[conf[cand] > cfg.tau]
            if len(sel) == 0:
                sel = cand[[np.argmax(conf[cand])]]
            masked[sel] = False
            top = sel[np.argmax(conf[sel])]
            cond[b] = z[top].argmax()
            assert out.draft_pos[b, k] == top - b * cfg.L and out.draft_tok[b, k] == cond[b]
    np.testing.assert_allclose(out.z, z, rtol=1e-11, atol=1e-11)
    np.testing.assert_array_equal(out.masked.astype(bool), masked)


def test_tv_bound_half_lipschitz_softmax():
    """TV(softmax(l + delta), softmax(l)) <= 0.5 * ||delta||_2 per row
    (appendix proof of the one-step contraction proposition)."""
    cfg, W, E, heads, h, z0 = _tiny_problem()
    # scale gamma down so that the bound is not vacuous
    hs = [(w1, w2, bits(np.full(cfg.d, 0.02))) for (w1, w2, _) in heads]
    oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 1, tau=cfg.tau)
    out = orc.chain_step(oc, E, W, hs[:1], z0, val(h))
    z_old = z0.astype(np.float64)
    delta = out.z - z_old
    p_old = np.exp(z_old - logsumexp(z_old, axis=1)[:, None])
    p_new = np.exp(out.z - out.lse[1][:, None])
    tv = 0.5 * np.abs(p_new - p_old).sum(1)
    bound = 0.5 * np.sqrt((delta * delta).sum(1))
    assert np.all(bound > 0) and np.all(bound < 1.0)
    assert np.all(tv <= bound + 1e-15)


# ------------------------------------------------------------------ reveal
def _reveal_once(conf, tau, L, r_min=1, max_accept=0, masked=None):
    M = len(conf); B = M // L
    cfg = orc.make_cfg(4, 8, B, L, 1, tau=tau, r_min=r_min, max_accept=max_accept)
    masked = np.ones(M, np.uint8) if masked is None else masked.copy()
    ra = np.full(M, -1, np.int8)
    tok = (np.arange(M) % 8).astype(np.int32)
    cond = np.full(B, 7, np.int32)
    dp, dt, tp = orc.reveal(cfg, 0, np.asarray(conf, np.float64), tok, masked, ra, cond)
    return masked, ra, dp, dt, cond, tok


def test_reveal_threshold_extremes():
    L = 8
    conf = RNG.uniform(0.01, 0.99, 3 * L)
    masked, ra, dp, dt, cond, tok = _reveal_once(conf, 0.0, L)
    assert masked.sum() == 0 and np.all(ra == 0)                      # tau = 0 reveals everything
    for tau in (1.0, 1.5):                                           # forced token only
        masked, ra, dp, dt, cond, tok = _reveal_once(conf, tau, L)
        for b in range(3):
            blk = slice(b * L, (b + 1) * L)
            assert (masked[blk] == 0).sum() == 1
            top = int(np.argmax(conf[blk]))
            assert masked[blk][top] == 0 and dp[b] == top and dt[b] == tok[b * L + top] == cond[b]
    # confidence exactly 1.0 does not exceed tau = 1.0 (direct decoding = forced reveals only)
    c = conf.copy(); c[3] = 1.0; c[5] = 1.0
    masked, *_ = _reveal_once(c, 1.0, L)
    assert (masked[:L] == 0).sum() == 1 and masked[3] == 0           # lowest position wins the tie


def test_reveal_monotone_in_tau_and_forced_minimum():
    L = 16
    conf = RNG.uniform(0, 1, 4 * L)
    prev = None
    for tau in (0.0, 0.2, 0.5, 0.8, 0.95, 1.0):
        masked, *_ = _reveal_once(conf, tau, L)
        revealed = masked == 0
        for b in range(4):
            blk = slice(b * L, (b + 1) * L)
            expect = conf[blk] > tau
            if not expect.any():
                expect = np.zeros(L, bool); expect[np.argmax(conf[blk])] = True
            np.testing.assert_array_equal(revealed[blk], expect)
        if prev is not None:
            assert np.all(revealed <= prev)                          # revealed set shrinks as tau grows
        prev = revealed
    # static decoding: tau = 1, r_min = r reveals exactly the r most confident masked rows
    pre = np.ones(4 * L, np.uint8); pre[::3] = 0
    masked, ra, *_ = _reveal_once(conf, 1.0, L, r_min=3, masked=pre)
    for b in range(4):
        blk = np.arange(b * L, (b + 1) * L)
        cand = blk[pre[blk] == 1]
        want = set(cand[np.argsort(-conf[cand], kind="stable")[:3]])
        got = set(blk[(pre[blk] == 1) & (masked[blk] == 0)])
        assert got == want
    # a sequence with nothing masked reveals nothing and keeps its conditioning token
    none = np.zeros(L, np.uint8)
    masked, ra, dp, dt, cond, _ = _reveal_once(conf[:L], 0.0, L, masked=none)
    assert dp[0] == -1 and dt[0] == -1 and cond[0] == 7 and np.all(ra == -1)


def test_max_accept_cap_values_and_effect():
    with open(os.path.join(HERE, "golden", "max_accept_cap.txt")) as f:
        rows = [tuple(map(int, ln.split())) for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 10
    for n, L, m in rows:
        assert orc.max_accept_cap(n, L) == m
    L = 16
    conf = RNG.uniform(0.6, 0.99, L)
    masked, *_ = _reveal_once(conf, 0.5, L, max_accept=1)             # all 16 clear tau, cap is 11
    assert (masked == 0).sum() == 11
    keep = np.argsort(-conf, kind="stable")[:11]
    assert np.all(masked[keep] == 0)
    masked, *_ = _reveal_once(conf, 0.5, L, max_accept=0)
    assert (masked == 0).sum() == 16


# ------------------------------------------------------------------ verify
def test_verify_accept_is_longest_matching_prefix_bruteforce():
    B, L = 1, 4
    for V in (4, 8, 16):
        for K in (1, 2, 3):
            for pattern in itertools.product([0, 1], repeat=K):
                verify = RNG.normal(0, 2, (B, L, V)).astype(np.float32)
                pos = RNG.permutation(L)[:K].astype(np.int32)
                tok = np.empty(K, np.int32)
                for j in range(K):
                    best = int(np.argmax(verify[0, pos[j]]))
                    tok[j] = best if pattern[j] else (best + 1 + RNG.integers(0, V - 1)) % V
                match, alen, corr = orc.verify_accept(verify, pos[None].copy(), tok[None].copy())
                # brute force: the largest a such that every one of the first a drafts matches
                brute = max(a for a in range(K + 1) if all(pattern[:a]))
                assert alen[0] == brute
                np.testing.assert_array_equal(match[0], np.array(pattern, np.uint8))
                if brute < K:
                    assert corr[0] == int(np.argmax(verify[0, pos[brute]]))
                else:
                    assert corr[0] == -1


def test_verify_missing_draft_and_ties():
    V, L = 8, 4
    verify = np.zeros((2, L, V), np.float32)
    verify[0, 2, 5] = 1.0
    verify[1, 1, 3] = 2.0; verify[1, 1, 6] = 2.0                       # tie -> lowest index 3
    pos = np.array([[2, -1, 0], [1, 0, 2]], np.int32)
    tok = np.array([[5, -1, 0], [6, 0, 0]], np.int32)
    match, alen, corr = orc.verify_accept(verify, pos, tok)
    assert list(match[0]) == [1, 0, 1] and alen[0] == 1 and corr[0] == -1   # missing draft ends the prefix
    assert list(match[1]) == [0, 1, 1] and alen[1] == 0 and corr[1] == 3


# ------------------------------------------------------------------ remask
def test_remask_set_inclusions():
    B, L = 3, 8
    M = B * L
    conf = RNG.uniform(0, 1, M)
    ra0 = RNG.integers(-2, 3, M).astype(np.int8)                       # -2 committed, -1 masked, 0..2 states
    m0 = (ra0 == -1).astype(np.uint8)
    protect = np.array([1, -1, 5], np.int32)
    state = 2
    elig = (ra0 >= 0) & (ra0 <= state - 1)
    for b in range(B):
        if protect[b] >= 0:
            elig[b * L + protect[b]] = False
    # tau_r = 0: nothing; tau_r > 1: every eligible row
    for tau_r, want in ((0.0, np.zeros(M, bool)), (1.5, elig), (0.4, elig & (conf < 0.4))):
        m, ra = m0.copy(), ra0.copy()
        rem = orc.remask(B, L, state, conf, tau_r, protect, m, ra).astype(bool)
        np.testing.assert_array_equal(rem, want)
        assert np.all(rem <= elig)
        np.testing.assert_array_equal(m, np.where(want, 1, m0))
        np.testing.assert_array_equal(ra, np.where(want, -1, ra0))
    # rows revealed by the current state are not eligible
    ra = np.full(M, 2, np.int8); m = np.zeros(M, np.uint8)
    assert orc.remask(B, L, 2, conf, 1.5, None, m, ra).sum() == 0
    # the comparison is strict (Algorithm 4: confidence below the threshold): a row exactly at the
    # threshold stays revealed, the next smaller double is remasked
    c2 = np.array([0.5, np.nextafter(0.5, 0.0), np.nextafter(0.5, 1.0), 0.5])
    rem = orc.remask(1, 4, 1, c2, 0.5, None, np.zeros(4, np.uint8), np.zeros(4, np.int8))
    np.testing.assert_array_equal(rem, [0, 1, 0, 0])


def test_chain_remask_and_reveal_control_flow():
    """Remask mode end to end on a straddling tiny case: the remasked rows are exactly the
    earlier-revealed, unprotected rows whose updated confidence is below the remask threshold."""
    cfg = mi.straddling(mi.config(0, B=6, L=8, V=512))
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    heads = [mi.head_weights(cfg, k) for k in range(cfg.K)]
    z0, h = mi.logits0(cfg), mi.hidden(cfg)
    oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, tau=0.5, tau_remask=0.3)
    out = orc.chain_step(oc, E, W, heads, z0, val(h))
    # replay the mask life cycle from the per-state outputs
    masked = np.ones(cfg.M, bool); ra = np.full(cfg.M, -1)
    n_rem = 0
    for k in range(cfg.K + 1):
        conf = out.conf[k]
        for b in range(cfg.B):
            rows = np.arange(b * cfg.L, (b + 1) * cfg.L)
            cand = rows[masked[rows]]
            if len(cand) == 0:
                assert out.draft_pos[b, k] == -1
                continue
            sel = cand[conf[cand] > 0.5]
            if len(sel) == 0:
                sel = cand[[np.argmax(conf[cand])]]
            masked[sel] = False; ra[sel] = k
            top = sel[np.argmax(conf[sel])]
            assert out.draft_pos[b, k] == top - b * cfg.L
            assert out.draft_tok[b, k] == out.tok[k][top]
            if k == 0:
                assert out.protect_pos[b] == top - b * cfg.L
        if k > 0:
            rem = (ra >= 0) & (ra <= k - 1) & (conf < 0.3)
            rem[np.arange(cfg.B) * cfg.L + out.protect_pos] = False
            np.testing.assert_array_equal(out.remasked[k].astype(bool), rem)
            masked[rem] = True; ra[rem] = -1
            n_rem += rem.sum()
    np.testing.assert_array_equal(out.masked.astype(bool), masked)
    np.testing.assert_array_equal(out.revealed_at, ra)
    assert n_rem > 0 and (out.revealed_at == 0).sum() > cfg.B     # both branches were exercised


# ---- decode loop around the chain: recorded token, committed-token remask, commit, block decode ----

@pytest.mark.parametrize("round_y,remask_mode,head_reveal", [(0, 0, 1), (1, 0, 1), (1, 1, 1), (0, 0, 0)])
def test_chain_resumed_head_by_head_equals_full_run(round_y, remask_mode, head_reveal):
    """A chain continued one head per call (state_offset = k - 1, run_state0 = 0, the previous call's
    z / h_run / masks / cond_tok / protect_pos / x_tok as inputs) gives, on every output, what the
    K-head call gives: the resumed form is what the GPU comparisons run the oracle in.  Straddling
    inputs with remask on, so that reveals above the threshold, forced reveals and remasks all occur."""
    cfg = mi.straddling(mi.config(0, B=7, L=8, V=640))
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    heads = [mi.head_weights(cfg, k) for k in range(cfg.K)]
    z0, h = mi.logits0(cfg).astype(np.float64), val(mi.hidden(cfg))
    kw = dict(tau=0.5, tau_remask=0.3 if head_reveal else 0.97, remask_mode=remask_mode, round_y=round_y,
              head_reveal=head_reveal)
    K = cfg.K
    full = orc.chain_step(orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, K, **kw), E, W, heads, z0, h)
    assert full.remasked.sum() > 0 and (full.revealed_at >= 0).sum() > cfg.B     # the case is not degenerate
    o = orc.chain_step(orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 0, **kw), E, W, [], z0, h)
    for f in ("tok", "conf", "lse", "gap", "remasked"):
        np.testing.assert_array_equal(getattr(o, f)[0], getattr(full, f)[0])
    np.testing.assert_array_equal(o.draft_pos[:, 0], full.draft_pos[:, 0])
    np.testing.assert_array_equal(o.draft_tok[:, 0], full.draft_tok[:, 0])
    for k in range(1, K + 1):
        ck = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 1, fresh_block=0, state_offset=k - 1, run_state0=0, **kw)
        o = orc.chain_step(ck, E, W, heads[k - 1:k], o.z, o.hrun, masked=o.masked, revealed_at=o.revealed_at,
                           cond_tok=o.cond_tok, protect_pos=o.protect_pos, x_tok=o.x_tok)
        for f in ("tok", "conf", "lse", "gap", "remasked"):
            np.testing.assert_array_equal(getattr(o, f)[1], getattr(full, f)[k], err_msg=f"{f} state {k}")
        np.testing.assert_array_equal(o.draft_pos[:, 1], full.draft_pos[:, k])
        np.testing.assert_array_equal(o.draft_tok[:, 1], full.draft_tok[:, k])
        assert np.all(o.draft_pos[:, 0] == -1)          # slot 0 of a resumed call is not written
    for f in ("z", "hrun", "masked", "revealed_at", "cond_tok", "protect_pos", "x_tok"):
        np.testing.assert_array_equal(getattr(o, f), getattr(full, f), err_msg=f)
    # an independent replay of what the state index means: a row revealed at state s carries s
    for s_idx in range(K + 1):
        rows = full.revealed_at == s_idx
        np.testing.assert_array_equal(full.x_tok[rows], full.tok[s_idx][rows])


def test_token_prob_against_library_softmax():
    """softmax(z)[x_tok] via scipy; it never exceeds the top-1 probability and equals it at the argmax."""
    from scipy.special import softmax
    z = RNG.normal(0, 2, (7, 300))
    tok, conf, lse = orc.reduce_rows(z)
    x = RNG.integers(0, 300, 7).astype(np.int32)
    x[2] = tok[2]; x[5] = -1
    p = orc.token_prob(z, lse, x)
    ref = softmax(z, axis=1)[np.arange(7), np.clip(x, 0, None)]
    ref[5] = 0.0
    np.testing.assert_allclose(p, ref, rtol=1e-12)
    assert np.all(p <= conf * (1 + 1e-12))
    np.testing.assert_allclose(p[2], conf[2], rtol=1e-12)


def test_commit_bookkeeping():
    B, L = 3, 5
    M = B * L
    ra = np.array([-2, -1, 0, 2, -1,   -1, -1, -1, -1, -1,   1, 0, -2, 3, 2], np.int8)
    masked = (ra == -1).astype(np.uint8)
    x_tok = np.arange(100, 100 + M, dtype=np.int32)
    x_out0 = np.full(M, -1, np.int32); x_out0[[0, 12]] = 7          # committed in earlier steps
    x_out, ra2, n = orc.commit(B, L, x_tok, ra, masked, x_out0)
    new = ra >= 0
    np.testing.assert_array_equal(x_out[new], x_tok[new])
    np.testing.assert_array_equal(x_out[~new], x_out0[~new])         # earlier commits and masked rows untouched
    np.testing.assert_array_equal(ra2, np.where(new, -2, ra))
    np.testing.assert_array_equal(n, [2, 5, 0])


def _decode_problem(B=4, L=8, V=512, K=2):
    cfg = mi.straddling(mi.config(0, B=B, L=L, V=V, K=K))
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    heads = [mi.head_weights(cfg, k) for k in range(cfg.K)]

    def backbone(step, x_out, masked):          # a stand-in backbone: fresh seeded logits / hidden states per step
        return mi.logits0(cfg, step=step).astype(np.float64), val(mi.hidden(cfg, step=step))
    return cfg, W, E, heads, backbone


def test_decode_block_static_and_threshold_limits():
    cfg, W, E, heads, backbone = _decode_problem()
    L, K = cfg.L, cfg.K
    # tau = 0: the backbone's own state reveals everything; one step, no head needed to finish
    oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, L, K, tau=0.0)
    x, steps, hist = orc.decode_block(oc, E, W, heads, backbone)
    assert steps == 1 and np.all(x >= 0)
    np.testing.assert_array_equal(x, hist[0].tok[0])                  # state 0 argmax everywhere
    # static decoding (tau >= 1): exactly r per state, K + 1 states per step
    for r in (1, 2):
        oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, L, K, tau=1.0, r_min=r)
        x, steps, hist = orc.decode_block(oc, E, W, heads, backbone)
        assert steps == -(-L // (r * (K + 1))) and np.all(x >= 0)
        for t, out in enumerate(hist):
            done_before = min(L, t * r * (K + 1))
            np.testing.assert_array_equal((out.masked.reshape(cfg.B, L) == 0).sum(1),
                                          np.full(cfg.B, min(L, done_before + r * (K + 1))))


def test_decode_block_remask_progress_and_monotone_commit():
    """Algorithm 4 (same threshold for reveal and remask) still commits at least one token per
    sequence and step (the protected state-0 row), so a block of L finishes within L steps; a
    committed token never changes afterwards."""
    cfg, W, E, heads, backbone = _decode_problem()
    for mode in (0, 1):
        oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, cfg.K, tau=0.6, tau_remask=0.6, head_reveal=0,
                          remask_mode=mode)
        x, steps, hist = orc.decode_block(oc, E, W, heads, backbone)
        assert steps <= cfg.L and np.all(x >= 0)
        committed = np.zeros(cfg.M, bool)
        n_prev = np.full(cfg.B, cfg.L)
        for out in hist:
            n_now = out.masked.reshape(cfg.B, cfg.L).sum(1)
            assert np.all((n_now < n_prev) | (n_prev == 0))           # progress in every unfinished sequence
            n_prev = n_now
            newly = (out.revealed_at >= 0)
            assert not np.any(newly & committed)
            np.testing.assert_array_equal(x[newly], out.x_tok[newly])
            committed |= newly


def test_committed_token_remask_is_at_least_as_strict():
    """p(revealed token) <= top-1 probability, so from identical inputs the committed-token rule
    remasks a superset of what the top-1 rule remasks at the first head."""
    cfg = mi.straddling(mi.config(0, B=6, L=8, V=512, K=1))
    W, E = mi.lm_head(cfg), mi.embedding(cfg)
    heads = [mi.head_weights(cfg, 0)]
    z0, h = mi.logits0(cfg), val(mi.hidden(cfg))
    outs = []
    for mode in (0, 1):
        oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 1, tau=0.3, tau_remask=0.8, remask_mode=mode)
        outs.append(orc.chain_step(oc, E, W, heads, z0, h))
    r0, r1 = outs[0].remasked[1].astype(bool), outs[1].remasked[1].astype(bool)
    assert np.all(r0 <= r1) and r1.sum() > 0
    # where the argmax did not move the two rules agree
    same_tok = outs[1].tok[1] == outs[1].x_tok
    np.testing.assert_array_equal(r0[same_tok], r1[same_tok])


def test_joint_candidate_verification_brute_force():
    """Draft j is checked against candidate j; equals the single-tensor rule when all candidates
    are the same tensor, and a brute-force longest matching prefix otherwise."""
    B, L, K = 5, 4, 3
    for V in (4, 8, 16):
        ver = RNG.normal(0, 2, (B, K + 1, L, V)).astype(np.float32)
        dpos = RNG.integers(-1, L, (B, K)).astype(np.int32)
        dtok = RNG.integers(0, V, (B, K)).astype(np.int32)
        # make about half of the drafts correct under their own candidate
        for b in range(B):
            for j in range(K):
                if dpos[b, j] >= 0 and RNG.random() < 0.6:
                    dtok[b, j] = int(np.argmax(ver[b, j, dpos[b, j]]))
        match, alen, corr = orc.verify_accept_joint(ver, dpos, dtok)
        for b in range(B):
            ok = [dpos[b, j] >= 0 and int(np.argmax(ver[b, j, dpos[b, j]])) == dtok[b, j] for j in range(K)]
            np.testing.assert_array_equal(match[b], ok)
            a = 0
            while a < K and ok[a]:
                a += 1
            assert alen[b] == a
            want = -1 if a == K or dpos[b, a] < 0 else int(np.argmax(ver[b, a, dpos[b, a]]))
            assert corr[b] == want
        same = np.repeat(ver[:, :1], K + 1, axis=1).copy()
        m1, a1, c1 = orc.verify_accept_joint(same, dpos, dtok)
        m0, a0, c0 = orc.verify_accept(np.ascontiguousarray(same[:, 0]), dpos, dtok)
        np.testing.assert_array_equal(m1, m0); np.testing.assert_array_equal(a1, a0); np.testing.assert_array_equal(c1, c0)


# ---------------------------------------------------------------------------------------------
# Training objective (Section 3.3, Equation 3)
def test_build_candidates_hand_example_and_nesting():
    """Figure 1 (d): candidate k = the block with the first k drafts written in.  A by-hand example,
    then on random inputs: candidate 0 is the block itself, candidate k differs from candidate k - 1
    exactly at draft k - 1's position (nothing if that draft is missing), masks are nested."""
    MASK = 99
    x_t = np.array([[5, -1, 7, -1, -1]], np.int32)
    m_t = np.array([[0, 1, 0, 1, 1]], np.uint8)
    dp = np.array([[3, 1, -1]], np.int32); dt = np.array([[40, 41, 42]], np.int32)
    ct, cm = orc.build_candidates(x_t, m_t, dp, dt, MASK)
    np.testing.assert_array_equal(ct[0], [[5, MASK, 7, MASK, MASK], [5, MASK, 7, 40, MASK], [5, 41, 7, 40, MASK],
                                          [5, 41, 7, 40, MASK]])
    np.testing.assert_array_equal(cm[0], [[0, 1, 0, 1, 1], [0, 1, 0, 0, 1], [0, 0, 0, 0, 1], [0, 0, 0, 0, 1]])
    rng = np.random.default_rng(7)
    B, L, K = 50, 16, 4
    m_t = (rng.random((B, L)) < 0.7).astype(np.uint8)
    x_t = rng.integers(0, 1000, (B, L)).astype(np.int32)
    dp = np.full((B, K), -1, np.int32); dt = rng.integers(1000, 2000, (B, K)).astype(np.int32)
    for b in range(B):                                   # drafts at distinct masked positions, some missing
        free = rng.permutation(np.flatnonzero(m_t[b]))[:K]
        dp[b, :len(free)] = free
        dp[b, rng.random(K) < 0.15] = -1
    ct, cm = orc.build_candidates(x_t, m_t, dp, dt, MASK)
    np.testing.assert_array_equal(cm[:, 0], m_t)
    np.testing.assert_array_equal(ct[:, 0], np.where(m_t == 1, MASK, x_t))
    for k in range(1, K + 1):
        for b in range(B):
            diff = np.flatnonzero((ct[b, k] != ct[b, k - 1]) | (cm[b, k] != cm[b, k - 1]))
            if dp[b, k - 1] < 0:
                assert len(diff) == 0
            else:
                np.testing.assert_array_equal(diff, [dp[b, k - 1]])
                assert ct[b, k, dp[b, k - 1]] == dt[b, k - 1] and cm[b, k, dp[b, k - 1]] == 0
        assert np.all(cm[:, k] <= cm[:, k - 1])
    assert np.all(ct[cm == 1] == MASK)
    # in candidate j the position of draft j is still masked: what the joint verification reads there
    for b in range(B):
        for j in range(K):
            if dp[b, j] >= 0:
                assert cm[b, j, dp[b, j]] == 1


def test_kl_loss_against_library_and_closed_forms():
    """KL(softmax(teacher) || softmax(student)) per row against scipy's softmax + rel_entr, a
    two-class closed form, shift invariance, and the zero at student = teacher + const."""
    from scipy.special import rel_entr, softmax
    M, V = 7, 333
    t = RNG.normal(0, 2, (M, V)).astype(np.float32)
    s = (t + RNG.normal(0, 1, (M, V))).astype(np.float32)
    loss, grad = orc.kl_loss(t, s)
    want = rel_entr(softmax(t.astype(np.float64), axis=1), softmax(s.astype(np.float64), axis=1)).sum(1)
    np.testing.assert_allclose(loss, want, rtol=1e-10, atol=1e-13)
    assert np.all(loss > 0)
    # an asymmetric pair: swapping the arguments gives a different number (catches a transposed operand)
    loss_sw, _ = orc.kl_loss(s, t)
    assert np.all(np.abs(loss_sw - loss) > 1e-6)
    # two classes: p = sigmoid(a), q = sigmoid(b)
    a, b = 1.25, -0.5
    two_t = np.array([[a, 0.0]], np.float32); two_s = np.array([[b, 0.0]], np.float32)
    p, q = 1 / (1 + np.exp(-a)), 1 / (1 + np.exp(-b))
    l2, g2 = orc.kl_loss(two_t, two_s)
    np.testing.assert_allclose(l2[0], p * np.log(p / q) + (1 - p) * np.log((1 - p) / (1 - q)), rtol=1e-12)
    np.testing.assert_allclose(g2[0], [q - p, p - q], rtol=1e-12)
    # softmax is shift invariant: a per-row constant on either side changes nothing; equal up to a constant -> 0
    shift = (s + np.float32(3.0)).astype(np.float32)
    l3, g3 = orc.kl_loss(t, shift)
    np.testing.assert_allclose(l3, loss, rtol=1e-5, atol=1e-7)      # (fp32 input rounding of s + 3)
    l0, g0 = orc.kl_loss(t, (t + np.float32(2.0)).astype(np.float32))
    np.testing.assert_allclose(l0, 0.0, atol=1e-6)
    np.testing.assert_allclose(g0, 0.0, atol=1e-6)
    # scale multiplies both outputs
    ls, gs = orc.kl_loss(t, s, scale=0.125)
    np.testing.assert_allclose(ls, 0.125 * loss, rtol=1e-14)
    np.testing.assert_allclose(gs, 0.125 * grad, rtol=1e-14)


def test_kl_loss_gradient_finite_differences_and_mask():
    """grad is d loss_i / d student[i][v]: central differences (student perturbed in fp32-exact
    steps of 2^-7), rows of the gradient sum to zero, unmasked rows contribute nothing."""
    M, V = 4, 41
    t = RNG.normal(0, 2, (M, V)).astype(np.float32)
    s = np.round((t + RNG.normal(0, 1, (M, V))) * 64) / 64          # on a 2^-6 grid: +-2^-7 is exact in fp32
    s = s.astype(np.float32)
    mask = np.array([1, 0, 1, 1], np.uint8)
    loss, grad = orc.kl_loss(t, s, mask, scale=0.5)
    assert loss[1] == 0.0 and np.all(grad[1] == 0.0)
    np.testing.assert_allclose(grad.sum(1), 0.0, atol=1e-14)
    full, _ = orc.kl_loss(t, s, None, scale=0.5)
    np.testing.assert_array_equal(loss[mask == 1], full[mask == 1])
    eps = 2.0 ** -7
    for i in (0, 2, 3):
        for v in range(V):
            sp, sm = s.copy(), s.copy()
            sp[i, v] += np.float32(eps); sm[i, v] -= np.float32(eps)
            lp, _ = orc.kl_loss(t, sp, mask, scale=0.5, want_grad=False)
            lm, _ = orc.kl_loss(t, sm, mask, scale=0.5, want_grad=False)
            fd = (lp[i] - lm[i]) / (2 * eps)
            assert abs(fd - grad[i, v]) < 2e-5, (i, v, fd, grad[i, v])   # O(eps^2) truncation
            assert lp[1] == 0.0


def test_kl_loss_one_hot_teacher_is_cross_entropy():
    """A teacher with one dominant logit makes Equation 3 the cross entropy -log q[target]."""
    from scipy.special import log_softmax
    M, V = 3, 64
    s = RNG.normal(0, 2, (M, V)).astype(np.float32)
    tgt = RNG.integers(0, V, M)
    t = np.full((M, V), -80.0, np.float32)
    t[np.arange(M), tgt] = 80.0
    loss, grad = orc.kl_loss(t, s)
    ce = -log_softmax(s.astype(np.float64), axis=1)[np.arange(M), tgt]
    np.testing.assert_allclose(loss, ce, rtol=1e-12)


# ---------------------------------------------------------------------------------------------
# Residual-magnitude measurement (Appendix B)
def test_residual_rms_hand_example_and_closed_forms():
    """A 3-state, 2-entry example worked by hand (3-4-5 triangles), a linear ramp
    X^(s) = s c whose r-step residual has RMS r |c| exactly, and numpy's vector norm."""
    X = np.array([[[0.0, 0.0], [3.0, 4.0], [6.0, 8.0]]])
    pair, delta = orc.residual_rms(X)
    s = np.sqrt(12.5)                                     # ||(3,4)||_RMS = sqrt(25/2)
    np.testing.assert_allclose(pair[0], [[0, s, 2 * s], [0, s, s], [0, 0, 2 * s]], rtol=1e-15)
    np.testing.assert_allclose(delta, [1.5 * s, s, 2 * s], rtol=1e-15)   # reference over s = 1, 2 only
    # ramp, two blocks with different slopes: mean over blocks of r |c|
    S, N = 6, 37
    c = RNG.normal(0, 1, (2, 1, N))
    ramp = np.ascontiguousarray(np.arange(S)[None, :, None] * c + 5.0)
    pair, delta = orc.residual_rms(ramp)
    crms = np.sqrt((c ** 2).mean(axis=(1, 2)))
    for r in range(1, S):
        np.testing.assert_allclose(delta[r], r * crms.mean(), rtol=1e-12)
        for t in range(S - r):
            np.testing.assert_allclose(pair[:, t, t + r], r * crms, rtol=1e-12)
    # the residual ignores a common offset, the reference line does not
    pair2, delta2 = orc.residual_rms(np.ascontiguousarray(ramp + 100.0))
    np.testing.assert_allclose(delta2[1:], delta[1:], rtol=1e-9)
    assert delta2[0] > delta[0] + 90
    # library norm on random states; order of subtraction must not matter, the pairing must
    X = RNG.normal(0, 2, (3, 5, 101))
    pair, delta = orc.residual_rms(X)
    for b in range(3):
        for t in range(5):
            for u in range(t, 5):
                want = np.linalg.norm(X[b, u] - X[b, t] if u > t else X[b, t]) / np.sqrt(101)
                np.testing.assert_allclose(pair[b, t, u], want, rtol=1e-13)
    np.testing.assert_allclose(delta[2], np.mean([pair[b, t, t + 2] for b in range(3) for t in range(3)]), rtol=1e-14)
    np.testing.assert_allclose(delta[0], np.mean([pair[b, s_, s_] for b in range(3) for s_ in range(1, 5)]), rtol=1e-14)


def test_residual_rms_random_walk_statistics_and_bf16_range():
    """The seeded stand-in states are a random walk with step deviation 0.4: the r-step residual
    has RMS 0.4 sqrt(r) and state s has RMS sqrt(4 + 0.16 s) up to sampling noise; differences far
    below a bf16 ulp of the states' sum of squares survive (the reason the paper computes in fp64)."""
    S, N = 17, 20000
    X = np.stack([mi.block_states(0, b, S, N) for b in range(2)]).astype(np.float64)
    pair, delta = orc.residual_rms(X)
    for r in range(1, S):
        assert abs(delta[r] / (0.4 * np.sqrt(r)) - 1) < 0.02, (r, delta[r])
    want_ref = np.mean([np.sqrt(4 + 0.16 * s) for s in range(1, S)])
    assert abs(delta[0] / want_ref - 1) < 0.02
    assert delta[1] < 0.25 * delta[0]                       # the magnitude gap the figure shows
    tiny = np.zeros((1, 2, 8)); tiny[0, 0, :] = 1.0; tiny[0, 1, :] = 1.0 + 2.0 ** -7
    pair, delta = orc.residual_rms(tiny)
    np.testing.assert_allclose(delta[1], 2.0 ** -7, rtol=1e-15)


# ---------------------------------------------------------------------------------------------
# Transformer head body (Section 3.2; D = 3 in Section 4.1)
def _tf_small(D=1, B=2, L=4, P_max=5, gain="normal"):
    cfg = mi.config(0, d=32, V=64, B=B, L=L, K=1)
    td = mi.TBodyDims(D, 4, 2, 8, 48, P_max, rope_theta=100.0)
    tc = orc.make_tcfg(td.D, td.n_heads, td.n_kv_heads, td.head_dim, td.d_ff, td.P_max, td.rope_theta)
    return cfg, td, tc, [mi.tf_layer(cfg, td, 0, l, gain=gain) for l in range(D)]


def test_rope_closed_forms_and_relative_position():
    """Rotary embedding: explicit 2-d and 4-d rotations, identity at position 0, norm kept, and
    q.k after rotation depends only on the position difference."""
    p, th = 3.0, 10000.0
    np.testing.assert_allclose(orc.rope([1.0, 0.0], p, th), [np.cos(p), np.sin(p)], rtol=1e-15)
    np.testing.assert_allclose(orc.rope([0.0, 1.0], p, th), [-np.sin(p), np.cos(p)], rtol=1e-15)
    # hd = 4: entry 0 pairs with 2 at angle p, entry 1 pairs with 3 at angle p / sqrt(theta)
    a2 = p / np.sqrt(th)
    np.testing.assert_allclose(orc.rope([1.0, 2.0, 0.0, 0.0], p, th),
                               [np.cos(p), 2 * np.cos(a2), np.sin(p), 2 * np.sin(a2)], rtol=1e-14)
    q, k = RNG.normal(size=16), RNG.normal(size=16)
    np.testing.assert_array_equal(orc.rope(q, 0.0, th), q)
    np.testing.assert_allclose(np.linalg.norm(orc.rope(q, 77.0, th)), np.linalg.norm(q), rtol=1e-14)
    d0 = orc.rope(q, 9.0, th) @ orc.rope(k, 4.0, th)
    d1 = orc.rope(q, 109.0, th) @ orc.rope(k, 104.0, th)
    np.testing.assert_allclose(d0, d1, rtol=1e-11)
    assert abs(orc.rope(q, 9.0, th) @ orc.rope(k, 5.0, th) - d0) > 1e-3


def _np_layer(td, layer, U, P, b, eps):
    """The same layer with numpy/scipy library calls (matmul, softmax), vectorised over rows and heads."""
    from scipy.special import softmax
    f = mi.bf16_bits_to_f64
    L, d = U.shape
    nh, nkv, hd, ff = td.n_heads, td.n_kv_heads, td.head_dim, td.d_ff
    rms = lambda x, g: x / np.sqrt((x ** 2).mean(-1, keepdims=True) + eps) * f(g)
    qkv = rms(U, layer["g1"]) @ f(layer["Wqkv"]).T
    q = qkv[:, :nh * hd].reshape(L, nh, hd)
    k = qkv[:, nh * hd:(nh + nkv) * hd].reshape(L, nkv, hd)
    v = qkv[:, (nh + nkv) * hd:].reshape(L, nkv, hd)
    pos = P + np.arange(L)
    inv = td.rope_theta ** (-np.arange(hd // 2) * 2.0 / hd)
    ang = pos[:, None] * inv[None, :]
    cs, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    rot = lambda x: np.concatenate([x[..., :hd // 2] * cs - x[..., hd // 2:] * sn,
                                    x[..., hd // 2:] * cs + x[..., :hd // 2] * sn], -1)
    q, k = rot(q), rot(k)
    K_all = np.concatenate([f(layer["kc"][b, :P]), k], 0)          # [T][nkv][hd]
    V_all = np.concatenate([f(layer["vc"][b, :P]), v], 0)
    K_all = np.repeat(K_all, nh // nkv, axis=1); V_all = np.repeat(V_all, nh // nkv, axis=1)
    sc = np.einsum("ihe,the->iht", q, K_all) / np.sqrt(hd)
    o = np.einsum("iht,the->ihe", softmax(sc, axis=-1), V_all).reshape(L, nh * hd)
    a = U + o @ f(layer["Wo"]).T
    gu = rms(a, layer["g2"]) @ f(layer["Wgu"]).T
    g, u = gu[:, :ff], gu[:, ff:]
    return a + (g / (1 + np.exp(-g)) * u) @ f(layer["Wdown"]).T


def test_transformer_layer_against_library_version():
    cfg, td, tc, layers = _tf_small()
    U = RNG.normal(0, 1, (cfg.L, cfg.d))
    for b, P in ((0, 0), (1, 5), (1, 3)):
        got = orc.tlayer(tc, layers[0], U, P, eps=1e-6, b=b)
        want = _np_layer(td, layers[0], U, P, b, 1e-6)
        np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # a different prefix or a different sequence's cache changes the result
    assert np.abs(orc.tlayer(tc, layers[0], U, 5, b=1) - orc.tlayer(tc, layers[0], U, 4, b=1)).max() > 1e-4
    assert np.abs(orc.tlayer(tc, layers[0], U, 5, b=1) - orc.tlayer(tc, layers[0], U, 5, b=0)).max() > 1e-4


def test_transformer_layer_special_cases():
    """Zero output projections make the layer the identity; zero keys make attention the plain mean
    of the values; one row without a prefix attends to itself only; the order of prefix entries is
    immaterial."""
    cfg, td, tc, layers = _tf_small(gain="ones")
    f = mi.bf16_bits_to_f64
    lay = {k: v.copy() for k, v in layers[0].items()}
    U = RNG.normal(0, 1, (cfg.L, cfg.d))
    z = dict(lay); z["Wo"] = np.zeros_like(lay["Wo"]); z["Wdown"] = np.zeros_like(lay["Wdown"])
    np.testing.assert_array_equal(orc.tlayer(tc, z, U, 5, b=1), U)
    # uniform attention: key rows of Wqkv and the key cache are zero; the MLP is switched off
    nh, nkv, hd = td.n_heads, td.n_kv_heads, td.head_dim
    m = dict(lay); m["Wdown"] = np.zeros_like(lay["Wdown"])
    m["Wqkv"] = lay["Wqkv"].copy(); m["Wqkv"][nh * hd:(nh + nkv) * hd] = 0
    m["kc"] = np.zeros_like(lay["kc"])
    P, b = 5, 1
    got = orc.tlayer(tc, m, U, P, b=b)
    n = U / np.sqrt((U ** 2).mean(-1, keepdims=True) + 1e-6)
    v_blk = (n @ f(m["Wqkv"][(nh + nkv) * hd:]).T).reshape(cfg.L, nkv, hd)
    v_mean = np.concatenate([f(m["vc"][b, :P]), v_blk], 0).mean(0)              # [nkv][hd]
    o = np.repeat(v_mean, nh // nkv, axis=0).reshape(-1)                        # same for every row
    np.testing.assert_allclose(got, U + (f(m["Wo"]) @ o)[None, :], rtol=1e-11, atol=1e-13)
    # a single row, no prefix: softmax over one key is 1, so o = its own value whatever q, k are
    s = dict(lay); s["Wdown"] = np.zeros_like(lay["Wdown"])
    U1 = U[:1]
    n1 = U1 / np.sqrt((U1 ** 2).mean(-1, keepdims=True) + 1e-6)
    v1 = (n1 @ f(s["Wqkv"][(nh + nkv) * hd:]).T).reshape(nkv, hd)
    o1 = np.repeat(v1, nh // nkv, axis=0).reshape(-1)
    np.testing.assert_allclose(orc.tlayer(tc, s, U1, 0, b=0), U1 + (f(s["Wo"]) @ o1)[None, :], rtol=1e-11, atol=1e-13)
    # permuting the prefix entries (keys and values together) changes nothing
    perm = RNG.permutation(5)
    pl = dict(lay); pl["kc"] = np.ascontiguousarray(lay["kc"][:, perm]); pl["vc"] = np.ascontiguousarray(lay["vc"][:, perm])
    np.testing.assert_allclose(orc.tlayer(tc, pl, U, 5, b=1), orc.tlayer(tc, lay, U, 5, b=1), rtol=1e-12, atol=1e-14)


def test_transformer_head_body_composition():
    """Fuse projection -> D layers -> RMSNorm/bf16, per sequence with its own prefix length and
    conditioning token; D = 0 is the bare fuse projection; the chain with this body equals the
    head-by-head composition with the LM head and the row reduction."""
    D = 2
    cfg, td, tc, layers = _tf_small(D=D, B=3)
    f = mi.bf16_bits_to_f64
    E, W = mi.embedding(cfg), mi.lm_head(cfg)
    w1, _, g = mi.head_weights(cfg, 0, gamma="normal")
    g = mi.f32_to_bf16_bits((1.0 + 10 * mi.bf16_bits_to_f32(g)).astype(np.float32))
    h = val(mi.hidden(cfg))
    ctok = np.array([3, 17, 60], np.int32)
    plen = np.array([0, 5, 2], np.int32)
    oc = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 1, tau=0.9, round_y=1)
    u, y, h_after = orc.head_transformer(oc, tc, w1, layers, plen, g, E, ctok, h)
    oc_plain = orc.make_cfg(cfg.d, cfg.V, cfg.B, cfg.L, 1, tau=0.9)
    u_p, y_p, _ = orc.head_transformer(oc_plain, tc, w1, layers, plen, g, E, ctok, h)
    np.testing.assert_array_equal(u_p, u)
    for b in range(cfg.B):
        rows = slice(b * cfg.L, (b + 1) * cfg.L)
        x = np.concatenate([h[rows], np.repeat(f(E[ctok[b]])[None], cfg.L, 0)], 1)
        U = x @ f(w1).T
        for l in range(D):
            U = _np_layer(td, layers[l], U, int(plen[b]), b, 1e-6)
        np.testing.assert_allclose(u[rows], U, rtol=1e-9, atol=1e-12)
        yn = U / np.sqrt((U ** 2).mean(-1, keepdims=True) + 1e-6) * f(g)
        np.testing.assert_allclose(y_p[rows], yn, rtol=1e-9, atol=1e-12)     # the definition: y not rounded
        yb = orc.bf16_round(yn)
        assert np.mean(y[rows] == yb) > 0.999          # (a rounding tie may flip under 1e-9 noise)
        np.testing.assert_allclose(y[rows], yb, rtol=2 ** -7)
    np.testing.assert_allclose(h_after, h + u, rtol=1e-14)
    tc0 = orc.make_tcfg(0, 4, 2, 8, 48, 5, 100.0)
    u0, _, _ = orc.head_transformer(oc, tc0, w1, [], plen, g, E, ctok, h)
    x = np.concatenate([h, np.repeat(f(E[ctok]), cfg.L, 0)], 1)
    np.testing.assert_allclose(u0, x @ f(w1).T, rtol=1e-12, atol=1e-14)
    # chain: state 0 picks cond_tok itself; compare with the composition around head_transformer
    z0 = mi.logits0(cfg)
    out = orc.chain_step(oc, E, W, [(w1, None, g)], z0, h, tbody=orc.TBody(tc, [layers], plen), dump_y=True)
    tok0, conf0, lse0 = orc.reduce_rows(z0.astype(np.float64))
    ct = np.zeros(cfg.B, np.int32)
    orc.reveal(oc, 0, conf0, tok0, np.ones(cfg.M, np.uint8), np.full(cfg.M, -1, np.int8), ct)
    u2, y2, _ = orc.head_transformer(oc, tc, w1, layers, plen, g, E, ct, h)
    np.testing.assert_array_equal(out.y[0], y2)
    np.testing.assert_allclose(out.z, z0 + y2 @ f(W).T, rtol=1e-12, atol=1e-12)
