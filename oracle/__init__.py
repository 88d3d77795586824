"""ctypes wrapper around the CPU oracle (``mrp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and ``bench.py``'s cpu_baseline leg; never by the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mrp_oracle.c")
_LIB = os.path.join(_HERE, "libmrp_oracle.so")
CFLAGS = ["-O2", "-fopenmp", "-std=c99", "-fPIC", "-shared", "-Wall"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("d", C.c_int), ("V", C.c_int), ("B", C.c_int), ("L", C.c_int), ("K", C.c_int),
                ("rms_eps", C.c_double), ("tau", C.c_double), ("r_min", C.c_int),
                ("max_accept", C.c_int), ("carry_hidden", C.c_int), ("tau_remask", C.c_double),
                ("head_reveal", C.c_int), ("fresh_block", C.c_int), ("state_offset", C.c_int),
                ("run_state0", C.c_int), ("remask_mode", C.c_int), ("round_y", C.c_int)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # (MRP_ORACLE_LIB: a library to load instead -- only the planted-mistake test sets it, to show that
        #  the pins fail on a deliberately wrong oracle)
        _lib = C.CDLL(os.environ.get("MRP_ORACLE_LIB") or build())
        _lib.orc_bf16_round.restype = C.c_double
        _lib.orc_bf16_round.argtypes = [C.c_double]
        _lib.orc_max_accept_cap.restype = C.c_int
        _lib.orc_max_accept_cap.argtypes = [C.c_int, C.c_int]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def make_cfg(d, V, B, L, K, tau=0.9, r_min=1, max_accept=0, carry_hidden=1, tau_remask=-1.0,
             head_reveal=1, fresh_block=1, state_offset=0, run_state0=1, rms_eps=1e-6,
             remask_mode=0, round_y=0) -> _Cfg:
    """round_y=0: the plain definition (no intermediate rounded); round_y=1: the LM-head operand y
    is rounded to bf16 (used to compare decisions with a bf16-operand implementation bit for bit)."""
    return _Cfg(d, V, B, L, K, rms_eps, tau, r_min, max_accept, carry_hidden, tau_remask,
                head_reveal, fresh_block, state_offset, run_state0, remask_mode, round_y)


def bf16_round(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty_like(x)
    lib().orc_bf16_round_array(_p(x), _p(out), C.c_long(x.size))
    return out


def threads() -> int:
    return lib().orc_threads()


def max_accept_cap(n_masked: int, L: int) -> int:
    return lib().orc_max_accept_cap(n_masked, L)


def reduce_rows(z: np.ndarray, with_gap: bool = False):
    z = _chk(z, np.float64)
    M, V = z.shape
    tok = np.empty(M, np.int32); conf = np.empty(M, np.float64); lse = np.empty(M, np.float64)
    gap = np.empty(M, np.float64) if with_gap else None
    lib().orc_reduce_rows(_p(z), M, V, _p(tok), _p(conf), _p(lse), _p(gap))
    return (tok, conf, lse, gap) if with_gap else (tok, conf, lse)


def head_mlp(cfg: _Cfg, W1, W2, gamma, E, cond_tok, hrun):
    """Returns (u, y); ``hrun`` [M][d] float64 is updated in place if carry_hidden."""
    M, d = cfg.B * cfg.L, cfg.d
    _chk(W1, np.uint16, (d, 2 * d)); _chk(W2, np.uint16, (d, d)); _chk(gamma, np.uint16, (d,))
    _chk(E, np.uint16); _chk(cond_tok, np.int32, (cfg.B,)); _chk(hrun, np.float64, (M, d))
    assert E.shape[1] == d and cond_tok.min() >= 0 and cond_tok.max() < E.shape[0]
    u = np.empty((M, d)); y = np.empty((M, d))
    lib().orc_head_mlp(C.byref(cfg), _p(W1), _p(W2), _p(gamma), _p(E), _p(cond_tok), _p(hrun), _p(u), _p(y))
    return u, y


def lm_head_add(W_lm, y, z):
    V, d = W_lm.shape
    M = y.shape[0]
    _chk(W_lm, np.uint16); _chk(y, np.float64, (M, d)); _chk(z, np.float64, (M, V))
    lib().orc_lm_head_add(_p(W_lm), _p(y), _p(z), M, V, d)


def reveal(cfg: _Cfg, state, conf, tok, masked, revealed_at, cond_tok):
    """In-place on masked / revealed_at / cond_tok; returns (draft_pos, draft_tok, top_pos)."""
    M = cfg.B * cfg.L
    _chk(conf, np.float64, (M,)); _chk(tok, np.int32, (M,)); _chk(masked, np.uint8, (M,))
    _chk(revealed_at, np.int8, (M,)); _chk(cond_tok, np.int32, (cfg.B,))
    dp = np.empty(cfg.B, np.int32); dt = np.empty(cfg.B, np.int32); tp = np.empty(cfg.B, np.int32)
    lib().orc_reveal(C.byref(cfg), int(state), _p(conf), _p(tok), _p(masked), _p(revealed_at),
                     _p(dp), _p(dt), _p(cond_tok), _p(tp))
    return dp, dt, tp


def remask(B, L, state, conf, tau_remask, protect_pos, masked, revealed_at):
    M = B * L
    _chk(conf, np.float64, (M,)); _chk(masked, np.uint8, (M,)); _chk(revealed_at, np.int8, (M,))
    if protect_pos is not None:
        _chk(protect_pos, np.int32, (B,))
    out = np.empty(M, np.uint8)
    lib().orc_remask(B, L, int(state), _p(conf), C.c_double(tau_remask), _p(protect_pos), _p(masked),
                     _p(revealed_at), _p(out))
    return out


def verify_accept(verify, draft_pos, draft_tok):
    B, L, V = verify.shape
    K = draft_pos.shape[1]
    _chk(verify, np.float32); _chk(draft_pos, np.int32, (B, K)); _chk(draft_tok, np.int32, (B, K))
    match = np.empty((B, K), np.uint8); alen = np.empty(B, np.int32); corr = np.empty(B, np.int32)
    lib().orc_verify_accept(B, L, V, K, _p(verify), _p(draft_pos), _p(draft_tok), _p(match), _p(alen), _p(corr))
    return match, alen, corr


def verify_accept_joint(verify, draft_pos, draft_tok):
    """verify: float32 [B][K+1][L][V], candidate k holding the first k drafts."""
    B, K1, L, V = verify.shape
    K = draft_pos.shape[1]
    assert K1 == K + 1
    _chk(verify, np.float32); _chk(draft_pos, np.int32, (B, K)); _chk(draft_tok, np.int32, (B, K))
    match = np.empty((B, K), np.uint8); alen = np.empty(B, np.int32); corr = np.empty(B, np.int32)
    lib().orc_verify_accept_joint(B, L, V, K, _p(verify), _p(draft_pos), _p(draft_tok), _p(match), _p(alen),
                                  _p(corr))
    return match, alen, corr


def build_candidates(x_t, masked_t, draft_pos, draft_tok, mask_token: int):
    """Candidate blocks of the joint verification.  x_t int32 [B][L], masked_t uint8 [B][L], drafts int32
    [B][K]; returns (cand_tok int32 [B][K+1][L], cand_masked uint8 [B][K+1][L])."""
    B, L = x_t.shape
    K = draft_pos.shape[1]
    _chk(x_t, np.int32); _chk(masked_t, np.uint8, (B, L)); _chk(draft_pos, np.int32, (B, K)); _chk(draft_tok, np.int32, (B, K))
    ct = np.empty((B, K + 1, L), np.int32); cm = np.empty((B, K + 1, L), np.uint8)
    lib().orc_build_candidates(B, L, K, _p(x_t), _p(masked_t), _p(draft_pos), _p(draft_tok), C.c_int32(mask_token),
                               _p(ct), _p(cm))
    return ct, cm


def kl_loss(teacher, student, row_mask=None, scale=1.0, want_grad=True):
    """Equation 3 per row and its gradient w.r.t. the student logits.  teacher/student float32 [M][V];
    returns (loss float64 [M], grad float64 [M][V] or None)."""
    M, V = teacher.shape
    _chk(teacher, np.float32); _chk(student, np.float32, (M, V))
    if row_mask is not None:
        _chk(row_mask, np.uint8, (M,))
    loss = np.empty(M, np.float64)
    grad = np.empty((M, V), np.float64) if want_grad else None
    lib().orc_kl_loss(M, V, _p(teacher), _p(student), _p(row_mask), C.c_double(scale), _p(loss), _p(grad))
    return loss, grad


def residual_rms(X):
    """Appendix B magnitudes.  X float64 [n_blocks][S][N]; returns (rms_pair [n_blocks][S][S], rms_delta [S])
    with rms_delta[0] the reference line and rms_delta[r] the mean RMS of the r-step residuals."""
    nb, S, N = X.shape
    _chk(X, np.float64)
    pair = np.empty((nb, S, S), np.float64); delta = np.empty(S, np.float64)
    lib().orc_residual_rms(nb, S, C.c_long(N), _p(X), _p(pair), _p(delta))
    return pair, delta


class _TCfg(C.Structure):
    _fields_ = [("D", C.c_int), ("n_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("d_ff", C.c_int), ("P_max", C.c_int), ("rope_theta", C.c_double)]


class _TBodyC(C.Structure):
    _fields_ = [("t", C.POINTER(_TCfg))] + [(n, C.POINTER(C.c_void_p)) for n in
                                             ("Wqkv", "Wo", "Wgu", "Wdown", "g1", "g2", "kc", "vc")] + \
               [("prefix_len", C.c_void_p)]


def make_tcfg(D, n_heads, n_kv_heads, head_dim, d_ff, P_max, rope_theta=1.0e6) -> _TCfg:
    assert n_heads % n_kv_heads == 0 and head_dim % 2 == 0
    return _TCfg(D, n_heads, n_kv_heads, head_dim, d_ff, P_max, rope_theta)


LAYER_FIELDS = ("Wqkv", "Wo", "Wgu", "Wdown", "g1", "g2", "kc", "vc")


def _check_layer(tc: _TCfg, d, B, layer):
    """layer: dict with the eight arrays of LAYER_FIELDS (uint16 bf16 bits)."""
    qd, kvd = tc.n_heads * tc.head_dim, tc.n_kv_heads * tc.head_dim
    _chk(layer["Wqkv"], np.uint16, (qd + 2 * kvd, d)); _chk(layer["Wo"], np.uint16, (d, qd))
    _chk(layer["Wgu"], np.uint16, (2 * tc.d_ff, d)); _chk(layer["Wdown"], np.uint16, (d, tc.d_ff))
    _chk(layer["g1"], np.uint16, (d,)); _chk(layer["g2"], np.uint16, (d,))
    _chk(layer["kc"], np.uint16, (B, tc.P_max, tc.n_kv_heads, tc.head_dim))
    _chk(layer["vc"], np.uint16, (B, tc.P_max, tc.n_kv_heads, tc.head_dim))


def _layer_arrays(tc, d, B, layers):
    """layers: flat list of layer dicts -> dict of ctypes pointer arrays."""
    n = max(len(layers), 1)
    out = {}
    for f in LAYER_FIELDS:
        out[f] = (C.c_void_p * n)(*[l[f].ctypes.data for l in layers])
    for l in layers:
        _check_layer(tc, d, B, l)
    return out


def rope(x, pos, theta):
    """Rotary embedding of one head vector (float64 [hd]) at position ``pos``; returns a new array."""
    x = np.array(x, np.float64)
    lib().orc_rope(_p(x), x.shape[0], C.c_double(pos), C.c_double(theta))
    return x


def tlayer(tc: _TCfg, layer, U, P, eps=1e-6, b=0):
    """One transformer layer over the block rows U float64 [L][d] of sequence ``b`` with ``P`` prefix
    positions; returns the new rows."""
    L, d = U.shape
    B = layer["kc"].shape[0]
    _check_layer(tc, d, B, layer)
    assert 0 <= P <= tc.P_max
    U = np.array(U, np.float64)
    off = b * tc.P_max * tc.n_kv_heads * tc.head_dim * 2
    lib().orc_tlayer(C.byref(tc), d, L, C.c_double(eps), _p(layer["Wqkv"]), _p(layer["Wo"]), _p(layer["Wgu"]),
                     _p(layer["Wdown"]), _p(layer["g1"]), _p(layer["g2"]),
                     C.c_void_p(layer["kc"].ctypes.data + off), C.c_void_p(layer["vc"].ctypes.data + off), P, _p(U))
    return U


def head_transformer(cfg: _Cfg, tc: _TCfg, Wf, layers, prefix_len, gamma, E, cond_tok, hrun):
    """Transformer head body on all rows.  Returns (u [M][d], y [M][d], hrun_after)."""
    M, d = cfg.B * cfg.L, cfg.d
    assert len(layers) == tc.D
    _chk(Wf, np.uint16, (d, 2 * d)); _chk(gamma, np.uint16, (d,)); _chk(E, np.uint16)
    prefix_len = _chk(np.ascontiguousarray(prefix_len, dtype=np.int32), np.int32, (cfg.B,))
    assert prefix_len.min() >= 0 and prefix_len.max() <= tc.P_max
    cond_tok = _chk(np.ascontiguousarray(cond_tok, dtype=np.int32), np.int32, (cfg.B,))
    hrun = np.array(_chk(np.ascontiguousarray(hrun, dtype=np.float64), np.float64, (M, d)))
    arr = _layer_arrays(tc, d, cfg.B, layers)
    u = np.empty((M, d)); y = np.empty((M, d))
    lib().orc_head_transformer(C.byref(cfg), C.byref(tc), _p(Wf), *[arr[f] for f in LAYER_FIELDS], _p(prefix_len),
                               _p(gamma), _p(E), _p(cond_tok), _p(hrun), _p(u), _p(y))
    return u, y, hrun


@dataclass
class TBody:
    """Transformer bodies of the K heads of a chain: layers[k][l] is a layer dict."""
    tcfg: _TCfg
    layers: Sequence
    prefix_len: np.ndarray


@dataclass
class ChainOut:
    z: np.ndarray            # [M][V] float64, final logit state
    hrun: np.ndarray         # [M][d] float64
    tok: np.ndarray          # [(K+1)][M]
    conf: np.ndarray
    lse: np.ndarray
    masked: np.ndarray
    revealed_at: np.ndarray
    cond_tok: np.ndarray
    protect_pos: np.ndarray
    draft_pos: np.ndarray    # [B][K+1]
    draft_tok: np.ndarray
    remasked: np.ndarray     # [(K+1)][M]
    y: Optional[np.ndarray]  # [K][M][d] LM-head operand (bf16-rounded when cfg.round_y)
    gap: np.ndarray          # [(K+1)][M] top-2 logit gap of every state
    x_tok: Optional[np.ndarray] = None   # [M] token recorded when a position was revealed (-1: none)


def chain_step(cfg: _Cfg, E, W_lm, heads: Sequence, z, hrun, masked=None, revealed_at=None,
               cond_tok=None, protect_pos=None, dump_y=False, x_tok=None, tbody: Optional[TBody] = None) -> ChainOut:
    """One chain step.  ``z`` [M][V] and ``hrun`` [M][d] float64 are copied, not modified.  With ``tbody``
    every head is (fuse projection W1, transformer layers, gamma); its W2 entry is ignored."""
    M, d, V, K, B = cfg.B * cfg.L, cfg.d, cfg.V, cfg.K, cfg.B
    assert len(heads) == K
    _chk(E, np.uint16); _chk(W_lm, np.uint16, (V, d))
    assert E.shape[1] == d
    z = np.array(_chk(np.ascontiguousarray(z, dtype=np.float64), np.float64, (M, V)))
    hrun = np.array(_chk(np.ascontiguousarray(hrun, dtype=np.float64), np.float64, (M, d)))
    for (w1, w2, g) in heads:
        _chk(w1, np.uint16, (d, 2 * d)); _chk(g, np.uint16, (d,))
        if tbody is None:
            _chk(w2, np.uint16, (d, d))
    PT = C.c_void_p * max(K, 1)
    w1s = PT(*[h[0].ctypes.data for h in heads])
    w2s = PT(*[h[1].ctypes.data for h in heads]) if tbody is None else None
    gs = PT(*[h[2].ctypes.data for h in heads])
    tok = np.full((K + 1, M), -1, np.int32); conf = np.zeros((K + 1, M)); lse = np.zeros((K + 1, M))
    masked = np.ones(M, np.uint8) if masked is None else np.array(masked, np.uint8)
    revealed_at = np.full(M, -1, np.int8) if revealed_at is None else np.array(revealed_at, np.int8)
    cond_tok = np.zeros(B, np.int32) if cond_tok is None else np.array(cond_tok, np.int32)
    protect_pos = np.full(B, -1, np.int32) if protect_pos is None else np.array(protect_pos, np.int32)
    assert cond_tok.min() >= 0 and cond_tok.max() < E.shape[0]
    dpos = np.empty((B, K + 1), np.int32); dtok = np.empty((B, K + 1), np.int32)
    rem = np.zeros((K + 1, M), np.uint8)
    y = np.empty((K, M, d)) if dump_y else None
    gap = np.full((K + 1, M), np.inf)
    x_tok = np.full(M, -1, np.int32) if x_tok is None else np.array(x_tok, np.int32)
    if tbody is None:
        lib().orc_chain_step(C.byref(cfg), _p(E), _p(W_lm), w1s, w2s, gs, _p(z), _p(hrun), _p(tok), _p(conf),
                             _p(lse), _p(masked), _p(revealed_at), _p(cond_tok), _p(protect_pos), _p(dpos),
                             _p(dtok), _p(rem), _p(y), _p(gap), _p(x_tok))
    else:
        tc = tbody.tcfg
        assert len(tbody.layers) == K and all(len(ls) == tc.D for ls in tbody.layers)
        flat = [l for ls in tbody.layers for l in ls]
        arr = _layer_arrays(tc, d, B, flat)
        plen = _chk(np.ascontiguousarray(tbody.prefix_len, dtype=np.int32), np.int32, (B,))
        assert plen.min() >= 0 and plen.max() <= tc.P_max
        tb = _TBodyC(C.pointer(tc), *[C.cast(arr[f], C.POINTER(C.c_void_p)) for f in LAYER_FIELDS],
                     C.c_void_p(plen.ctypes.data))
        lib().orc_chain_step_tf(C.byref(cfg), _p(E), _p(W_lm), w1s, gs, _p(z), _p(hrun), _p(tok), _p(conf),
                                _p(lse), _p(masked), _p(revealed_at), _p(cond_tok), _p(protect_pos), _p(dpos),
                                _p(dtok), _p(rem), _p(y), _p(gap), _p(x_tok), C.byref(tb))
    return ChainOut(z, hrun, tok, conf, lse, masked, revealed_at, cond_tok, protect_pos, dpos, dtok, rem, y, gap,
                    x_tok)


def token_prob(z, lse, x_tok) -> np.ndarray:
    """softmax(z[i])[x_tok[i]] per row (0 where x_tok[i] < 0)."""
    z = _chk(np.ascontiguousarray(z, dtype=np.float64), np.float64)
    M, V = z.shape
    lse = _chk(np.ascontiguousarray(lse, dtype=np.float64), np.float64, (M,))
    x_tok = _chk(np.ascontiguousarray(x_tok, dtype=np.int32), np.int32, (M,))
    p = np.empty(M)
    lib().orc_token_prob(_p(z), M, V, _p(lse), _p(x_tok), _p(p))
    return p


def commit(B, L, x_tok, revealed_at, masked, x_out):
    """End of a denoising step.  Returns (x_out, revealed_at, n_masked); inputs are copied."""
    M = B * L
    x_tok = _chk(np.ascontiguousarray(x_tok, dtype=np.int32), np.int32, (M,))
    revealed_at = np.array(revealed_at, np.int8); masked = np.array(masked, np.uint8)
    x_out = np.array(x_out, np.int32)
    n = np.empty(B, np.int32)
    lib().orc_commit(B, L, _p(x_tok), _p(revealed_at), _p(masked), _p(x_out), _p(n))
    return x_out, revealed_at, n


def decode_block(cfg: _Cfg, E, W_lm, heads: Sequence, backbone, max_steps=None):
    """Decode one block per sequence to completion (Algorithm 2 with tau >= 1 / r_min = r, Algorithm 4
    with tau_remask set): every denoising step asks ``backbone(step, x_out, masked)`` for the
    prior logits z [M][V] and hidden states h [M][d] of that step, runs one chain step on the
    still-masked positions, and commits what it revealed.  Returns (x_out, steps, history) where
    history[t] is the ChainOut of step t."""
    B, L = cfg.B, cfg.L
    M = B * L
    x_out = np.full(M, -1, np.int32)
    masked = np.ones(M, np.uint8)
    revealed_at = np.full(M, -1, np.int8)
    history = []
    max_steps = L if max_steps is None else max_steps
    steps = 0
    step_cfg = _Cfg.from_buffer_copy(cfg)
    step_cfg.fresh_block = 0
    while masked.any() and steps < max_steps:
        z, h = backbone(steps, x_out.copy(), masked.copy())
        out = chain_step(step_cfg, E, W_lm, heads, z, h, masked=masked, revealed_at=revealed_at)
        x_out, revealed_at, _ = commit(B, L, out.x_tok, out.revealed_at, out.masked, x_out)
        masked = out.masked
        history.append(out)
        steps += 1
    return x_out, steps, history
