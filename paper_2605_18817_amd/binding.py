"""ctypes binding of include/mrp.h — same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

from . import build as _build

EXPORTED_SYMBOLS = [
    "mrp_create", "mrp_destroy", "mrp_workspace_bytes", "mrp_last_error", "mrp_packed_bytes",
    "mrp_pack_weight", "mrp_pack_body_weight", "mrp_chain_step", "mrp_remask", "mrp_commit", "mrp_verify_accept", "mrp_verify_accept_joint", "mrp_kl_loss", "mrp_residual_rms", "mrp_tbody_create", "mrp_chain_step_tf",
    "mrp_profile_enable", "mrp_profile_read", "mrp_verify_accept_static", "mrp_verify_accept_static_scratch_bytes",
    "mrp_build_candidates", "mrp_poll_error", "mrp_probe_lm_traffic",
]

MRP_MAX_HEADS = 16


class MrpError(RuntimeError):
    pass


class _Dims(C.Structure):
    _fields_ = [("d", C.c_int), ("V", C.c_int), ("max_rows", C.c_int), ("block_len", C.c_int),
                ("rms_eps", C.c_float)]


class _Head(C.Structure):
    _fields_ = [("W1_packed", C.c_void_p), ("W2_packed", C.c_void_p), ("gamma", C.c_void_p)]


class _TBodyDims(C.Structure):
    _fields_ = [("D", C.c_int), ("n_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("d_ff", C.c_int), ("max_prefix", C.c_int), ("rope_theta", C.c_float)]


class _TLayer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Wqkv_packed", "Wo_packed", "Wgu_packed", "Wdown_packed", "g1", "g2",
                                          "k_cache", "v_cache")]


class _RevealCfg(C.Structure):
    _fields_ = [("tau", C.c_float), ("r_min", C.c_int), ("max_accept", C.c_int), ("carry_hidden", C.c_int),
                ("tau_remask", C.c_float), ("head_reveal", C.c_int), ("fresh_block", C.c_int),
                ("state_offset", C.c_int), ("run_state0", C.c_int), ("remask_mode", C.c_int)]


class _StepIO(C.Structure):
    _fields_ = [("tok", C.c_void_p), ("conf", C.c_void_p), ("lse", C.c_void_p), ("revealed_at", C.c_void_p),
                ("masked", C.c_void_p), ("cond_tok", C.c_void_p), ("protect_pos", C.c_void_p),
                ("draft_pos", C.c_void_p), ("draft_tok", C.c_void_p), ("remasked", C.c_void_p),
                ("x_tok", C.c_void_p)]


_lib = None


def library_path() -> str:
    return _build.LIB


def load_library():
    """Load the built library (building it only if no library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    lib = C.CDLL(_build.LIB)
    lib.mrp_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_Dims)]
    lib.mrp_destroy.argtypes = [C.c_void_p]
    lib.mrp_workspace_bytes.argtypes = [C.POINTER(_Dims)]
    lib.mrp_workspace_bytes.restype = C.c_size_t
    lib.mrp_last_error.argtypes = [C.c_void_p]
    lib.mrp_last_error.restype = C.c_char_p
    lib.mrp_packed_bytes.argtypes = [C.c_int, C.c_int]
    lib.mrp_packed_bytes.restype = C.c_size_t
    lib.mrp_pack_weight.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.mrp_pack_body_weight.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.mrp_chain_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.POINTER(_Head), C.c_void_p, C.POINTER(_RevealCfg),
                                   C.POINTER(_StepIO)]
    lib.mrp_remask.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_float, C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_void_p]
    lib.mrp_verify_accept_joint.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.mrp_kl_loss.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                C.c_void_p, C.c_void_p]
    lib.mrp_residual_rms.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_long, C.c_void_p, C.c_int,
                                     C.c_void_p, C.c_void_p]
    lib.mrp_tbody_create.argtypes = [C.c_void_p, C.POINTER(_TBodyDims)]
    lib.mrp_chain_step_tf.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.POINTER(_Head), C.POINTER(_TLayer), C.c_void_p, C.c_void_p,
                                      C.POINTER(_RevealCfg), C.POINTER(_StepIO)]
    lib.mrp_commit.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.c_void_p]
    lib.mrp_verify_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.mrp_verify_accept_static.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.mrp_verify_accept_static_scratch_bytes.restype = C.c_size_t
    lib.mrp_build_candidates.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int, C.c_int32, C.c_void_p, C.c_void_p]
    lib.mrp_poll_error.argtypes = [C.c_void_p, C.c_void_p]
    lib.mrp_probe_lm_traffic.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.mrp_profile_enable.argtypes = [C.c_void_p, C.c_int]
    lib.mrp_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None stays NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MrpError("tensor must be a contiguous device tensor")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def packed_bytes(rows: int, cols: int) -> int:
    return load_library().mrp_packed_bytes(rows, cols)


def pack_weight(w, body: bool = False):
    """bf16 (or int16 bit pattern) device tensor [rows][cols] -> packed device tensor (uint8).
    body=True: a head-body weight (converted to fp16 while packing); False: the LM head."""
    import torch
    rows, cols = w.shape
    n = packed_bytes(rows, cols)
    if n == 0:
        raise MrpError(f"cannot pack a {rows}x{cols} matrix (cols must be a multiple of 16)")
    out = torch.empty(n, dtype=torch.uint8, device=w.device)
    fn = load_library().mrp_pack_body_weight if body else load_library().mrp_pack_weight
    rc = fn(_stream(), _ptr(w), rows, cols, _ptr(out))
    if rc != 0:
        raise MrpError(f"mrp_pack_weight failed: {rc}")
    return out


def verify_accept_static(B: int, L: int, V: int, K: int, verify, draft_pos, draft_tok, draft_stride: int, match,
                         accept_len, correction_tok) -> int:
    """mrp_verify_accept_static: no context, no allocation; returns the status code."""
    return load_library().mrp_verify_accept_static(_stream(), B, L, V, K, _ptr(verify), _ptr(draft_pos),
                                                   _ptr(draft_tok), draft_stride, _ptr(match), _ptr(accept_len),
                                                   _ptr(correction_tok))


@dataclass
class Head:
    W1_packed: object
    W2_packed: object
    gamma: object


@dataclass
class TLayer:
    """One transformer layer of a head body (device tensors; weights packed with pack_weight(body=True))."""
    Wqkv_packed: object
    Wo_packed: object
    Wgu_packed: object
    Wdown_packed: object
    g1: object
    g2: object
    k_cache: object
    v_cache: object


@dataclass
class RevealCfg:
    tau: float = 0.9
    r_min: int = 1
    max_accept: int = 0
    carry_hidden: int = 1
    tau_remask: float = -1.0
    head_reveal: int = 1
    fresh_block: int = 1
    state_offset: int = 0
    run_state0: int = 1
    remask_mode: int = 0


class StepIO:
    """Device buffers of one chain step (allocated with torch)."""

    def __init__(self, B: int, L: int, K: int, device="cuda"):
        import torch
        M = B * L
        self.B, self.L, self.K = B, L, K
        self.tok = torch.full((K + 1, M), -1, dtype=torch.int32, device=device)
        self.conf = torch.zeros((K + 1, M), dtype=torch.float32, device=device)
        self.lse = torch.zeros((K + 1, M), dtype=torch.float32, device=device)
        self.revealed_at = torch.full((M,), -1, dtype=torch.int8, device=device)
        self.masked = torch.ones((M,), dtype=torch.uint8, device=device)
        self.cond_tok = torch.zeros((B,), dtype=torch.int32, device=device)
        self.protect_pos = torch.full((B,), -1, dtype=torch.int32, device=device)
        self.draft_pos = torch.full((B, K + 1), -1, dtype=torch.int32, device=device)
        self.draft_tok = torch.full((B, K + 1), -1, dtype=torch.int32, device=device)
        self.remasked = torch.zeros((K + 1, M), dtype=torch.uint8, device=device)
        self.x_tok = torch.full((M,), -1, dtype=torch.int32, device=device)

    def c_struct(self) -> _StepIO:
        return _StepIO(_ptr(self.tok), _ptr(self.conf), _ptr(self.lse), _ptr(self.revealed_at), _ptr(self.masked),
                       _ptr(self.cond_tok), _ptr(self.protect_pos), _ptr(self.draft_pos), _ptr(self.draft_tok),
                       _ptr(self.remasked), _ptr(self.x_tok))


class MrpContext:
    """Owns an ``mrp_ctx`` (workspace) for fixed (d, V, max_rows, block_len)."""

    def __init__(self, d: int, V: int, max_rows: int, block_len: int, rms_eps: float = 1e-6):
        import torch
        if not torch.cuda.is_available():
            raise MrpError("no GPU: the MRP chain has no CPU path")
        self.lib = load_library()
        self.d, self.V, self.max_rows, self.L = d, V, max_rows, block_len
        self._dims = _Dims(d, V, max_rows, block_len, rms_eps)
        h = C.c_void_p()
        rc = self.lib.mrp_create(C.byref(h), C.byref(self._dims))
        if rc != 0:
            raise MrpError(f"mrp_create failed: {rc}")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self.lib.mrp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self) -> int:
        return self.lib.mrp_workspace_bytes(C.byref(self._dims))

    def last_error(self) -> str:
        return self.lib.mrp_last_error(self._h).decode()

    def _check(self, rc: int, what: str):
        if rc < 0:
            raise MrpError(f"{what} failed ({rc}): {self.last_error()}")
        return rc

    def chain_step(self, B: int, K: int, h, h_run, E, W_lm_packed, heads: Sequence[Head], z, cfg: RevealCfg,
                   io: StepIO, check: bool = True) -> int:
        harr = (_Head * max(len(heads), 1))(*[_Head(_ptr(x.W1_packed), _ptr(x.W2_packed), _ptr(x.gamma))
                                              for x in heads])
        if len(heads) < K <= MRP_MAX_HEADS:
            raise MrpError("fewer heads than K")
        ccfg = _RevealCfg(cfg.tau, cfg.r_min, cfg.max_accept, cfg.carry_hidden, cfg.tau_remask, cfg.head_reveal,
                          cfg.fresh_block, cfg.state_offset, cfg.run_state0, cfg.remask_mode)
        cio = io.c_struct()
        rc = self.lib.mrp_chain_step(self._h, _stream(), B, K, _ptr(h), _ptr(h_run), _ptr(E), _ptr(W_lm_packed),
                                     harr, _ptr(z), C.byref(ccfg), C.byref(cio))
        return self._check(rc, "mrp_chain_step") if check else rc

    def tbody_create(self, D: int, n_heads: int, n_kv_heads: int, d_ff: int, max_prefix: int,
                     rope_theta: float = 1.0e6, head_dim: int = 128, check: bool = True) -> int:
        dims = _TBodyDims(D, n_heads, n_kv_heads, head_dim, d_ff, max_prefix, rope_theta)
        rc = self.lib.mrp_tbody_create(self._h, C.byref(dims))
        return self._check(rc, "mrp_tbody_create") if check else rc

    def chain_step_tf(self, B: int, K: int, h, h_run, E, W_lm_packed, heads: Sequence[Head],
                      layers: Sequence[TLayer], prefix_len, z, cfg: RevealCfg, io: StepIO, check: bool = True) -> int:
        """layers: K * D entries, head k's layer l at [k * D + l]."""
        harr = (_Head * max(len(heads), 1))(*[_Head(_ptr(x.W1_packed), _ptr(x.W2_packed), _ptr(x.gamma))
                                              for x in heads])
        larr = (_TLayer * max(len(layers), 1))(*[
            _TLayer(_ptr(l.Wqkv_packed), _ptr(l.Wo_packed), _ptr(l.Wgu_packed), _ptr(l.Wdown_packed), _ptr(l.g1),
                    _ptr(l.g2), _ptr(l.k_cache), _ptr(l.v_cache)) for l in layers])
        if len(heads) < K <= MRP_MAX_HEADS:
            raise MrpError("fewer heads than K")
        ccfg = _RevealCfg(cfg.tau, cfg.r_min, cfg.max_accept, cfg.carry_hidden, cfg.tau_remask, cfg.head_reveal,
                          cfg.fresh_block, cfg.state_offset, cfg.run_state0, cfg.remask_mode)
        cio = io.c_struct()
        rc = self.lib.mrp_chain_step_tf(self._h, _stream(), B, K, _ptr(h), _ptr(h_run), _ptr(E), _ptr(W_lm_packed),
                                        harr, larr if len(layers) else None, _ptr(prefix_len), _ptr(z),
                                        C.byref(ccfg), C.byref(cio))
        return self._check(rc, "mrp_chain_step_tf") if check else rc

    def remask(self, B: int, state: int, conf_new, tau_remask: float, protect_pos, revealed_at, masked,
               remasked_out, check: bool = True) -> int:
        rc = self.lib.mrp_remask(self._h, _stream(), B, state, _ptr(conf_new), tau_remask, _ptr(protect_pos),
                                 _ptr(revealed_at), _ptr(masked), _ptr(remasked_out))
        return self._check(rc, "mrp_remask") if check else rc

    def commit(self, B: int, x_tok, revealed_at, masked, x_out, n_masked, check: bool = True) -> int:
        rc = self.lib.mrp_commit(self._h, _stream(), B, _ptr(x_tok), _ptr(revealed_at), _ptr(masked), _ptr(x_out),
                                 _ptr(n_masked))
        return self._check(rc, "mrp_commit") if check else rc

    def decode_block(self, B: int, K: int, backbone, E, W_lm_packed, heads: Sequence[Head], cfg: RevealCfg,
                     max_steps: Optional[int] = None):
        """Decode one block per sequence to completion: each denoising step takes the prior logits
        ``z`` (fp32 [M][V], device) and hidden states ``h`` (bf16 [M][d], device) from
        ``backbone(step, x_out, masked)``, runs one chain step on the still-masked rows and commits
        what it revealed (mrp_commit).  Only the count of masked rows comes back to the host, once
        per step, to end the loop.  Returns (x_out [M] int32 device, steps, io)."""
        import torch
        L = self.L
        M = B * L
        io = StepIO(B, L, K)
        x_out = torch.full((M,), -1, dtype=torch.int32, device="cuda")
        n_masked = torch.empty((B,), dtype=torch.int32, device="cuda")
        h_run = torch.empty((M, self.d), dtype=torch.float32, device="cuda")
        step_cfg = RevealCfg(**{**cfg.__dict__, "fresh_block": 0})
        max_steps = L if max_steps is None else max_steps
        steps = 0
        while steps < max_steps:
            z, h = backbone(steps, x_out, io.masked)
            self.chain_step(B, K, h, h_run, E, W_lm_packed, heads, z, step_cfg, io)
            self.commit(B, io.x_tok, io.revealed_at, io.masked, x_out, n_masked)
            steps += 1
            if int(n_masked.sum().item()) == 0:
                break
        return x_out, steps, io

    def verify_accept(self, B: int, K: int, verify, draft_pos, draft_tok, draft_stride: int, match, accept_len,
                      correction_tok, check: bool = True) -> int:
        rc = self.lib.mrp_verify_accept(self._h, _stream(), B, K, _ptr(verify), _ptr(draft_pos), _ptr(draft_tok),
                                        draft_stride, _ptr(match), _ptr(accept_len), _ptr(correction_tok))
        return self._check(rc, "mrp_verify_accept") if check else rc

    def verify_accept_joint(self, B: int, K: int, verify, draft_pos, draft_tok, draft_stride: int, match,
                            accept_len, correction_tok, check: bool = True) -> int:
        rc = self.lib.mrp_verify_accept_joint(self._h, _stream(), B, K, _ptr(verify), _ptr(draft_pos),
                                              _ptr(draft_tok), draft_stride, _ptr(match), _ptr(accept_len),
                                              _ptr(correction_tok))
        return self._check(rc, "mrp_verify_accept_joint") if check else rc

    def build_candidates(self, B: int, K: int, x_t, masked_t, draft_pos, draft_tok, draft_stride: int,
                         mask_token: int, cand_tok, cand_masked, check: bool = True) -> int:
        rc = self.lib.mrp_build_candidates(self._h, _stream(), B, K, _ptr(x_t), _ptr(masked_t), _ptr(draft_pos),
                                           _ptr(draft_tok), draft_stride, mask_token, _ptr(cand_tok),
                                           _ptr(cand_masked))
        return self._check(rc, "mrp_build_candidates") if check else rc

    def probe_lm_traffic(self, mode: int, M: int, W_lm_packed, z, check: bool = True) -> int:
        rc = self.lib.mrp_probe_lm_traffic(self._h, _stream(), mode, M, _ptr(W_lm_packed), _ptr(z))
        return self._check(rc, "mrp_probe_lm_traffic") if check else rc

    def poll_error(self) -> int:
        """Wait for the current stream; bits of the device error word set since the last poll (cleared)."""
        return self._check(self.lib.mrp_poll_error(self._h, _stream()), "mrp_poll_error")

    def kl_loss(self, M: int, teacher, student, row_mask, scale: float, loss_rows, grad=None,
                check: bool = True) -> int:
        rc = self.lib.mrp_kl_loss(self._h, _stream(), M, _ptr(teacher), _ptr(student), _ptr(row_mask), scale,
                                  _ptr(loss_rows), _ptr(grad))
        return self._check(rc, "mrp_kl_loss") if check else rc

    def residual_rms(self, n_blocks: int, S: int, N: int, X, bf16: bool, rms_pair, rms_delta,
                     check: bool = True) -> int:
        rc = self.lib.mrp_residual_rms(self._h, _stream(), n_blocks, S, N, _ptr(X), 1 if bf16 else 0,
                                       _ptr(rms_pair), _ptr(rms_delta))
        return self._check(rc, "mrp_residual_rms") if check else rc

    def profile_enable(self, on: bool):
        self._check(self.lib.mrp_profile_enable(self._h, 1 if on else 0), "mrp_profile_enable")

    def profile_read(self, cap: int = 4096) -> List[float]:
        buf = (C.c_float * cap)()
        n = self._check(self.lib.mrp_profile_read(self._h, buf, cap), "mrp_profile_read")
        return [buf[i] for i in range(n)]
