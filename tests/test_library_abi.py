"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-only entry points behave (no GPU, no compute calls)."""
import ctypes
import os
import re

import paper_2605_18817_amd as mrp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "mrp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mrp_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = mrp.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(mrp.EXPORTED_SYMBOLS) == declared


def test_host_only_entry_points():
    lib = mrp.load_library()
    assert lib.mrp_packed_bytes(100, 64) == 128 * 64 * 2          # rows padded to a multiple of 32
    assert lib.mrp_packed_bytes(32, 10) == 0                      # columns must be a multiple of 16
    assert lib.mrp_pack_weight(None, None, 32, 16, None) == -1    # NULL pointers are rejected before any launch
    assert lib.mrp_last_error(None) == b"null context"
    assert lib.mrp_destroy(None) == -1
    h = ctypes.c_void_p()
    assert lib.mrp_create(ctypes.byref(h), None) == -1
    # every other entry point refuses a NULL context (or NULL buffers) before anything is launched
    assert lib.mrp_pack_body_weight(None, None, 32, 16, None) == -1
    assert lib.mrp_tbody_create(None, None) == -1
    assert lib.mrp_chain_step(None, None, 1, 0, None, None, None, None, None, None, None, None) == -1
    assert lib.mrp_chain_step_tf(None, None, 1, 0, None, None, None, None, None, None, None, None, None, None) == -1
    assert lib.mrp_kl_loss(None, None, 1, None, None, None, 1.0, None, None) == -1
    assert lib.mrp_residual_rms(None, None, 1, 5, 64, None, 0, None, None) == -1
    assert lib.mrp_commit(None, None, 1, None, None, None, None, None) == -1
    assert lib.mrp_profile_enable(None, 1) == -1


def test_no_cpu_fallback_without_gpu():
    import pytest
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(mrp.MrpError):
        mrp.MrpContext(256, 4096, 4, 4)
