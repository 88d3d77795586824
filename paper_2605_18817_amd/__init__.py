"""MI355X-native MRP chain step: thin Python binding over the C-ABI HIP library.

Everything the chain computes runs in ``libmrp.so`` (``csrc/*.hip``); this
package only marshals arguments.  PyTorch is used for device memory and
streams.  There is no CPU fallback: without the built library, or without a
GPU, calls fail loudly.
"""
from .binding import (MrpContext, RevealCfg, StepIO, Head, TLayer, load_library, library_path,  # noqa: F401
                      MrpError, pack_weight, packed_bytes, verify_accept_static, EXPORTED_SYMBOLS)
